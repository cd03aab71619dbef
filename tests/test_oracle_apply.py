"""Pins for the oracle's bitmask packing and -inf apply (section 2.1)."""

import numpy as np

import oracle


def test_pack_layout_by_hand():
    allowed = np.zeros(70, dtype=bool)
    allowed[[0, 1, 31, 32, 69]] = True
    w = oracle.pack_bitmask(allowed).view(np.uint32)
    assert w.shape == (3,)
    assert w[0] == (1 | 2 | (1 << 31)) and w[1] == 1 and w[2] == (1 << 5)
    assert np.array_equal(oracle.unpack_bitmask(w.view(np.int32), 70), allowed)


def test_apply_by_hand_bf16_patterns():
    # bf16 bit patterns: 1.0, -0.0, +inf, NaN, smallest subnormal, -2.5
    bits = np.array([[0x3F80, 0x8000, 0x7F80, 0x7FC1, 0x0001, 0xC020]], dtype=np.uint16)
    allowed = np.array([[True, False, True, True, False, True]])
    out = oracle.apply_mask(bits, allowed, 0xFF80)
    assert out.tolist() == [[0x3F80, 0xFF80, 0x7F80, 0x7FC1, 0xFF80, 0xC020]]
    # fp32, with a logits row wider than the mask: the extra columns are masked
    b32 = np.array([[0x3F800000, 0x7FC00001, 0x00000001, 0x80000000]], dtype=np.uint32)
    out = oracle.apply_mask(b32, np.array([[True, True, False]]), 0xFF800000)
    assert out.tolist() == [[0x3F800000, 0x7FC00001, 0xFF800000, 0xFF800000]]
    assert np.float32(np.array([0xFF800000], dtype=np.uint32).view(np.float32)[0]) == -np.inf
