"""Seeded synthetic vocabularies (token byte strings in CSR form).

Two recipes:

* ``arith``: 1024 distinct tokens of 1-4 bytes, bytes uniform over the
  15-symbol alphabet ``0-9+*() ``; always contains the 15 one-symbol tokens
  and one zero-byte stop token.
* ``bpe``: a BPE-shaped vocabulary: all 256 single bytes, one zero-byte stop
  token, the rest drawn with length ~ truncated geometric on 1..16 (draw
  parameter 0.30; after de-duplication saturates the short lengths the
  realised mean is about 5 bytes) and byte content 70 % ASCII letters with an optional leading
  space, 20 % punctuation/digits, 10 % multibyte UTF-8 text (2-4 byte
  characters, one in ten cut in the middle of a character); de-duplicated.

Token ids are a seeded random permutation, so id order is unrelated to byte
order (as in a real tokenizer).
"""

from __future__ import annotations

from dataclasses import dataclass
from functools import lru_cache

import numpy as np

ARITH_ALPHABET = b"0123456789+*() "
_LETTERS = b"abcdefghijklmnopqrstuvwxyzABCDEFGHIJKLMNOPQRSTUVWXYZ"
_PUNCT = b"!\"#$%&'()*+,-./:;<=>?@[\\]^_`{|}~0123456789"
_MAX_LEN = 16
_GEOM_P = 0.30


@dataclass(frozen=True)
class Vocab:
    data: np.ndarray      # uint8, all token bytes back to back (id order)
    offsets: np.ndarray   # int64 [V+1]
    stop_ids: np.ndarray  # int32

    @property
    def size(self) -> int:
        return int(self.offsets.shape[0] - 1)

    def token(self, i: int) -> bytes:
        return self.data[self.offsets[i]:self.offsets[i + 1]].tobytes()

    def tokens(self) -> list:
        d = self.data.tobytes()
        o = self.offsets
        return [d[o[i]:o[i + 1]] for i in range(self.size)]


def _pack(tokens: list, stop_ids: list) -> Vocab:
    lens = np.fromiter((len(t) for t in tokens), dtype=np.int64, count=len(tokens))
    offsets = np.zeros(len(tokens) + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    data = np.frombuffer(b"".join(tokens), dtype=np.uint8).copy()
    return Vocab(data=data, offsets=offsets, stop_ids=np.asarray(stop_ids, dtype=np.int32))


def _random_codepoint(rng: np.random.Generator) -> int:
    k = int(rng.integers(0, 3))
    if k == 0:
        return int(rng.integers(0x80, 0x800))
    if k == 1:
        while True:
            c = int(rng.integers(0x800, 0x10000))
            if not (0xD800 <= c <= 0xDFFF):
                return c
    return int(rng.integers(0x10000, 0x110000))


def _draw_bpe_token(rng: np.random.Generator) -> bytes:
    # truncated geometric length on 1.._MAX_LEN
    while True:
        n = int(rng.geometric(_GEOM_P))
        if n <= _MAX_LEN:
            break
    u = rng.random()
    if u < 0.70:
        lead = n >= 2 and rng.random() < 0.5
        k = n - 1 if lead else n
        body = bytes(_LETTERS[j] for j in rng.integers(0, len(_LETTERS), size=k))
        return (b" " + body) if lead else body
    if u < 0.90:
        return bytes(_PUNCT[j] for j in rng.integers(0, len(_PUNCT), size=n))
    out = b""
    while len(out) < max(n, 2):
        enc = chr(_random_codepoint(rng)).encode("utf-8")
        if len(out) + len(enc) > _MAX_LEN:
            break
        out += enc
    if not out:
        out = chr(_random_codepoint(rng)).encode("utf-8")
    if rng.random() < 0.1 and len(out) >= 2:
        out = out[:-1]  # cut inside the last character
    return out


@lru_cache(maxsize=8)
def make_vocab(kind: str, size: int, seed: int = 0) -> Vocab:
    """Build a vocabulary of ``size`` tokens (including one stop token)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    seen = set()
    toks = []
    if kind == "arith":
        for b in ARITH_ALPHABET:
            t = bytes([b])
            seen.add(t)
            toks.append(t)
        while len(toks) < size - 1:
            n = int(rng.integers(1, 5))
            t = bytes(ARITH_ALPHABET[j] for j in rng.integers(0, len(ARITH_ALPHABET), size=n))
            if t not in seen:
                seen.add(t)
                toks.append(t)
    elif kind == "bpe":
        if size < 258:
            raise ValueError("bpe vocabulary needs at least 258 tokens")
        for b in range(256):
            t = bytes([b])
            seen.add(t)
            toks.append(t)
        while len(toks) < size - 1:
            t = _draw_bpe_token(rng)
            if t not in seen:
                seen.add(t)
                toks.append(t)
    else:
        raise ValueError(f"unknown vocabulary kind {kind!r}")
    toks.append(b"")  # the stop token has no bytes
    perm = rng.permutation(size)
    shuffled = [None] * size
    for src, dst in enumerate(perm):
        shuffled[int(dst)] = toks[src]
    stop = int(perm[size - 1])
    return _pack(shuffled, [stop])
