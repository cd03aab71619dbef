"""The fill entry point that allocates nothing (xgm_fill_next_token_bitmask_static:
per-call staging in a fixed array of device memory) against the entry point it
is a variant of, bit for bit and against the oracle, on two calls in a row, the
second with a smaller batch; then its size limit."""

import numpy as np
import pytest

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _stream():
    return int(torch.cuda.current_stream().cuda_stream)


def test_static_staging_fill_equals_the_allocating_fill_twice_in_a_row():
    import paper_2411_15100_amd as xgm
    from paper_2411_15100_amd import workloads as wl

    vocab = si.make_vocab("bpe", 32000, 0)
    xv = wl.make_xgm_vocab(vocab)
    texts = [si.JSON_GRAMMAR, si.make_schema_grammar(2, string_heavy=True), si.JSON_GRAMMAR, si.make_schema_grammar(4)]
    caches = [xgm.Cache(xgm.Grammar(t, "root"), xv) for t in texts]
    B, W = 12, xgm.bitmask_words(vocab.size)
    walker = wl.BatchWalker([caches[b % 4] for b in range(B)], vocab, seed=31, structural_bias=0.4)
    oms = [oracle.EarleyMatcher(oracle.Grammar(texts[b % 4], "root")) for b in range(B)]
    toks = vocab.tokens()
    for step in range(14):           # rows in different states, several of them inside strings
        picks = walker.step()
        for b in range(B):
            if not walker.history[b]:
                oms[b] = oracle.EarleyMatcher(oracle.Grammar(texts[b % 4], "root"))
            else:
                assert oms[b].advance(toks[int(picks[b])])
    before = xgm.overflow_total()
    want = oracle.pack_bitmask(np.stack([om.mask(vocab) for om in oms]))
    d_ref = torch.full((B, W), -1, dtype=torch.int32, device="cuda")
    d_new = torch.full((B, W), -1, dtype=torch.int32, device="cuda")
    # first call: the whole batch
    xgm.fill_next_token_bitmask(walker.matchers, d_ref.data_ptr(), _stream())
    xgm.fill_next_token_bitmask_static(walker.matchers, d_new.data_ptr(), _stream())
    torch.cuda.synchronize()
    assert np.array_equal(d_new.cpu().numpy(), d_ref.cpu().numpy())
    assert np.array_equal(d_new.cpu().numpy(), want)
    # second call, right after the first, with a smaller batch (rows 7, 2, 9, 4, 0): what the first call left in the
    # staging array must not matter
    rows = [7, 2, 9, 4, 0]
    sub = [walker.matchers[b] for b in rows]
    d_ref.fill_(-1)
    d_new.fill_(-1)
    xgm.fill_next_token_bitmask_static(sub, d_new.data_ptr(), _stream())
    xgm.fill_next_token_bitmask(sub, d_ref.data_ptr(), _stream())
    torch.cuda.synchronize()
    got = d_new.cpu().numpy()
    assert np.array_equal(got, d_ref.cpu().numpy())
    assert np.array_equal(got[:len(rows)], want[rows])
    assert (got[len(rows):] == -1).all()          # rows beyond the batch are not written
    # a third and a fourth call back to back on the stream, no synchronisation in between
    d_a = torch.full((B, W), -1, dtype=torch.int32, device="cuda")
    xgm.fill_next_token_bitmask_static(walker.matchers, d_a.data_ptr(), _stream())
    xgm.fill_next_token_bitmask_static(sub, d_new.data_ptr(), _stream())
    torch.cuda.synchronize()
    assert np.array_equal(d_a.cpu().numpy(), want)
    assert np.array_equal(d_new.cpu().numpy()[:len(rows)], want[rows])
    assert xgm.overflow_total() == before


def test_static_staging_fill_rejects_what_does_not_fit():
    import paper_2411_15100_amd as xgm
    from paper_2411_15100_amd import workloads as wl

    vocab = si.make_vocab("bpe", 32000, 0)
    cache = xgm.Cache(xgm.Grammar(si.JSON_GRAMMAR, "root"), wl.make_xgm_vocab(vocab))
    m = xgm.Matcher(cache=cache)
    m.accept_bytes(b"[" * 1800)                    # 1800 or more frames in one stack
    B = 400                                        # 400 x 1800 frames x 2 bytes > 1 MiB
    W = xgm.bitmask_words(vocab.size)
    d = torch.full((B, W), -1, dtype=torch.int32, device="cuda")
    with pytest.raises(xgm.XgmError) as e:
        xgm.fill_next_token_bitmask_static([m] * B, d.data_ptr(), _stream())
    assert e.value.status == -9 and "static" in str(e.value)
    torch.cuda.synchronize()
    assert (d.cpu().numpy() == -1).all()           # nothing was enqueued
    xgm.fill_next_token_bitmask([m] * B, d.data_ptr(), _stream())     # the allocating entry point takes it
    om = oracle.EarleyMatcher(oracle.Grammar(si.JSON_GRAMMAR, "root"))
    assert om.advance(b"[" * 1800)
    assert np.array_equal(d.cpu().numpy(), np.tile(oracle.pack_bitmask(om.mask(vocab)), (B, 1)))
