"""GPU parity at the benchmark's full size: the serving decode step (batch 128,
vocabulary 151936, 128 distinct string-heavy schema grammars) in the launch
configuration that bench.py times, checked on sampled rows against the oracle's
brute-force Earley masks, and apply checked on the whole batch by definition."""

import sys

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_serving_step_full_size_sampled_rows():
    import paper_2411_15100_amd as xgm
    from paper_2411_15100_amd import workloads as wl

    before = xgm.overflow_total()
    say("serving workload: building 128 caches at V=151936 (one state set)")
    work = wl.ServingWorkload(pool=1, n_logit_buffers=1, log=lambda *a: None)
    stream = wl.current_stream()
    work.fill(0, stream)
    torch.cuda.synchronize()
    words = work.d_mask.cpu().numpy()
    w = work.sets[0]
    toks = work.vocab.tokens()
    entries = np.array([sum(c.num_uncertain(m.stack(s)[-1]) for s in range(m.num_stacks()))
                        for m, c in zip(w.matchers, work.caches)])
    # the rows with the longest context-dependent lists, the deepest stacks, and a seeded sample of the rest
    rng = np.random.Generator(np.random.PCG64(99))
    depth = np.array([w.depth(b) for b in range(work.B)])
    rows = sorted(set(np.argsort(-entries)[:4].tolist()) | set(np.argsort(-depth)[:2].tolist())
                  | set(int(x) for x in rng.choice(work.B, size=6, replace=False)))
    threads = oracle.default_threads()
    allowed_rows = {}
    oracle_rows = {}
    for b in rows:
        og = oracle.Grammar(work.texts[b], "root")
        om = oracle.EarleyMatcher(og)
        for t in w.history[b]:
            assert om.advance(toks[t])
        want = om.mask(work.vocab, threads)
        assert np.array_equal(words[b], oracle.pack_bitmask(want)), f"row {b}"
        allowed_rows[b] = want
        oracle_rows[b] = om
        say(f"  row {b}: {int(entries[b])} list entries, depth {int(depth[b])}, {int(want.sum())} allowed: bit-exact")
    # properties that hold for every row: bits beyond V are zero, zero-byte tokens are never allowed
    V, W = work.V, work.W
    bits = np.unpackbits(words.view(np.uint8), axis=1, bitorder="little")
    assert not bits[:, V:].any()
    empty = np.array([len(t) == 0 for t in toks])
    stop = np.zeros(V, dtype=bool)
    stop[work.vocab.stop_ids] = True
    assert not bits[:, :V][:, empty & ~stop].any()
    # apply on the whole batch: by definition, from the mask the kernel produced
    t = work.logits[0]
    view = t.view(torch.int16)
    old = view.cpu().numpy().view(np.uint16).copy()
    work.apply(0, stream)
    torch.cuda.synchronize()
    new = view.cpu().numpy().view(np.uint16)
    want = oracle.apply_mask(old, bits[:, :V].astype(bool), 0xFF80)
    assert np.array_equal(new, want)
    # the fused call on fresh logits: same mask, same logits
    work.refresh_logits()
    torch.cuda.synchronize()
    old = view.cpu().numpy().view(np.uint16).copy()
    d_mask2 = torch.full_like(work.d_mask, -1)
    xgm.fill_and_apply(w.batch, d_mask2.data_ptr(), t.data_ptr(), xgm.DTYPE_BF16, V, t.stride(0), stream=stream)
    torch.cuda.synchronize()
    assert np.array_equal(d_mask2.cpu().numpy(), words)
    assert np.array_equal(view.cpu().numpy().view(np.uint16), oracle.apply_mask(old, bits[:, :V].astype(bool), 0xFF80))
    # the same states resident on the device: one launch, no packing, same mask and logits
    work.refresh_logits()
    torch.cuda.synchronize()
    old = view.cpu().numpy().view(np.uint16).copy()
    d_mask2.fill_(-1)
    work.device_sets[0].fill_next_token_bitmask(d_mask2.data_ptr(), stream)
    assert np.array_equal(d_mask2.cpu().numpy(), words)
    d_mask2.fill_(-1)
    work.device_sets[0].fill_and_apply(d_mask2.data_ptr(), t.data_ptr(), xgm.DTYPE_BF16, V, t.stride(0), stream=stream)
    torch.cuda.synchronize()
    assert np.array_equal(d_mask2.cpu().numpy(), words)
    assert np.array_equal(view.cpu().numpy().view(np.uint16), oracle.apply_mask(old, bits[:, :V].astype(bool), 0xFF80))
    # one decode step of the whole batch on the device: every row accepts a token of its mask
    # (stop tokens aside), states and next masks equal the host matchers', sampled rows the oracle's
    import synth_inputs as si
    allowed = wl.unpack_rows(words, V)
    allowed[:, work.vocab.stop_ids] = False
    picks = si.pick_tokens(rng, allowed, w.info.structural, w.info.is_stop, 0.35)
    assert (picks >= 0).sum() > work.B // 2   # rows whose text is complete have only the stop token left: they sit out
    batch = xgm.DeviceBatch(w.matchers, history=2, stream=stream)
    batch.accept_tokens(torch.tensor(picks, dtype=torch.int32, device="cuda").data_ptr(), stream)
    status = batch.status(stream)
    assert not status.any(), status
    scratch = [xgm.Matcher(cache=c) for c in work.caches]
    for b in range(work.B):
        if picks[b] >= 0:
            w.matchers[b].accept_token(int(picks[b]))
        batch.get_row(b, scratch[b], stream)
        assert [scratch[b].stack(s) for s in range(scratch[b].num_stacks())] == \
               [w.matchers[b].stack(s) for s in range(w.matchers[b].num_stacks())], f"row {b}"
    batch.fill_next_token_bitmask(d_mask2.data_ptr(), stream)
    work.fill(0, stream)
    torch.cuda.synchronize()
    words2 = d_mask2.cpu().numpy()
    assert np.array_equal(words2, work.d_mask.cpu().numpy())
    for b in rows:
        if picks[b] >= 0:
            assert oracle_rows[b].advance(toks[int(picks[b])])
        assert np.array_equal(words2[b], oracle.pack_bitmask(oracle_rows[b].mask(work.vocab, threads))), f"row {b}"
    say(f"  one device-side decode step of all {work.B} rows: states and masks equal the host's; {len(rows)} rows checked against the oracle")
    assert xgm.overflow_total() == before
