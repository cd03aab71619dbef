"""GPU parity of the device-resident matcher states (xgm_batch_*): tokens are
accepted by a kernel, the fill reads the states where they are.  Expected
masks come from the CPU oracle; expected stacks and status codes from the
library's host matchers, which the CPU suite pins to the oracle."""

import sys

import numpy as np
import pytest

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def xgm():
    import paper_2411_15100_amd as lib
    lib.load_library()
    return lib


@pytest.fixture(scope="module")
def wl():
    from paper_2411_15100_amd import workloads
    return workloads


def _stream():
    return int(torch.cuda.current_stream().cuda_stream)


def _stacks(m):
    return None if m.is_terminated() else [m.stack(s) for s in range(m.num_stacks())]


def _dev(values):
    return torch.tensor(list(values), dtype=torch.int32, device="cuda")


class _Rows:
    """B rows over one vocabulary: host matchers, oracle matchers, a device batch."""

    def __init__(self, xgm, wl, specs, vocab, history):
        self.vocab = vocab
        self.xv = wl.make_xgm_vocab(vocab)
        self.caches = [xgm.Cache(xgm.Grammar(t, r), self.xv) for t, r in specs]
        self.ogs = [oracle.Grammar(t, r) for t, r in specs]
        self.ms = [xgm.Matcher(cache=c) for c in self.caches]
        self.scratch = [xgm.Matcher(cache=c) for c in self.caches]
        self.oms = [oracle.EarleyMatcher(o) for o in self.ogs]
        self.B = len(specs)
        self.W = xgm.bitmask_words(vocab.size)
        self.batch = xgm.DeviceBatch(self.ms, history=history, stream=_stream())
        self.d_dev = torch.zeros((self.B, self.W), dtype=torch.int32, device="cuda")
        self.d_host = torch.zeros((self.B, self.W), dtype=torch.int32, device="cuda")

    def masks(self, xgm):
        """(mask from the device states, mask from the host matchers), both packed on the host;
        walks over the on-chip limits (the markup grammar has a few) are decided after each fill."""
        self.d_dev.fill_(-1)
        self.batch.fill_next_token_bitmask(self.d_dev.data_ptr(), _stream())
        self.batch.fill_overflow_fixup(_stream())
        xgm.fill_next_token_bitmask(self.ms, self.d_host.data_ptr(), _stream())
        xgm.fill_overflow_fixup(_stream())
        return self.d_dev.cpu().numpy(), self.d_host.cpu().numpy()

    def check_states(self):
        for b in range(self.B):
            self.batch.get_row(b, self.scratch[b], _stream())
            assert _stacks(self.scratch[b]) == _stacks(self.ms[b]), f"row {b}"


MIXED = [(si.JSON_GRAMMAR, "root"), (si.CSQL_GRAMMAR, "root"), (si.XML_GRAMMAR, "root"), (si.ARITH_GRAMMAR, "expr"), (si.PYDSL_GRAMMAR, "root"),
         (si.make_schema_grammar(0, string_heavy=True), "root"), (si.make_schema_grammar(1), "root"),
         (si.JSON_GRAMMAR, "root"), (si.make_schema_grammar(2, string_heavy=True), "root")]


def test_device_accept_follows_host_matchers_and_oracle(xgm, wl):
    vocab = si.make_vocab("bpe", 32000, 0)
    rows = _Rows(xgm, wl, MIXED, vocab, history=4)
    info = wl.TokenInfo(vocab)
    toks = vocab.tokens()
    nonempty = np.array([len(t) > 0 for t in toks])
    rng = np.random.Generator(np.random.PCG64(2024))
    n_ok = n_rejected = n_skipped = n_stopped = n_after_stop = n_host = 0
    fresh_overflow = xgm.overflow_total()
    for step in range(60):
        got, host = rows.masks(xgm)
        assert np.array_equal(got, host), f"step {step}: rows {np.flatnonzero((got != host).any(axis=1))}"
        if step % 6 == 0:
            want = np.stack([np.zeros(vocab.size, dtype=bool) if m.is_terminated() else om.mask(vocab)
                             for m, om in zip(rows.ms, rows.oms)])
            for b, m in enumerate(rows.ms):
                if m.is_terminated():
                    want[b, vocab.stop_ids] = True
            assert np.array_equal(got, oracle.pack_bitmask(want)), f"step {step}"
        allowed = wl.unpack_rows(got, vocab.size)
        picks = si.pick_tokens(rng, allowed, info.structural, info.is_stop, 0.35)
        tokens = np.array(picks, dtype=np.int64)
        for b in range(rows.B):
            u = rng.random()
            if rows.ms[b].is_terminated():
                tokens[b] = int(rng.integers(0, vocab.size))      # anything: the row reports that it has terminated
            elif u < 0.12:
                bad = np.flatnonzero(~allowed[b] & nonempty)
                tokens[b] = int(bad[rng.integers(0, bad.size)])
            elif u < 0.2:
                tokens[b] = -1
        status_before = rows.batch.status(_stream())
        rows.batch.accept_tokens(_dev(tokens).data_ptr(), _stream())
        status = rows.batch.status(_stream())
        for b in range(rows.B):
            t = int(tokens[b])
            if t < 0:
                assert status[b] == status_before[b]
                n_skipped += 1
                continue
            rc = rows.ms[b].try_accept_token(t)
            if rc == 0 and status[b] in (-8, -9):
                # beyond what the device holds or walks: the host's state becomes the row's next state
                rows.batch.set_row(b, rows.ms[b], _stream())
                n_host += 1
            else:
                assert status[b] == rc, (step, b, toks[t], status[b], rc)
            if rc == 0 and rows.ms[b].is_terminated():
                n_stopped += 1
            elif rc == 0:
                assert rows.oms[b].advance(toks[t])
                n_ok += 1
            elif rc == -7:
                n_after_stop += 1
                # start the row again, through the host
                rows.ms[b].reset()
                rows.oms[b] = oracle.EarleyMatcher(rows.ogs[b])
                rows.batch.set_row(b, rows.ms[b], _stream())
            else:
                assert rc == -6
                n_rejected += 1
        rows.check_states()
    say(f"  accepted {n_ok}, rejected {n_rejected}, skipped {n_skipped}, stop tokens {n_stopped}, "
        f"tokens after the stop {n_after_stop}, through the host {n_host}; walks over the limits in these fills: {xgm.overflow_total() - fresh_overflow}")
    assert n_ok > 250 and n_rejected > 20 and n_skipped > 10 and n_host < 10


def test_rollback_returns_to_earlier_states(xgm, wl):
    vocab = si.make_vocab("bpe", 32000, 0)
    specs = [(si.JSON_GRAMMAR, "root"), (si.make_schema_grammar(3, string_heavy=True), "root"),
             (si.CSQL_GRAMMAR, "root"), (si.JSON_GRAMMAR, "root")]
    rows = _Rows(xgm, wl, specs, vocab, history=5)
    info = wl.TokenInfo(vocab)
    toks = vocab.tokens()
    rng = np.random.Generator(np.random.PCG64(77))
    accepted = [[] for _ in range(rows.B)]

    def advance(n_steps):
        for _ in range(n_steps):
            got, host = rows.masks(xgm)
            assert np.array_equal(got, host)
            allowed = wl.unpack_rows(got, vocab.size)
            allowed[:, vocab.stop_ids] = False
            picks = si.pick_tokens(rng, allowed, info.structural, info.is_stop, 0.35)
            rows.batch.accept_tokens(_dev(picks).data_ptr(), _stream())
            assert not rows.batch.status(_stream()).any()
            for b in range(rows.B):
                rows.ms[b].accept_token(int(picks[b]))
                accepted[b].append(int(picks[b]))

    def replay():
        for b in range(rows.B):
            rows.ms[b].reset()
            rows.oms[b] = oracle.EarleyMatcher(rows.ogs[b])
            for t in accepted[b]:
                rows.ms[b].accept_token(t)
                assert rows.oms[b].advance(toks[t])

    advance(7)
    back = [0, 2, 5, 6]          # the ring keeps 5 older states: row 3 asks for too much
    rows.batch.rollback(_dev(back).data_ptr(), _stream())
    status = rows.batch.status(_stream())
    assert list(status) == [0, 0, 0, -1]
    for b, k in enumerate(back[:3]):
        accepted[b] = accepted[b][: len(accepted[b]) - k]
    replay()
    rows.check_states()
    got, host = rows.masks(xgm)
    assert np.array_equal(got, host)
    want = np.stack([om.mask(vocab) for om in rows.oms])
    assert np.array_equal(got, oracle.pack_bitmask(want))
    # going on from the restored states, then back again by what the ring holds now
    advance(3)
    rows.check_states()
    rows.batch.rollback(_dev([3, 1, 0, 3]).data_ptr(), _stream())
    assert not rows.batch.status(_stream()).any()
    for b, k in enumerate([3, 1, 0, 3]):
        accepted[b] = accepted[b][: len(accepted[b]) - k]
    replay()
    rows.check_states()
    got, host = rows.masks(xgm)
    assert np.array_equal(got, host)
    want = np.stack([om.mask(vocab) for om in rows.oms])
    assert np.array_equal(got, oracle.pack_bitmask(want))


@pytest.mark.parametrize("dtype_name", ["bf16", "f32"])
def test_batch_fused_fill_and_apply(xgm, wl, dtype_name):
    vocab = si.make_vocab("bpe", 9000, 0)
    specs = [(si.JSON_GRAMMAR, "root"), (si.make_schema_grammar(4, string_heavy=True), "root"), (si.ARITH_GRAMMAR, "expr")]
    rows = _Rows(xgm, wl, specs, vocab, history=0)
    for m, om, text in zip(rows.ms, rows.oms, [b'{"a', b"{", b"(1+"]):
        m.accept_bytes(text)
        assert om.advance(text)
    for b in range(rows.B):
        rows.batch.set_row(b, rows.ms[b], _stream())
    tdt, code, ninf = (torch.bfloat16, xgm.DTYPE_BF16, 0xFF80) if dtype_name == "bf16" else (torch.float32, xgm.DTYPE_F32, 0xFF800000)
    Vl = 9008
    logits = torch.from_numpy(si.make_logits(rows.B, Vl, seed=9)).to("cuda").to(tdt).contiguous()
    before = logits.clone()
    rows.batch.fill_and_apply(rows.d_dev.data_ptr(), logits.data_ptr(), code, Vl, logits.stride(0), _stream())
    want = np.stack([om.mask(vocab) for om in rows.oms])
    assert np.array_equal(rows.d_dev.cpu().numpy(), oracle.pack_bitmask(want))
    raw = lambda t: t.view(torch.int16 if tdt == torch.bfloat16 else torch.int32).cpu().numpy()
    out, src = raw(logits), raw(before)
    full = np.zeros((rows.B, Vl), dtype=bool)
    full[:, : vocab.size] = want
    ninf_signed = np.array(ninf, dtype=np.uint16 if tdt == torch.bfloat16 else np.uint32).view(out.dtype)
    assert np.array_equal(out, np.where(full, src, ninf_signed))
    with pytest.raises(xgm.XgmError):
        rows.batch.fill_and_apply(rows.d_dev.data_ptr(), logits.data_ptr(), code, 100, logits.stride(0), _stream())


def test_device_limits_are_reported_and_the_host_takes_over(xgm, wl):
    toks = [b"x", b"p", b"q", b"xx", b"[", b"]", b"1", b","] + [b""]
    V = len(toks)

    class V_:
        data = np.frombuffer(b"".join(toks), dtype=np.uint8).copy()
        offsets = np.concatenate([[0], np.cumsum([len(t) for t in toks])]).astype(np.int64)
        stop_ids = np.array([8], dtype=np.int32)
        size = V

    xv = xgm.Vocab(V_.data, V_.offsets, V_.stop_ids)
    amb = 'root ::= a | b\na ::= "x" root? "p"\nb ::= "x" root? "q"'
    nest = 'root ::= "[" (root ("," root)*)? "]" | "1"'
    ca, cn = xgm.Cache(xgm.Grammar(amb, "root"), xv), xgm.Cache(xgm.Grammar(nest, "root"), xv)
    ma, mn = xgm.Matcher(cache=ca), xgm.Matcher(cache=cn)
    oa, on = oracle.EarleyMatcher(oracle.Grammar(amb, "root")), oracle.EarleyMatcher(oracle.Grammar(nest, "root"))
    batch = xgm.DeviceBatch([ma, mn], history=2, stream=_stream())
    d = torch.zeros((2, 1), dtype=torch.int32, device="cuda")
    # row 0 doubles its stacks with every "x" (2, 4, 8, 16, then 32: over the device limit of 16);
    # row 1 nests deeper with every "[" until a stack passes 128 frames
    depth_hit = None
    for step in range(140):
        batch.accept_tokens(_dev([0 if step < 5 else -1, 4]).data_ptr(), _stream())
        st = batch.status(_stream())
        if step < 4:
            assert st[0] == 0
            ma.accept_token(0)
            assert oa.advance(b"x")
        elif step == 4:
            assert st[0] == -8            # too many stacks for the device: the row keeps its 16
        if st[1] == 0:
            mn.accept_token(4)
            assert on.advance(b"[")
        else:
            assert st[1] == -9
            depth_hit = step
            break
    assert depth_hit is not None and max(len(s) for s in _stacks(mn)) >= 127
    say(f"  row 1 reached the device's depth limit after {depth_hit} tokens")
    batch.fill_next_token_bitmask(d.data_ptr(), _stream())
    got = d.cpu().numpy()
    assert np.array_equal(got[0], oracle.pack_bitmask(oa.mask(V_)))
    assert np.array_equal(got[1], oracle.pack_bitmask(on.mask(V_)))
    sa, sn = xgm.Matcher(cache=ca), xgm.Matcher(cache=cn)
    batch.get_row(0, sa, _stream())
    batch.get_row(1, sn, _stream())
    assert _stacks(sa) == _stacks(ma) and ma.num_stacks() == 16
    assert _stacks(sn) == _stacks(mn)
    # the host can go on where the device cannot, but such a state does not go back to the device
    sa.accept_token(0)
    assert sa.num_stacks() == 32
    with pytest.raises(xgm.XgmError):
        batch.set_row(0, sa, _stream())
    sn.accept_token(4)
    with pytest.raises(xgm.XgmError):
        batch.set_row(1, sn, _stream())
    # a state within the limits does: close one level on the host, hand it back
    sn.accept_token(6)
    sn.accept_token(5)
    sn.accept_token(5)
    assert on.advance(b"[1]]")
    batch.set_row(1, sn, _stream())
    batch.fill_next_token_bitmask(d.data_ptr(), _stream())
    assert np.array_equal(d.cpu().numpy()[1], oracle.pack_bitmask(on.mask(V_)))
    # creation refuses what the device cannot hold, and bad arguments
    with pytest.raises(xgm.XgmError):
        xgm.DeviceBatch([sa], history=2, stream=_stream())
    with pytest.raises(xgm.XgmError):
        xgm.DeviceBatch([ma], history=64, stream=_stream())
    with pytest.raises(xgm.XgmError):
        xgm.DeviceBatch([xgm.Matcher(grammar=xgm.Grammar(nest, "root"), vocab=xv)], history=1, stream=_stream())


def test_batch_fill_walks_over_the_limits_are_fixed_up(xgm, wl):
    """A token that pushes more than 64 frames: the fill records it, the fixup
    decides it on the host from the state read back from the device; accepting
    it on the device reports the limit and the host takes the row over."""
    deep = b")+" + b"(" * 30
    toks = [b"1", b"(", b")", b"+", deep, deep + b"+", b"1" * 20, b")" * 4, b""]
    V = len(toks)

    class V_:
        data = np.frombuffer(b"".join(toks), dtype=np.uint8).copy()
        offsets = np.concatenate([[0], np.cumsum([len(t) for t in toks])]).astype(np.int64)
        stop_ids = np.array([8], dtype=np.int32)
        size = V

    xv = xgm.Vocab(V_.data, V_.offsets, V_.stop_ids)
    cache = xgm.Cache(xgm.Grammar(si.ARITH_GRAMMAR, "expr"), xv)
    og = oracle.Grammar(si.ARITH_GRAMMAR, "expr")
    m = xgm.Matcher(cache=cache)
    om = oracle.EarleyMatcher(og)
    text = b"(" * 5 + b"1"
    m.accept_bytes(text)
    assert om.advance(text)
    want = om.mask(V_)
    assert want[4] and not want[5]
    batch = xgm.DeviceBatch([m], history=1, stream=_stream())
    d = torch.zeros((1, 1), dtype=torch.int32, device="cuda")
    before = xgm.overflow_total()
    batch.fill_next_token_bitmask(d.data_ptr(), _stream())
    torch.cuda.synchronize()
    assert xgm.overflow_total() - before == 2
    # the batch's own counter, read without synchronising the device (a 4-byte copy on the stream)
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    import ctypes
    import os
    hip = ctypes.CDLL(os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so"))   # the runtime torch has loaded
    hip.hipMemcpyAsync.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
    assert hip.hipMemcpyAsync(count.data_ptr(), batch.overflow_count_device(), 4, 3, _stream()) == 0
    assert int(count.cpu()[0]) == 2
    assert xgm.fill_overflow_fixup(_stream()) == 0          # nothing of this belongs to the host-state fills
    assert batch.fill_overflow_fixup(_stream()) == 2
    assert np.array_equal(d.cpu().numpy()[0], oracle.pack_bitmask(want))
    assert batch.fill_overflow_fixup(_stream()) == 0         # every record is decided once
    batch.accept_tokens(_dev([4]).data_ptr(), _stream())
    assert list(batch.status(_stream())) == [-9]
    m.accept_token(4)
    assert om.advance(deep)
    batch.set_row(0, m, _stream())
    batch.fill_next_token_bitmask(d.data_ptr(), _stream())
    batch.fill_overflow_fixup(_stream())
    assert np.array_equal(d.cpu().numpy()[0], oracle.pack_bitmask(om.mask(V_)))


def test_walk_records_of_two_batches_on_two_streams_stay_apart(xgm, wl):
    """Two batches whose fills interleave on two streams; only the first has a state in which a token's
    walk exceeds the on-chip limits.  Each batch keeps its own records: the fixup of either decides
    exactly its own, in any order, and a record whose row has moved on is reported, not guessed."""
    deep = b")+" + b"(" * 30
    toks = [b"1", b"(", b")", b"+", deep, deep + b"+", b"1" * 20, b")" * 4, b""]
    V = len(toks)

    class V_:
        data = np.frombuffer(b"".join(toks), dtype=np.uint8).copy()
        offsets = np.concatenate([[0], np.cumsum([len(t) for t in toks])]).astype(np.int64)
        stop_ids = np.array([8], dtype=np.int32)
        size = V

    xv = xgm.Vocab(V_.data, V_.offsets, V_.stop_ids)
    cache = xgm.Cache(xgm.Grammar(si.ARITH_GRAMMAR, "expr"), xv)
    og = oracle.Grammar(si.ARITH_GRAMMAR, "expr")
    texts_a = [b"(" * 5 + b"1", b"1+", b"((1"]      # rows 0 and 2 are inside parentheses: `deep` needs a walk there
    texts_b = [b"1", b"1+1"]                        # no parentheses open: nothing to walk
    ms_a, ms_b, oms_a, oms_b = [], [], [], []
    for texts, ms, oms in ((texts_a, ms_a, oms_a), (texts_b, ms_b, oms_b)):
        for t in texts:
            m = xgm.Matcher(cache=cache)
            m.accept_bytes(t)
            om = oracle.EarleyMatcher(og)
            assert om.advance(t)
            ms.append(m)
            oms.append(om)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    batch_a = xgm.DeviceBatch(ms_a, history=2, stream=s1.cuda_stream)
    batch_b = xgm.DeviceBatch(ms_b, history=2, stream=s2.cuda_stream)
    d_a = torch.zeros((3, 1), dtype=torch.int32, device="cuda")
    d_a2 = torch.zeros((3, 1), dtype=torch.int32, device="cuda")
    d_b = torch.zeros((2, 1), dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = xgm.overflow_total()
    batch_a.fill_next_token_bitmask(d_a.data_ptr(), s1.cuda_stream)
    batch_b.fill_next_token_bitmask(d_b.data_ptr(), s2.cuda_stream)
    batch_a.fill_next_token_bitmask(d_a2.data_ptr(), s1.cuda_stream)      # a second fill of the same states, another buffer
    batch_b.fill_next_token_bitmask(d_b.data_ptr(), s2.cuda_stream)
    want_a = oracle.pack_bitmask(np.stack([om.mask(V_) for om in oms_a]))
    want_b = oracle.pack_bitmask(np.stack([om.mask(V_) for om in oms_b]))
    assert batch_b.fill_overflow_fixup(s2.cuda_stream) == 0               # the other batch's fixup first: it has nothing
    assert np.array_equal(d_b.cpu().numpy(), want_b)
    n = batch_a.fill_overflow_fixup(s1.cuda_stream)
    assert n > 0 and n % 2 == 0                                           # both fills of batch a, the same pairs each
    assert xgm.overflow_total() - before == n
    assert np.array_equal(d_a.cpu().numpy(), want_a)
    assert np.array_equal(d_a2.cpu().numpy(), want_a)
    assert xgm.fill_overflow_fixup(s1.cuda_stream) == 0                   # and none of it reached the host-state fills' log
    # a record whose row has left the state it was made in cannot be decided any more: reported as an error
    batch_a.fill_next_token_bitmask(d_a.data_ptr(), s1.cuda_stream)
    torch.cuda.synchronize()
    batch_a.accept_tokens(_dev([1, -1, 1]).data_ptr(), s1.cuda_stream)    # "(" right after a digit is refused:
    assert list(batch_a.status(s1.cuda_stream)) == [-6, 0, -6]             # the states stay, so the fixup still works
    assert batch_a.fill_overflow_fixup(s1.cuda_stream) == n // 2
    assert np.array_equal(d_a.cpu().numpy(), want_a)
    batch_a.fill_next_token_bitmask(d_a.data_ptr(), s1.cuda_stream)
    torch.cuda.synchronize()
    batch_a.accept_tokens(_dev([3, -1, 3]).data_ptr(), s1.cuda_stream)    # "+" moves rows 0 and 2 on
    assert not batch_a.status(s1.cuda_stream).any()
    with pytest.raises(xgm.XgmError) as e:
        batch_a.fill_overflow_fixup(s1.cuda_stream)
    assert e.value.status == -9 and "left" in str(e.value)
    assert batch_a.fill_overflow_fixup(s1.cuda_stream) == 0               # reported once


def test_stop_token_and_termination_on_the_device(xgm, wl):
    toks = [b"1", b"2", b"+", b"*", b"(", b")", b" ", b"12", b"+1", b")*", b"", b"((", b"1)", b"", b"3 "]
    V = len(toks)

    class V_:
        data = np.frombuffer(b"".join(toks), dtype=np.uint8).copy()
        offsets = np.concatenate([[0], np.cumsum([len(t) for t in toks])]).astype(np.int64)
        stop_ids = np.array([10, 13], dtype=np.int32)
        size = V

    xv = xgm.Vocab(V_.data, V_.offsets, V_.stop_ids)
    cache = xgm.Cache(xgm.Grammar(si.ARITH_GRAMMAR, "expr"), xv)
    og = oracle.Grammar(si.ARITH_GRAMMAR, "expr")
    ms = [xgm.Matcher(cache=cache) for _ in range(3)]
    oms = [oracle.EarleyMatcher(og) for _ in range(3)]
    batch = xgm.DeviceBatch(ms, history=3, stream=_stream())
    d = torch.zeros((3, 1), dtype=torch.int32, device="cuda")

    def expect():
        want = np.stack([om.mask(V_) for om in oms])
        for b, m in enumerate(ms):
            if m.is_terminated():
                want[b] = False
                want[b, [10, 13]] = True
        batch.fill_next_token_bitmask(d.data_ptr(), _stream())
        assert np.array_equal(d.cpu().numpy(), oracle.pack_bitmask(want))

    # stop before anything is written: rejected; a token without bytes that is no stop token: id 10/13 are both stops,
    # so use an id beyond the vocabulary for the argument check
    batch.accept_tokens(_dev([10, 0, V]).data_ptr(), _stream())
    assert list(batch.status(_stream())) == [-6, 0, -1]
    ms[1].accept_token(0)
    assert oms[1].advance(b"1")
    expect()
    # row 1 may stop now (second stop id), row 0 writes "(", row 2 "12"
    batch.accept_tokens(_dev([4, 13, 7]).data_ptr(), _stream())
    assert list(batch.status(_stream())) == [0, 0, 0]
    ms[0].accept_token(4)
    ms[1].accept_token(13)
    ms[2].accept_token(7)
    assert oms[0].advance(b"(") and oms[2].advance(b"12")
    assert ms[1].is_terminated()
    expect()
    s = xgm.Matcher(cache=cache)
    batch.get_row(1, s, _stream())
    assert s.is_terminated()
    # after the stop token nothing is accepted, not even another stop
    batch.accept_tokens(_dev([-1, 10, 10]).data_ptr(), _stream())
    assert list(batch.status(_stream())) == [0, -7, 0]
    ms[2].accept_token(10)
    expect()
    # one step back: rows 1 and 2 are open again
    batch.rollback(_dev([0, 1, 1]).data_ptr(), _stream())
    assert list(batch.status(_stream())) == [0, 0, 0]
    for b, text in ((1, b"1"), (2, b"12")):
        ms[b].reset()
        ms[b].accept_bytes(text)
    expect()
    batch.get_row(1, s, _stream())
    assert not s.is_terminated() and _stacks(s) == _stacks(ms[1])


def test_many_rows_fill_from_resident_states_equals_host_states(xgm, wl):
    """1000 rows of a mid-sized vocabulary: the fill from device-resident states agrees with the fill from
    host-side states, and both with the oracle for the distinct states."""
    vocab = si.make_vocab("bpe", 32000, 0)
    xv = wl.make_xgm_vocab(vocab)
    texts = (si.JSON_GRAMMAR, si.make_schema_grammar(1, string_heavy=True))
    caches = [xgm.Cache(xgm.Grammar(t, "root"), xv) for t in texts]
    prefixes = [b"", b'{"a": "x', b"[1, ", b'{"k', b"[", b'["abc", ']
    ms, keys = [], []
    for b in range(1000):
        m = xgm.Matcher(cache=caches[0] if b % 3 else caches[1])
        if b % 3:
            m.accept_bytes(prefixes[b % len(prefixes)])
        ms.append(m)
        keys.append((0, prefixes[b % len(prefixes)]) if b % 3 else (1, b""))
    batch = xgm.DeviceBatch(ms, history=0, stream=_stream())
    W = xgm.bitmask_words(vocab.size)
    d_dev = torch.zeros((len(ms), W), dtype=torch.int32, device="cuda")
    d_host = torch.zeros((len(ms), W), dtype=torch.int32, device="cuda")
    batch.fill_next_token_bitmask(d_dev.data_ptr(), _stream())
    xgm.fill_next_token_bitmask(ms, d_host.data_ptr(), _stream())
    assert torch.equal(d_dev, d_host)
    got = d_dev.cpu().numpy()
    want = {}
    for b, key in enumerate(keys):
        if key not in want:
            om = oracle.EarleyMatcher(oracle.Grammar(texts[key[0]], "root"))
            assert om.advance(key[1]) or not key[1]
            want[key] = oracle.pack_bitmask(om.mask(vocab))
        assert np.array_equal(got[b], want[key]), f"row {b}"
    say(f"  1000 rows ({len(want)} distinct states): resident and host-side fills agree with the oracle")


def test_fork_continues_one_state_in_several_rows(xgm, wl):
    vocab = si.make_vocab("bpe", 32000, 0)
    gj = xgm.Grammar(si.JSON_GRAMMAR, "root")
    xv = wl.make_xgm_vocab(vocab)
    cj, cs = xgm.Cache(gj, xv), xgm.Cache(xgm.Grammar(si.make_schema_grammar(1), "root"), xv)
    caches = [cj, cj, cj, cj, cs]
    ogs = [oracle.Grammar(si.JSON_GRAMMAR, "root")] * 4 + [oracle.Grammar(si.make_schema_grammar(1), "root")]
    texts = [b'{"a": [1, ', b'[true', b'"x', b'{', b'{']
    ms = [xgm.Matcher(cache=c) for c in caches]
    for m, t in zip(ms, texts):
        m.accept_bytes(t)
    batch = xgm.DeviceBatch(ms, history=3, stream=_stream())
    W = xgm.bitmask_words(vocab.size)
    d = torch.zeros((5, W), dtype=torch.int32, device="cuda")

    def expect(texts_now):
        batch.fill_next_token_bitmask(d.data_ptr(), _stream())
        got = d.cpu().numpy()
        for b, t in enumerate(texts_now):
            om = oracle.EarleyMatcher(ogs[b])
            assert om.advance(t)
            assert np.array_equal(got[b], oracle.pack_bitmask(om.mask(vocab))), f"row {b}"
            s = xgm.Matcher(cache=caches[b])
            batch.get_row(b, s, _stream())
            r = xgm.Matcher(cache=caches[b])
            r.accept_bytes(t)
            assert _stacks(s) == _stacks(r), f"row {b}"

    expect(texts)
    # rows 1 and 2 both continue row 0; row 0 continues row 2 as it was before the call; row 3 stays;
    # row 4 has another grammar than row 0 and is refused; an index beyond the batch is refused too
    batch.fork(_dev([2, 0, 0, -1, 0]).data_ptr(), _stream())
    assert list(batch.status(_stream())) == [0, 0, 0, 0, -1]
    now = [texts[2], texts[0], texts[0], texts[3], texts[4]]
    expect(now)
    batch.fork(_dev([-1, -1, -1, 7, -1]).data_ptr(), _stream())
    assert list(batch.status(_stream())) == [0, 0, 0, -1, -1]
    expect(now)
    # forked rows go their own ways, and a fork can be taken back like a token
    tok = {t: i for i, t in enumerate(vocab.tokens())}
    batch.accept_tokens(_dev([tok[b'"'], tok[b'2'], tok[b'{'], -1, -1]).data_ptr(), _stream())
    assert list(batch.status(_stream()))[:3] == [0, 0, 0]
    expect([now[0] + b'"', now[1] + b'2', now[2] + b'{', now[3], now[4]])
    batch.rollback(_dev([2, 1, 2, 0, 0]).data_ptr(), _stream())
    assert list(batch.status(_stream()))[:3] == [0, 0, 0]
    expect([texts[0], now[1], texts[2], now[3], now[4]])
    # a batch without history has no room for a forked state
    flat = xgm.DeviceBatch(ms[:2], history=0, stream=_stream())
    with pytest.raises(xgm.XgmError):
        flat.fork(_dev([1, -1]).data_ptr(), _stream())


def test_random_grammars_cache_fill_and_device_accept(xgm, wl):
    """Seeded random grammars (nested groups, repetition, recursive and tail references, empty
    alternatives, ambiguity): mask cache, fill from host-side and device-resident states, and the accept
    kernel, against the oracle and the host matchers at every step."""
    from test_host_library import _random_grammar_text
    from test_oracle_misc import TinyVocab
    rng = np.random.Generator(np.random.PCG64(777))
    pieces = [bytes(p) for p in (b"a", b"b", b"c", b"d", b"(", b")", b"ab", b"ba", b"a(", b")b", b"cd)", b"((", b"))", b"abc", b"dcba", b"(a)")]
    vocab = TinyVocab(pieces + [b""], [len(pieces)])
    vocab.size = len(pieces) + 1
    xv = xgm.Vocab(vocab.data, vocab.offsets, vocab.stop_ids)
    texts = []
    while len(texts) < 24:
        text = _random_grammar_text(rng)
        try:
            xgm.Grammar(text, "root")
        except xgm.XgmError:
            continue
        texts.append(text)
    caches = [xgm.Cache(xgm.Grammar(t, "root"), xv) for t in texts]
    ogs = [oracle.Grammar(t, "root") for t in texts]
    B = len(texts)
    n_checked = n_host = n_multi = 0
    for walk in range(3):
        ms = [xgm.Matcher(cache=c) for c in caches]
        oms = [oracle.EarleyMatcher(o) for o in ogs]
        batch = xgm.DeviceBatch(ms, history=2, stream=_stream())
        d_dev = torch.zeros((B, 1), dtype=torch.int32, device="cuda")
        d_host = torch.zeros((B, 1), dtype=torch.int32, device="cuda")
        frozen = np.zeros(B, dtype=bool)
        for step in range(10):
            batch.fill_next_token_bitmask(d_dev.data_ptr(), _stream())
            batch.fill_overflow_fixup(_stream())
            xgm.fill_next_token_bitmask(ms, d_host.data_ptr(), _stream())
            xgm.fill_overflow_fixup(_stream())
            want = np.stack([om.mask(vocab) for om in oms])
            for b, m in enumerate(ms):
                if m.is_terminated():
                    want[b] = False
                    want[b, vocab.stop_ids] = True
            packed = oracle.pack_bitmask(want)
            assert np.array_equal(d_host.cpu().numpy(), packed), (walk, step, np.flatnonzero((d_host.cpu().numpy() != packed).any(axis=1)))
            assert np.array_equal(d_dev.cpu().numpy(), packed), (walk, step, np.flatnonzero((d_dev.cpu().numpy() != packed).any(axis=1)))
            n_checked += B
            tokens = np.full(B, -1, dtype=np.int64)
            for b in range(B):
                allowed = np.flatnonzero(want[b][: len(pieces)])
                if frozen[b] or ms[b].is_terminated() or allowed.size == 0:
                    frozen[b] = True
                    continue
                tokens[b] = int(allowed[rng.integers(0, allowed.size)])
            batch.accept_tokens(_dev(tokens).data_ptr(), _stream())
            status = batch.status(_stream())
            for b in range(B):
                t = int(tokens[b])
                if t < 0:
                    continue
                rc = ms[b].try_accept_token(t)
                if rc == -8:                      # the host's own limit of 64 stacks: the row stops here
                    frozen[b] = True
                    if status[b] == 0:            # the device went on: take it one step back
                        back = np.zeros(B, dtype=np.int64)
                        back[b] = 1
                        batch.rollback(_dev(back).data_ptr(), _stream())
                        assert batch.status(_stream())[b] == 0
                    continue
                assert rc == 0
                assert oms[b].advance(pieces[t])
                if status[b] in (-8, -9):         # device limits: through the host
                    try:
                        batch.set_row(b, ms[b], _stream())
                    except xgm.XgmError:
                        frozen[b] = True          # the state no longer fits the device: leave the row alone
                        ms[b] = None
                    n_host += 1
                else:
                    assert status[b] == 0, (walk, step, b, status[b])
                n_multi += ms[b] is not None and ms[b].num_stacks() > 1
            alive = [b for b in range(B) if ms[b] is not None]
            if len(alive) < B:
                # drop rows that left the device's limits: rebuild the batch from the remaining host matchers
                ms = [ms[b] for b in alive]
                oms = [oms[b] for b in alive]
                frozen = frozen[alive]
                B = len(ms)
                batch = xgm.DeviceBatch(ms, history=2, stream=_stream())
                d_dev = torch.zeros((B, 1), dtype=torch.int32, device="cuda")
                d_host = torch.zeros((B, 1), dtype=torch.int32, device="cuda")
                continue
        B = len(texts)
    say(f"  {n_checked} masks of random grammars bit-exact on both paths; {n_multi} steps with parallel stacks; {n_host} through the host")
    assert n_checked > 400 and n_multi > 20


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_grammars_one_launch_form(xgm, wl, seed):
    """The same family of seeded random grammars through the call that fills the mask and writes the
    logits in one launch, from host-side and from device-resident states: masks and logits (bit
    patterns; untouched where allowed) against the oracle at every step, with parallel stacks."""
    from test_host_library import _random_grammar_text
    from test_oracle_misc import TinyVocab
    rng = np.random.Generator(np.random.PCG64(seed))
    pieces = [bytes(p) for p in (b"a", b"b", b"c", b"d", b"(", b")", b"ab", b"ba", b"a(", b")b", b"cd)", b"((", b"))", b"abc", b"dcba",
                                 b"(a)", b"aa", b"bb", b"ccd", b"d(", b"()", b")(", b"abcd", b"a)b(", b"ddd", b"c(c", b"b)", b"(((",
                                 b")))", b"ad", b"da", b"cab")]
    vocab = TinyVocab(pieces + [b""], [len(pieces)])
    vocab.size = len(pieces) + 1
    V = vocab.size
    stride = (V + 3) // 4 * 4
    W = xgm.bitmask_words(V)
    xv = xgm.Vocab(vocab.data, vocab.offsets, vocab.stop_ids)
    texts = []
    while len(texts) < 24:
        text = _random_grammar_text(rng)
        try:
            xgm.Grammar(text, "root")
        except xgm.XgmError:
            continue
        texts.append(text)
    caches = [xgm.Cache(xgm.Grammar(t, "root"), xv) for t in texts]
    ogs = [oracle.Grammar(t, "root") for t in texts]
    B = len(texts)
    n_rows = n_multi = 0
    for walk in range(2):
        ms = [xgm.Matcher(cache=c) for c in caches]
        oms = [oracle.EarleyMatcher(o) for o in ogs]
        frozen = np.zeros(B, dtype=bool)
        for step in range(10):
            want = np.stack([om.mask(vocab) for om in oms])
            for b, m in enumerate(ms):
                if m.is_terminated():
                    want[b] = False
                    want[b, vocab.stop_ids] = True
            packed = oracle.pack_bitmask(want)
            base = rng.standard_normal((B, stride)).astype(np.float32)
            expect = base.copy()
            expect[:, :V][~want] = -np.inf
            try:
                batch = xgm.DeviceBatch(ms, history=0, stream=_stream())
            except xgm.XgmError:      # a state beyond the device's limits: host-side states only
                batch = None
            for kind in ("host", "device"):
                if kind == "device" and batch is None:
                    continue
                d = torch.zeros((B, W), dtype=torch.int32, device="cuda")
                lg = torch.from_numpy(base.copy()).cuda()
                if kind == "host":
                    xgm.fill_and_apply(ms, d.data_ptr(), lg.data_ptr(), xgm.DTYPE_F32, V, stride, _stream())
                else:
                    batch.fill_and_apply(d.data_ptr(), lg.data_ptr(), xgm.DTYPE_F32, V, stride, _stream())
                    batch.fill_overflow_fixup(_stream())
                xgm.fill_overflow_fixup(_stream())
                assert np.array_equal(d.cpu().numpy(), packed), (walk, step, kind)
                assert np.array_equal(lg.cpu().numpy().view(np.uint32), expect.view(np.uint32)), (walk, step, kind)
            n_rows += B
            n_multi += sum(m.num_stacks() > 1 for m in ms)
            for b in range(B):
                allowed = np.flatnonzero(want[b][: len(pieces)])
                if frozen[b] or ms[b].is_terminated() or allowed.size == 0:
                    frozen[b] = True
                    continue
                t = int(allowed[rng.integers(0, allowed.size)])
                rc = ms[b].try_accept_token(t)
                if rc == -8:          # the host's limit of 64 stacks: the row stops here
                    frozen[b] = True
                    continue
                assert rc == 0
                assert oms[b].advance(pieces[t])
    say(f"one-launch form on random grammars (seed {seed}): {n_rows} rows bit-exact on both paths, {n_multi} with parallel stacks")
    assert n_multi > 10
