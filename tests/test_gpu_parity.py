"""GPU parity: the HIP path (through the C ABI) against the CPU oracle,
bit for bit, on the five workloads and on edge cases.  Every expected value
comes from `oracle/`; nothing here is read from a file written by the GPU."""

import sys
import zlib

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


@pytest.fixture
def no_overflow(xgm):
    """The test must not record a single walk that exceeded the on-chip limits
    (so no result in it came from the host slow path)."""
    before = xgm.overflow_total()
    yield
    assert xgm.overflow_total() == before


def _apply_and_check(xgm, logits_np, dtype_code, torch_dtype, neg_inf_bits, d_mask, allowed, V):
    """Apply on the GPU and compare raw bit patterns with the oracle's apply."""
    B = logits_np.shape[0]
    t = torch.from_numpy(logits_np).to("cuda").to(torch_dtype).contiguous()
    view = torch.int32 if torch_dtype == torch.float32 else torch.int16
    before = t.view(view).cpu().numpy().view(np.uint32 if view == torch.int32 else np.uint16)
    xgm.apply_token_bitmask_inplace(t.data_ptr(), dtype_code, B, t.shape[1], t.stride(0), d_mask.data_ptr(), V,
                                    stream=_stream())
    after = t.view(view).cpu().numpy().view(before.dtype)
    want = oracle.apply_mask(before, allowed, neg_inf_bits)
    assert np.array_equal(after, want)
    return after


# --------------------------------------------------------------------------
# workload 1: arithmetic grammar, vocabulary 1024, batch 1, 64 steps, fp32
# --------------------------------------------------------------------------
def test_workload1_arith_every_step(xgm, wl, no_overflow):
    say("workload 1: arith V=1024 B=1 steps=64")
    vocab = si.make_vocab("arith", 1024, 0)
    g = xgm.Grammar(si.ARITH_GRAMMAR, "expr")
    cache = xgm.Cache(g, wl.make_xgm_vocab(vocab))
    assert cache.host_classified == 0
    walker = wl.BatchWalker([cache], vocab, seed=0, structural_bias=0.0)
    og = oracle.Grammar(si.ARITH_GRAMMAR, "expr")
    om = oracle.EarleyMatcher(og)
    toks = vocab.tokens()
    for step in range(64):
        words = walker.fill()
        want = om.mask(vocab)
        assert np.array_equal(words, oracle.pack_bitmask(want)[None, :]), f"step {step}"
        logits = si.make_logits(1, 1024, seed=1000 + step)
        _apply_and_check(xgm, logits, xgm.DTYPE_F32, torch.float32, 0xFF800000, walker.d_mask, want[None, :], 1024)
        t = int(walker.step(words)[0])
        if not walker.history[0]:      # the request terminated and was re-seeded
            om = oracle.EarleyMatcher(og)
        else:
            assert om.advance(toks[t])


# --------------------------------------------------------------------------
# workload 2: JSON, vocabulary 32000, batch 1, 256 steps, fp32
# --------------------------------------------------------------------------
def test_workload2_json_every_step(xgm, wl, no_overflow):
    say("workload 2: json V=32000 B=1 steps=256")
    vocab = si.make_vocab("bpe", 32000, 0)
    g = xgm.Grammar(si.JSON_GRAMMAR, "root")
    cache = xgm.Cache(g, wl.make_xgm_vocab(vocab))
    assert cache.host_classified == 0
    walker = wl.BatchWalker([cache], vocab, seed=2, structural_bias=0.35)
    og = oracle.Grammar(si.JSON_GRAMMAR, "root")
    om = oracle.EarleyMatcher(og)
    toks = vocab.tokens()
    n_multi = 0
    for step in range(256):
        words = walker.fill()
        want = om.mask(vocab)
        assert np.array_equal(words, oracle.pack_bitmask(want)[None, :]), f"step {step}"
        n_multi += walker.matchers[0].num_stacks() > 1
        if step % 16 == 0:
            logits = si.make_logits(1, 32000, seed=2000 + step)
            _apply_and_check(xgm, logits, xgm.DTYPE_F32, torch.float32, 0xFF800000, walker.d_mask, want[None, :], 32000)
        t = int(walker.step(words)[0])
        if not walker.history[0]:
            om = oracle.EarleyMatcher(og)
        else:
            assert om.advance(toks[t])
    say(f"  steps with several parallel stacks: {n_multi}")


# --------------------------------------------------------------------------
# workload 3: schema grammar, vocabulary 128256, batch 16, 512 steps, bf16
# --------------------------------------------------------------------------
def test_workload3_schema_batch16(xgm, wl, no_overflow):
    say("workload 3: schema V=128256 B=16 steps=512 (oracle on every 16th step of every row)")
    vocab = si.make_vocab("bpe", 128256, 0)
    text = si.make_schema_grammar(0)
    g = xgm.Grammar(text, "root")
    cache = xgm.Cache(g, wl.make_xgm_vocab(vocab))
    assert cache.host_classified == 0
    B = 16
    walker = wl.BatchWalker([cache] * B, vocab, seed=3, structural_bias=0.35)
    og = oracle.Grammar(text, "root")
    oms = [oracle.EarleyMatcher(og) for _ in range(B)]
    toks = vocab.tokens()
    checked = 0
    for step in range(512):
        words = walker.fill()
        if step % 16 == 0:
            want = np.stack([om.mask(vocab) for om in oms])
            assert np.array_equal(words, oracle.pack_bitmask(want)), f"step {step}"
            checked += B
            logits = si.make_logits(B, 128256, seed=3000 + step, sigma=2.0)
            _apply_and_check(xgm, logits, xgm.DTYPE_BF16, torch.bfloat16, 0xFF80, walker.d_mask, want, 128256)
            say(f"  step {step}: {B} rows bit-exact")
        picks = walker.step(words)
        for b in range(B):
            if not walker.history[b]:
                oms[b] = oracle.EarleyMatcher(og)
            else:
                assert oms[b].advance(toks[int(picks[b])])
    assert checked == 512


# --------------------------------------------------------------------------
# workload 4: mask-cache build, 128256 tokens at every node
# --------------------------------------------------------------------------
def _check_cache_classes(xgm, cache, g, og, vocab, nodes):
    """Oracle classes: 2 accepted, 1 context-dependent, 4 context-dependent by
    section 3.1 alone (dropped by the one-byte narrowing), 0 rejected."""
    n1 = n4 = 0
    for node in nodes:
        want = og.classify(g.rule_name(g.node_rule(node)), g.node_path(node), vocab)
        acc, unc = cache.copy_node_bits(node)
        plain = cache.copy_node_plain(node)
        assert np.array_equal(acc, oracle.pack_bitmask(want == 2)), ("accepted", node, g.node_path(node))
        assert np.array_equal(unc, oracle.pack_bitmask(want == 1)), ("uncertain", node, g.node_path(node))
        assert np.array_equal(plain, oracle.pack_bitmask(want == 4)), ("uncertain, 3.1 only", node, g.node_path(node))
        assert cache.num_uncertain(node) == int((want == 1).sum())
        assert cache.num_uncertain_plain(node) == int((want == 4).sum())
        n1 += int((want == 1).sum())
        n4 += int((want == 4).sum())
    return n1, n4


def test_workload4_cache_build_json_all_nodes(xgm, wl, no_overflow):
    say("workload 4(i): json cache, V=128256, every node")
    vocab = si.make_vocab("bpe", 128256, 0)
    g = xgm.Grammar(si.JSON_GRAMMAR, "root")
    cache = xgm.Cache(g, wl.make_xgm_vocab(vocab), keep_plain=True)
    assert cache.host_classified == 0
    og = oracle.Grammar(si.JSON_GRAMMAR, "root")
    n1, n4 = _check_cache_classes(xgm, cache, g, og, vocab, range(g.num_nodes))
    say(f"  {g.num_nodes} nodes x {vocab.size} tokens bit-exact; kernel {cache.build_kernel_seconds*1e3:.2f} ms; "
        f"context-dependent pairs {n1 + n4} by section 3.1, {n1} after the one-byte narrowing")


def test_cache_build_in_batches_of_nodes_gives_the_same_classes(xgm, wl):
    """A grammar too large for one batch of rank-space rows is classified batch after batch; forced here with 32
    nodes per batch.  The markup grammar also has walks over the on-chip limits, which are then decided on the
    host per batch."""
    say("cache build in batches of 32 nodes: JSON (every node) and markup (a seeded sample), V=32000")
    vocab = si.make_vocab("bpe", 32000, 0)
    xv = wl.make_xgm_vocab(vocab)
    xgm.debug_set_build_batch_nodes(32)
    try:
        for text, count in ((si.JSON_GRAMMAR, None), (si.XML_GRAMMAR, 24)):
            g = xgm.Grammar(text, "root")
            assert g.num_nodes > 64
            before = xgm.overflow_total()
            cache = xgm.Cache(g, xv, keep_plain=True)
            assert cache.host_classified == xgm.overflow_total() - before
            og = oracle.Grammar(text, "root")
            nodes = range(g.num_nodes) if count is None else sorted(
                int(n) for n in np.random.Generator(np.random.PCG64(9)).choice(g.num_nodes, size=count, replace=False))
            n1, n4 = _check_cache_classes(xgm, cache, g, og, vocab, nodes)
            # and the masks that come out of such a cache
            m = xgm.Matcher(cache=cache)
            om = oracle.EarleyMatcher(og)
            d_mask = torch.zeros(1, xgm.bitmask_words(vocab.size), dtype=torch.int32, device="cuda")
            xgm.fill_next_token_bitmask([m], d_mask.data_ptr(), _stream())
            xgm.fill_overflow_fixup(_stream())
            torch.cuda.synchronize()
            assert np.array_equal(d_mask.cpu().numpy(), oracle.pack_bitmask(om.mask(vocab))[None, :])
            say(f"  {g.num_nodes} nodes in {-(-g.num_nodes // 32)} batches: classes of {len(nodes)} nodes and the first mask "
                f"bit-exact ({cache.host_classified} pairs decided on the host)")
    finally:
        xgm.debug_set_build_batch_nodes(0)


def test_workload4_cache_build_csql_sample(xgm, wl):
    say("workload 4(ii): C/SQL-like cache, V=128256, 8 % of the nodes (the longest lists + a seeded sample)")
    vocab = si.make_vocab("bpe", 128256, 0)
    g = xgm.Grammar(si.CSQL_GRAMMAR, "root")
    before = xgm.overflow_total()
    cache = xgm.Cache(g, wl.make_xgm_vocab(vocab), keep_plain=True)
    # every walk over the on-chip limits is recorded and then decided on the host: the two counts agree
    assert cache.host_classified == xgm.overflow_total() - before
    say(f"  pairs decided on the host after exceeding a walk limit: {cache.host_classified}")
    og = oracle.Grammar(si.CSQL_GRAMMAR, "root")
    rng = np.random.Generator(np.random.PCG64(44))
    by_list = np.argsort([-cache.num_uncertain(n) for n in range(g.num_nodes)], kind="stable")
    nodes = sorted(set(int(n) for n in by_list[:12]) | set(int(n) for n in rng.choice(g.num_nodes, size=48, replace=False)))
    assert len(nodes) >= 0.05 * g.num_nodes
    n1, n4 = _check_cache_classes(xgm, cache, g, og, vocab, nodes)
    say(f"  {len(nodes)} of {g.num_nodes} nodes bit-exact ({n1} context-dependent pairs, {n4} more by section 3.1 alone); "
        f"kernel {cache.build_kernel_seconds*1e3:.2f} ms")


# --------------------------------------------------------------------------
# workload 5 (reduced batch; the full batch-128 configuration is checked in
# test_gpu_serving.py): distinct string-heavy schema grammars, V = 151936
# --------------------------------------------------------------------------
def test_workload5_distinct_grammars_batch8(xgm, wl, no_overflow):
    say("workload 5 (8 distinct grammars): V=151936 bf16")
    vocab = si.make_vocab("bpe", 151936, 0)
    xv = wl.make_xgm_vocab(vocab)
    texts = [si.make_schema_grammar(s, string_heavy=True) for s in range(8)]
    caches = [xgm.Cache(xgm.Grammar(t, "root"), xv) for t in texts]
    walker = wl.BatchWalker(caches, vocab, seed=5, structural_bias=0.35)
    ogs = [oracle.Grammar(t, "root") for t in texts]
    oms = [oracle.EarleyMatcher(o) for o in ogs]
    toks = vocab.tokens()
    for step in range(40):
        words = walker.fill()
        if step % 8 == 7:
            want = np.stack([om.mask(vocab) for om in oms])
            assert np.array_equal(words, oracle.pack_bitmask(want)), f"step {step}"
            logits = si.make_logits(8, 151936, seed=5000 + step)
            _apply_and_check(xgm, logits, xgm.DTYPE_BF16, torch.bfloat16, 0xFF80, walker.d_mask, want, 151936)
            say(f"  step {step}: 8 rows bit-exact; uncertain fraction at the tops "
                f"{wl.uncertain_fraction(walker, caches).mean():.3f}")
        picks = walker.step(words)
        for b in range(8):
            if not walker.history[b]:
                oms[b] = oracle.EarleyMatcher(ogs[b])
            else:
                assert oms[b].advance(toks[int(picks[b])])


# --------------------------------------------------------------------------
# a second grammar family: markup (elements, attributes, text, comments)
# --------------------------------------------------------------------------
def test_markup_grammar_every_step_and_every_node(xgm, wl):
    """The white-space runs of this grammar are ambiguous (`attrs ws`), so a few
    tokens made of many blanks exceed the walk's 24 pending alternatives: those
    pairs are decided by the host slow path, at build time and - through
    xgm_fill_overflow_fixup - at fill time.  Everything stays bit-exact."""
    say("markup grammar: V=32000 B=2 steps=160, classes at every node")
    vocab = si.make_vocab("bpe", 32000, 0)
    g = xgm.Grammar(si.XML_GRAMMAR, "root")
    cache = xgm.Cache(g, wl.make_xgm_vocab(vocab), keep_plain=True)
    assert cache.host_classified < 200
    og = oracle.Grammar(si.XML_GRAMMAR, "root")
    _check_cache_classes(xgm, cache, g, og, vocab, range(g.num_nodes))
    walker = wl.BatchWalker([cache, cache], vocab, seed=21, structural_bias=0.5)
    oms = [oracle.EarleyMatcher(og) for _ in range(2)]
    toks = vocab.tokens()
    n_multi = n_fixed = 0
    for step in range(160):
        words = walker.fill()
        fixed = xgm.fill_overflow_fixup(_stream())
        if fixed:
            n_fixed += fixed
            words = walker.d_mask.cpu().numpy()
        want = np.stack([om.mask(vocab) for om in oms])
        assert np.array_equal(words, oracle.pack_bitmask(want)), f"step {step}"
        n_multi += sum(m.num_stacks() > 1 for m in walker.matchers)
        picks = walker.step(words)
        for b in range(2):
            if not walker.history[b]:
                oms[b] = oracle.EarleyMatcher(og)
            else:
                assert oms[b].advance(toks[int(picks[b])])
    say(f"  (row, step) pairs with several parallel stacks: {n_multi}; build pairs on the host: "
        f"{cache.host_classified}; fill pairs fixed up: {n_fixed}")


# --------------------------------------------------------------------------
# storage of the cache (section 3.1): a bitset row where many tokens are accepted (every distinct row
# once), a list where few are; either way the node's accepted set is the oracle's
# --------------------------------------------------------------------------
def test_cache_storage_is_adaptive_and_exact(xgm, wl):
    vocab = si.make_vocab("bpe", 32000, 0)
    xv = wl.make_xgm_vocab(vocab)
    W = xgm.bitmask_words(vocab.size)
    for name, text, root in [("json", si.JSON_GRAMMAR, "root"), ("csql", si.CSQL_GRAMMAR, "root"),
                             ("schema", si.make_schema_grammar(3, string_heavy=True), "root")]:
        g = xgm.Grammar(text, root)
        cache = xgm.Cache(g, xv)
        og = oracle.Grammar(text, root)
        rows, as_list = {}, 0
        rng = np.random.Generator(np.random.PCG64(zlib.crc32(name.encode())))
        sample = set(int(n) for n in rng.choice(cache.num_nodes, size=min(cache.num_nodes, 24), replace=False))
        for node in range(cache.num_nodes):
            acc, _ = cache.copy_node_bits(node, with_uncertain=False)
            n_acc = int(np.unpackbits(acc.view(np.uint8)).sum())
            if 2 * n_acc <= W:
                as_list += 1          # few accepted tokens: kept as a list of token ids
            else:
                rows.setdefault(acc.tobytes(), []).append(node)
            if node in sample:        # (every node of these grammars is checked by the class tests at V = 128256)
                want = og.classify(g.rule_name(g.node_rule(node)), g.node_path(node), vocab)
                assert np.array_equal(acc, oracle.pack_bitmask(want == 2)), (name, node)
        st = cache.stats
        say(f"{name}: {cache.num_nodes} nodes: {as_list} keep a list, {len(rows)} distinct bitsets among the others, "
            f"{cache.num_accept_rows} rows kept; {st['entries']} list entries under {st['keys']} keys; "
            f"{cache.device_bytes / 1e6:.2f} MB on the device")
        assert cache.num_accept_rows == len(rows) == st["bitset_rows"]
        assert cache.device_bytes >= cache.num_accept_rows * W * 4 + 4 * st["entries"]
        # the schema grammars of the serving workload: far below one bitset per node (the C-like grammar, whose
        # rules are used in dozens of places each, spends its memory on the per-context lists instead)
        if name == "schema":
            assert cache.device_bytes < 0.25 * cache.num_nodes * W * 4


# --------------------------------------------------------------------------
# a third grammar family: a scripting language with word operators and one-line bodies
# --------------------------------------------------------------------------
def test_scripting_grammar_every_step_and_every_node(xgm, wl):
    say("scripting grammar: V=32000 B=2 steps=160, classes at every node")
    vocab = si.make_vocab("bpe", 32000, 0)
    g = xgm.Grammar(si.PYDSL_GRAMMAR, "root")
    cache = xgm.Cache(g, wl.make_xgm_vocab(vocab), keep_plain=True)
    og = oracle.Grammar(si.PYDSL_GRAMMAR, "root")
    _check_cache_classes(xgm, cache, g, og, vocab, range(g.num_nodes))
    walker = wl.BatchWalker([cache, cache], vocab, seed=23, structural_bias=0.5)
    oms = [oracle.EarleyMatcher(og) for _ in range(2)]
    toks = vocab.tokens()
    n_multi = n_fixed = 0
    for step in range(160):
        words = walker.fill()
        fixed = xgm.fill_overflow_fixup(_stream())
        if fixed:
            n_fixed += fixed
            words = walker.d_mask.cpu().numpy()
        want = np.stack([om.mask(vocab) for om in oms])
        assert np.array_equal(words, oracle.pack_bitmask(want)), f"step {step}"
        n_multi += sum(m.num_stacks() > 1 for m in walker.matchers)
        picks = walker.step(words)
        for b in range(2):
            if not walker.history[b]:
                oms[b] = oracle.EarleyMatcher(og)
            else:
                assert oms[b].advance(toks[int(picks[b])])
    say(f"  nodes {g.num_nodes}; (row, step) pairs with several parallel stacks: {n_multi}; build pairs on the host: "
        f"{cache.host_classified}; fill pairs fixed up: {n_fixed}")


# --------------------------------------------------------------------------
# caches resolved fewer frames deep at build time: more is walked at fill time, the masks are the same
# --------------------------------------------------------------------------
@pytest.mark.parametrize("depth", [1, 2])
def test_shallower_caches_give_the_same_masks(xgm, wl, depth):
    say(f"caches built {depth} frame(s) deep: JSON, a schema grammar and the scripting grammar, V=32000, 96 steps")
    vocab = si.make_vocab("bpe", 32000, 0)
    xv = wl.make_xgm_vocab(vocab)
    texts = [si.JSON_GRAMMAR, si.make_schema_grammar(1, string_heavy=True), si.PYDSL_GRAMMAR]
    grammars = [xgm.Grammar(t, "root") for t in texts]
    caches = [xgm.Cache(g, xv, depth=depth) for g in grammars]
    full = [xgm.Cache(g, xv) for g in grammars]
    for c, f in zip(caches, full):
        assert c.stats["keys"] < f.stats["keys"]   # (not fewer entries: what the deeper levels reject stays listed, to be walked)
    walker = wl.BatchWalker(caches, vocab, seed=31 + depth, structural_bias=0.4)
    oms = [oracle.EarleyMatcher(oracle.Grammar(t, "root")) for t in texts]
    toks = vocab.tokens()
    B, W = len(texts), xgm.bitmask_words(vocab.size)
    d_mask2 = torch.zeros((B, W), dtype=torch.int32, device="cuda")
    steps_walked = n_fixed = 0
    for step in range(96):
        words = walker.fill()
        fixed = xgm.fill_overflow_fixup(_stream())
        if fixed:
            n_fixed += fixed
            words = walker.d_mask.cpu().numpy()
        want = np.stack([om.mask(vocab) for om in oms])
        assert np.array_equal(words, oracle.pack_bitmask(want)), f"step {step}"
        if step % 8 == 0:   # the same states resident on the device, and how much was walked
            db = xgm.DeviceBatch(walker.matchers, history=0, stream=_stream())
            db.fill_next_token_bitmask(d_mask2.data_ptr(), _stream())
            db.fill_overflow_fixup(_stream())
            torch.cuda.synchronize()
            assert np.array_equal(d_mask2.cpu().numpy(), oracle.pack_bitmask(want)), f"step {step}, resident states"
            steps_walked += xgm.debug_fill_count_steps(walker.batch, d_mask2.data_ptr(), _stream())
        picks = walker.step(words)
        for b in range(B):
            if not walker.history[b]:
                oms[b] = oracle.EarleyMatcher(oracle.Grammar(texts[b], "root"))
            else:
                assert oms[b].advance(toks[int(picks[b])])
    assert steps_walked > 0   # (with all three levels these states need next to no walks)
    say(f"  96 steps x {B} rows bit-exact from host-side and resident states; automaton steps walked in 12 sampled fills: "
        f"{steps_walked}; pairs fixed up on the host: {n_fixed}")


# --------------------------------------------------------------------------
# fused fill + apply: same masks, same logits as the two calls / as the oracle
# --------------------------------------------------------------------------
# (vocabularies above 8192 tokens have segments that lie wholly inside the row: the one-launch kernel masks those
# by a path of their own)
@pytest.mark.parametrize("dtype_name,V,pad", [("bf16", 4100, 0), ("f32", 4100, 0), ("f16", 4099, 13), ("bf16", 9000, 24),
                                              ("f32", 9000, 0), ("f16", 17001, 5), ("f32", 16384, 4)])
def test_fused_fill_and_apply_matches_oracle(xgm, wl, no_overflow, dtype_name, V, pad):
    say(f"fused fill+apply: json V={V} logits width {V + pad} {dtype_name}")
    tdt, code, ninf, view, npv = {"f32": (torch.float32, xgm.DTYPE_F32, 0xFF800000, torch.int32, np.uint32),
                                  "bf16": (torch.bfloat16, xgm.DTYPE_BF16, 0xFF80, torch.int16, np.uint16),
                                  "f16": (torch.float16, xgm.DTYPE_F16, 0xFC00, torch.int16, np.uint16)}[dtype_name]
    vocab = si.make_vocab("bpe", V, 1)
    xv = wl.make_xgm_vocab(vocab)
    texts = [si.JSON_GRAMMAR, si.make_schema_grammar(2, string_heavy=True), si.JSON_GRAMMAR]
    roots = ["root"] * 3
    caches = [xgm.Cache(xgm.Grammar(t, r), xv) for t, r in zip(texts, roots)]
    walker = wl.BatchWalker(caches, vocab, seed=11, structural_bias=0.35)
    oms = [oracle.EarleyMatcher(oracle.Grammar(t, r)) for t, r in zip(texts, roots)]
    toks = vocab.tokens()
    B, W = 3, xgm.bitmask_words(V)
    Vl = V + pad
    stride = ((Vl * (4 if dtype_name == "f32" else 2) + 15) // 16 * 16) // (4 if dtype_name == "f32" else 2)
    d_mask = torch.zeros((B, W), dtype=torch.int32, device="cuda")
    for step in range(24):
        words = walker.fill()
        if step % 4 == 3:
            want = np.stack([om.mask(vocab) for om in oms])
            buf = torch.zeros((B, stride), dtype=tdt, device="cuda")
            buf[:, :Vl] = torch.from_numpy(si.make_logits(B, Vl, seed=900 + step)).to("cuda").to(tdt)
            before = buf.view(view).cpu().numpy().view(npv).copy()
            d_mask.fill_(-1)
            xgm.fill_and_apply(walker.batch, d_mask.data_ptr(), buf.data_ptr(), code, Vl, stride, stream=_stream())
            torch.cuda.synchronize()
            assert np.array_equal(d_mask.cpu().numpy(), oracle.pack_bitmask(want)), f"step {step}"
            after = buf.view(view).cpu().numpy().view(npv)
            expect = before.copy()
            expect[:, :Vl] = oracle.apply_mask(before[:, :Vl], want, ninf)
            assert np.array_equal(after, expect), f"step {step}"      # the padding of the rows is untouched, too
        picks = walker.step(words)
        for b in range(B):
            if not walker.history[b]:
                oms[b] = oracle.EarleyMatcher(oracle.Grammar(texts[b], roots[b]))
            else:
                assert oms[b].advance(toks[int(picks[b])])


def test_fused_fill_and_apply_argument_errors(xgm, wl):
    vocab = si.make_vocab("arith", 1024, 0)
    cache = xgm.Cache(xgm.Grammar(si.ARITH_GRAMMAR, "expr"), wl.make_xgm_vocab(vocab))
    m = xgm.Matcher(cache=cache)
    d_mask = torch.zeros((1, 32), dtype=torch.int32, device="cuda")
    buf = torch.zeros((1, 1040), dtype=torch.float32, device="cuda")
    with pytest.raises(xgm.XgmError):      # rows narrower than the vocabulary
        xgm.fill_and_apply([m], d_mask.data_ptr(), buf.data_ptr(), xgm.DTYPE_F32, 1000, 1040, stream=_stream())
    with pytest.raises(xgm.XgmError):      # misaligned base
        xgm.fill_and_apply([m], d_mask.data_ptr(), buf.data_ptr() + 4, xgm.DTYPE_F32, 1024, 1032, stream=_stream())
    with pytest.raises(xgm.XgmError):      # row pitch not a multiple of 16 bytes
        xgm.fill_and_apply([m], d_mask.data_ptr(), buf.data_ptr(), xgm.DTYPE_F32, 1024, 1025, stream=_stream())
    with pytest.raises(xgm.XgmError):
        xgm.fill_and_apply([m], d_mask.data_ptr(), 0, xgm.DTYPE_F32, 1024, 1024, stream=_stream())


# --------------------------------------------------------------------------
# apply: dtypes, ragged sizes, row subsets, strides, special values
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype_name", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("V,Vl", [(1000, 1000), (1003, 1003), (37, 41), (4097, 4100), (64, 64)])
def test_apply_shapes_and_special_values(xgm, dtype_name, V, Vl):
    code, tdt, ninf, udt = {
        "f32": (xgm.DTYPE_F32, torch.float32, 0xFF800000, np.uint32),
        "bf16": (xgm.DTYPE_BF16, torch.bfloat16, 0xFF80, np.uint16),
        "f16": (xgm.DTYPE_F16, torch.float16, 0xFC00, np.uint16),
    }[dtype_name]
    rng = np.random.Generator(np.random.PCG64(V * 7 + Vl))
    B = 5
    allowed = rng.random((B, V)) < 0.5
    allowed[0] = True
    allowed[1] = False
    allowed[2, : V // 2] = True
    # raw bit patterns, including NaNs, infinities, zeros and subnormals
    bits = rng.integers(0, 2 ** (16 if udt == np.uint16 else 32), size=(B, Vl), dtype=np.uint64).astype(udt)
    view = torch.int32 if udt == np.uint32 else torch.int16
    sview = np.int32 if udt == np.uint32 else np.int16
    for stride in (Vl, Vl + 3, ((Vl + 7) // 8) * 8):
        buf = torch.zeros((B, stride), dtype=view, device="cuda")
        buf[:, :Vl] = torch.from_numpy(bits.view(sview)).cuda()
        t = buf.view(tdt)
        d_mask = torch.from_numpy(oracle.pack_bitmask(allowed)).cuda()
        xgm.apply_token_bitmask_inplace(t.data_ptr(), code, B, Vl, stride, d_mask.data_ptr(), V, stream=_stream())
        got = buf[:, :Vl].cpu().numpy().view(udt)
        assert np.array_equal(got, oracle.apply_mask(bits, allowed, ninf)), (dtype_name, V, Vl, stride)
        assert (buf[:, Vl:].cpu().numpy() == 0).all()  # padding beyond the row is never written


def test_apply_row_subset(xgm):
    V, B = 5000, 6
    rng = np.random.Generator(np.random.PCG64(17))
    allowed = rng.random((3, V)) < 0.3
    bits = rng.integers(0, 2 ** 16, size=(B, V), dtype=np.uint64).astype(np.uint16)
    t = torch.from_numpy(bits.view(np.int16)).cuda()
    rows = np.array([4, 0, 3], dtype=np.int32)
    d_rows = torch.from_numpy(rows).cuda()
    d_mask = torch.from_numpy(oracle.pack_bitmask(allowed)).cuda()
    xgm.apply_token_bitmask_inplace(t.data_ptr(), xgm.DTYPE_BF16, B, V, V, d_mask.data_ptr(), V,
                                    d_row_index=d_rows.data_ptr(), n_rows=3, stream=_stream())
    got = t.cpu().numpy().view(np.uint16)
    want = bits.copy()
    for j, r in enumerate(rows):
        want[r] = oracle.apply_mask(bits[r:r + 1], allowed[j:j + 1], 0xFF80)[0]
    assert np.array_equal(got, want)


def test_apply_argument_errors(xgm):
    t = torch.zeros((2, 64), dtype=torch.float32, device="cuda")
    m = torch.zeros((2, 2), dtype=torch.int32, device="cuda")
    for kwargs in [dict(d_logits=0), dict(dtype=7), dict(V_logits=0), dict(row_stride=10), dict(n_rows=1)]:
        args = dict(d_logits=t.data_ptr(), dtype=xgm.DTYPE_F32, B=2, V_logits=64, row_stride=64,
                    d_bitmask=m.data_ptr(), V_mask=64, n_rows=2)
        args.update(kwargs)
        with pytest.raises(xgm.XgmError) as e:
            xgm.apply_token_bitmask_inplace(**args)
        assert e.value.status == -1


# --------------------------------------------------------------------------
# fill: edge cases
# --------------------------------------------------------------------------
def test_fill_terminated_rows_ragged_vocab_and_stop_tokens(xgm, wl):
    # vocabulary size not a multiple of 32, two stop tokens
    toks = [b"1", b"2", b"+", b"*", b"(", b")", b" ", b"12", b"+1", b")*", b"", b"((", b"1)", b"", b"3 "] + \
           [bytes([48 + k % 10]) * (1 + k % 3) + b"+" for k in range(28)]
    V = len(toks)
    assert V % 32 != 0

    class V_:  # minimal vocabulary object for both sides
        data = np.frombuffer(b"".join(toks), dtype=np.uint8).copy()
        offsets = np.concatenate([[0], np.cumsum([len(t) for t in toks])]).astype(np.int64)
        stop_ids = np.array([10, 13], dtype=np.int32)

    xv = xgm.Vocab(V_.data, V_.offsets, V_.stop_ids)
    g = xgm.Grammar(si.ARITH_GRAMMAR, "expr")
    cache = xgm.Cache(g, xv)
    og = oracle.Grammar(si.ARITH_GRAMMAR, "expr")
    ms = [xgm.Matcher(cache=cache) for _ in range(4)]
    oms = [oracle.EarleyMatcher(og) for _ in range(4)]
    for m, om, text in zip(ms, oms, [b"", b"1", b"(1+2", b"1 "]):
        if text:
            m.accept_bytes(text)
            assert om.advance(text)
    ms[1].accept_token(10)  # stop: row 1 is terminated now
    W = xgm.bitmask_words(V)
    d = torch.full((4, W), -1, dtype=torch.int32, device="cuda")
    xgm.fill_next_token_bitmask(ms, d.data_ptr(), _stream())
    got = d.cpu().numpy()
    want = np.stack([om.mask(V_) for om in oms])
    want[1] = False
    want[1, [10, 13]] = True  # a terminated request allows only the stop tokens
    assert np.array_equal(got, oracle.pack_bitmask(want))
    assert not want[0, 10] and want[3].sum() > 0
    with pytest.raises(xgm.XgmError):
        xgm.fill_next_token_bitmask([], d.data_ptr(), _stream())


def test_fill_deep_stacks_and_many_parallel_stacks(xgm, wl, no_overflow):
    vocab = si.make_vocab("bpe", 32000, 0)
    xv = wl.make_xgm_vocab(vocab)
    g = xgm.Grammar(si.JSON_GRAMMAR, "root")
    cache = xgm.Cache(g, xv)
    og = oracle.Grammar(si.JSON_GRAMMAR, "root")
    text = b"[" * 300 + b'{"a":' + b"[" * 200 + b"1"
    m = xgm.Matcher(cache=cache)
    m.accept_bytes(text)
    assert len(m.stack(0)) > 400
    om = oracle.EarleyMatcher(og)
    assert om.advance(text)
    # ambiguous grammar: 64 parallel stacks
    amb = 'root ::= a | b\na ::= "x" root? "p"\nb ::= "x" root? "q"'
    ga = xgm.Grammar(amb, "root")
    ca = xgm.Cache(ga, xv)
    ma = xgm.Matcher(cache=ca)
    ma.accept_bytes(b"xxxxxx")
    assert ma.num_stacks() == 64
    oa = oracle.EarleyMatcher(oracle.Grammar(amb, "root"))
    assert oa.advance(b"xxxxxx")
    W = xgm.bitmask_words(32000)
    d = torch.zeros((2, W), dtype=torch.int32, device="cuda")
    xgm.fill_next_token_bitmask([m, ma], d.data_ptr(), _stream())
    got = d.cpu().numpy()
    assert np.array_equal(got[0], oracle.pack_bitmask(om.mask(vocab)))
    assert np.array_equal(got[1], oracle.pack_bitmask(oa.mask(vocab)))


def test_walk_limits_are_reported_and_fixed_up_exactly(xgm, wl):
    """Tokens that exceed the on-chip limits (here: longer than 255 bytes, and
    30 nested parentheses = more than 64 frames) are decided exactly by the
    host slow path, at build time and at fill time."""
    toks = [b"1", b"(", b")", b"+", b"1" * 300, b"(" * 30, b"1" * 20, b")" * 40, b""]
    V = len(toks)

    class V_:
        data = np.frombuffer(b"".join(toks), dtype=np.uint8).copy()
        offsets = np.concatenate([[0], np.cumsum([len(t) for t in toks])]).astype(np.int64)
        stop_ids = np.array([8], dtype=np.int32)

    xv = xgm.Vocab(V_.data, V_.offsets, V_.stop_ids)
    g = xgm.Grammar(si.ARITH_GRAMMAR, "expr")
    before = xgm.overflow_total()
    cache = xgm.Cache(g, xv, keep_plain=True)
    assert cache.host_classified > 0
    og = oracle.Grammar(si.ARITH_GRAMMAR, "expr")
    _check_cache_classes(xgm, cache, g, og, V_, range(g.num_nodes))
    # fill: after "(" * 41 + "1", the token ")" * 40 pops 40 x 3 live frames (fine on chip);
    # the 300-digit token is context-dependent at a digit node and exceeds the byte limit
    m = xgm.Matcher(cache=cache)
    om = oracle.EarleyMatcher(og)
    text = b"(" * 41 + b"1"
    m.accept_bytes(text)
    assert om.advance(text)
    d = torch.zeros((1, 1), dtype=torch.int32, device="cuda")
    xgm.fill_next_token_bitmask([m], d.data_ptr(), _stream())
    n_fixed = xgm.fill_overflow_fixup(_stream())
    got = d.cpu().numpy()
    assert np.array_equal(got[0], oracle.pack_bitmask(om.mask(V_)))
    say(f"  build: {cache.host_classified} pairs on the host; fill: {n_fixed} pairs fixed up; "
        f"log grew by {xgm.overflow_total() - before}")


def test_fused_path_leaves_undecided_tokens_allowed_until_the_fixup(xgm, wl):
    """Walks over the on-chip limits in the fused call: the token's logit is
    left untouched and its bit set; the fixup then writes the exact bit, set
    (token 4, allowed) or cleared (token 5, not allowed), and a second apply
    finishes the logits."""
    deep = b")+" + b"(" * 30          # closes one level, then opens 30: more than 64 frames in one token
    toks = [b"1", b"(", b")", b"+", deep, deep + b"+", b"1" * 20, b")" * 40, b""]
    V = len(toks)

    class V_:
        data = np.frombuffer(b"".join(toks), dtype=np.uint8).copy()
        offsets = np.concatenate([[0], np.cumsum([len(t) for t in toks])]).astype(np.int64)
        stop_ids = np.array([8], dtype=np.int32)

    xv = xgm.Vocab(V_.data, V_.offsets, V_.stop_ids)
    g = xgm.Grammar(si.ARITH_GRAMMAR, "expr")
    cache = xgm.Cache(g, xv)
    og = oracle.Grammar(si.ARITH_GRAMMAR, "expr")
    m = xgm.Matcher(cache=cache)
    om = oracle.EarleyMatcher(og)
    text = b"(" * 41 + b"1"
    m.accept_bytes(text)
    assert om.advance(text)
    want = om.mask(V_)
    assert want[4] and not want[5]
    d = torch.zeros((1, 1), dtype=torch.int32, device="cuda")
    logits = torch.arange(1, 17, dtype=torch.float32, device="cuda").reshape(1, 16).contiguous()
    before = xgm.overflow_total()
    xgm.fill_and_apply([m], d.data_ptr(), logits.data_ptr(), xgm.DTYPE_F32, 16, 16, stream=_stream())
    torch.cuda.synchronize()
    assert xgm.overflow_total() - before == 2
    out = logits.cpu().numpy()[0]
    for i in range(V):
        if want[i] or i in (4, 5):     # allowed, or undecided so far
            assert out[i] == float(i + 1), i
        else:
            assert out[i] == float("-inf"), i
    assert np.all(out[V:] == float("-inf"))          # columns beyond the vocabulary are masked
    assert xgm.fill_overflow_fixup(_stream()) == 2
    assert np.array_equal(d.cpu().numpy()[0], oracle.pack_bitmask(want))
    xgm.apply_token_bitmask_inplace(logits.data_ptr(), xgm.DTYPE_F32, 1, 16, 16, d.data_ptr(), V, stream=_stream())
    out = logits.cpu().numpy()[0]
    for i in range(V):
        assert (out[i] == float(i + 1)) == bool(want[i]), i
    # the two-call path on the same state: undecided tokens are not allowed until the fixup
    d.zero_()
    xgm.fill_next_token_bitmask([m], d.data_ptr(), _stream())
    got = d.cpu().numpy()[0].copy()
    assert not (int(got[0]) >> 4) & 1 and not (int(got[0]) >> 5) & 1
    assert xgm.fill_overflow_fixup(_stream()) == 2
    assert np.array_equal(d.cpu().numpy()[0], oracle.pack_bitmask(want))


def test_fill_states_with_the_longest_lists(xgm, wl, no_overflow):
    """States whose stack tops have tens of thousands of context-dependent tokens (inside a string, after a
    value), at the full vocabulary: host-side and device-resident states, mask only and with the logits."""
    vocab = si.make_vocab("bpe", 151936, 0)
    xv = wl.make_xgm_vocab(vocab)
    specs = [(si.JSON_GRAMMAR, b'{"key": "val'), (si.make_schema_grammar(5, string_heavy=True), None), (si.JSON_GRAMMAR, b'[1, ')]
    caches = [xgm.Cache(xgm.Grammar(t, "root"), xv) for t, _ in specs]
    ms = [xgm.Matcher(cache=c) for c in caches]
    oms = [oracle.EarleyMatcher(oracle.Grammar(t, "root")) for t, _ in specs]
    toks = vocab.tokens()
    for b, (m, om, (_, text)) in enumerate(zip(ms, oms, specs)):
        if text is not None:
            m.accept_bytes(text)
            assert om.advance(text)
        else:   # walk the schema grammar into a string value: the state with the longest lists
            info = wl.TokenInfo(vocab)
            rng = np.random.Generator(np.random.PCG64(3))
            for _ in range(120):
                tops = [m.stack(s)[-1] for s in range(m.num_stacks())]
                if max(caches[b].num_uncertain(t) for t in tops) > 10000:
                    break
                want = om.mask(vocab)
                want[vocab.stop_ids] = False
                t = int(si.pick_tokens(rng, want[None, :], info.structural, info.is_stop, 0.35)[0])
                m.accept_token(t)
                assert om.advance(toks[t])
    entries = [sum(c.num_uncertain(m.stack(s)[-1]) for s in range(m.num_stacks())) for m, c in zip(ms, caches)]
    assert max(entries) > 10000, entries
    want = oracle.pack_bitmask(np.stack([om.mask(vocab) for om in oms]))
    W = xgm.bitmask_words(vocab.size)
    d = torch.zeros((3, W), dtype=torch.int32, device="cuda")
    xgm.fill_next_token_bitmask(ms, d.data_ptr(), _stream())
    assert np.array_equal(d.cpu().numpy(), want)
    batch = xgm.DeviceBatch(ms, history=0, stream=_stream())
    d.zero_()
    batch.fill_next_token_bitmask(d.data_ptr(), _stream())
    assert np.array_equal(d.cpu().numpy(), want)
    bits = np.unpackbits(want.view(np.uint8), axis=1, bitorder="little")[:, :vocab.size].astype(bool)
    for fill_and_apply in (lambda lg: xgm.fill_and_apply(ms, d.data_ptr(), lg.data_ptr(), xgm.DTYPE_BF16, vocab.size,
                                                          vocab.size, _stream()),
                           lambda lg: batch.fill_and_apply(d.data_ptr(), lg.data_ptr(), xgm.DTYPE_BF16, vocab.size,
                                                           vocab.size, _stream())):
        logits = torch.from_numpy(si.make_logits(3, vocab.size, 77)).to(torch.bfloat16).cuda()
        before = logits.view(torch.int16).cpu().numpy().view(np.uint16).copy()
        d.zero_()
        fill_and_apply(logits)
        assert np.array_equal(d.cpu().numpy(), want)
        after = logits.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(after, np.where(bits, before, np.uint16(0xFF80)))
    say(f"  context-dependent tokens at the stack tops per row {entries}: masks and logits bit-exact")


def test_grammars_from_the_schema_front_end_every_step(xgm, wl):
    """Schemas with optional members, bounded arrays, unions and free-form parts, turned into grammars by
    xgm_schema_to_grammar: rules with empty alternatives and ambiguous white space on the HIP path."""
    import json
    from test_schema_frontend import HANDWRITTEN, to_json_schema
    vocab = si.make_vocab("bpe", 32000, 0)
    xv = wl.make_xgm_vocab(vocab)
    rng = np.random.Generator(np.random.PCG64(8))
    schemas = [HANDWRITTEN] + [to_json_schema(si.random_schema(s, max_depth=3, string_heavy=True), rng) for s in (11, 12, 13)]
    texts = [xgm.schema_to_grammar(json.dumps(s, ensure_ascii=False)) for s in schemas]
    caches = [xgm.Cache(xgm.Grammar(t, "root"), xv) for t in texts]
    walker = wl.BatchWalker(caches, vocab, seed=21, structural_bias=0.4)
    ogs = [oracle.Grammar(t, "root") for t in texts]
    oms = [oracle.EarleyMatcher(o) for o in ogs]
    toks = vocab.tokens()
    before = xgm.overflow_total()
    for step in range(48):
        words = walker.fill()
        if xgm.overflow_total() != before:          # ambiguous white space: a few walks over the limits
            xgm.fill_overflow_fixup(_stream())
            words = walker.d_mask.cpu().numpy()
            before = xgm.overflow_total()
        want = np.stack([om.mask(vocab) for om in oms])
        assert np.array_equal(words, oracle.pack_bitmask(want)), f"step {step}: rows {np.flatnonzero((words != oracle.pack_bitmask(want)).any(axis=1))}"
        picks = walker.step(words)
        for b in range(len(oms)):
            if not walker.history[b]:
                oms[b] = oracle.EarleyMatcher(ogs[b])
            else:
                assert oms[b].advance(toks[int(picks[b])])
    say(f"  4 front-end grammars x 48 steps bit-exact; most parallel stacks in a row: {max(m.num_stacks() for m in walker.matchers)}")
