"""CPU tests of the library's host side: C-ABI surface, grammar compilation,
matcher state, error codes.  The automaton is compared with the oracle on
membership and on token classes (the oracle never sees the library's tables;
a node is named by its rule and a symbol path from the rule's start)."""

import ctypes
import os
import re
import zlib

import numpy as np
import pytest

import oracle
import paper_2411_15100_amd as xgm
from paper_2411_15100_amd import binding
import synth_inputs as si
from test_oracle_misc import TinyVocab

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

GRAMMARS = {
    "arith": (si.ARITH_GRAMMAR, "expr", b"0123456789+*() "),
    "json": (si.JSON_GRAMMAR, "root", b' \n"{}[],:\\/abfnrtu0123456789.eE+-\xc3\xa9\xe4\xb8\xad\xf0\x9f\x98\x80xyz'),
    "csql": (si.CSQL_GRAMMAR, "root", b" \n(){}[];,.*+-/%<>=!&|^~?:'\"\\_abcdefhilnorstuwxSELCTFROMWHNDBYGUPIAV0123459"),
    "xml": (si.XML_GRAMMAR, "root", b" \n\t<>/=\"'&;#!-._abcxyzAZ019"),
    "pydsl": (si.PYDSL_GRAMMAR, "root", b" \n()[]{}:;,.=+-*/%<>!~#'\"\\xzuv_ab019ifelsnotrdwhpcTFNm"),
    "schema": (si.make_schema_grammar(3), "root", b' \n"{}[],:\\abcdefghijklmnopqrstuvwxyz_0123456789.eE+-tfu'),
}


def test_every_declared_symbol_is_exported_and_bound():
    header = open(os.path.join(ROOT, "include", "xgm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(xgm_[a-z_0-9]+)\s*\(", header))
    assert len(declared) >= 30
    lib = xgm.load_library()
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared but not exported"
        assert name in binding.SIGNATURES, f"{name} has no binding"
    assert set(binding.SIGNATURES) == declared


@pytest.mark.parametrize("name", list(GRAMMARS))
def test_membership_matches_oracle_on_random_byte_walks(name):
    text, root, alphabet = GRAMMARS[name]
    g = xgm.Grammar(text, root)
    og = oracle.Grammar(text, root)
    rng = np.random.Generator(np.random.PCG64(zlib.crc32(name.encode())))
    n_accept = n_reject = 0
    for trial in range(12):
        m = xgm.Matcher(grammar=g)
        prefix = b""
        for step in range(60):
            assert m.can_terminate() == (og.recognize(prefix) == 2), prefix
            # try several random bytes; the oracle must agree on every verdict
            progressed = False
            for b in rng.permutation(list(alphabet))[:8]:
                cand = prefix + bytes([int(b)])
                rc = m.try_accept_bytes(bytes([int(b)]))
                want = og.recognize(cand) > 0
                assert (rc == 0) == want, (cand, rc)
                if rc == 0:
                    n_accept += 1
                    prefix = cand
                    progressed = True
                    break
                assert rc == -6  # TOKEN_REJECTED, state unchanged
                n_reject += 1
            if not progressed:
                # steer with the oracle's completion so the walk keeps going
                tail = oracle.EarleyMatcher(og)
                assert tail.advance(prefix)
                nxt = tail.completion()[:1]
                if not nxt:
                    break
                m.accept_bytes(nxt)
                prefix += nxt
    assert n_accept > 50 and n_reject > 100


def test_multibyte_chunks_equal_single_bytes():
    g = xgm.Grammar(si.JSON_GRAMMAR, "root")
    doc = '{"k\\u00e9": [1.5e3, "中\U0001f600", true, null, {"x": -0}]}'.encode()
    rng = np.random.Generator(np.random.PCG64(2))
    for _ in range(20):
        m = xgm.Matcher(grammar=g)
        pos = 0
        while pos < len(doc):
            k = int(rng.integers(1, 7))
            m.accept_bytes(doc[pos:pos + k])
            pos += k
        assert m.can_terminate()
        assert m.num_stacks() >= 1


def _classes_for_all_nodes(text, root, vocab, nodes=None):
    g = xgm.Grammar(text, root)
    og = oracle.Grammar(text, root)
    toks = vocab.tokens() if hasattr(vocab, "tokens") else vocab.toks
    seen = set()
    for node in (range(g.num_nodes) if nodes is None else nodes):
        rule = g.rule_name(g.node_rule(node))
        path = g.node_path(node)
        want = og.classify(rule, path, vocab)
        got = np.array([g.debug_classify_host(node, t) for t in toks], dtype=np.uint8)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, (rule, path, toks[bad[0]], int(got[bad[0]]), int(want[bad[0]]))
        seen |= set(got.tolist())
    return seen


def test_host_classes_match_oracle_arith_all_nodes():
    vocab = si.make_vocab("arith", 1024, 0)
    assert _classes_for_all_nodes(si.ARITH_GRAMMAR, "expr", vocab) == {0, 1, 2, 4}


def test_host_classes_match_oracle_json_all_nodes():
    import itertools
    alphabet = [b'"', b"\\", b"{", b"}", b"[", b"]", b",", b":", b" ", b"1", b"0", b"-", b".", b"e", b"t", b"r", b"u",
                b"a", b"\xc3", b"\xa9", b"\xf0", b"\x9f", b"n"]
    toks = [b"".join(t) for n in (1, 2) for t in itertools.product(alphabet, repeat=n)]
    toks += [b"true", b"null", b"fals", b'"ab"', b'":', b'",', b'"}', b"\\u00e9", b"1.5e3", b"", b"\xe4\xb8\xad", b"\xe4\xb8"]
    vocab = TinyVocab(toks)
    assert _classes_for_all_nodes(si.JSON_GRAMMAR, "root", vocab) == {0, 1, 2, 4}


def test_host_classes_match_oracle_csql_sample():
    vocab = si.make_vocab("bpe", 2048, 1)
    g = xgm.Grammar(si.CSQL_GRAMMAR, "root")
    rng = np.random.Generator(np.random.PCG64(4))
    nodes = sorted(set(int(n) for n in rng.integers(0, g.num_nodes, size=25)))
    _classes_for_all_nodes(si.CSQL_GRAMMAR, "root", vocab, nodes)


def test_compile_errors():
    def status(text, root="root"):
        with pytest.raises(xgm.XgmError) as e:
            xgm.Grammar(text, root)
        return e.value.status

    assert status('root ::= "a') == -2
    assert status("root ::= [a") == -2
    assert status('root ::= ("a"') == -2
    assert status('root ::= "a")') == -2
    assert status('root = "a"') == -2
    assert status("") == -2
    assert status('root ::= "a"\nroot ::= "b"') == -2
    assert status('root ::= "\\q"') == -2
    assert status("root ::= other") == -3
    assert status('a ::= "x"') == -3
    assert status('root ::= root "a" | "b"') == -4
    assert status('root ::= a "x" | "z"\na ::= b? root\nb ::= "y"') == -4      # hidden behind a nullable prefix
    assert status('root ::= "a" root') == -5
    assert status('root ::= dead\ndead ::= "x" dead') == -5


def test_left_recursion_rejection_is_conservative():
    """The library refuses left-recursive grammars; the oracle's Earley side
    takes them, which shows nothing else is affected by the refusal."""
    text = 'E ::= E "+" "n" | "n"'
    assert oracle.Grammar(text, "E").recognize(b"n+n") == 2
    with pytest.raises(xgm.XgmError) as e:
        xgm.Grammar(text, "E")
    assert e.value.status == -4


def test_unproductive_and_unreachable_parts_are_dropped():
    g = xgm.Grammar('root ::= "a" dead | "a" "b"\ndead ::= "x" dead\nunused ::= "zzz"', "root")
    assert g.num_rules == 1
    m = xgm.Matcher(grammar=g)
    m.accept_bytes(b"a")
    assert m.try_accept_bytes(b"x") == -6
    m.accept_bytes(b"b")
    assert m.can_terminate()


def test_nullable_rules_and_loops():
    text = 'root ::= (e | "a")* "b"\ne ::= "c"?'
    g = xgm.Grammar(text, "root")
    og = oracle.Grammar(text, "root")
    import itertools
    for n in range(0, 6):
        for tup in itertools.product(b"abc", repeat=n):
            s = bytes(tup)
            m = xgm.Matcher(grammar=g)
            ok = m.try_accept_bytes(s) == 0
            want = og.recognize(s)
            assert ok == (want > 0), s
            if ok:
                assert m.can_terminate() == (want == 2), s


def test_token_level_errors_and_termination():
    vocab = si.make_vocab("arith", 1024, 0)
    toks = vocab.tokens()
    index = {t: i for i, t in enumerate(toks)}
    stop = int(vocab.stop_ids[0])
    g = xgm.Grammar(si.ARITH_GRAMMAR, "expr")
    v = xgm.Vocab(vocab.data, vocab.offsets, vocab.stop_ids)
    m = xgm.Matcher(grammar=g, vocab=v)
    assert m.try_accept_token(stop) == -6          # empty text is not an expression
    assert m.try_accept_token(index[b")"]) == -6
    assert m.stack(0) == xgm.Matcher(grammar=g, vocab=v).stack(0)  # unchanged
    m.accept_token(index[b"1"])
    assert m.can_terminate() and not m.is_terminated()
    assert m.try_accept_token(-1) == -1 and m.try_accept_token(1024) == -1
    m.accept_token(stop)
    assert m.is_terminated() and m.num_stacks() == 0
    assert m.try_accept_token(index[b"1"]) == -7
    m.reset()
    assert not m.is_terminated() and m.num_stacks() == 1


def test_parallel_stacks_and_their_limit():
    # "1 " may continue the term or the expression: two parallel stacks
    g = xgm.Grammar(si.ARITH_GRAMMAR, "expr")
    m = xgm.Matcher(grammar=g)
    m.accept_bytes(b"1 ")
    assert m.num_stacks() == 2
    # nested binary choices that stay on the stack: 2^k stacks after k bytes
    rules = ['root ::= a | b', 'a ::= "x" root? "p"', 'b ::= "x" root? "q"']
    g2 = xgm.Grammar("\n".join(rules), "root")
    m2 = xgm.Matcher(grammar=g2)
    m2.accept_bytes(b"xxxxxx")
    assert m2.num_stacks() == 64
    before = [m2.stack(s) for s in range(64)]
    assert m2.try_accept_bytes(b"x") == -8
    assert [m2.stack(s) for s in range(64)] == before


def test_vocab_argument_checks():
    lib = xgm.load_library()
    h = ctypes.c_void_p()
    off = np.array([0, 1, 0], dtype=np.int64)
    data = np.zeros(4, dtype=np.uint8)
    assert lib.xgm_vocab_create(data.ctypes.data, off.ctypes.data, 2, None, 0, ctypes.byref(h)) == -1
    off = np.array([0, 1, 2], dtype=np.int64)
    stops = np.array([5], dtype=np.int32)
    assert lib.xgm_vocab_create(data.ctypes.data, off.ctypes.data, 2, stops.ctypes.data, 1, ctypes.byref(h)) == -1
    assert lib.xgm_vocab_create(data.ctypes.data, off.ctypes.data, 0, None, 0, ctypes.byref(h)) == -1
    assert b"" != lib.xgm_last_error()
    assert xgm.bitmask_words(151936) == 4748 and xgm.bitmask_words(33) == 2 and xgm.bitmask_words(0) == 0


# ---------------------------------------------------------------------------
# the GPU kernels' token walk, compiled for the host from the same source
# ---------------------------------------------------------------------------
def _walk_classes_for_nodes(text, root, vocab, nodes=None):
    g = xgm.Grammar(text, root)
    og = oracle.Grammar(text, root)
    toks = vocab.tokens() if hasattr(vocab, "tokens") else vocab.toks
    n_over = 0
    for node in (range(g.num_nodes) if nodes is None else nodes):
        want = og.classify(g.rule_name(g.node_rule(node)), g.node_path(node), vocab)
        for t, w in zip(toks, want):
            got = g.debug_walk_host([node], t, True)
            if got == 3:
                n_over += 1
                got = g.debug_classify_host(node, t)
            assert got == w, (node, g.node_path(node), t, got, int(w))
    return n_over


def test_kernel_walk_classes_match_oracle_arith():
    vocab = si.make_vocab("arith", 1024, 0)
    assert _walk_classes_for_nodes(si.ARITH_GRAMMAR, "expr", vocab) == 0


def test_kernel_walk_classes_match_oracle_json_and_csql_samples():
    vocab = si.make_vocab("bpe", 3000, 2)
    assert _walk_classes_for_nodes(si.JSON_GRAMMAR, "root", vocab, range(0, 74, 3)) == 0
    g = xgm.Grammar(si.CSQL_GRAMMAR, "root")
    rng = np.random.Generator(np.random.PCG64(9))
    nodes = sorted(set(int(n) for n in rng.integers(0, g.num_nodes, size=12)))
    assert _walk_classes_for_nodes(si.CSQL_GRAMMAR, "root", vocab, nodes) == 0


@pytest.mark.parametrize("name", ["arith", "json", "csql", "schema", "xml"])
def test_kernel_walk_masks_match_oracle_along_walks(name):
    """Two-way walk with the full live stack (what the fill kernel runs for
    every stack) OR-ed over the stacks == the oracle's mask, for all tokens."""
    text, root, _ = GRAMMARS[name]
    vocab = si.make_vocab("arith", 1024, 0) if name == "arith" else si.make_vocab("bpe", 4000, 3)
    toks = vocab.tokens()
    first = np.array([t[0] if t else -1 for t in toks], dtype=np.int16)
    g = xgm.Grammar(text, root)
    og = oracle.Grammar(text, root)
    v = xgm.Vocab(vocab.data, vocab.offsets, vocab.stop_ids)
    m = xgm.Matcher(grammar=g, vocab=v)
    om = oracle.EarleyMatcher(og)
    rng = np.random.Generator(np.random.PCG64(zlib.crc32(name.encode()) + 1))
    for step in range(14):
        want = om.mask(vocab)
        stacks = [m.stack(s) for s in range(m.num_stacks())]
        got = np.zeros(len(toks), dtype=bool)
        for i, t in enumerate(toks):
            if not t:
                continue
            for st in stacks:
                r = g.debug_walk_host(st, t, False)
                assert r in (0, 2), (name, st, t, r)
                if r == 2:
                    got[i] = True
                    break
        if m.can_terminate():
            got[vocab.stop_ids] = True
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, (name, step, toks[bad[0]], bool(got[bad[0]]))
        t = si.pick_token(rng, want, first, vocab.stop_ids, structural_bias=0.4)
        if t < 0 or t == int(vocab.stop_ids[0]):
            break
        m.accept_token(t)
        assert om.advance(toks[t])


@pytest.mark.parametrize("name", ["arith", "json", "csql", "schema", "xml"])
def test_frame_below_is_always_a_listed_context(name):
    """Along random walks, the node below every frame of every stack is one of
    the contexts the compiler lists for that frame's rule (the mask cache names
    a stack's token lists by these indices, two frames deep)."""
    text, root, _ = GRAMMARS[name]
    vocab = si.make_vocab("arith", 1024, 0) if name == "arith" else si.make_vocab("bpe", 4000, 3)
    toks = vocab.tokens()
    first = np.array([t[0] if t else -1 for t in toks], dtype=np.int16)
    g = xgm.Grammar(text, root)
    og = oracle.Grammar(text, root)
    v = xgm.Vocab(vocab.data, vocab.offsets, vocab.stop_ids)
    seen = 0
    for seed in range(3):
        m = xgm.Matcher(grammar=g, vocab=v)
        om = oracle.EarleyMatcher(og)
        rng = np.random.Generator(np.random.PCG64(zlib.crc32(name.encode()) + 31 * seed))
        for step in range(40):
            for s in range(m.num_stacks()):
                st = m.stack(s)
                for k in range(len(st) - 1, 0, -1):
                    assert g.debug_context_index(st[k], st[k - 1]) >= 0, (name, seed, step, st, k)
                    seen += 1
            want = om.mask(vocab)
            t = si.pick_token(rng, want, first, vocab.stop_ids, structural_bias=0.4)
            if t < 0 or t == int(vocab.stop_ids[0]):
                break
            m.accept_token(t)
            assert om.advance(toks[t])
    assert seen > 10


def test_kernel_walk_reports_overflow_instead_of_guessing():
    g = xgm.Grammar(si.ARITH_GRAMMAR, "expr")
    start = [n for n in range(g.num_nodes) if g.rule_name(g.node_rule(n)) == "expr" and g.node_path(n) == []][0]
    # every "(" pushes three frames (expr, term, factor): 64 frames are used up
    assert g.debug_walk_host([start], b"(" * 30, True) == 3
    assert g.debug_classify_host(start, b"(" * 30) == 2
    assert g.debug_walk_host([start], b"(" * 15, True) == 2
    assert g.debug_walk_host([start], b"1" * 300, True) == 3     # longer than 255 bytes
    assert g.debug_classify_host(start, b"1" * 300) == 2


def test_vocabulary_size_limit():
    n = 589825
    with pytest.raises(xgm.XgmError) as e:
        xgm.Vocab(np.zeros(1, dtype=np.uint8), np.zeros(n + 1, dtype=np.int64), np.zeros(0, dtype=np.int32))
    assert e.value.args[0] == -10 or "MAX_VOCAB" in str(e.value)


AMBIGUOUS_GRAMMAR = 'root ::= a | b | c\na ::= "a"* "x"\nb ::= "a"* "y" tail\nc ::= ("a" "a")* "z"\ntail ::= "(" root ")" | ""\n'


def _same_state(m1, m2):
    assert m1.is_terminated() == m2.is_terminated()
    if m1.is_terminated():
        return
    s1 = [m1.stack(s) for s in range(m1.num_stacks())]
    s2 = [m2.stack(s) for s in range(m2.num_stacks())]
    assert s1 == s2


@pytest.mark.parametrize("name", ["arith", "json", "csql", "schema", "xml", "ambiguous"])
def test_depth_first_accept_gives_the_engines_stacks(name):
    """The routine the device uses to move stacks on by a token (an enumerating
    depth-first walk over the flattened tables) against the host engine (a
    breadth-first run of the structured automaton): same verdict for every
    token tried and the same set of stacks, in the same order, after every
    accepted one."""
    if name == "ambiguous":
        text, root = AMBIGUOUS_GRAMMAR, "root"
        vocab = TinyVocab([b"a", b"aa", b"aaa", b"x", b"y", b"z", b"ax", b"aay(", b"(", b")", b"y(a", b"))", b"az", b""], [13])
        toks = vocab.toks
    else:
        text, root, _ = GRAMMARS[name]
        vocab = si.make_vocab("arith", 1024, 0) if name == "arith" else si.make_vocab("bpe", 4000, 3)
        toks = vocab.tokens()
    first = np.array([t[0] if t else -1 for t in toks], dtype=np.int16)
    g = xgm.Grammar(text, root)
    og = oracle.Grammar(text, root)
    v = xgm.Vocab(vocab.data, vocab.offsets, vocab.stop_ids)
    n_ok = n_rejected = n_multi = 0
    for seed in range(20 if name == "ambiguous" else 3):
        m1, m2 = xgm.Matcher(grammar=g, vocab=v), xgm.Matcher(grammar=g, vocab=v)
        om = oracle.EarleyMatcher(og)
        rng = np.random.Generator(np.random.PCG64(zlib.crc32(name.encode()) + 77 * seed))
        for step in range(40):
            want = om.mask(vocab)
            # a few random tokens, allowed or not: same verdict, and a rejection leaves the state alone
            for t in rng.integers(0, len(toks), 6):
                if want[t] or not toks[t]:
                    continue
                assert m1.try_accept_token(int(t)) == -6
                assert m2.debug_try_accept_token_walk(int(t)) == -6
                n_rejected += 1
                _same_state(m1, m2)
            t = si.pick_token(rng, want, first, vocab.stop_ids, structural_bias=0.4)
            if t < 0:
                break
            assert m1.try_accept_token(t) == 0
            assert m2.debug_try_accept_token_walk(t) == 0, (name, seed, step, toks[t])
            _same_state(m1, m2)
            n_ok += 1
            if m1.is_terminated():
                assert m2.debug_try_accept_token_walk(t) == -7
                break
            n_multi += m1.num_stacks() > 1
            assert om.advance(toks[t])
    assert n_ok > 20 and n_rejected > 20, (n_ok, n_rejected)
    if name == "ambiguous":
        assert n_multi > 3


def _random_grammar_text(rng) -> str:
    """A small random grammar over the bytes a-d, '(' and ')': nested groups, repetition, optional parts,
    references (also recursive and in tail position), empty alternatives - the shapes that produce
    parallel stacks, tail calls, shortcuts and returns through several frames."""
    n_rules = int(rng.integers(2, 6))
    names = ["root"] + [f"r{k}" for k in range(1, n_rules)]

    def item(depth):
        u = rng.random()
        if u < 0.40 or depth > 2:
            lit = "".join(rng.choice(list("abcd()")) for _ in range(int(rng.integers(1, 4))))
            return '"' + lit + '"'
        if u < 0.55:
            return "[" + "".join(sorted(set(rng.choice(list("abcd"), size=int(rng.integers(1, 4)))))) + "]"
        if u < 0.80:
            return names[int(rng.integers(0, n_rules))]
        return "( " + alts(depth + 1) + " )"

    def seq(depth):
        parts = []
        for _ in range(int(rng.integers(1, 4))):
            parts.append(item(depth) + rng.choice(["", "", "", "*", "+", "?"]))
        return " ".join(parts)

    def alts(depth):
        k = int(rng.integers(1, 4))
        out = [seq(depth) for _ in range(k)]
        if rng.random() < 0.15:
            out.append('""')
        return " | ".join(out)

    return "\n".join(f"{name} ::= {alts(0)}" for name in names) + "\n"


def test_depth_first_accept_on_random_grammars():
    """Seeded random grammars (those the library accepts: no left recursion, productive root): for random
    byte strings fed a few bytes at a time as tokens, the depth-first accept (what the device runs), the
    host engine and the oracle's recogniser agree on every verdict, and the two library routes on the stacks."""
    rng = np.random.Generator(np.random.PCG64(424242))
    pieces = [bytes(p) for p in (b"a", b"b", b"c", b"d", b"(", b")", b"ab", b"ba", b"a(", b")b", b"cd)", b"((", b"))", b"abc", b"dcba", b"(a)")]
    vocab = TinyVocab(pieces + [b""], [len(pieces)])
    n_grammars = n_multi = n_steps = 0
    for trial in range(400):
        text = _random_grammar_text(rng)
        try:
            g = xgm.Grammar(text, "root")
        except xgm.XgmError as e:
            assert e.status in (-4, -5), (text, e)    # left recursion, or nothing derivable
            continue
        og = oracle.Grammar(text, "root")
        v = xgm.Vocab(vocab.data, vocab.offsets, vocab.stop_ids)
        n_grammars += 1
        for walk in range(6):
            m1, m2 = xgm.Matcher(grammar=g, vocab=v), xgm.Matcher(grammar=g, vocab=v)
            prefix = b""
            for step in range(12):
                assert m1.can_terminate() == (og.recognize(prefix) == 2), (text, prefix)
                order = rng.permutation(len(pieces))
                moved = False
                for t in order:
                    rc1 = m1.try_accept_token(int(t))
                    rc2 = m2.debug_try_accept_token_walk(int(t))
                    want = og.recognize(prefix + pieces[t]) > 0
                    if rc1 == -8:          # more than 64 parallel stacks: the engine gives up, state unchanged
                        assert want
                        if rc2 == 0:       # the walk has no such limit: put its matcher back
                            m2 = xgm.Matcher(grammar=g, vocab=v)
                            assert prefix == b"" or m2.try_accept_bytes(prefix) == 0
                            _same_state(m1, m2)
                        continue
                    assert (rc1 == 0) == want, (text, prefix, pieces[t], rc1)
                    assert rc2 == rc1 or (rc2 == -9 and rc1 == 0), (text, prefix, pieces[t], rc1, rc2)
                    if rc2 == -9:          # the walk's limits; take the host's state on both sides
                        m2 = xgm.Matcher(grammar=g, vocab=v)
                        assert m2.try_accept_bytes(prefix + pieces[t]) == 0
                    _same_state(m1, m2)
                    n_steps += 1
                    if rc1 == 0:
                        prefix += pieces[t]
                        n_multi += m1.num_stacks() > 1
                        moved = True
                        break
                if not moved:
                    break
    assert n_grammars > 100 and n_steps > 3000 and n_multi > 100, (n_grammars, n_steps, n_multi)
