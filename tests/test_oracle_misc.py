"""More oracle pins: regular special case (Python ``re`` / ``regex`` as
library recognisers), Dyck counting closed forms, union over parallel stacks,
unproductive and left-recursive grammars, UTF-8 classes."""

import itertools
import math
import re

import numpy as np
import pytest
import regex  # third-party engine with partial matching: viable-prefix test

import oracle
import synth_inputs as si


class TinyVocab:
    def __init__(self, tokens, stop_ids=()):
        self.data = np.frombuffer(b"".join(tokens), dtype=np.uint8).copy()
        self.offsets = np.zeros(len(tokens) + 1, dtype=np.int64)
        np.cumsum([len(t) for t in tokens], out=self.offsets[1:])
        self.stop_ids = np.asarray(stop_ids, dtype=np.int32)
        self.toks = list(tokens)


# ---------------------------------------------------------------------------
# P3: grammars without recursion are regular expressions
# ---------------------------------------------------------------------------
REGULAR_CASES = [
    # (grammar text, root, equivalent Python regex, alphabet)
    ('root ::= "a" ("b" | "c")* "d"?', "root", r"a(b|c)*d?", b"abcd"),
    ('root ::= x+ y\nx ::= "ab" | "a"\ny ::= "b"* "c"', "root", r"(ab|a)+b*c", b"abc"),
    ('root ::= [a-c]+ "-" [0-9] [0-9]?', "root", r"[a-c]+-[0-9][0-9]?", b"ab-01c"),
    ('root ::= ("a" | "") ("aa")* "b"', "root", r"(a|)(aa)*b", b"ab"),
    ('root ::= [^ab]* "a"', "root", r"[^ab]*a", b"abc\n"),
    ('root ::= (("a" "b"?)+ | "c")*', "root", r"((ab?)+|c)*", b"abc"),
]


@pytest.mark.parametrize("text,root,pattern,alphabet", REGULAR_CASES)
def test_regular_grammars_match_regex_engines(text, root, pattern, alphabet):
    g = oracle.Grammar(text, root)
    full = re.compile(pattern.encode(), re.DOTALL)
    part = regex.compile(pattern.encode(), regex.DOTALL)
    for n in range(0, 8):
        for tup in itertools.product(sorted(set(alphabet)), repeat=n):
            s = bytes(tup)
            is_sentence = full.fullmatch(s) is not None
            is_viable = part.fullmatch(s, partial=True) is not None
            want = 2 if is_sentence else (1 if is_viable else 0)
            assert g.recognize(s) == want, (s, want)
            assert g.recognize_pda(s) == want, (s, want)


# ---------------------------------------------------------------------------
# P4: Dyck language, counting closed forms
# ---------------------------------------------------------------------------
def test_dyck_counts():
    g = oracle.Grammar('S ::= ("(" S ")")*', "S")
    for n in range(0, 15):
        sentences = viable = 0
        for tup in itertools.product(b"()", repeat=n):
            r = g.recognize(bytes(tup))
            sentences += r == 2
            viable += r >= 1
        catalan = math.comb(n, n // 2) // (n // 2 + 1) if n % 2 == 0 else 0
        assert sentences == catalan, n
        assert viable == math.comb(n, n // 2), n


# ---------------------------------------------------------------------------
# P8: the mask of a state with several parallel stacks is the union of the
# masks of its stacks taken one by one (section 3.1 / Algorithm 1)
# ---------------------------------------------------------------------------
def test_union_over_parallel_stacks():
    text = 'S ::= A | B\nA ::= "a"* "x" C\nB ::= "a"* "y" "q"\nC ::= "p"'
    g = oracle.Grammar(text, "S")
    toks = [b"a", b"x", b"y", b"ax", b"ay", b"aax", b"xp", b"yq", b"xq", b"yp", b"axp", b"p", b"q", b""]
    vocab = TinyVocab(toks, stop_ids=[len(toks) - 1])
    m = oracle.PdaMatcher(g)
    assert m.advance(b"aa")
    assert m.num_configs() >= 2
    full = m.mask(vocab)
    union = np.zeros(len(toks), dtype=bool)
    singles = []
    for k in range(m.num_configs()):
        one = m.mask(vocab, single=k)
        singles.append(one)
        union |= one
    assert np.array_equal(full[:-1], union[:-1])
    assert any(not np.array_equal(s, union) for s in singles)  # the union is not trivial
    want = {b"a", b"x", b"y", b"ax", b"ay", b"aax", b"xp", b"yq", b"axp"}
    assert {t for t, ok in zip(toks, full) if ok} == want
    e = oracle.EarleyMatcher(g)
    assert e.advance(b"aa")
    assert np.array_equal(e.mask(vocab), full)


# ---------------------------------------------------------------------------
# grammars with dead parts, nullable loops, left recursion
# ---------------------------------------------------------------------------
def test_unproductive_alternatives_are_ignored():
    # "dead" can never finish, so the branch through it does not count
    g = oracle.Grammar('root ::= "a" dead | "a" "b"\ndead ::= "x" dead', "root")
    assert g.recognize(b"a") == 1
    assert g.recognize(b"ax") == 0
    assert g.recognize_pda(b"ax") == 0
    assert g.recognize(b"ab") == 2
    with pytest.raises(oracle.OracleError):
        oracle.Grammar('root ::= "a" root', "root")


def test_nullable_loops_terminate():
    g = oracle.Grammar('root ::= (e | "a")* "b"\ne ::= "c"?', "root")
    for s, want in [(b"", 1), (b"b", 2), (b"acab", 2), (b"ba", 0), (b"cc", 1)]:
        assert g.recognize(s) == want, s
        assert g.recognize_pda(s) == want, s


def test_left_recursion_earley_only():
    g = oracle.Grammar('E ::= E "+" "n" | "n"', "E")
    assert g.recognize(b"n+n+n") == 2
    assert g.recognize(b"n+") == 1
    assert g.recognize(b"+") == 0
    with pytest.raises(oracle.OracleError):
        g.recognize_pda(b"n+n")


def test_parse_errors():
    for bad in ['root ::= "a', "root ::= [a", "root ::= (a", "root ::= undefined_rule", 'root = "a"',
                'root ::= "a"\nroot ::= "b"', ""]:
        with pytest.raises(oracle.OracleError):
            oracle.Grammar(bad, "root")
    with pytest.raises(oracle.OracleError):
        oracle.Grammar('a ::= "x"', "root")


# ---------------------------------------------------------------------------
# byte level: a class is the set of UTF-8 encodings of its code points
# ---------------------------------------------------------------------------
def test_classes_are_utf8_encodings():
    g = oracle.Grammar('root ::= [^"\\\\\\x00-\\x1f]', "root")
    rng = np.random.Generator(np.random.PCG64(1))
    cps = [0x20, 0x21, 0x22, 0x5B, 0x5C, 0x5D, 0x7F, 0x80, 0x7FF, 0x800, 0xD7FF, 0xE000, 0xFFFF, 0x10000, 0x10FFFF, 0x1F, 0x0]
    cps += [int(c) for c in rng.integers(0, 0x110000, size=400)]
    for cp in cps:
        if 0xD800 <= cp <= 0xDFFF:
            continue
        enc = chr(cp).encode("utf-8")
        want = 2 if (cp >= 0x20 and cp not in (0x22, 0x5C)) else 0
        assert g.recognize(enc) == want, hex(cp)
        if want == 2:
            for k in range(1, len(enc)):
                assert g.recognize(enc[:k]) == 1  # a token may stop inside a character
    for bad in [b"\x80", b"\xc0\xaf", b"\xc1\xbf", b"\xe0\x80\x80", b"\xed\xa0\x80", b"\xf0\x80\x80\x80", b"\xf4\x90\x80\x80", b"\xf5", b"\xff"]:
        assert g.recognize(bad) == 0, bad
    g2 = oracle.Grammar('root ::= [\u00e9\u4e2d-\u4e2f\\u00df]', "root")
    for s, want in [("é", 2), ("中", 2), ("丯", 2), ("丰", 0), ("ß", 2), ("e", 0)]:
        assert g2.recognize(s.encode()) == want, s


def test_literal_escapes():
    g = oracle.Grammar(r'root ::= "\x41\n\t\"\\\u00e9" "/"', "root")
    assert g.recognize('A\n\t"\\é/'.encode()) == 2
    assert g.recognize(b"A\n\t") == 1
