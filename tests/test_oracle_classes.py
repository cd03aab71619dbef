"""Pins for the three-way token classes of section 3.1.

For grammars whose rules have small finite languages the classes have a
plain language-level definition that needs no automaton: let X be the set of
byte strings the rest of the rule can still produce from the position (its
own frame and deeper ones only).  Token t is
  accepted  iff t is a prefix of some string of X (t is used up inside the
            frame; using it up exactly at the end of the rule still counts),
  uncertain iff not accepted and some *proper* prefix of t is in X (the rule
            ends while bytes remain: what follows depends on the context),
  rejected  otherwise.
The enumerator below works on a hand-written Python structure of the same
tiny grammars, not on the oracle's parser or automata.

The narrowing by one byte of context (section 3.2 in its smallest form) has a
plain definition too: FOLLOW(R) is the set of bytes found right after some
instance of R in some sentence, read off a brute-force enumeration of all
derivations; an uncertain token stays uncertain (class 1) iff one of the
proper prefixes in X is followed, inside the token, by a byte of FOLLOW(R),
otherwise it is uncertain by section 3.1 alone (class 4).
"""

import itertools

import numpy as np
import pytest

import oracle
import synth_inputs as si
from test_oracle_misc import TinyVocab

# grammar as Python data: rule -> list of alternatives; an alternative is a
# list of symbols; a symbol is bytes (literal) or a rule name
G1 = {
    "root": [[b"<", "word", b">"], [b"<", "num", b"/>"]],
    "word": [[b"a"], [b"a", b"b"], [b"b", "word2"]],
    "word2": [[b"a"], [b"a", b"a"]],
    "num": [[b"1"], [b"1", b"2"], []],
}
G1_TEXT = '''
root  ::= "<" word ">" | "<" num "/>"
word  ::= "a" | "a" "b" | "b" word2
word2 ::= "a" | "a" "a"
num   ::= "1" | "1" "2" | ""
'''


def expand(gr, symbols):
    """All byte strings a symbol sequence produces (finite grammars only)."""
    out = {b""}
    for s in symbols:
        if isinstance(s, bytes):
            out = {x + s for x in out}
        else:
            sub = set()
            for alt in gr[s]:
                sub |= expand(gr, alt)
            out = {x + y for x in out for y in sub}
    return out


def residuals(gr, rule, path):
    """Strings the rest of `rule` can produce after the symbol path (bytes
    consumed one at a time inside literals, rule names as whole symbols).
    References to rules that can produce "" may be skipped by the path."""
    rests = []
    for alt in gr[rule]:
        # flatten literals to single bytes so that a path can stop inside one
        flat = []
        for s in alt:
            if isinstance(s, bytes):
                flat.extend(bytes([c]) for c in s)
            else:
                flat.append(s)
        frontier = [0]
        for sym in path:
            nxt = []
            for k in frontier:
                # skip nullable references
                ks = [k]
                j = k
                while j < len(flat) and isinstance(flat[j], str) and b"" in expand(gr, [flat[j]]):
                    j += 1
                    ks.append(j)
                for kk in ks:
                    if kk < len(flat) and flat[kk] == (bytes([sym]) if isinstance(sym, int) else sym):
                        nxt.append(kk + 1)
            frontier = nxt
        for k in frontier:
            rests.append(flat[k:])
    out = set()
    for r in rests:
        out |= expand(gr, r)
    return out


def derivations(gr, symbols):
    """All (string, [(rule, end offset), ...]) a symbol sequence derives."""
    out = [(b"", [])]
    for s in symbols:
        nxt = []
        if isinstance(s, bytes):
            nxt = [(x + s, inst) for x, inst in out]
        else:
            subs = []
            for alt in gr[s]:
                subs.extend(derivations(gr, alt))
            for x, inst in out:
                for y, inst2 in subs:
                    moved = [(r, len(x) + e) for r, e in inst2]
                    nxt.append((x + y, inst + moved + [(s, len(x) + len(y))]))
        out = nxt
    return out


def brute_force_follow(gr, root):
    follow = {r: set() for r in gr}
    for text, instances in derivations(gr, [root]):
        for rule, end in instances:
            if end < len(text):
                follow[rule].add(text[end])
    return follow


def want_class(X, t, follow=None):
    """0 rejected, 2 accepted, 1 uncertain; with `follow` (bytes that may come
    after the rule) an uncertain token none of whose exits is in front of such
    a byte is 4."""
    if len(t) == 0:
        return 0
    if any(x.startswith(t) for x in X):
        return 2
    exits = [len(x) for x in X if t.startswith(x) and len(x) < len(t)]
    if not exits:
        return 0
    if follow is None or any(t[k] in follow for k in exits):
        return 1
    return 4


POSITIONS = [
    ("root", []), ("root", [ord("<")]), ("root", [ord("<"), "word"]), ("root", [ord("<"), "num"]),
    ("root", [ord("<"), "num", ord("/")]), ("root", [ord("<"), ord("/")]),
    ("word", []), ("word", [ord("a")]), ("word", [ord("b")]), ("word", [ord("b"), "word2"]), ("word", [ord("a"), ord("b")]),
    ("word2", []), ("word2", [ord("a")]), ("word2", [ord("a"), ord("a")]),
    ("num", []), ("num", [ord("1")]), ("num", [ord("1"), ord("2")]),
]


def test_classes_against_language_level_definition():
    g = oracle.Grammar(G1_TEXT, "root")
    alphabet = b"<>/ab12"
    toks = [bytes(t) for n in range(1, 5) for t in itertools.product(alphabet, repeat=n)] + [b""]
    vocab = TinyVocab(toks)
    follow = brute_force_follow(G1, "root")
    assert follow == {"root": set(), "word": {ord(">")}, "word2": {ord(">")}, "num": {ord("/")}}
    for rule in G1:
        assert g.follow(rule) == follow[rule], rule
    seen = set()
    for rule, path in POSITIONS:
        X = residuals(G1, rule, path)
        assert X, (rule, path)
        got = g.classify(rule, path, vocab)
        for t, c in zip(toks, got):
            # section 3.1 alone: classes 1 and 4 together are "uncertain"
            assert {0: 0, 1: 1, 2: 2, 4: 1}[int(c)] == want_class(X, t), (rule, path, t, int(c))
            # with the one-byte narrowing
            assert c == want_class(X, t, follow[rule]), (rule, path, t, int(c), want_class(X, t, follow[rule]))
        seen |= set(int(c) for c in got)
    assert seen == {0, 1, 2, 4}


def test_hand_values():
    """A handful of values anyone can check by eye on  root ::= "<" word ">"."""
    g = oracle.Grammar('root ::= "<" word ">"\nword ::= [ab]+', "root")
    toks = [b"ab", b"a>", b">", b"c", b"ca", b"b", b"a>x", b"<", b"<a", b"<>", b""]
    vocab = TinyVocab(toks)
    REJ, UNC, ACC, UN4 = 0, 1, 2, 4
    # only ">" can come after word, and nothing after root
    assert g.follow("word") == {ord(">")} and g.follow("root") == set()
    # inside word after one letter: the rule may end here; leaving it in front
    # of anything but ">" is hopeless in every context (4)
    assert list(g.classify("word", [ord("a")], vocab)) == [ACC, UNC, UNC, UN4, UN4, ACC, UNC, UN4, UN4, UN4, REJ]
    # at the start of word: it cannot end yet
    assert list(g.classify("word", [], vocab)) == [ACC, UNC, REJ, REJ, REJ, ACC, UNC, REJ, REJ, REJ, REJ]
    # in root after "<": leaving word returns into root's own frame, which is known;
    # "a>x" leaves root itself in front of "x"
    assert list(g.classify("root", [ord("<")], vocab)) == [ACC, ACC, REJ, REJ, REJ, ACC, UN4, REJ, REJ, REJ, REJ]
    # at root's start
    assert list(g.classify("root", [], vocab)) == [REJ, REJ, REJ, REJ, REJ, REJ, REJ, ACC, ACC, REJ, REJ]


def test_classes_consistent_with_masks_on_json():
    """accepted => allowed and rejected => not allowed, whatever lies below
    the top frame; only uncertain tokens may go either way."""
    g = oracle.Grammar(si.JSON_GRAMMAR, "root")
    vocab = si.make_vocab("bpe", 32000, 0)
    # (accepted text, rule of the top frame, path to the position inside it)
    cases = [
        (b'{"ab', "char", [ord("b")]),
        (b'[1', "int", [ord("1")]),
        (b'[12', "int", [ord("1"), ord("2")]),
        (b'{"a":1.5', "frac", [ord("."), ord("5")]),
        (b'[ ', "ws", [ord(" ")]),
        (b'["\\', "char", [ord("\\")]),
        (b'["\\u0', "hex", [ord("0")]),
        (b'[tr', "value", [ord("t"), ord("r")]),
        (b'{', "object", [ord("{")]),
        (b'["a"', "string", [ord('"'), "char", ord('"')]),
    ]
    n_unc_allowed = n_unc_refused = n_narrowed = 0
    for text, rule, path in cases:
        cls = g.classify(rule, path, vocab)
        m = oracle.EarleyMatcher(g)
        assert m.advance(text)
        mask = m.mask(vocab)
        mask[vocab.stop_ids] = False
        assert mask[cls == 2].all(), (text, rule)
        assert not mask[cls == 0].any(), (text, rule)
        assert not mask[cls == 4].any(), (text, rule)   # the narrowing only drops tokens no context allows
        n_unc_allowed += int(mask[cls == 1].sum())
        n_unc_refused += int((~mask[cls == 1]).sum())
        n_narrowed += int((cls == 4).sum())
    assert n_unc_allowed > 0 and n_unc_refused > 0 and n_narrowed > 1000
