"""Pins for the oracle on the arithmetic workload (5-rule grammar).

The expected values here are written by hand or come from a closed-form
checker of the arithmetic language that shares nothing with the oracle: it
never sees the grammar text, only the rules of the language stated in words
(operands and operators alternate, parentheses balance, digit runs are not
broken by spaces, spaces may separate lexemes except at the two ends of the
whole expression).
"""

import itertools

import numpy as np
import pytest

import oracle
import synth_inputs as si

ALPHABET = si.ARITH_ALPHABET


@pytest.fixture(scope="module")
def grammar():
    return oracle.Grammar(si.ARITH_GRAMMAR, "expr")


# ---------------------------------------------------------------------------
# closed form: 0 = not a viable prefix, 1 = viable prefix, 2 = sentence
# ---------------------------------------------------------------------------
def arith_status(s: bytes) -> int:
    depth = 0
    need_operand = True      # the next lexeme must be an operand
    prev = None              # previous byte
    for i, c in enumerate(s):
        ch = chr(c)
        if ch.isdigit():
            if need_operand:
                need_operand = False
            elif not (prev is not None and chr(prev).isdigit()):
                return 0     # digit after a finished operand
        elif ch == "(":
            if not need_operand:
                return 0
            depth += 1
        elif ch == ")":
            if need_operand or depth == 0:
                return 0
            depth -= 1
        elif ch in "+*":
            if need_operand:
                return 0
            need_operand = True
        elif ch == " ":
            if i == 0:
                return 0     # no leading space before the whole expression
        else:
            return 0
        prev = c
    done = (not need_operand) and depth == 0 and (prev is not None and prev != ord(" "))
    return 2 if done else 1


def test_closed_form_spot_checks():
    # the checker itself, against statements anyone can verify by eye
    assert arith_status(b"") == 1
    assert arith_status(b"1") == 2
    assert arith_status(b"12+3*(4)") == 2
    assert arith_status(b"1 2") == 0
    assert arith_status(b" 1") == 0
    assert arith_status(b"1 ") == 1
    assert arith_status(b"( 1 )") == 2
    assert arith_status(b"(1") == 1
    assert arith_status(b"1)") == 0
    assert arith_status(b"1++") == 0
    assert arith_status(b"()") == 0


def test_exhaustive_against_closed_form(grammar):
    """Every string over the 15-symbol alphabet up to length 5 (813,615 of
    them, visited as a tree; a non-viable prefix settles all its extensions)."""
    m = oracle.EarleyMatcher(grammar)
    checked = 0

    def visit(prefix: bytes, matcher, depth: int):
        nonlocal checked
        for c in ALPHABET:
            s = prefix + bytes([c])
            want = arith_status(s)
            child = matcher.clone()
            ok = child.advance(bytes([c]))
            got = 0 if not ok else (2 if child.complete() else 1)
            assert got == want, (s, got, want)
            checked += 1
            if ok and depth + 1 < 5:
                visit(s, child, depth + 1)
            elif not ok and depth + 1 < 5:
                # all extensions of a dead prefix are dead in the closed form too
                for ext in (b"1", b")", b" ", b"+"):
                    assert arith_status(s + ext) == 0

    assert arith_status(b"") == 1 and not m.complete()
    visit(b"", m, 0)
    assert checked > 20000


def test_recognize_matches_closed_form_random_long(grammar):
    rng = np.random.Generator(np.random.PCG64(7))
    for _ in range(3000):
        n = int(rng.integers(6, 24))
        # biased draw so that long viable strings occur
        s = bytes(rng.choice(list(b"11223()+* "), size=n).tolist())
        assert grammar.recognize(s) == arith_status(s), s
        assert grammar.recognize_pda(s) == arith_status(s), s


# ---------------------------------------------------------------------------
# hand-enumerated masks: allowed one-symbol tokens after named prefixes
# ---------------------------------------------------------------------------
DIG = set(b"0123456789")
HAND = {
    b"": DIG | set(b"("),
    b"1": DIG | set(b"+* "),
    b"1+": DIG | set(b"( "),
    b"(": DIG | set(b"( "),
    b"(1": DIG | set(b"+*) "),
    b"(1)": set(b"+* "),
    b"1 ": set(b"+* "),
    b"1*(": DIG | set(b"( "),
    b"((": DIG | set(b"( "),
    b"12": DIG | set(b"+* "),
    b"(1 ": set(b"+*) "),
    b"1 + ": DIG | set(b"( "),
}
# a few multi-symbol tokens judged by hand: prefix -> {token: allowed}
HAND_MULTI = {
    b"": {b"12": True, b"(1": True, b"1)": False, b"1 +": True, b" 1": False, b"((": True, b"1 2": False, b"()": False},
    b"(1": {b")+": True, b"))": False, b" )": True, b")(": False, b"2 3": False, b"+ (": True, b") *": True},
    b"1 ": {b"+1": True, b"1": False, b" +": True, b"*(": True, b")": False},
}


def test_hand_enumerated_masks(grammar):
    vocab = si.make_vocab("arith", 1024, 0)
    toks = vocab.tokens()
    index = {t: i for i, t in enumerate(toks)}
    for prefix, allowed_chars in HAND.items():
        m = oracle.EarleyMatcher(grammar)
        assert m.advance(prefix)
        mask = m.mask(vocab)
        for c in ALPHABET:
            assert bool(mask[index[bytes([c])]]) == (c in allowed_chars), (prefix, chr(c))
        # every token of the vocabulary, against the closed form
        for i, t in enumerate(toks):
            if len(t) == 0:
                continue
            assert bool(mask[i]) == (arith_status(prefix + t) > 0), (prefix, t)
        # stop token: allowed iff the prefix is a complete expression
        assert bool(mask[vocab.stop_ids[0]]) == (arith_status(prefix) == 2)
    for prefix, cases in HAND_MULTI.items():
        m = oracle.EarleyMatcher(grammar)
        assert m.advance(prefix)
        for t, want in cases.items():
            assert (arith_status(prefix + t) > 0) == want, ("closed form disagrees with hand value", prefix, t)
            g = m.clone()
            assert g.advance(t) == want, (prefix, t)


def test_pda_matcher_agrees_on_hand_prefixes(grammar):
    vocab = si.make_vocab("arith", 1024, 0)
    for prefix in HAND:
        e = oracle.EarleyMatcher(grammar)
        p = oracle.PdaMatcher(grammar)
        assert e.advance(prefix) and p.advance(prefix)
        assert np.array_equal(e.mask(vocab), p.mask(vocab)), prefix


def test_random_walk_prefix_invariant(grammar):
    """Concatenated allowed tokens always form a prefix of the language; the
    completion returned by the oracle makes a sentence (closed form judges)."""
    vocab = si.make_vocab("arith", 1024, 0)
    toks = vocab.tokens()
    first = np.array([t[0] if t else -1 for t in toks], dtype=np.int16)
    rng = np.random.Generator(np.random.PCG64(0))
    m = oracle.EarleyMatcher(grammar)
    text = b""
    for step in range(64):
        mask = m.mask(vocab)
        t = si.pick_token(rng, mask, first, vocab.stop_ids)
        assert t >= 0
        if t == int(vocab.stop_ids[0]):
            assert arith_status(text) == 2
            break
        assert m.advance(toks[t])
        text += toks[t]
        assert arith_status(text) > 0, text
        if step % 8 == 0:
            tail = m.completion()
            assert arith_status(text + tail) == 2, (text, tail)
