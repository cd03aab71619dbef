"""Pins for the oracle on the JSON workload.

Python's ``json`` module is the independent recogniser for complete texts:
seeded random documents (written by a generator in this file that knows JSON,
not the grammar) must be sentences, and byte-level mutations of them are
sentences exactly when ``json.loads`` (strict, constants refused) takes them.
"""

import json

import numpy as np
import pytest

import oracle
import synth_inputs as si


@pytest.fixture(scope="module")
def grammar():
    return oracle.Grammar(si.JSON_GRAMMAR, "root")


@pytest.fixture(scope="module")
def vocab():
    return si.make_vocab("bpe", 32000, 0)


def _refuse(name):
    raise ValueError(name)


def json_ok(data: bytes) -> bool:
    # strict UTF-8 first (json.loads on bytes would let encoded surrogates pass)
    try:
        json.loads(data.decode("utf-8"), parse_constant=_refuse)
        return True
    except (ValueError, RecursionError):
        return False


def _rand_string(rng) -> str:
    n = int(rng.integers(0, 8))
    out = []
    for _ in range(n):
        k = int(rng.integers(0, 10))
        if k < 5:
            out.append(chr(int(rng.integers(0x20, 0x7F))))
        elif k < 6:
            out.append(chr(int(rng.integers(0xA0, 0x800))))
        elif k < 7:
            c = int(rng.integers(0x800, 0xFFFF))
            out.append(chr(c) if not (0xD800 <= c <= 0xDFFF) else "x")
        elif k < 8:
            out.append(chr(int(rng.integers(0x10000, 0x110000))))
        else:
            out.append("\n\t\"\\/\b\f\r"[int(rng.integers(0, 8))])
    return "".join(out)


def _rand_value(rng, depth=0):
    k = int(rng.integers(0, 8 if depth < 4 else 6))
    if k == 0:
        return None
    if k == 1:
        return bool(rng.integers(0, 2))
    if k == 2:
        return int(rng.integers(-10**6, 10**6))
    if k == 3:
        return float(rng.standard_normal()) * 10.0 ** int(rng.integers(-8, 9))
    if k in (4, 5):
        return _rand_string(rng)
    if k == 6:
        return [_rand_value(rng, depth + 1) for _ in range(int(rng.integers(0, 4)))]
    return {_rand_string(rng): _rand_value(rng, depth + 1) for _ in range(int(rng.integers(0, 4)))}


def _serialise(rng, v) -> bytes:
    style = int(rng.integers(0, 3))
    if style == 0:
        s = json.dumps(v, ensure_ascii=False)
    elif style == 1:
        s = json.dumps(v, ensure_ascii=True, indent=int(rng.integers(0, 3)))
    else:
        s = json.dumps(v, separators=(",", ":"))
    return s.encode("utf-8")


def test_random_documents_and_mutations(grammar):
    rng = np.random.Generator(np.random.PCG64(11))
    n_valid_mut = n_invalid_mut = 0
    for _ in range(300):
        doc = _serialise(rng, _rand_value(rng))
        assert json_ok(doc)
        assert grammar.recognize(doc) == 2, doc
        assert grammar.recognize_pda(doc) == 2, doc
        for _ in range(6):
            b = bytearray(doc)
            op = int(rng.integers(0, 3))
            pos = int(rng.integers(0, len(b) + (1 if op == 0 else 0))) if len(b) else 0
            if op == 0 or not b:
                b.insert(pos, int(rng.choice(list(b' "{}[],:\\0123456789.eE-+tfnu') + [int(rng.integers(0, 256))])))
            elif op == 1:
                del b[pos]
            else:
                b[pos] = int(rng.integers(0, 256))
            mutated = bytes(b)
            want = json_ok(mutated)
            got = grammar.recognize(mutated) == 2
            assert got == want, mutated
            assert (grammar.recognize_pda(mutated) == 2) == want, mutated
            n_valid_mut += want
            n_invalid_mut += not want
    assert n_valid_mut > 20 and n_invalid_mut > 200


def test_handwritten_edge_documents(grammar):
    good = [b"0", b"-0", b"1e5", b"1E+5", b"1.5e-3", b'""', b'"\\u00e9\\ud800"', b" [ ] ", b"{ }",
            b'{"a":{"b":[1,2,{"c":null}]}}', b"\t\n\r 1 \t\n\r", b'"\xf4\x8f\xbf\xbf"', b'"\x7f"']
    bad = [b"", b"01", b"1.", b".5", b"+1", b"1e", b"[1,]", b"{,}", b'{"a" 1}', b"'a'", b'"\x1f"',
           b'"\\x41"', b'"\\u12"', b"nul", b"True", b"NaN", b"Infinity", b'"\xc0\xaf"', b'"\xed\xa0\x80"',
           b'"\xf4\x90\x80\x80"', b'"\xff"', b"[1 2]", b"1 1", b"\x0c1"]
    for d in good:
        assert json_ok(d), d
        assert grammar.recognize(d) == 2, d
    for d in bad:
        assert not json_ok(d), d
        assert grammar.recognize(d) != 2, d


def test_every_tokenisation_is_allowed(grammar, vocab):
    """Each token of a random tokenisation of a valid document has its mask
    bit set at its step, and the stop bit is set exactly at the end."""
    toks = vocab.tokens()
    by_first = {}
    for i, t in enumerate(toks):
        if t:
            by_first.setdefault(t[0], []).append(i)
    rng = np.random.Generator(np.random.PCG64(5))
    stop = int(vocab.stop_ids[0])
    for _ in range(6):
        doc = _serialise(rng, _rand_value(rng))[:60]
        # cut at 60 bytes: the text is then a prefix, which is all this test needs
        m = oracle.EarleyMatcher(grammar)
        pos = 0
        while pos < len(doc):
            cands = [i for i in by_first[doc[pos]] if doc.startswith(toks[i], pos)]
            t = cands[int(rng.integers(0, len(cands)))]
            mask = m.mask(vocab)
            assert mask[t], (doc, pos, toks[t])
            assert bool(mask[stop]) == (grammar.recognize(doc[:pos]) == 2)
            assert m.advance(toks[t])
            pos += len(toks[t])
        assert m.complete() == json_ok(doc)


def _walk(grammar, vocab, seed, steps, bias=0.35):
    toks = vocab.tokens()
    first = np.array([t[0] if t else -1 for t in toks], dtype=np.int16)
    rng = np.random.Generator(np.random.PCG64(seed))
    m = oracle.EarleyMatcher(grammar)
    text = b""
    for _ in range(steps):
        mask = m.mask(vocab)
        t = si.pick_token(rng, mask, first, vocab.stop_ids, structural_bias=bias)
        if t < 0 or t == int(vocab.stop_ids[0]):
            break
        assert m.advance(toks[t])
        text += toks[t]
        yield m, text, mask


def test_walk_invariants(grammar, vocab):
    """P5 byte-at-a-time, P6 prefix closure, P7 completion soundness, and
    O1 == O2 along a seeded random walk."""
    toks = vocab.tokens()
    order = sorted(range(len(toks)), key=lambda i: toks[i])
    done = 0
    for step, (m, text, mask_before) in enumerate(_walk(grammar, vocab, 3, 40)):
        if step % 5:
            continue
        mask = m.mask(vocab)
        # O1 == O2
        p2 = oracle.PdaMatcher(grammar)
        assert p2.advance(text)
        assert np.array_equal(mask, p2.mask(vocab)), text
        # P6: a vocabulary token that is a proper prefix of an allowed token is allowed
        allowed_sorted = [i for i in order if mask[i] and toks[i]]
        allowed_set = {toks[i] for i in allowed_sorted}
        for i in allowed_sorted[::50]:
            # all single bytes are in the vocabulary
            assert toks[i][:1] in allowed_set, (text, toks[i])
        # P5: token allowed <=> feeding its bytes one at a time succeeds
        rng = np.random.Generator(np.random.PCG64(step))
        for i in rng.integers(0, len(toks), size=300):
            t = toks[int(i)]
            if not t:
                continue
            c = m.clone()
            ok = all(c.advance(bytes([b])) for b in t)
            assert ok == bool(mask[int(i)]), (text, t)
        # P7: the completion makes a sentence by json.loads
        tail = m.completion()
        assert json_ok(text + tail), (text, tail)
        assert grammar.recognize(text + tail) == 2
        done += 1
    assert done >= 4


def test_prefix_closure_full(grammar, vocab):
    toks = vocab.tokens()
    index = {t: i for i, t in enumerate(toks)}
    for text in [b"", b'{"k', b'[1', b'{"a":', b'[tr', b'"\\']:
        m = oracle.EarleyMatcher(grammar)
        assert m.advance(text)
        mask = m.mask(vocab)
        for i, t in enumerate(toks):
            if mask[i]:
                for k in range(1, len(t)):
                    j = index.get(t[:k])
                    if j is not None:
                        assert mask[j], (text, t, t[:k])
