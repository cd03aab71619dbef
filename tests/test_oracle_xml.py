"""Oracle on the markup grammar, pinned against expat (Python's XML parser):
documents generated here with matching tag names, unique attributes and the
predefined entities are well-formed XML, so expat must parse them and the
oracle must accept them; every byte prefix must be viable; hand-written
malformed documents are refused by both."""

import xml.parsers.expat

import numpy as np
import pytest

import oracle
import synth_inputs as si


def _expat_ok(data: bytes) -> bool:
    p = xml.parsers.expat.ParserCreate()
    try:
        p.Parse(data, True)
        return True
    except xml.parsers.expat.ExpatError:
        return False


def _name(rng):
    first = "abcdefgXYZ_"
    rest = "abcxyz019_.-"
    return rng.choice(list(first)) + "".join(rng.choice(list(rest)) for _ in range(int(rng.integers(0, 5))))


def _ws(rng, at_least_one=False):
    n = int(rng.integers(1 if at_least_one else 0, 3))
    return "".join(rng.choice([" ", "\t", "\n"]) for _ in range(n))


def _element(rng, depth):
    name = _name(rng)
    attrs = ""
    used = set()
    for _ in range(int(rng.integers(0, 3))):
        a = _name(rng)
        if a in used:
            continue
        used.add(a)
        q = rng.choice(['"', "'"])
        val = "".join(rng.choice(list("abc 123/>=")) for _ in range(int(rng.integers(0, 6))))
        attrs += _ws(rng, True) + a + _ws(rng) + "=" + _ws(rng) + q + val + q
    if rng.random() < 0.25:
        return "<" + name + attrs + _ws(rng) + "/>"
    body = ""
    for _ in range(int(rng.integers(0, 4))):
        kind = rng.integers(0, 4)
        if kind == 0 and depth < 3:
            body += _element(rng, depth + 1)
        elif kind == 1:
            body += "".join(rng.choice(list("hello wor1d>\"'\n")) for _ in range(int(rng.integers(1, 8))))
        elif kind == 2:
            body += rng.choice(["&amp;", "&lt;", "&gt;", "&quot;", "&apos;", "&#65;", "&#120;"])
        else:
            body += "<!--" + "".join(rng.choice(list("ab -c<>&")) for _ in range(int(rng.integers(0, 8)))).replace("--", "- ").rstrip("-") + "-->"
    return "<" + name + attrs + _ws(rng) + ">" + body + "</" + name + _ws(rng) + ">"


def test_generated_documents_are_accepted_by_the_oracle_and_by_expat():
    og = oracle.Grammar(si.XML_GRAMMAR, "root")
    rng = np.random.Generator(np.random.PCG64(2024))
    n = 0
    for _ in range(120):
        doc = (_ws(rng) + _element(rng, 0) + _ws(rng)).encode()
        assert _expat_ok(doc), doc
        assert og.recognize(doc) == 2, doc
        assert og.recognize_pda(doc) == 2, doc
        # every proper prefix is a viable prefix and (except trailing white space) not a sentence
        for cut in rng.integers(0, len(doc), size=6):
            r = og.recognize(doc[:int(cut)])
            assert r >= 1, (doc, int(cut))
        n += 1
    assert n == 120


@pytest.mark.parametrize("doc", [
    b"<a>", b"<a></a", b"<a x=1/>", b"<a x=\"1/>", b"<a x=\"<\"/>", b"<a>&amp</a>", b"<a><!-- x -- y --></a>",
    b"<a/><b/>", b"text", b"<1a/>", b"<a x='1'y='2'/>", b"< a/>", b"<a>&;</a>",
])
def test_malformed_documents_are_refused_by_both(doc):
    og = oracle.Grammar(si.XML_GRAMMAR, "root")
    assert not _expat_ok(doc)
    assert og.recognize(doc) != 2
    assert og.recognize_pda(doc) != 2
