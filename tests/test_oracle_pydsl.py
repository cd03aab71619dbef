"""Oracle on the scripting grammar, pinned against Python's own parser: every
sentence of the grammar is meant to be a Python module, so programs generated
here must be accepted by the oracle and by `ast.parse`, every byte prefix must
be viable, and whatever the oracle accepts among randomly damaged programs
`ast.parse` must accept too (the grammar describes a subset of the language,
so the converse does not hold)."""

import ast
import warnings

import numpy as np
import pytest

import oracle
import synth_inputs as si


def _python_ok(src: bytes) -> bool:
    try:
        with warnings.catch_warnings():
            warnings.simplefilter("ignore")
            ast.parse(src.decode("utf-8"))
        return True
    except (SyntaxError, ValueError, UnicodeDecodeError, RecursionError, MemoryError):
        return False


def _name(rng):
    return rng.choice(list("xzuv_")) + "".join(rng.choice(list("abYZ019_")) for _ in range(int(rng.integers(0, 4))))


def _sp(rng):
    return " " * int(rng.integers(0, 3))


def _string(rng):
    q = rng.choice(['"', "'"])
    plain = [c for c in "abc xyz=()[]{}:;,.+-#\"'" if c != q] + ["é", "中"]
    body = ""
    for _ in range(int(rng.integers(0, 6))):
        if rng.integers(0, 8) == 0:
            body += rng.choice(["\\n", "\\t", "\\\\", "\\'", '\\"'])
        else:
            body += rng.choice(plain)
    return q + body + q


def _atom(rng, depth):
    k = int(rng.integers(0, 10 if depth < 2 else 5))
    if k == 0:
        return str(int(rng.integers(0, 1000)))
    if k == 1:
        return f"{int(rng.integers(0, 50))}.{int(rng.integers(0, 100)):02d}"
    if k == 2:
        return _string(rng)
    if k == 3:
        return rng.choice(["True", "False", "None"])
    if k == 4:
        return _name(rng)
    if k == 5:
        prim = "(" + _sp(rng) + _expr(rng, depth + 1) + _sp(rng) + ")"
    elif k == 6:
        prim = "[" + _sp(rng) + (_sp(rng) + "," + _sp(rng)).join(_expr(rng, depth + 1) for _ in range(int(rng.integers(0, 3)))) + _sp(rng) + "]"
    elif k == 7:
        items = [_expr(rng, depth + 1) + _sp(rng) + ":" + _sp(rng) + _expr(rng, depth + 1) for _ in range(int(rng.integers(0, 3)))]
        prim = "{" + _sp(rng) + (_sp(rng) + "," + _sp(rng)).join(items) + _sp(rng) + "}"
    else:
        prim = _name(rng)
    for _ in range(int(rng.integers(0, 2))):
        t = int(rng.integers(0, 3))
        if t == 0:
            prim += "(" + _sp(rng) + (_sp(rng) + "," + _sp(rng)).join(_expr(rng, depth + 1) for _ in range(int(rng.integers(0, 3)))) + _sp(rng) + ")"
        elif t == 1:
            prim += "[" + _sp(rng) + _expr(rng, depth + 1) + _sp(rng) + "]"
        else:
            prim += "." + _name(rng)
    return prim


def _arith(rng, depth):
    def factor():
        f = "".join(rng.choice(list("+-~")) for _ in range(int(rng.integers(0, 2)))) + _atom(rng, depth)
        if rng.random() < 0.15:
            f += _sp(rng) + "**" + _sp(rng) + rng.choice(["", "-"]) + _atom(rng, depth + 1)
        return f
    def term():
        t = factor()
        for _ in range(int(rng.integers(0, 2))):
            t += _sp(rng) + rng.choice(["*", "/", "//", "%"]) + _sp(rng) + factor()
        return t
    a = term()
    for _ in range(int(rng.integers(0, 2))):
        a += _sp(rng) + rng.choice(["+", "-"]) + _sp(rng) + term()
    return a


def _or(rng, depth):
    def cmp_():
        c = _arith(rng, depth)
        for _ in range(int(rng.integers(0, 2))):
            op = rng.choice(["==", "!=", "<=", ">=", "<", ">", " in ", " not in ", " is ", " is not "])
            c += (op if op.startswith(" ") else _sp(rng) + op + _sp(rng)) + _arith(rng, depth)
        return c
    def not_():
        return "not " * int(rng.integers(0, 2) if rng.random() < 0.3 else 0) + cmp_()
    def and_():
        return " and ".join(not_() for _ in range(int(rng.integers(1, 3)) if rng.random() < 0.3 else 1))
    return " or ".join(and_() for _ in range(int(rng.integers(1, 3)) if rng.random() < 0.3 else 1))


def _expr(rng, depth=0):
    r = rng.random()
    if r < 0.1 and depth < 3:
        params = (_sp(rng) + "," + _sp(rng)).join(_name(rng) for _ in range(int(rng.integers(0, 3))))
        return "lambda" + (" " + params if params else "") + ":" + _sp(rng) + _expr(rng, depth + 1)
    t = _or(rng, depth)
    if r > 0.85 and depth < 3:
        t += " if " + _or(rng, depth + 1) + " else " + _expr(rng, depth + 1)
    return t


def _simple(rng):
    smalls = []
    for _ in range(int(rng.integers(1, 3))):
        k = int(rng.integers(0, 8))
        if k == 0:
            smalls.append(rng.choice(["pass", "break", "continue", "return"]))
        elif k == 1:
            smalls.append("return " + _expr(rng))
        elif k <= 5:
            target = _name(rng)
            for _ in range(int(rng.integers(0, 2))):
                target += ("." + _name(rng)) if rng.random() < 0.5 else ("[" + _sp(rng) + _expr(rng, 2) + _sp(rng) + "]")
            smalls.append(target + _sp(rng) + rng.choice(["=", "+=", "-=", "*=", "/=", "//=", "%="]) + _sp(rng) + _expr(rng))
        else:
            smalls.append(_expr(rng))
    return (_sp(rng) + ";" + _sp(rng)).join(smalls)


def _stmt(rng):
    k = int(rng.integers(0, 8))
    if k == 0:
        s = "if " + _expr(rng, 1) + ":" + _sp(rng) + _simple(rng)
        for _ in range(int(rng.integers(0, 2))):
            s += "\n" + "elif " + _expr(rng, 1) + ":" + _sp(rng) + _simple(rng)
        if rng.random() < 0.5:
            s += "\n" + "else:" + _sp(rng) + _simple(rng)
        return s
    if k == 1:
        return "while " + _expr(rng, 1) + ":" + _sp(rng) + _simple(rng)
    if k == 2:
        return "for " + _name(rng) + " in " + _expr(rng, 1) + ":" + _sp(rng) + _simple(rng)
    if k == 3:
        params = (_sp(rng) + "," + _sp(rng)).join(_name(rng) for _ in range(int(rng.integers(0, 3))))
        return "def " + _name(rng) + "(" + _sp(rng) + params + _sp(rng) + "):" + _sp(rng) + _simple(rng)
    return _simple(rng)


def make_program(rng, lines=4):
    out = []
    for _ in range(lines):
        line = _stmt(rng)
        if rng.random() < 0.2:
            line += _sp(rng) + "#" + "".join(rng.choice(list("note: x=1 é")) for _ in range(int(rng.integers(0, 8))))
        out.append(line)
    return ("\n" * 1).join(out) + ("\n" if rng.random() < 0.5 else "")


def test_generated_programs_are_accepted_by_the_oracle_and_by_python():
    og = oracle.Grammar(si.PYDSL_GRAMMAR, "root")
    rng = np.random.Generator(np.random.PCG64(31))
    for k in range(150):
        src = make_program(rng, lines=int(rng.integers(1, 5))).encode("utf-8")
        assert _python_ok(src), src
        assert og.recognize(src) == 2, src
        assert og.recognize_pda(src) == 2, src
        for cut in rng.integers(0, len(src), size=5):
            assert og.recognize(src[:int(cut)]) >= 1, (src, int(cut))


def test_what_the_oracle_accepts_among_damaged_programs_python_accepts_too():
    og = oracle.Grammar(si.PYDSL_GRAMMAR, "root")
    rng = np.random.Generator(np.random.PCG64(32))
    alphabet = list(b" \n()[]{}:;,.=+-*/%<>!~#'\"\\xzuv_ab019ifelsnotrdwhpcTFN")
    n_accepted = n_refused = 0
    for k in range(400):
        src = bytearray(make_program(rng, lines=int(rng.integers(1, 3))).encode("utf-8"))
        for _ in range(int(rng.integers(1, 3))):
            pos = int(rng.integers(0, len(src)))
            kind = int(rng.integers(0, 3))
            if kind == 0:
                del src[pos]
            elif kind == 1:
                src.insert(pos, int(rng.choice(alphabet)))
            else:
                src[pos] = int(rng.choice(alphabet))
        src = bytes(src)
        verdict = og.recognize(src) == 2
        assert verdict == (og.recognize_pda(src) == 2), src
        if verdict:
            n_accepted += 1
            assert _python_ok(src), src
        else:
            n_refused += 1
    assert n_accepted >= 30 and n_refused >= 150, (n_accepted, n_refused)


@pytest.mark.parametrize("src", [
    b"x = 01", b"if = 3", b"x = 1.z", b"x = (1", b"if x: if z: pass", b"x = 'a", b"x = 1 +", b"def (x): pass",
    b"x = lambda x y: 1", b"for 1 in x: pass", b"x = y = ", b" x = 1", b"x = 1 if z", b"else: pass", b"x = [1, 2",
])
def test_malformed_programs_are_refused_by_both(src):
    og = oracle.Grammar(si.PYDSL_GRAMMAR, "root")
    assert not _python_ok(src)
    assert og.recognize(src) != 2
    assert og.recognize_pda(src) != 2
