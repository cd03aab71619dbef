"""TEST INFRASTRUCTURE ONLY: the slow, plain CPU oracle.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the GPU
library and never imports it.

What it computes (arxiv 2411.15100):

* ``EarleyMatcher`` (O1): the definition of the next-token mask of sections
  1-2: token t is allowed iff accepted-text + bytes(t) can still be extended
  to a sentence of the grammar.  No automaton, no cache; an Earley recogniser
  on productions over byte sets, brute force over the vocabulary.
* ``PdaMatcher`` / ``classify`` (O2): the pushdown automaton of Appendix A
  simulated literally on Thompson NFAs (sets of (state, stack) with a visited
  set), and from it the accepted / rejected / context-dependent token classes
  of section 3.1 for a position inside a rule, plus their narrowing by one
  byte of context (section 3.2 in its smallest form: FOLLOW sets).
* ``apply_mask``: section 2.1, logits of disallowed tokens become -inf, all
  other logits keep their bit pattern.

Pins (see tests/test_oracle_*.py): hand-enumerated masks and a closed-form
checker on the arithmetic language, Python's ``json`` and ``re`` modules as
independent recognisers, Catalan/central-binomial counts on the Dyck
language, byte-at-a-time equivalence, prefix closure, completion soundness,
union over parallel stacks, and O1 == O2 on random walks.
"""

from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_SOURCES = ["capi.cpp", "grammar.hpp", "utf8dag.hpp", "earley.hpp", "pda.hpp"]
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (host only)."""
    srcs = [os.path.join(_HERE, "src", s) for s in _SOURCES]
    if not force and os.path.exists(_LIB_PATH):
        if os.path.getmtime(_LIB_PATH) >= max(os.path.getmtime(s) for s in srcs):
            return _LIB_PATH
    cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-pthread", "-Wall",
           "-o", _LIB_PATH, srcs[0]]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, cp, i32, i64 = ctypes.c_void_p, ctypes.c_char_p, ctypes.c_int, ctypes.c_int64
    sig = {
        "orc_last_error": (cp, []),
        "orc_grammar_new": (vp, [cp, i64, cp]),
        "orc_grammar_free": (None, [vp]),
        "orc_rule_index": (i32, [vp, cp]),
        "orc_num_rules": (i32, [vp]),
        "orc_follow": (i32, [vp, i32, vp]),
        "orc_recognize": (i32, [vp, cp, i64]),
        "orc_recognize_pda": (i32, [vp, cp, i64]),
        "orc_earley_new": (vp, [vp]),
        "orc_earley_clone": (vp, [vp]),
        "orc_earley_free": (None, [vp]),
        "orc_earley_advance": (i32, [vp, cp, i64]),
        "orc_earley_complete": (i32, [vp]),
        "orc_earley_length": (i32, [vp]),
        "orc_earley_mask": (i32, [vp, vp, vp, i64, vp, i32]),
        "orc_earley_completion": (i64, [vp, vp, i64]),
        "orc_pda_new": (vp, [vp]),
        "orc_pda_free": (None, [vp]),
        "orc_pda_advance": (i32, [vp, cp, i64]),
        "orc_pda_complete": (i32, [vp]),
        "orc_pda_num_configs": (i32, [vp]),
        "orc_pda_mask": (i32, [vp, vp, vp, i64, vp, i32]),
        "orc_pda_mask_single": (i32, [vp, i32, vp, vp, i64, vp, i32]),
        "orc_positions": (vp, [vp, i32, vp, i32]),
        "orc_positions_free": (None, [vp]),
        "orc_positions_size": (i32, [vp]),
        "orc_classify": (i32, [vp, vp, vp, vp, i64, vp, i32]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


class OracleError(RuntimeError):
    pass


def _err() -> str:
    return _load().orc_last_error().decode("utf-8", "replace")


def default_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


class _VocabView:
    """Pointers to a vocabulary's bytes/offsets (any object with .data/.offsets)."""

    def __init__(self, vocab):
        self.data = np.ascontiguousarray(vocab.data, dtype=np.uint8)
        if self.data.size == 0:
            self.data = np.zeros(1, dtype=np.uint8)
        self.offsets = np.ascontiguousarray(vocab.offsets, dtype=np.int64)
        self.V = int(self.offsets.shape[0] - 1)


class Grammar:
    def __init__(self, text: str, root: str = "root"):
        lib = _load()
        raw = text.encode("utf-8")
        self._h = lib.orc_grammar_new(raw, len(raw), root.encode())
        if not self._h:
            raise OracleError(_err())

    def __del__(self):
        if getattr(self, "_h", None) and _load is not None:   # (module globals are gone at interpreter exit)
            _load().orc_grammar_free(self._h)
            self._h = None

    def rule_index(self, name: str) -> int:
        return _load().orc_rule_index(self._h, name.encode())

    def recognize(self, data: bytes) -> int:
        """2 = sentence, 1 = viable prefix only, 0 = not a viable prefix (Earley)."""
        r = _load().orc_recognize(self._h, data, len(data))
        if r < 0:
            raise OracleError(_err())
        return r

    def recognize_pda(self, data: bytes) -> int:
        """Same question answered by the literal pushdown automaton."""
        r = _load().orc_recognize_pda(self._h, data, len(data))
        if r < 0:
            raise OracleError(_err())
        return r

    def follow(self, rule: str) -> set:
        """Bytes that can come right after an instance of ``rule`` in some context."""
        out = np.zeros(256, dtype=np.uint8)
        if _load().orc_follow(self._h, self.rule_index(rule), out.ctypes.data) < 0:
            raise OracleError(f"unknown rule {rule!r}")
        return set(int(c) for c in np.flatnonzero(out))

    def classify(self, rule: str, path, vocab, nthreads: int | None = None) -> np.ndarray:
        """Token classes at the position of ``rule`` reached from its start by
        ``path`` (a list whose items are ints = bytes or rule names =
        references): 0 rejected, 2 accepted, 1 context-dependent, 4
        context-dependent by section 3.1 alone but refused in every context
        by the one-byte narrowing (so: section 3.1's class is {1, 4}, the
        narrowed class is {1})."""
        lib = _load()
        r = self.rule_index(rule)
        if r < 0:
            raise OracleError(f"unknown rule {rule!r}")
        syms = []
        for s in path:
            if isinstance(s, str):
                k = self.rule_index(s)
                if k < 0:
                    raise OracleError(f"unknown rule {s!r} in path")
                syms.append(256 + k)
            else:
                syms.append(int(s))
        arr = np.asarray(syms, dtype=np.int32)
        pos = lib.orc_positions(self._h, r, arr.ctypes.data if arr.size else None, int(arr.size))
        if not pos:
            raise OracleError(_err())
        try:
            if lib.orc_positions_size(pos) == 0:
                raise OracleError(f"no position of {rule!r} is reached by path {path!r}")
            vv = _VocabView(vocab)
            out = np.zeros(vv.V, dtype=np.uint8)
            rc = lib.orc_classify(self._h, pos, vv.data.ctypes.data, vv.offsets.ctypes.data, vv.V,
                                  out.ctypes.data, nthreads or default_threads())
            if rc < 0:
                raise OracleError(_err())
            return out
        finally:
            lib.orc_positions_free(pos)


class EarleyMatcher:
    """O1: accepted text + brute-force mask over a vocabulary."""

    def __init__(self, grammar: Grammar, _handle=None):
        self.grammar = grammar
        self._h = _handle if _handle is not None else _load().orc_earley_new(grammar._h)
        if not self._h:
            raise OracleError(_err())

    def __del__(self):
        if getattr(self, "_h", None) and _load is not None:   # (module globals are gone at interpreter exit)
            _load().orc_earley_free(self._h)
            self._h = None

    def clone(self) -> "EarleyMatcher":
        return EarleyMatcher(self.grammar, _load().orc_earley_clone(self._h))

    def advance(self, data: bytes) -> bool:
        r = _load().orc_earley_advance(self._h, data, len(data))
        if r < 0:
            raise OracleError(_err())
        return bool(r)

    def complete(self) -> bool:
        return bool(_load().orc_earley_complete(self._h))

    def length(self) -> int:
        return _load().orc_earley_length(self._h)

    def mask(self, vocab, nthreads: int | None = None) -> np.ndarray:
        """bool [V]: allowed tokens; stop tokens are allowed iff the accepted
        text is a sentence; other zero-byte tokens are never allowed."""
        vv = _VocabView(vocab)
        out = np.zeros(vv.V, dtype=np.uint8)
        rc = _load().orc_earley_mask(self._h, vv.data.ctypes.data, vv.offsets.ctypes.data, vv.V,
                                     out.ctypes.data, nthreads or default_threads())
        if rc < 0:
            raise OracleError(_err())
        m = out.astype(bool)
        if self.complete():
            m[np.asarray(vocab.stop_ids, dtype=np.int64)] = True
        return m

    def completion(self) -> bytes:
        buf = np.zeros(1 << 20, dtype=np.uint8)
        n = _load().orc_earley_completion(self._h, buf.ctypes.data, buf.size)
        if n < 0:
            raise OracleError(_err())
        return buf[:n].tobytes()


class PdaMatcher:
    """O2: literal Appendix-A automaton on the accepted text."""

    def __init__(self, grammar: Grammar):
        self.grammar = grammar
        self._h = _load().orc_pda_new(grammar._h)
        if not self._h:
            raise OracleError(_err())

    def __del__(self):
        if getattr(self, "_h", None) and _load is not None:   # (module globals are gone at interpreter exit)
            _load().orc_pda_free(self._h)
            self._h = None

    def advance(self, data: bytes) -> bool:
        r = _load().orc_pda_advance(self._h, data, len(data))
        if r < 0:
            raise OracleError(_err())
        return bool(r)

    def complete(self) -> bool:
        r = _load().orc_pda_complete(self._h)
        if r < 0:
            raise OracleError(_err())
        return bool(r)

    def num_configs(self) -> int:
        return _load().orc_pda_num_configs(self._h)

    def mask(self, vocab, nthreads: int | None = None, single: int | None = None) -> np.ndarray:
        vv = _VocabView(vocab)
        out = np.zeros(vv.V, dtype=np.uint8)
        lib = _load()
        if single is None:
            rc = lib.orc_pda_mask(self._h, vv.data.ctypes.data, vv.offsets.ctypes.data, vv.V,
                                  out.ctypes.data, nthreads or default_threads())
        else:
            rc = lib.orc_pda_mask_single(self._h, single, vv.data.ctypes.data, vv.offsets.ctypes.data,
                                         vv.V, out.ctypes.data, nthreads or default_threads())
        if rc < 0:
            raise OracleError(_err())
        m = out.astype(bool)
        if single is None and self.complete():
            m[np.asarray(vocab.stop_ids, dtype=np.int64)] = True
        return m


def pack_bitmask(allowed: np.ndarray) -> np.ndarray:
    """bool [..., V] -> int32 [..., ceil(V/32)]; token i is bit i%32 of word
    i//32 (least significant bit first), 1 = allowed, tail bits 0."""
    allowed = np.asarray(allowed, dtype=bool)
    V = allowed.shape[-1]
    W = (V + 31) // 32
    pad = np.zeros(allowed.shape[:-1] + (W * 32,), dtype=bool)
    pad[..., :V] = allowed
    b = np.packbits(pad.reshape(allowed.shape[:-1] + (W, 32)), axis=-1, bitorder="little")
    return b.view(np.uint32).reshape(allowed.shape[:-1] + (W,)).view(np.int32)


def unpack_bitmask(words: np.ndarray, V: int) -> np.ndarray:
    w = np.ascontiguousarray(words).view(np.uint32)
    bits = np.unpackbits(w.view(np.uint8).reshape(w.shape + (4,)), axis=-1, bitorder="little")
    return bits.reshape(w.shape[:-1] + (-1,))[..., :V].astype(bool)




def apply_mask(logit_bits: np.ndarray, allowed: np.ndarray, neg_inf_bits: int) -> np.ndarray:
    """Section 2.1: out = logits where allowed else -inf, on raw bit patterns.

    ``logit_bits``: unsigned integer view [B, Vl] of the logits (uint16 for
    bf16/fp16, uint32 for fp32); ``allowed``: bool [B, V]; columns >= V (a
    padded LM head) count as not allowed.  ``neg_inf_bits``: the pattern of
    -inf in that type (0xFF800000 fp32, 0xFF80 bf16, 0xFC00 fp16).
    """
    out = logit_bits.copy()
    B, Vl = out.shape
    ok = np.zeros((B, Vl), dtype=bool)
    V = min(Vl, allowed.shape[1])
    ok[:, :V] = allowed[:, :V]
    out[~ok] = neg_inf_bits
    return out
