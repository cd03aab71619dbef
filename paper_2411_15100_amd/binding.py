"""ctypes binding of libxgm.so: argument marshalling only.

Every function here has the name of the C entry point it calls (minus the
``xgm_`` prefix).  Device buffers are passed as integer addresses
(``tensor.data_ptr()``) and streams as integer handles
(``torch.cuda.current_stream().cuda_stream``); torch itself is not imported.
The library is loaded from this directory; if it has not been built the
import of any entry point fails loudly (there is no fallback).
"""

from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libxgm.so")
_lib = None

DTYPE_F32, DTYPE_BF16, DTYPE_F16 = 0, 1, 2

# name -> (restype, argtypes); must list every symbol include/xgm.h declares
_vp, _cp, _i32, _i64, _sz = ctypes.c_void_p, ctypes.c_char_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
_pp = ctypes.POINTER(ctypes.c_void_p)
SIGNATURES = {
    "xgm_last_error": (_cp, []),
    "xgm_bitmask_words": (_i32, [_i32]),
    "xgm_vocab_create": (_i32, [_vp, _vp, _i32, _vp, _i32, _pp]),
    "xgm_vocab_destroy": (None, [_vp]),
    "xgm_vocab_size": (_i32, [_vp]),
    "xgm_grammar_compile": (_i32, [_cp, _sz, _cp, _pp]),
    "xgm_grammar_destroy": (None, [_vp]),
    "xgm_schema_to_grammar": (_i32, [_cp, _sz, _vp, _sz, _vp]),
    "xgm_grammar_num_nodes": (_i32, [_vp]),
    "xgm_grammar_num_rules": (_i32, [_vp]),
    "xgm_grammar_rule_name": (_cp, [_vp, _i32]),
    "xgm_grammar_node_rule": (_i32, [_vp, _i32]),
    "xgm_grammar_node_path": (_i32, [_vp, _i32, _vp, _i32]),
    "xgm_grammar_node_is_final": (_i32, [_vp, _i32]),
    "xgm_debug_classify_host": (_i32, [_vp, _i32, _cp, _i32]),
    "xgm_debug_walk_host": (_i32, [_vp, _vp, _i32, _cp, _i32, _i32, _vp]),
    "xgm_debug_context_index": (_i32, [_vp, _i32, _i32]),
    "xgm_cache_build": (_i32, [_vp, _vp, _vp, _pp]),
    "xgm_cache_build_ex": (_i32, [_vp, _vp, _vp, ctypes.c_uint32, _pp]),
    "xgm_cache_num_uncertain_plain": (_i32, [_vp, _i32]),
    "xgm_cache_copy_node_plain": (_i32, [_vp, _i32, _vp]),
    "xgm_cache_destroy": (None, [_vp]),
    "xgm_cache_num_nodes": (_i32, [_vp]),
    "xgm_cache_copy_node_bits": (_i32, [_vp, _i32, _vp, _vp]),
    "xgm_cache_num_uncertain": (_i32, [_vp, _i32]),
    "xgm_cache_host_classified": (_i64, [_vp]),
    "xgm_cache_build_kernel_seconds": (ctypes.c_double, [_vp]),
    "xgm_cache_build_seconds": (ctypes.c_double, [_vp]),
    "xgm_cache_build_classify_seconds": (ctypes.c_double, [_vp]),
    "xgm_debug_set_build_batch_nodes": (None, [ctypes.c_int32]),
    "xgm_cache_num_accept_rows": (_i32, [_vp]),
    "xgm_cache_device_bytes": (ctypes.c_int64, [_vp]),
    "xgm_cache_stats": (_i32, [_vp, _vp]),
    "xgm_matcher_create": (_i32, [_vp, _pp]),
    "xgm_matcher_create_host": (_i32, [_vp, _vp, _pp]),
    "xgm_matcher_destroy": (None, [_vp]),
    "xgm_matcher_reset": (_i32, [_vp]),
    "xgm_matcher_accept_token": (_i32, [_vp, _i32]),
    "xgm_matcher_accept_bytes": (_i32, [_vp, _cp, _i32]),
    "xgm_matcher_is_terminated": (_i32, [_vp]),
    "xgm_matcher_can_terminate": (_i32, [_vp]),
    "xgm_matcher_num_stacks": (_i32, [_vp]),
    "xgm_matcher_stack": (_i32, [_vp, _i32, _vp, _i32]),
    "xgm_fill_next_token_bitmask": (_i32, [_vp, _i32, _vp, _vp]),
    "xgm_fill_next_token_bitmask_static": (_i32, [_vp, _i32, _vp, _vp]),
    "xgm_fill_and_apply": (_i32, [_vp, _i32, _vp, _vp, _i32, _i32, ctypes.c_int64, _vp]),
    "xgm_debug_fill_count_steps": (_i32, [_vp, _i32, _vp, _vp, _vp]),
    "xgm_debug_matcher_fill_work": (_i32, [_vp, _vp]),
    "xgm_debug_fill_timed": (_i32, [_vp, _i32, _vp, _vp, _vp]),
    "xgm_batch_create": (_i32, [_vp, _i32, _i32, _vp, _pp]),
    "xgm_batch_destroy": (None, [_vp]),
    "xgm_batch_size": (_i32, [_vp]),
    "xgm_batch_accept_tokens": (_i32, [_vp, _vp, _vp]),
    "xgm_batch_rollback": (_i32, [_vp, _vp, _vp]),
    "xgm_batch_fork": (_i32, [_vp, _vp, _vp]),
    "xgm_batch_status": (_i32, [_vp, _vp, _vp]),
    "xgm_batch_get_row": (_i32, [_vp, _i32, _vp, _vp]),
    "xgm_batch_set_row": (_i32, [_vp, _i32, _vp, _vp]),
    "xgm_batch_fill_next_token_bitmask": (_i32, [_vp, _vp, _vp]),
    "xgm_batch_fill_and_apply": (_i32, [_vp, _vp, _vp, _i32, _i32, ctypes.c_int64, _vp]),
    "xgm_debug_matcher_accept_token_walk": (_i32, [_vp, _i32]),
    "xgm_debug_lds_lookup_rate": (_i32, [_vp, _vp]),
    "xgm_fill_overflow_fixup": (_i32, [_vp]),
    "xgm_fill_overflow_count_device": (_vp, []),
    "xgm_batch_fill_overflow_fixup": (_i32, [_vp, _vp]),
    "xgm_batch_overflow_count_device": (_vp, [_vp]),
    "xgm_overflow_total": (_i64, []),
    "xgm_apply_token_bitmask_inplace": (_i32, [_vp, _i32, _i32, _i32, _i64, _vp, _i32, _vp, _i32, _vp]),
}

STATUS_NAMES = {
    0: "OK", -1: "BAD_ARG", -2: "PARSE", -3: "UNDEFINED_RULE", -4: "LEFT_RECURSION", -5: "UNPRODUCTIVE",
    -6: "TOKEN_REJECTED", -7: "TERMINATED", -8: "TOO_MANY_STACKS", -9: "TOO_LARGE", -10: "HIP", -11: "INTERNAL",
}


class XgmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"XGM_ERR_{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


def _preload_hip_runtime():
    """One process must hold one HIP runtime.  PyTorch ships its own copy of
    libamdhip64 and loads it by file path; if this library were loaded first it
    would pull in the system copy under the same soname and the process would
    end up with two runtimes that do not see each other's devices or memory.
    So, when PyTorch is installed, its copy is loaded first (without importing
    torch); libxgm's dependency then resolves to it by soname."""
    import importlib.util
    import sys
    if "torch" in sys.modules:
        return
    spec = importlib.util.find_spec("torch")
    if spec is None or not spec.origin:
        return
    path = os.path.join(os.path.dirname(spec.origin), "lib", "libamdhip64.so")
    if os.path.exists(path):
        ctypes.CDLL(path, mode=ctypes.RTLD_GLOBAL)


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2411_15100_amd.build` "
            "(there is no fallback implementation)")
    _preload_hip_runtime()
    lib = ctypes.CDLL(_LIB_PATH)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    _handles["lib"] = lib
    return lib


_handles = {"lib": None}  # filled by load_library(); bound into _destroy so that it survives module teardown


def _destroy(fn_name: str, obj, _state=_handles) -> None:
    """Release a handle; safe during interpreter shutdown, when module globals may be gone."""
    try:
        h = obj.__dict__.get("_h")
        lib = _state["lib"]
        if h and lib is not None:
            getattr(lib, fn_name)(h)
        obj.__dict__["_h"] = None
    except Exception:
        pass


def _check(rc: int) -> int:
    if rc < 0:
        raise XgmError(rc, load_library().xgm_last_error().decode("utf-8", "replace"))
    return rc


def bitmask_words(V: int) -> int:
    return load_library().xgm_bitmask_words(V)


class Vocab:
    def __init__(self, data: np.ndarray, offsets: np.ndarray, stop_ids):
        lib = load_library()
        data = np.ascontiguousarray(data, dtype=np.uint8)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        stops = np.ascontiguousarray(np.asarray(stop_ids, dtype=np.int32))
        h = ctypes.c_void_p()
        _check(lib.xgm_vocab_create(data.ctypes.data if data.size else None, offsets.ctypes.data,
                                    int(offsets.shape[0] - 1), stops.ctypes.data if stops.size else None,
                                    int(stops.size), ctypes.byref(h)))
        self._h = h
        self.size = int(offsets.shape[0] - 1)

    def __del__(self, _destroy=_destroy):
        _destroy("xgm_vocab_destroy", self)


def schema_to_grammar(schema_json: str) -> str:
    """Grammar text (root rule `root`) for a JSON schema given as text; see xgm_schema_to_grammar."""
    lib = load_library()
    raw = schema_json.encode("utf-8")
    n = ctypes.c_size_t(0)
    _check(lib.xgm_schema_to_grammar(raw, len(raw), None, 0, ctypes.byref(n)))
    buf = ctypes.create_string_buffer(n.value + 1)
    _check(lib.xgm_schema_to_grammar(raw, len(raw), buf, n.value + 1, ctypes.byref(n)))
    return buf.raw[: n.value].decode("utf-8")


class Grammar:
    def __init__(self, text: str, root: str = "root"):
        lib = load_library()
        raw = text.encode("utf-8")
        h = ctypes.c_void_p()
        _check(lib.xgm_grammar_compile(raw, len(raw), root.encode(), ctypes.byref(h)))
        self._h = h

    def __del__(self, _destroy=_destroy):
        _destroy("xgm_grammar_destroy", self)

    @property
    def num_nodes(self) -> int:
        return _check(load_library().xgm_grammar_num_nodes(self._h))

    @property
    def num_rules(self) -> int:
        return _check(load_library().xgm_grammar_num_rules(self._h))

    def rule_name(self, r: int) -> str:
        s = load_library().xgm_grammar_rule_name(self._h, r)
        if s is None:
            raise XgmError(-1, "rule index out of range")
        return s.decode()

    def node_rule(self, node: int) -> int:
        return _check(load_library().xgm_grammar_node_rule(self._h, node))

    def node_is_final(self, node: int) -> bool:
        return bool(_check(load_library().xgm_grammar_node_is_final(self._h, node)))

    def node_path(self, node: int) -> list:
        """Path from the start of the node's rule: ints are bytes, strings are rule names."""
        lib = load_library()
        n = _check(lib.xgm_grammar_node_path(self._h, node, None, 0))
        buf = np.zeros(max(n, 1), dtype=np.int32)
        _check(lib.xgm_grammar_node_path(self._h, node, buf.ctypes.data, n))
        return [int(s) if s < 256 else self.rule_name(int(s) - 256) for s in buf[:n]]

    def debug_classify_host(self, node: int, data: bytes) -> int:
        return _check(load_library().xgm_debug_classify_host(self._h, node, data, len(data)))

    def debug_walk_host(self, stack, data: bytes, build: bool, with_steps: bool = False):
        arr = np.asarray(stack, dtype=np.int32)
        steps = ctypes.c_int32(0)
        rc = _check(load_library().xgm_debug_walk_host(self._h, arr.ctypes.data, int(arr.size), data, len(data),
                                                       1 if build else 0, ctypes.byref(steps)))
        return (rc, int(steps.value)) if with_steps else rc


    def debug_context_index(self, top: int, below: int) -> int:
        """Index of `below` among the contexts of top's rule; -1000 not a context."""
        return int(load_library().xgm_debug_context_index(self._h, int(top), int(below)))



class Cache:
    def __init__(self, grammar: Grammar, vocab: Vocab, stream: int = 0, keep_plain: bool = False, depth: int = 0):
        """depth: resolve context-dependent tokens at most that many frames deep at build time (0: the default, 3)."""
        h = ctypes.c_void_p()
        if not 0 <= depth <= 7:
            raise ValueError("depth")
        _check(load_library().xgm_cache_build_ex(grammar._h, vocab._h, ctypes.c_void_p(stream),
                                                 (1 if keep_plain else 0) | (depth << 4), ctypes.byref(h)))
        self._h = h
        self.grammar = grammar
        self.vocab = vocab

    def __del__(self, _destroy=_destroy):
        _destroy("xgm_cache_destroy", self)

    @property
    def num_nodes(self) -> int:
        return _check(load_library().xgm_cache_num_nodes(self._h))

    def num_uncertain(self, node: int) -> int:
        return _check(load_library().xgm_cache_num_uncertain(self._h, node))

    def num_uncertain_plain(self, node: int) -> int:
        return _check(load_library().xgm_cache_num_uncertain_plain(self._h, node))

    def copy_node_plain(self, node: int):
        plain = np.zeros(bitmask_words(self.vocab.size), dtype=np.int32)
        _check(load_library().xgm_cache_copy_node_plain(self._h, node, plain.ctypes.data))
        return plain

    @property
    def host_classified(self) -> int:
        return load_library().xgm_cache_host_classified(self._h)

    @property
    def build_kernel_seconds(self) -> float:
        return load_library().xgm_cache_build_kernel_seconds(self._h)

    @property
    def build_seconds(self) -> float:
        return load_library().xgm_cache_build_seconds(self._h)

    @property
    def build_classify_seconds(self) -> float:
        """The part of build_seconds spent until the section 3.1 classes of every node were known."""
        return load_library().xgm_cache_build_classify_seconds(self._h)

    @property
    def num_accept_rows(self) -> int:
        """Distinct accepted bitsets kept (at most one per node)."""
        return _check(load_library().xgm_cache_num_accept_rows(self._h))

    @property
    def device_bytes(self) -> int:
        """Bytes of device memory the cache holds."""
        return int(load_library().xgm_cache_device_bytes(self._h))

    def copy_node_bits(self, node: int, with_uncertain: bool = True):
        """(accepted, context-dependent) bitsets of a node; the second needs keep_plain=True at build time
        (None with with_uncertain=False)."""
        W = bitmask_words(self.vocab.size)
        acc = np.zeros(W, dtype=np.int32)
        unc = np.zeros(W, dtype=np.int32) if with_uncertain else None
        _check(load_library().xgm_cache_copy_node_bits(self._h, node, acc.ctypes.data,
                                                       unc.ctypes.data if with_uncertain else None))
        return acc, unc

    @property
    def stats(self) -> dict:
        """Sizes of the cache (xgm_cache_stats)."""
        out = np.zeros(8, dtype=np.int64)
        _check(load_library().xgm_cache_stats(self._h, out.ctypes.data))
        names = ["keys", "keys_level1", "keys_level2", "entries", "entries_level0", "context_dependent_pairs",
                 "pair_context_items", "bitset_rows"]
        return {k: int(v) for k, v in zip(names, out)}


class Matcher:
    def __init__(self, cache: Cache = None, grammar: Grammar = None, vocab: Vocab = None):
        lib = load_library()
        h = ctypes.c_void_p()
        if cache is not None:
            _check(lib.xgm_matcher_create(cache._h, ctypes.byref(h)))
            self._keep = (cache,)
        else:
            _check(lib.xgm_matcher_create_host(grammar._h, vocab._h if vocab is not None else None, ctypes.byref(h)))
            self._keep = (grammar, vocab)
        self._h = h

    def __del__(self, _destroy=_destroy):
        _destroy("xgm_matcher_destroy", self)

    def reset(self):
        _check(load_library().xgm_matcher_reset(self._h))

    def accept_token(self, token_id: int):
        _check(load_library().xgm_matcher_accept_token(self._h, int(token_id)))

    def accept_bytes(self, data: bytes):
        _check(load_library().xgm_matcher_accept_bytes(self._h, data, len(data)))

    def debug_fill_work(self) -> np.ndarray:
        """[stacks with a bitset row, entries of the level-0 / level-1 / level-2 lists] a fill reads for this state."""
        out = np.zeros(4, dtype=np.int64)
        _check(load_library().xgm_debug_matcher_fill_work(self._h, out.ctypes.data))
        return out

    def try_accept_bytes(self, data: bytes) -> int:
        return load_library().xgm_matcher_accept_bytes(self._h, data, len(data))

    def try_accept_token(self, token_id: int) -> int:
        return load_library().xgm_matcher_accept_token(self._h, int(token_id))

    def debug_try_accept_token_walk(self, token_id: int) -> int:
        """accept_token through the depth-first walk the device uses (status code)."""
        return load_library().xgm_debug_matcher_accept_token_walk(self._h, int(token_id))

    def is_terminated(self) -> bool:
        return bool(_check(load_library().xgm_matcher_is_terminated(self._h)))

    def can_terminate(self) -> bool:
        return bool(_check(load_library().xgm_matcher_can_terminate(self._h)))

    def num_stacks(self) -> int:
        return _check(load_library().xgm_matcher_num_stacks(self._h))

    def stack(self, s: int) -> list:
        lib = load_library()
        n = _check(lib.xgm_matcher_stack(self._h, s, None, 0))
        buf = np.zeros(max(n, 1), dtype=np.int32)
        _check(lib.xgm_matcher_stack(self._h, s, buf.ctypes.data, n))
        return buf[:n].tolist()


def fill_next_token_bitmask(matchers, d_bitmask: int, stream: int = 0):
    """d_bitmask: device address of int32 [len(matchers), bitmask_words(V)]."""
    arr = (ctypes.c_void_p * len(matchers))(*[m._h for m in matchers])
    _check(load_library().xgm_fill_next_token_bitmask(arr, len(matchers), ctypes.c_void_p(d_bitmask),
                                                      ctypes.c_void_p(stream)))


def fill_next_token_bitmask_static(matchers, d_bitmask: int, stream: int = 0):
    """As fill_next_token_bitmask, staged in fixed memory (the call allocates nothing)."""
    arr = (ctypes.c_void_p * len(matchers))(*[m._h for m in matchers])
    _check(load_library().xgm_fill_next_token_bitmask_static(arr, len(matchers), ctypes.c_void_p(d_bitmask),
                                                             ctypes.c_void_p(stream)))


STATIC_STAGING_BYTES = 1 << 20


class MatcherBatch:
    """A fixed batch of matchers with the pointer array prepared once."""

    def __init__(self, matchers):
        self.matchers = list(matchers)
        self._arr = (ctypes.c_void_p * len(self.matchers))(*[m._h for m in self.matchers])

    def fill_next_token_bitmask(self, d_bitmask: int, stream: int = 0):
        _check(load_library().xgm_fill_next_token_bitmask(self._arr, len(self.matchers), ctypes.c_void_p(d_bitmask),
                                                          ctypes.c_void_p(stream)))


class DeviceBatch:
    """Matcher states of a fixed batch kept in device memory (xgm_batch_*).

    All pointer arguments are device addresses (ints); token ids and rollback
    steps are int32 [B] device arrays."""

    def __init__(self, matchers, history: int = 8, stream: int = 0):
        lib = load_library()
        arr = (ctypes.c_void_p * len(matchers))(*[m._h for m in matchers])
        h = ctypes.c_void_p()
        _check(lib.xgm_batch_create(arr, len(matchers), int(history), ctypes.c_void_p(stream), ctypes.byref(h)))
        self._h = h
        self.size = len(matchers)

    def __del__(self, _destroy=_destroy):
        _destroy("xgm_batch_destroy", self)

    def accept_tokens(self, d_token_ids: int, stream: int = 0):
        _check(load_library().xgm_batch_accept_tokens(self._h, ctypes.c_void_p(d_token_ids), ctypes.c_void_p(stream)))

    def rollback(self, d_steps: int, stream: int = 0):
        _check(load_library().xgm_batch_rollback(self._h, ctypes.c_void_p(d_steps), ctypes.c_void_p(stream)))

    def fork(self, d_src_rows: int, stream: int = 0):
        _check(load_library().xgm_batch_fork(self._h, ctypes.c_void_p(d_src_rows), ctypes.c_void_p(stream)))

    def status(self, stream: int = 0) -> np.ndarray:
        out = np.zeros(self.size, dtype=np.int32)
        _check(load_library().xgm_batch_status(self._h, out.ctypes.data, ctypes.c_void_p(stream)))
        return out

    def get_row(self, row: int, matcher: "Matcher", stream: int = 0):
        _check(load_library().xgm_batch_get_row(self._h, int(row), matcher._h, ctypes.c_void_p(stream)))

    def set_row(self, row: int, matcher: "Matcher", stream: int = 0):
        _check(load_library().xgm_batch_set_row(self._h, int(row), matcher._h, ctypes.c_void_p(stream)))

    def fill_overflow_fixup(self, stream: int = 0) -> int:
        return _check(load_library().xgm_batch_fill_overflow_fixup(self._h, ctypes.c_void_p(stream)))

    def overflow_count_device(self) -> int:
        """Device address of the batch's counter of walks over the limits."""
        return int(load_library().xgm_batch_overflow_count_device(self._h) or 0)

    def fill_next_token_bitmask(self, d_bitmask: int, stream: int = 0):
        _check(load_library().xgm_batch_fill_next_token_bitmask(self._h, ctypes.c_void_p(d_bitmask),
                                                                ctypes.c_void_p(stream)))

    def fill_and_apply(self, d_bitmask: int, d_logits: int, dtype: int, v_logits: int, row_stride: int,
                       stream: int = 0):
        _check(load_library().xgm_batch_fill_and_apply(self._h, ctypes.c_void_p(d_bitmask), ctypes.c_void_p(d_logits),
                                                       int(dtype), int(v_logits), int(row_stride),
                                                       ctypes.c_void_p(stream)))


def fill_and_apply(matchers, d_bitmask: int, d_logits: int, dtype: int, v_logits: int, row_stride: int,
                   stream: int = 0):
    """Fill the bitmask and mask the logits in one launch (rows 16-byte aligned)."""
    batch = matchers if isinstance(matchers, MatcherBatch) else MatcherBatch(matchers)
    _check(load_library().xgm_fill_and_apply(batch._arr, len(batch.matchers), ctypes.c_void_p(d_bitmask),
                                             ctypes.c_void_p(d_logits), int(dtype), int(v_logits), int(row_stride),
                                             ctypes.c_void_p(stream)))


def debug_fill_count_steps(batch: "MatcherBatch", d_bitmask: int, stream: int = 0) -> int:
    """Automaton steps taken by all walks of one fill of this batch (instrumentation)."""
    n = ctypes.c_int64(0)
    _check(load_library().xgm_debug_fill_count_steps(batch._arr, len(batch.matchers), ctypes.c_void_p(d_bitmask),
                                                     ctypes.c_void_p(stream), ctypes.byref(n)))
    return int(n.value)


def debug_set_build_batch_nodes(nodes: int) -> None:
    """Test knob: the following cache builds classify `nodes` nodes per batch (0: the default, all at once)."""
    load_library().xgm_debug_set_build_batch_nodes(int(nodes))


def debug_lds_lookup_rate(stream: int = 0) -> float:
    """Dependent LDS reads per second of the whole device (measurement aid)."""
    out = ctypes.c_double(0.0)
    _check(load_library().xgm_debug_lds_lookup_rate(ctypes.c_void_p(stream), ctypes.byref(out)))
    return float(out.value)


def debug_fill_timed(batch: "MatcherBatch", d_bitmask: int, stream: int = 0):
    """One fill with HIP events around its kernels: (upload kernel us, fill kernel us)."""
    us = (ctypes.c_float * 2)()
    _check(load_library().xgm_debug_fill_timed(batch._arr, len(batch.matchers), ctypes.c_void_p(d_bitmask),
                                               ctypes.c_void_p(stream), us))
    return float(us[0]), float(us[1])


def fill_overflow_fixup(stream: int = 0) -> int:
    return _check(load_library().xgm_fill_overflow_fixup(ctypes.c_void_p(stream)))


def fill_overflow_count_device() -> int:
    """Device address of the counter of walks over the limits recorded by fills from host-side states."""
    return int(load_library().xgm_fill_overflow_count_device() or 0)


def overflow_total() -> int:
    return _check(load_library().xgm_overflow_total())


def apply_token_bitmask_inplace(d_logits: int, dtype: int, B: int, V_logits: int, row_stride: int, d_bitmask: int,
                                V_mask: int, d_row_index: int = 0, n_rows: int = None, stream: int = 0):
    if n_rows is None:
        n_rows = B
    _check(load_library().xgm_apply_token_bitmask_inplace(
        ctypes.c_void_p(d_logits), dtype, B, V_logits, row_stride, ctypes.c_void_p(d_bitmask), V_mask,
        ctypes.c_void_p(d_row_index) if d_row_index else None, n_rows, ctypes.c_void_p(stream)))
