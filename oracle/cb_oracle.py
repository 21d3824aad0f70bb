"""ctypes loader for the C oracle -- TEST INFRASTRUCTURE (tests, smoke check, benchmark baseline only).

Argument marshalling only; every number comes out of ``cb_oracle.c``.  ``case`` arguments are
duck-typed objects carrying numpy arrays (dtype, B, Hq, Hkv, D, V, block_size, kv_len,
node_offsets, parent, tokens, q, k, v, logits, block_table); this module imports nothing from the
HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcb_oracle.so")
_lib = None


def _configure(L):
    L.cbo_num_threads.restype = C.c_int
    L.cbo_attention_rows.restype = C.c_int
    L.cbo_attention_rows.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int64,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_double, C.c_int,
                                     C.c_void_p, C.c_void_p, C.c_int]
    L.cbo_argmax.restype = None
    L.cbo_argmax.argtypes = [C.c_int, C.c_void_p, C.c_int, C.c_int64, C.c_void_p]
    L.cbo_accept.restype = C.c_int
    L.cbo_accept.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
    L.cbo_compact.restype = C.c_int
    L.cbo_compact.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int64, C.c_void_p, C.c_void_p,
                              C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]
    return L


def load_library(path: str):
    """Open an oracle shared object (the tests also load deliberately broken builds this way)."""
    return _configure(C.CDLL(path))


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        _lib = load_library(_LIB_PATH)
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dt(dtype: str) -> int:
    return {"f32": 0, "bf16": 1}[dtype]


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def num_threads() -> int:
    return int(lib().cbo_num_threads())


def attention_rows(case, rows: np.ndarray, scale: Optional[float] = None, threads: int = 1) -> np.ndarray:
    """Tree attention of the listed (sequence, head, node) rows -> float64 [nrows, D]."""
    rows = _c(rows, np.int32).reshape(-1, 3)
    out = np.empty((rows.shape[0], case.D), dtype=np.float64)
    if scale is None:
        scale = 1.0 / np.sqrt(case.D)
    want = np.float32 if case.dtype == "f32" else np.uint16
    q, k, v = _c(case.q, want), _c(case.k, want), _c(case.v, want)
    paged = case.block_size > 0
    capacity = k.shape[0] if paged else k.shape[1]
    bt = _c(case.block_table, np.int32) if paged else None
    kv_len, offs, par = _c(case.kv_len, np.int32), _c(case.node_offsets, np.int32), _c(case.parent, np.int32)
    rc = lib().cbo_attention_rows(_dt(case.dtype), case.Hq, case.Hkv, case.D, case.block_size, capacity,
                                  _p(q), _p(k), _p(v), _p(bt), bt.shape[1] if paged else 0,
                                  _p(kv_len), _p(offs), _p(par), float(scale), rows.shape[0], _p(rows), _p(out),
                                  int(threads))
    if rc != 0:
        raise MemoryError("oracle attention ran out of memory")
    return out


def all_rows(case) -> np.ndarray:
    """Every (sequence, head, node) triple in the order of the attention output [node, head]."""
    rows = []
    for b in range(case.B):
        n = int(case.node_offsets[b + 1] - case.node_offsets[b])
        for i in range(n):
            for h in range(case.Hq):
                rows.append((b, h, i))
    return np.asarray(rows, dtype=np.int32)


def attention(case, scale: Optional[float] = None, threads: int = 1) -> np.ndarray:
    """Full attention output, float64 [sum_nodes, Hq, D]."""
    out = attention_rows(case, all_rows(case), scale, threads)
    return out.reshape(int(case.node_offsets[-1]), case.Hq, case.D)


def argmax(logits: np.ndarray, dtype: str) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    lg = _c(logits, want)
    out = np.empty(lg.shape[0], dtype=np.int32)
    lib().cbo_argmax(_dt(dtype), _p(lg), lg.shape[0], lg.shape[1], _p(out))
    return out


def accept(parent: Sequence[int], tokens: Sequence[int], a: Sequence[int]) -> Tuple[int, np.ndarray, np.ndarray]:
    """One tree -> (accepted_len L, path[L+1], accepted_tokens[L+1])."""
    par, tok, aa = _c(parent, np.int32), _c(tokens, np.int32), _c(a, np.int32)
    n = par.shape[0]
    path = np.empty(n, dtype=np.int32)
    toks = np.empty(n, dtype=np.int32)
    L = int(lib().cbo_accept(_p(par), _p(tok), _p(aa), n, _p(path), _p(toks)))
    return L, path[:L + 1].copy(), toks[:L + 1].copy()


def verify(case):
    """argmax + acceptance for every sequence of a case -> (a, [(L, path, tokens) per sequence])."""
    a = argmax(case.logits, case.dtype)
    res = []
    for b in range(case.B):
        lo, hi = int(case.node_offsets[b]), int(case.node_offsets[b + 1])
        res.append(accept(case.parent[lo:hi], case.tokens[lo:hi], a[lo:hi]))
    return a, res


def compact(case, k: np.ndarray, v: np.ndarray, seq: int, path: Sequence[int]) -> int:
    """Compacts sequence ``seq`` of the given (writable, C-contiguous) cache arrays in place; returns the new length."""
    assert k.flags.c_contiguous and v.flags.c_contiguous and k.flags.writeable and v.flags.writeable
    paged = case.block_size > 0
    capacity = k.shape[0] if paged else k.shape[1]
    bt = _c(case.block_table, np.int32) if paged else None
    pth = _c(path, np.int32)
    L = pth.shape[0] - 1
    S = int(case.kv_len[seq])
    rc = lib().cbo_compact(k.itemsize, case.Hkv, case.D, case.block_size, capacity, _p(k), _p(v), _p(bt),
                           bt.shape[1] if paged else 0, seq, S, L, _p(pth))
    if rc != 0:
        raise MemoryError("oracle compaction ran out of memory")
    return S + L + 1
