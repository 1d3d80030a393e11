"""ctypes front end of the plain-C checker in densify_oracle.c.

TEST INFRASTRUCTURE ONLY.  Marshals numpy arrays, nothing else: every number it
returns is produced by the C file, which states the passages of the paper it
follows (Section 4, Listing 1; Section 6, Algorithm 2).
"""
from __future__ import annotations

import ctypes as C
import os
import time
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

ROW_FP32 = 0
ROW_BF16 = 1
OUT_FP32 = 0
OUT_BF16 = 1

_lib = None


def _load():
    global _lib
    if _lib is None:
        # TS_SANITIZE=1: the build with the address and undefined-behaviour sanitizers
        path = _build.build(force=False, sanitize=os.environ.get("TS_SANITIZE") == "1")
        lib = C.CDLL(path)
        lib.oracle_accumulate.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                          C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.oracle_accumulate.restype = None
        lib.oracle_finish.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                      C.c_int32, C.c_void_p, C.c_void_p]
        lib.oracle_finish.restype = None
        lib.oracle_densify.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                       C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.oracle_densify.restype = C.c_int
        lib.oracle_unique_ids.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        lib.oracle_unique_ids.restype = C.c_int32
        lib.oracle_buffer_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                            C.c_void_p, C.c_void_p]
        lib.oracle_buffer_bytes.restype = None
        lib.oracle_bf16_from_double_array.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
        lib.oracle_bf16_from_double_array.restype = None
        lib.oracle_finish_scaled.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                             C.c_int32, C.c_float, C.c_int32, C.c_void_p, C.c_void_p,
                                             C.c_void_p]
        lib.oracle_finish_scaled.restype = None
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class OracleResult:
    out: np.ndarray          # float32 [V, d], the float64 sum rounded once (uint16 bf16 bit patterns for OUT_BF16)
    exact: np.ndarray        # float64 [V, d], the unrounded sum
    abs_sum: np.ndarray      # float64 [V, d], sum of |terms| per element (tolerance scale)
    count: np.ndarray        # int32 [V], pairs received per row
    unique_ids: np.ndarray   # int32 [n_unique], ascending
    n_bad: int               # pairs skipped because the id was outside [0, V)


def _as_rows(rows: np.ndarray, row_dtype: int, d: int) -> np.ndarray:
    want = np.uint16 if row_dtype == ROW_BF16 else np.float32
    r = np.ascontiguousarray(rows, dtype=want)
    assert r.size % max(d, 1) == 0
    return r


def densify(ids_k: Sequence[np.ndarray], rows_k: Sequence[np.ndarray], d: int, V: int,
            dense_in: Optional[np.ndarray], row_dtype: int = ROW_FP32, scale: Optional[float] = None,
            out_dtype: int = OUT_FP32) -> OracleResult:
    """Densify k contributions (k may be 1), taken in list order, and add dense_in.

    With scale given (or out_dtype = OUT_BF16) the finish step is the one with the
    write-back epilogue: out = cast(scale * sum)."""
    lib = _load()
    acc = np.zeros((V, d), dtype=np.float64)
    abs_sum = np.zeros((V, d), dtype=np.float64)
    count = np.zeros(V, dtype=np.int32)
    n_bad = np.zeros(1, dtype=np.int64)
    for ids, rows in zip(ids_k, rows_k):
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        rows = _as_rows(rows, row_dtype, d)
        assert rows.size == ids.size * d, (rows.shape, ids.shape, d)
        lib.oracle_accumulate(_ptr(ids), _ptr(rows), ids.size, d, V, row_dtype,
                              _ptr(acc), _ptr(abs_sum), _ptr(count), _ptr(n_bad))
    dn = None if dense_in is None else np.ascontiguousarray(dense_in, dtype=np.float32)
    if dn is not None:
        assert dn.shape == (V, d)
    exact = np.empty((V, d), dtype=np.float64)
    if scale is None and out_dtype == OUT_FP32:
        out = np.empty((V, d), dtype=np.float32)
        lib.oracle_finish(_ptr(acc), _ptr(abs_sum), _ptr(count), _ptr(dn), d, V, _ptr(out), _ptr(exact))
    else:
        sc = np.float32(1.0 if scale is None else scale)
        assert np.isfinite(sc)
        out = np.empty((V, d), dtype=np.uint16 if out_dtype == OUT_BF16 else np.float32)
        lib.oracle_finish_scaled(_ptr(acc), _ptr(abs_sum), _ptr(count), _ptr(dn), d, V, float(sc), out_dtype,
                                 _ptr(out) if out_dtype == OUT_FP32 else None,
                                 _ptr(out) if out_dtype == OUT_BF16 else None, _ptr(exact))
    return OracleResult(out=out, exact=exact, abs_sum=abs_sum, count=count,
                        unique_ids=unique_ids(count), n_bad=int(n_bad[0]))


def bf16_round(x: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) of float64 values, rounded once, ties to even."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint16)
    lib.oracle_bf16_from_double_array(_ptr(x), x.size, _ptr(out))
    return out


def unique_ids(count: np.ndarray) -> np.ndarray:
    lib = _load()
    count = np.ascontiguousarray(count, dtype=np.int32)
    buf = np.empty(count.size, dtype=np.int32)
    m = lib.oracle_unique_ids(_ptr(count), count.size, _ptr(buf))
    return buf[:m].copy()


def buffer_bytes(k: int, N: int, d: int, V: int, row_dtype: int = ROW_FP32):
    """(gathered_bytes, dense_bytes) of the two accumulate strategies."""
    lib = _load()
    g = np.zeros(1, dtype=np.int64)
    dn = np.zeros(1, dtype=np.int64)
    lib.oracle_buffer_bytes(k, N, d, V, row_dtype, _ptr(g), _ptr(dn))
    return int(g[0]), int(dn[0])


def _one_shot(lib, ids, rows, d, V, dn, row_dtype):
    """One call of oracle_densify on marshalled arrays: (out, count, n_bad, seconds)."""
    out = np.empty((V, d), dtype=np.float32)
    count = np.zeros(V, dtype=np.int32)
    n_bad = np.zeros(1, dtype=np.int64)
    t0 = time.perf_counter()
    rc = lib.oracle_densify(_ptr(ids), _ptr(rows), ids.size, d, V, row_dtype, _ptr(dn),
                            _ptr(out), _ptr(count), _ptr(n_bad))
    t1 = time.perf_counter()
    if rc != 0:
        raise MemoryError("oracle_densify could not allocate its accumulator")
    return out, count, int(n_bad[0]), t1 - t0


def densify_one_shot(ids: np.ndarray, rows: np.ndarray, d: int, V: int, dense_in: Optional[np.ndarray],
                     row_dtype: int = ROW_FP32):
    """(out, count, n_bad) of the one-shot form oracle_densify: the same definition as
    densify() on a single contribution, with the function's own float64 array.  This is
    the form densify_timed() times; the pins compare its output with densify()'s."""
    lib = _load()
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    rows = _as_rows(rows, row_dtype, d)
    assert rows.size == ids.size * d, (rows.shape, ids.shape, d)
    dn = None if dense_in is None else np.ascontiguousarray(dense_in, dtype=np.float32)
    if dn is not None:
        assert dn.shape == (V, d)
    out, count, n_bad, _ = _one_shot(lib, ids, rows, d, V, dn, row_dtype)
    return out, count, n_bad


def densify_timed(ids: np.ndarray, rows: np.ndarray, d: int, V: int, dense_in: Optional[np.ndarray],
                  row_dtype: int = ROW_FP32, repeats: int = 3) -> List[float]:
    """Seconds per call of the one-shot form (own zeroed float64 array, single
    thread), after one untimed call.  Used only as a reported CPU baseline."""
    lib = _load()
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    rows = _as_rows(rows, row_dtype, d)
    dn = None if dense_in is None else np.ascontiguousarray(dense_in, dtype=np.float32)
    times = []
    for it in range(repeats + 1):
        seconds = _one_shot(lib, ids, rows, d, V, dn, row_dtype)[3]
        if it > 0:
            times.append(seconds)
    return times
