"""ctypes binding of libts_densify.so: the same names as include/ts_densify.h and
include/ts_densify_tools.h (the calls for tests, benchmarks and tuning).

Argument marshalling only.  Tensors are PyTorch tensors on the GPU (PyTorch is
used for device memory and streams, nothing else); every step of the path runs
in the library's kernels.  There is no fallback: if the library is missing or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

TS_OK = 0
TS_ERR_NULL, TS_ERR_SHAPE, TS_ERR_ALIGN, TS_ERR_WORKSPACE, TS_ERR_HIP, TS_ERR_OVERFLOW, TS_ERR_CAPACITY = 1, 2, 3, 4, 5, 6, 7
TS_GRAD_DENSE, TS_GRAD_SLICES = 0, 1
TS_RULE_TF, TS_RULE_PROPOSED = 1, 2
TS_ACC_PASS_THROUGH, TS_ACC_REDUCE, TS_ACC_DENSIFY_REDUCE, TS_ACC_GATHER = 0, 1, 2, 3
TS_ROW_FP32, TS_ROW_BF16 = 0, 1
TS_OUT_FP32, TS_OUT_BF16 = 0, 1
TS_MAX_SHARDS = 64

# TS_SANITIZE=1 selects the build whose host code runs under ASan + UBSan (build.py, sanitize=True)
LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)),
                        "libts_densify_san.so" if os.environ.get("TS_SANITIZE") == "1" else "libts_densify.so")

_lib = None


class TsGrad(C.Structure):
    """ts_grad of include/ts_densify.h."""
    _fields_ = [("kind", C.c_int32), ("reserved", C.c_int32), ("ids", C.c_void_p), ("values", C.c_void_p),
                ("n", C.c_int64)]


class TsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib():
    """The loaded library.  Raises if it has not been built (run build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1905_04035_amd.build`")
        l = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        l.ts_densify.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
        l.ts_densify_bf16.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
        l.ts_densify_static.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
        l.ts_densify_multi.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, vp]
        l.ts_densify_scaled.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, i32, C.c_float, vp]
        l.ts_fusion_place.argtypes = [i64, i64, i32, i32, i32, vp, vp]
        l.ts_densify_range.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp]
        l.ts_buffer_bytes.argtypes = [i64, i64, i32, i32, i32, vp, vp]
        l.ts_accumulate_strategy.argtypes = [vp, i32, i32, vp]
        l.ts_accumulate.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, i64, vp, vp, vp]
        l.ts_workspace_bytes.argtypes = [i64, i32, i32, vp]
        l.ts_call_workspace_bytes.argtypes = [i64, i32, i32, i32, vp]
        l.ts_bind_workspace.argtypes = [vp, i64]
        l.ts_last_views.argtypes = [vp, vp, vp, vp, vp]
        l.ts_read_views.argtypes = [vp, vp, i64, vp, i64, vp, vp, vp]
        l.ts_unique_ids.argtypes = [vp, vp, vp]
        l.ts_last_launch_info.argtypes = [vp]
        l.ts_profile_begin.argtypes = [i32]
        l.ts_profile_end.argtypes = [vp, i32, vp]
        l.ts_set_piece_tokens.argtypes = [i32]
        l.ts_set_overlap_bytes.argtypes = [i64]
        l.ts_set_sort_part.argtypes = [i32]
        l.ts_set_short_rows.argtypes = [i32]
        l.ts_status_string.argtypes = [C.c_int]
        l.ts_status_string.restype = C.c_char_p
        for name in ("ts_densify", "ts_densify_static", "ts_densify_bf16", "ts_densify_multi", "ts_buffer_bytes",
                     "ts_densify_scaled", "ts_fusion_place", "ts_densify_range",
                     "ts_accumulate_strategy", "ts_accumulate",
                     "ts_workspace_bytes", "ts_call_workspace_bytes", "ts_bind_workspace", "ts_last_views", "ts_read_views", "ts_unique_ids",
                     "ts_last_launch_info",
                     "ts_profile_begin", "ts_profile_end", "ts_set_piece_tokens", "ts_set_overlap_bytes", "ts_set_sort_part", "ts_set_short_rows"):
            getattr(l, name).restype = C.c_int
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().ts_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != TS_OK:
        raise TsError(status, where)


def _p(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check_dense(d: int, V: int, dense_in, dense_out):
    assert dense_out.is_cuda and dense_out.dtype == torch.float32 and dense_out.is_contiguous()
    assert tuple(dense_out.shape) == (V, d)
    if dense_in is not None:
        assert dense_in.is_cuda and dense_in.dtype == torch.float32 and dense_in.is_contiguous()
        assert tuple(dense_in.shape) == (V, d)


def _check_pair(ids, rows, d: int, dtype):
    assert ids.is_cuda and ids.dtype == torch.int32 and ids.is_contiguous()
    assert rows.is_cuda and rows.dtype == dtype and rows.is_contiguous()
    assert rows.numel() == ids.numel() * d


# ---- raw calls (return the status; used by the error-path tests) -------------------------------
def ts_densify_raw(ids_ptr, rows_ptr, n, d, V, dense_in_ptr, dense_out_ptr, stream_ptr=None) -> int:
    return lib().ts_densify(ids_ptr, rows_ptr, n, d, V, dense_in_ptr, dense_out_ptr, stream_ptr)


# ---- the entry points ----------------------------------------------------------------------------
def ts_densify(ids: torch.Tensor, rows: torch.Tensor, d: int, V: int,
               dense_in: Optional[torch.Tensor], dense_out: torch.Tensor, stream=None) -> None:
    _check_pair(ids, rows, d, torch.float32)
    _check_dense(d, V, dense_in, dense_out)
    _check(lib().ts_densify(_p(ids), _p(rows), ids.numel(), d, V, _p(dense_in), _p(dense_out),
                            _stream(stream)), "ts_densify")


TS_STATIC_SCRATCH_BYTES = 16 << 20


def ts_densify_static(ids: torch.Tensor, rows: torch.Tensor, d: int, V: int,
                      dense_in: Optional[torch.Tensor], dense_out: torch.Tensor, stream=None) -> None:
    """ts_densify on the library's built-in workspace: nothing is allocated or bound."""
    _check_pair(ids, rows, d, torch.float32)
    _check_dense(d, V, dense_in, dense_out)
    _check(lib().ts_densify_static(_p(ids), _p(rows), ids.numel(), d, V, _p(dense_in), _p(dense_out),
                                   _stream(stream)), "ts_densify_static")


def ts_densify_bf16(ids: torch.Tensor, rows: torch.Tensor, d: int, V: int,
                    dense_in: Optional[torch.Tensor], dense_out: torch.Tensor, stream=None) -> None:
    """rows: uint16 / int16 / bfloat16 tensor holding bf16 bit patterns."""
    assert rows.element_size() == 2
    _check_pair(ids, rows, d, rows.dtype)
    _check_dense(d, V, dense_in, dense_out)
    _check(lib().ts_densify_bf16(_p(ids), _p(rows), ids.numel(), d, V, _p(dense_in), _p(dense_out),
                                 _stream(stream)), "ts_densify_bf16")


def ts_densify_multi(ids_k: Sequence[torch.Tensor], rows_k: Sequence[torch.Tensor], row_dtype: int,
                     d: int, V: int, dense_in: Optional[torch.Tensor], dense_out: torch.Tensor,
                     stream=None) -> None:
    k = len(ids_k)
    assert k == len(rows_k)
    for i, r in zip(ids_k, rows_k):
        assert r.element_size() == (2 if row_dtype == TS_ROW_BF16 else 4)
        _check_pair(i, r, d, r.dtype)
    _check_dense(d, V, dense_in, dense_out)
    ids_arr = (C.c_void_p * max(k, 1))(*[i.data_ptr() for i in ids_k])
    rows_arr = (C.c_void_p * max(k, 1))(*[r.data_ptr() for r in rows_k])
    n_arr = (C.c_int64 * max(k, 1))(*[i.numel() for i in ids_k])
    _check(lib().ts_densify_multi(ids_arr, rows_arr, n_arr, k, row_dtype, d, V, _p(dense_in),
                                  _p(dense_out), _stream(stream)), "ts_densify_multi")


def ts_densify_scaled(ids_k: Sequence[torch.Tensor], rows_k: Sequence[torch.Tensor], row_dtype: int,
                      d: int, V: int, dense_in: Optional[torch.Tensor], out: torch.Tensor, scale: float,
                      stream=None) -> None:
    """out: [V, d] float32, or a 2-byte dtype (bfloat16 / int16 / uint16) for bf16 output; it may
    be a view into a larger buffer (a fusion buffer at the offset ts_fusion_place gives)."""
    k = len(ids_k)
    assert k == len(rows_k)
    for i, r in zip(ids_k, rows_k):
        assert r.element_size() == (2 if row_dtype == TS_ROW_BF16 else 4)
        _check_pair(i, r, d, r.dtype)
    assert out.is_cuda and out.is_contiguous() and out.numel() == V * d
    assert out.dtype == torch.float32 or out.element_size() == 2
    out_dtype = TS_OUT_FP32 if out.dtype == torch.float32 else TS_OUT_BF16
    if dense_in is not None:
        assert dense_in.is_cuda and dense_in.dtype == torch.float32 and dense_in.is_contiguous()
        assert tuple(dense_in.shape) == (V, d)
    ids_arr = (C.c_void_p * max(k, 1))(*[i.data_ptr() for i in ids_k])
    rows_arr = (C.c_void_p * max(k, 1))(*[r.data_ptr() for r in rows_k])
    n_arr = (C.c_int64 * max(k, 1))(*[i.numel() for i in ids_k])
    _check(lib().ts_densify_scaled(ids_arr, rows_arr, n_arr, k, row_dtype, d, V, _p(dense_in), _p(out),
                                   out_dtype, C.c_float(scale), _stream(stream)), "ts_densify_scaled")


def ts_densify_range(ids_k: Sequence[torch.Tensor], rows_k: Sequence[torch.Tensor], row_dtype: int,
                     d: int, V: int, v_begin: int, v_end: int, dense_in: Optional[torch.Tensor],
                     dense_out: torch.Tensor, stream=None) -> None:
    """dense_in / dense_out: the [v_end - v_begin, d] slice of the owner of rows v_begin .. v_end - 1."""
    k = len(ids_k)
    assert k == len(rows_k)
    for i, r in zip(ids_k, rows_k):
        assert r.element_size() == (2 if row_dtype == TS_ROW_BF16 else 4)
        _check_pair(i, r, d, r.dtype)
    _check_dense(d, v_end - v_begin, dense_in, dense_out)
    ids_arr = (C.c_void_p * max(k, 1))(*[i.data_ptr() for i in ids_k])
    rows_arr = (C.c_void_p * max(k, 1))(*[r.data_ptr() for r in rows_k])
    n_arr = (C.c_int64 * max(k, 1))(*[i.numel() for i in ids_k])
    _check(lib().ts_densify_range(ids_arr, rows_arr, n_arr, k, row_dtype, d, V, v_begin, v_end, _p(dense_in),
                                  _p(dense_out), _stream(stream)), "ts_densify_range")


def ts_fusion_place(capacity_bytes: int, used_bytes: int, d: int, V: int, out_dtype: int = TS_OUT_FP32):
    """(offset_bytes, used_after_bytes) of a [V, d] result in a fusion buffer."""
    off, used = C.c_int64(-1), C.c_int64(-1)
    _check(lib().ts_fusion_place(capacity_bytes, used_bytes, d, V, out_dtype, C.byref(off), C.byref(used)),
           "ts_fusion_place")
    return off.value, used.value


def _grad_array(grads):
    """grads: list of ("dense", tensor[V, d]) or ("slices", ids[n], rows[n, d]) -> ts_grad array."""
    arr = (TsGrad * max(len(grads), 1))()
    for i, g in enumerate(grads):
        if g[0] == "dense":
            t = g[1]
            assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
            arr[i] = TsGrad(TS_GRAD_DENSE, 0, None, t.data_ptr(), 0)
        else:
            ids, rows = g[1], g[2]
            assert ids.is_cuda and ids.dtype == torch.int32 and ids.is_contiguous()
            assert rows.is_cuda and rows.dtype == torch.float32 and rows.is_contiguous()
            arr[i] = TsGrad(TS_GRAD_SLICES, 0, ids.data_ptr(), rows.data_ptr(), ids.numel())
    return arr


def ts_accumulate_strategy(grads, rule: int) -> int:
    st = C.c_int32(-1)
    _check(lib().ts_accumulate_strategy(_grad_array(grads), len(grads), rule, C.byref(st)),
           "ts_accumulate_strategy")
    return st.value


def ts_accumulate(grads, rule: int, d: int, V: int, dense_out: Optional[torch.Tensor] = None,
                  ids_out: Optional[torch.Tensor] = None, rows_out: Optional[torch.Tensor] = None, stream=None):
    """Returns (strategy, n_slices); n_slices is None when the result is dense."""
    cap = 0 if ids_out is None else ids_out.numel()
    if rows_out is not None:
        assert rows_out.is_cuda and rows_out.dtype == torch.float32 and rows_out.numel() >= cap * d
    n_out, st = C.c_int64(-1), C.c_int32(-1)
    _check(lib().ts_accumulate(_grad_array(grads), len(grads), rule, d, V, _p(dense_out), _p(ids_out),
                               _p(rows_out), cap, C.byref(n_out), C.byref(st), _stream(stream)), "ts_accumulate")
    return st.value, (n_out.value if n_out.value >= 0 else None)


def ts_buffer_bytes(k: int, N: int, d: int, V: int, row_dtype: int = TS_ROW_FP32):
    g, dn = C.c_int64(0), C.c_int64(0)
    _check(lib().ts_buffer_bytes(k, N, d, V, row_dtype, C.byref(g), C.byref(dn)), "ts_buffer_bytes")
    return g.value, dn.value


def ts_workspace_bytes(n_total: int, d: int, V: int) -> int:
    b = C.c_int64(0)
    _check(lib().ts_workspace_bytes(n_total, d, V, C.byref(b)), "ts_workspace_bytes")
    return b.value


def ts_call_workspace_bytes(n_total: int, row_dtype: int, d: int, V: int) -> int:
    """Bytes of workspace a call of exactly this shape uses (host arithmetic)."""
    b = C.c_int64(0)
    _check(lib().ts_call_workspace_bytes(n_total, row_dtype, d, V, C.byref(b)), "ts_call_workspace_bytes")
    return b.value


def ts_bind_workspace(ws: Optional[torch.Tensor]) -> None:
    if ws is None:
        _check(lib().ts_bind_workspace(None, 0), "ts_bind_workspace")
        return
    assert ws.is_cuda and ws.is_contiguous()
    _check(lib().ts_bind_workspace(_p(ws), ws.numel() * ws.element_size()), "ts_bind_workspace")


class Workspace:
    """Device scratch for calls of up to n_total pairs; keeps the tensor alive while bound."""

    def __init__(self, n_total: int, d: int, V: int, device="cuda:0"):
        self.bytes = ts_workspace_bytes(n_total, d, V)
        self.tensor = torch.empty(self.bytes, dtype=torch.uint8, device=device)
        ts_bind_workspace(self.tensor)

    def close(self):
        ts_bind_workspace(None)
        self.tensor = None


def ts_read_views(V: int, n: int):
    """(count[V], row_start[V+1], perm[n_valid], n_valid, n_bad_ids) of the last call as host
    tensors (the library waits for the current stream and copies); perm is the input position of
    every sorted pair."""
    count = torch.empty(V, dtype=torch.int32)
    row_start = torch.empty(V + 1, dtype=torch.int32)
    records = torch.empty((max(n, 1), 8), dtype=torch.int32)        # TS_SORTED_PAIR_BYTES = 32
    n_valid, n_bad = C.c_int32(0), C.c_int32(0)
    _check(lib().ts_read_views(C.c_void_p(count.data_ptr()), C.c_void_p(row_start.data_ptr()), V,
                               C.c_void_p(records.data_ptr()), n, C.byref(n_valid), C.byref(n_bad),
                               _stream(None)), "ts_read_views")
    return count, row_start, records[:n_valid.value, 3].contiguous(), n_valid.value, n_bad.value


def ts_last_views():
    """Device addresses (ints) of count, row_start, the sorted records, n_valid and n_bad_ids of
    the last call, inside the bound workspace."""
    ptrs = [C.c_void_p() for _ in range(5)]
    _check(lib().ts_last_views(*[C.byref(p) for p in ptrs]), "ts_last_views")
    return tuple(p.value for p in ptrs)


def ts_unique_ids(capacity: int, stream=None, device="cuda:0"):
    """Ascending ids that received at least one pair in the last call (host tensor)."""
    out = torch.empty(max(capacity, 1), dtype=torch.int32, device=device)
    n_out = torch.zeros(1, dtype=torch.int32, device=device)
    _check(lib().ts_unique_ids(_p(out), _p(n_out), _stream(stream)), "ts_unique_ids")
    m = int(n_out.cpu()[0])
    return out[:m].cpu()


def ts_last_launch_info() -> dict:
    buf = (C.c_int32 * 8)()
    _check(lib().ts_last_launch_info(buf), "ts_last_launch_info")
    keys = ["piece_tokens", "sort_copy_rows_end", "reduce_copy_rows_end", "sort_slices", "sort_part",
            "pieces", "combine_levels", "in_place"]
    info = dict(zip(keys, list(buf)))
    info["short_rows"] = info["in_place"] >> 1      # 0 in the pieces, 1 / 2 row by row
    info["in_place"] &= 1
    return info


def ts_profile_begin(capacity: int) -> None:
    _check(lib().ts_profile_begin(capacity), "ts_profile_begin")


def ts_profile_end(capacity: int):
    buf = (C.c_float * max(capacity, 1))()
    n = C.c_int32(0)
    _check(lib().ts_profile_end(buf, capacity, C.byref(n)), "ts_profile_end")
    return [buf[i] for i in range(n.value)]


def ts_set_piece_tokens(piece_tokens: int) -> None:
    _check(lib().ts_set_piece_tokens(piece_tokens), "ts_set_piece_tokens")


def ts_set_overlap_bytes(sort_bytes: int) -> None:
    _check(lib().ts_set_overlap_bytes(sort_bytes), "ts_set_overlap_bytes")


def ts_set_sort_part(part: int) -> None:
    _check(lib().ts_set_sort_part(part), "ts_set_sort_part")


def ts_set_short_rows(mode: int) -> None:
    _check(lib().ts_set_short_rows(mode), "ts_set_short_rows")
