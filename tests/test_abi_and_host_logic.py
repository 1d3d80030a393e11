"""No GPU needed: the C-ABI library loads, exports every symbol the header declares, and its
host-side checks and byte arithmetic behave as documented.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

from paper_1905_04035_amd import binding as ts
from paper_1905_04035_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", "ts_densify.h"), os.path.join(ROOT, "include", "ts_densify_tools.h")]


@pytest.fixture(scope="module")
def lib():
    hip_build.build(force=False)
    return ts.lib()


def declared_functions(headers=HEADERS):
    names = set()
    for h in headers:
        text = open(h).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(ts_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"ts_densify", "ts_densify_bf16", "ts_densify_multi", "ts_buffer_bytes"} <= set(names)
    # the library's own calls and the calls for tests, benchmarks and tuning live in separate headers
    api, tools = set(declared_functions(HEADERS[:1])), set(declared_functions(HEADERS[1:]))
    assert {"ts_read_views", "ts_last_launch_info", "ts_profile_begin", "ts_set_piece_tokens"} <= tools
    assert not (api & tools)
    assert not any(n.startswith(("ts_set_", "ts_profile_")) for n in api)
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in the header but not exported"


def test_the_binding_offers_the_same_names():
    for name in declared_functions():
        if name in ("ts_status_string",):
            continue
        assert hasattr(ts, name) or hasattr(ts, name + "_raw"), name


def test_buffer_bytes_formulas_and_errors(lib):
    assert ts.ts_buffer_bytes(16, 16384, 1024, 32768) == (16 * 16384 * (4 + 4 * 1024), 4 * 32768 * 1024)
    assert ts.ts_buffer_bytes(16, 16384, 1024, 32768) == (1074790400, 134217728)
    assert ts.ts_buffer_bytes(2, 65536, 1024, 32768, ts.TS_ROW_BF16)[0] == 2 * 65536 * (4 + 2 * 1024)
    g1, d1 = ts.ts_buffer_bytes(1, 1000, 64, 1000)
    g64, d64 = ts.ts_buffer_bytes(64, 1000, 64, 1000)
    assert g64 == 64 * g1 and d64 == d1              # a gather grows with the workers, a reduce does not
    assert ts.ts_buffer_bytes(0, 0, 4, 1) == (0, 16)
    g, d = C.c_int64(0), C.c_int64(0)
    assert lib.ts_buffer_bytes(1, 1, 0, 1, 0, C.byref(g), C.byref(d)) == ts.TS_ERR_SHAPE
    assert lib.ts_buffer_bytes(1, 1, 4, 1, 7, C.byref(g), C.byref(d)) == ts.TS_ERR_SHAPE
    assert lib.ts_buffer_bytes(-1, 1, 4, 1, 0, C.byref(g), C.byref(d)) == ts.TS_ERR_SHAPE
    assert lib.ts_buffer_bytes(1, 1, 4, 1, 0, None, C.byref(d)) == ts.TS_ERR_NULL
    assert lib.ts_buffer_bytes(2 ** 40, 2 ** 40, 1024, 1, 0, C.byref(g), C.byref(d)) == ts.TS_ERR_OVERFLOW


def test_workspace_bytes(lib):
    small = ts.ts_workspace_bytes(16384, 1024, 32768)
    big = ts.ts_workspace_bytes(262144, 1024, 32768)
    assert 0 < small < big < 2 ** 30
    assert ts.ts_workspace_bytes(0, 4, 1) > 0
    prev = 0
    for n in (1, 100, 16384, 16385, 32768, 32769, 100000, 1000000):
        b = ts.ts_workspace_bytes(n, 256, 5000)
        assert b >= prev
        prev = b
    out = C.c_int64(0)
    assert lib.ts_workspace_bytes(10, 6, 10, C.byref(out)) == ts.TS_ERR_SHAPE        # d % 4 != 0
    assert lib.ts_workspace_bytes(-1, 4, 10, C.byref(out)) == ts.TS_ERR_SHAPE
    assert lib.ts_workspace_bytes(2 ** 31, 4, 10, C.byref(out)) == ts.TS_ERR_OVERFLOW
    assert lib.ts_workspace_bytes(10, 4, 10, None) == ts.TS_ERR_NULL


@pytest.mark.parametrize("V,d", [(32768, 1024), (32768, 64), (3000, 8), (1 << 20, 64), (1000, 260)])
def test_workspace_bound_once_serves_every_smaller_call(lib, V, d):
    # ts_workspace_bytes(n) must never shrink as n grows, and must cover what any call of at most
    # n pairs uses -- also where the sort changes its split: one slice up to 57344 pairs, slices of
    # 16384 pairs beyond, longer slices beyond 64 of them (where the slice count can drop again)
    edges = [0, 1, 1023, 1024, 16384, 16385, 57344, 57345, 65536, 131072, 262144, 1048576, 1048577,
             1048576 + 16384, 1500000, 2000000, 3000000, 20000000]
    grid = sorted(set(edges + [e + k for e in edges for k in (-1, 1, 2, 1025) if e + k >= 0]
                      + list(range(1040000, 1120000, 1777))))
    prev = 0
    for n in grid:
        bound = ts.ts_workspace_bytes(n, d, V)
        assert bound >= prev, (n, bound, prev)
        prev = bound
        for dt in (ts.TS_ROW_FP32, ts.TS_ROW_BF16):
            assert ts.ts_call_workspace_bytes(n, dt, d, V) <= bound, (n, dt)
    # a workspace sized for n_total serves every smaller call, smaller V and d included
    for n_total in (57345, 1048576, 1100000, 20000000):
        bound = ts.ts_workspace_bytes(n_total, d, V)
        for n in grid:
            if n <= n_total:
                assert ts.ts_call_workspace_bytes(n, ts.TS_ROW_FP32, d, V) <= bound, (n_total, n)
                assert ts.ts_call_workspace_bytes(n, ts.TS_ROW_BF16, d, max(1, V // 3)) <= bound, (n_total, n)


def test_argument_checks_happen_before_any_launch(lib):
    ts.ts_bind_workspace(None)
    fake = 0x1000      # 16-byte aligned, never dereferenced: every call below fails a host check first
    f = lambda *a: lib.ts_densify(*a)
    assert f(fake, fake, 4, 8, 16, None, None, None) == ts.TS_ERR_NULL
    assert f(None, fake, 4, 8, 16, None, fake, None) == ts.TS_ERR_NULL
    assert f(fake, None, 4, 8, 16, None, fake, None) == ts.TS_ERR_NULL
    assert f(fake, fake, -1, 8, 16, None, fake, None) == ts.TS_ERR_SHAPE
    assert f(fake, fake, 4, 6, 16, None, fake, None) == ts.TS_ERR_SHAPE
    assert f(fake, fake, 4, 8, 0, None, fake, None) == ts.TS_ERR_SHAPE
    assert f(fake, fake, 2 ** 31, 8, 16, None, fake, None) == ts.TS_ERR_OVERFLOW
    assert f(fake, fake + 4, 4, 8, 16, None, fake, None) == ts.TS_ERR_ALIGN
    assert f(fake, fake, 4, 8, 16, fake + 8, fake, None) == ts.TS_ERR_ALIGN
    assert f(fake, fake, 4, 8, 16, None, fake, None) == ts.TS_ERR_WORKSPACE      # nothing bound
    ids = (C.c_void_p * 1)(fake)
    n = (C.c_int64 * 1)(4)
    assert lib.ts_densify_multi(ids, ids, n, 0, 0, 8, 16, None, fake, None) == ts.TS_ERR_SHAPE
    assert lib.ts_densify_multi(ids, ids, n, ts.TS_MAX_SHARDS + 1, 0, 8, 16, None, fake, None) == ts.TS_ERR_SHAPE
    assert lib.ts_densify_multi(ids, ids, n, 1, 9, 8, 16, None, fake, None) == ts.TS_ERR_SHAPE
    assert lib.ts_densify_multi(None, ids, n, 1, 0, 8, 16, None, fake, None) == ts.TS_ERR_NULL
    assert lib.ts_bind_workspace(C.c_void_p(fake + 8), 1 << 20) == ts.TS_ERR_ALIGN
    assert lib.ts_last_views(None, None, None, None, None) == ts.TS_ERR_WORKSPACE
    assert lib.ts_read_views(None, None, 0, None, 0, None, None, None) == ts.TS_ERR_WORKSPACE


def test_accumulation_rule_branches_are_host_logic(lib):
    # Section 3, Algorithm 1 and Section 6, Algorithm 2: the branch depends on the kinds only
    fake = 0x1000

    def branch(kinds, rule):
        arr = (ts.TsGrad * len(kinds))()
        for i, k in enumerate(kinds):
            arr[i] = ts.TsGrad(k, 0, fake, fake, 5)
        out = C.c_int32(-1)
        assert lib.ts_accumulate_strategy(arr, len(kinds), rule, C.byref(out)) == ts.TS_OK
        return out.value

    D, S = ts.TS_GRAD_DENSE, ts.TS_GRAD_SLICES
    for rule in (ts.TS_RULE_TF, ts.TS_RULE_PROPOSED):
        assert branch([D], rule) == branch([S], rule) == ts.TS_ACC_PASS_THROUGH
        assert branch([D, D, D], rule) == ts.TS_ACC_REDUCE
        assert branch([S, S], rule) == ts.TS_ACC_GATHER
    assert branch([S, S, D], ts.TS_RULE_TF) == ts.TS_ACC_GATHER
    assert branch([S, S, D], ts.TS_RULE_PROPOSED) == ts.TS_ACC_DENSIFY_REDUCE
    assert branch([D, S], ts.TS_RULE_PROPOSED) == ts.TS_ACC_DENSIFY_REDUCE
    arr = (ts.TsGrad * 1)(ts.TsGrad(5, 0, fake, fake, 1))
    out = C.c_int32(-1)
    assert lib.ts_accumulate_strategy(arr, 1, ts.TS_RULE_TF, C.byref(out)) == ts.TS_ERR_SHAPE
    assert lib.ts_accumulate_strategy(arr, 0, ts.TS_RULE_TF, C.byref(out)) == ts.TS_ERR_SHAPE
    assert lib.ts_accumulate_strategy(None, 1, ts.TS_RULE_TF, C.byref(out)) == ts.TS_ERR_NULL


def test_scaled_entry_point_checks_and_fusion_placement(lib):
    ts.ts_bind_workspace(None)
    fake = 0x1000
    ids = (C.c_void_p * 1)(fake)
    n = (C.c_int64 * 1)(4)
    f = lambda out, dt, scale, dn=None: lib.ts_densify_scaled(ids, ids, n, 1, 0, 8, 16, dn, out, dt, C.c_float(scale), None)
    assert f(fake, 2, 1.0) == ts.TS_ERR_SHAPE                       # unknown output type
    assert f(fake, ts.TS_OUT_FP32, float("inf")) == ts.TS_ERR_SHAPE
    assert f(fake, ts.TS_OUT_FP32, float("nan")) == ts.TS_ERR_SHAPE
    assert f(fake, ts.TS_OUT_BF16, 1.0, fake) == ts.TS_ERR_SHAPE    # bf16 output cannot alias dense_in
    assert f(None, ts.TS_OUT_BF16, 1.0) == ts.TS_ERR_NULL
    assert f(fake + 8, ts.TS_OUT_BF16, 0.5) == ts.TS_ERR_ALIGN
    assert f(fake, ts.TS_OUT_BF16, 0.5) == ts.TS_ERR_WORKSPACE      # passes every check, nothing bound
    assert f(fake, ts.TS_OUT_FP32, 0.5, fake) == ts.TS_ERR_WORKSPACE
    # Section 5, runtime settings: a fusion buffer of 134217728 bytes holds exactly one
    # [32768, 1024] fp32 gradient, or two bf16 ones
    cap = 134217728
    assert ts.ts_fusion_place(cap, 0, 1024, 32768, ts.TS_OUT_FP32) == (0, cap)
    off, used = ts.ts_fusion_place(cap, 0, 1024, 32768, ts.TS_OUT_BF16)
    assert (off, used) == (0, cap // 2)
    assert ts.ts_fusion_place(cap, used, 1024, 32768, ts.TS_OUT_BF16) == (cap // 2, cap)
    assert ts.ts_fusion_place(10000, 1, 4, 8, ts.TS_OUT_FP32) == (256, 256 + 128)
    assert ts.ts_fusion_place(10000, 256, 4, 8, ts.TS_OUT_BF16) == (256, 256 + 64)
    o, u = C.c_int64(-7), C.c_int64(-7)
    assert lib.ts_fusion_place(cap, 1, 1024, 32768, 0, C.byref(o), C.byref(u)) == ts.TS_ERR_CAPACITY
    assert (o.value, u.value) == (-7, -7)
    assert lib.ts_fusion_place(cap, 0, 1024, 32768, 5, C.byref(o), C.byref(u)) == ts.TS_ERR_SHAPE
    assert lib.ts_fusion_place(-1, 0, 4, 8, 0, C.byref(o), C.byref(u)) == ts.TS_ERR_SHAPE
    assert lib.ts_fusion_place(cap, 0, 4, 8, 0, None, C.byref(u)) == ts.TS_ERR_NULL
    assert lib.ts_fusion_place(2 ** 62, 2 ** 63 - 100, 4, 8, 0, C.byref(o), C.byref(u)) == ts.TS_ERR_OVERFLOW
    assert lib.ts_fusion_place(2 ** 62, 0, 2 ** 31 - 1, 2 ** 31 - 1, 0, C.byref(o), C.byref(u)) == ts.TS_ERR_OVERFLOW


def test_range_entry_point_checks(lib):
    ts.ts_bind_workspace(None)
    fake = 0x1000
    ids = (C.c_void_p * 1)(fake)
    n = (C.c_int64 * 1)(4)
    f = lambda v0, v1, V=16: lib.ts_densify_range(ids, ids, n, 1, 0, 8, V, v0, v1, None, fake, None)
    assert f(-1, 4) == ts.TS_ERR_SHAPE
    assert f(4, 4) == ts.TS_ERR_SHAPE
    assert f(5, 4) == ts.TS_ERR_SHAPE
    assert f(0, 17) == ts.TS_ERR_SHAPE
    assert f(0, -1) == ts.TS_ERR_SHAPE
    assert f(0, 1, 0) == ts.TS_ERR_SHAPE
    assert f(3, 9) == ts.TS_ERR_WORKSPACE        # passes every check, nothing bound


def test_tuning_setters_validate(lib):
    assert lib.ts_set_piece_tokens(7) == ts.TS_ERR_SHAPE
    assert lib.ts_set_piece_tokens(0) == ts.TS_OK
    assert lib.ts_set_sort_part(100) == ts.TS_ERR_SHAPE
    assert lib.ts_set_sort_part(0) == ts.TS_OK
    assert lib.ts_set_overlap_bytes(-2) == ts.TS_ERR_SHAPE
    assert lib.ts_set_overlap_bytes(-1) == ts.TS_OK
    assert lib.ts_set_short_rows(2) == ts.TS_ERR_SHAPE
    assert lib.ts_set_short_rows(-2) == ts.TS_ERR_SHAPE
    assert lib.ts_set_short_rows(1) == ts.TS_OK
    assert lib.ts_set_short_rows(-1) == ts.TS_OK


def test_status_strings(lib):
    seen = {ts.status_string(i) for i in range(8)}
    assert len(seen) == 8 and "ok" in seen
    assert "unknown" in ts.status_string(99)


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(ts, "_lib", None)
    monkeypatch.setattr(ts, "LIB_PATH", "/nonexistent/libts_densify.so")
    with pytest.raises(FileNotFoundError):
        ts.lib()
