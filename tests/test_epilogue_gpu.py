"""GPU parity of ts_densify_scaled (write-back epilogue: out = cast(scale * sum), fp32 or
bf16, possibly inside a fusion buffer) against the CPU checker, element by element."""
import numpy as np
import pytest
import torch

import oracle
from oracle import reference as R
from paper_1905_04035_amd import binding as ts
from paper_1905_04035_amd import workloads as wl

from parity import TOL, DEV, to_dev

pytestmark = pytest.mark.gpu


def bf16_value(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def run_scaled(w, scale, out_dtype, group=1, dense=True, in_place=False, buffer_offset=None):
    """Returns (out as a host array, count); with buffer_offset the output lies in a larger
    buffer whose other bytes must stay as they were."""
    V, d = w.V, w.d
    dn = to_dev(w.dense_in if dense else None)
    elem = 2 if out_dtype == ts.TS_OUT_BF16 else 4
    tdt = torch.int16 if out_dtype == ts.TS_OUT_BF16 else torch.float32
    buf = None
    if in_place:
        out = dn
    elif buffer_offset is not None:
        buf = torch.full((buffer_offset + V * d * elem + 512,), 0x5A, dtype=torch.uint8, device=DEV)
        out = buf[buffer_offset:buffer_offset + V * d * elem].view(tdt).view(V, d)
    else:
        out = torch.full((V, d), -1 if elem == 2 else float("nan"), dtype=tdt, device=DEV)
    ids_k, rows_k = w.grouped(group)
    ws = ts.Workspace(max(w.n_total, 1), d, V, DEV)
    try:
        ts.ts_densify_scaled([to_dev(i) for i in ids_k], [to_dev(r) for r in rows_k], w.row_dtype, d, V, dn,
                             out, scale)
        torch.cuda.synchronize()
        count, _, _, _, _ = ts.ts_read_views(V, w.n_total)
        host = out.cpu().numpy()
        if buf is not None:
            b = buf.cpu().numpy()
            assert (b[:buffer_offset] == 0x5A).all() and (b[buffer_offset + V * d * elem:] == 0x5A).all(), \
                "bytes outside the output's place in the buffer were written"
    finally:
        ws.close()
    if out_dtype == ts.TS_OUT_BF16:
        host = host.view(np.uint16)
    return host, count.numpy()


def check_scaled(w, scale, out_dtype, exact_bits=False, **kw):
    dense = kw.get("dense", True)
    got, count = run_scaled(w, scale, out_dtype, **kw)
    r = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in if dense else None, w.row_dtype, scale=scale,
                       out_dtype=R.OUT_BF16 if out_dtype == ts.TS_OUT_BF16 else R.OUT_FP32)
    assert np.array_equal(count, r.count)
    untouched = r.count == 0
    bits_t = np.uint16 if out_dtype == ts.TS_OUT_BF16 else np.uint32
    # rows without pairs: one fp32 product (and one rounding to bf16), the same bits on both sides
    assert np.array_equal(got[untouched].view(bits_t), r.out[untouched].view(bits_t)), \
        "a row that received no pair is not scale * dense_in"
    if exact_bits:
        assert np.array_equal(got.view(bits_t), r.out.view(bits_t))
        return
    t = ~untouched
    tol = TOL * r.abs_sum[t]            # abs_sum already carries |scale|
    if out_dtype == ts.TS_OUT_FP32:
        err = np.abs(got[t].astype(np.float64) - r.exact[t])
        assert (err <= tol).all(), f"worst {float(np.max(err / np.maximum(r.abs_sum[t], 1e-300)))}"
    else:
        # the fp32 value that the GPU rounds lies within tol of the exact one, and rounding is
        # monotonic: the result lies between the roundings of the interval's ends
        lo = bf16_value(R.bf16_round(r.exact[t] - tol))
        hi = bf16_value(R.bf16_round(r.exact[t] + tol))
        v = bf16_value(got[t])
        assert ((v >= lo) & (v <= hi)).all(), f"{int(((v < lo) | (v > hi)).sum())} bf16 outputs outside the rounded interval"
        # and almost all of them are the correctly rounded exact value
        if got[t].size > 1000:
            assert np.mean(got[t] == r.out[t]) > 0.99


@pytest.mark.parametrize("out_dtype", [ts.TS_OUT_FP32, ts.TS_OUT_BF16])
@pytest.mark.parametrize("name,scale,group", [("tiny", 0.5, 1), ("transformer_base", 1.0 / 3.0, 1),
                                              ("transformer_big", 1.0 / 64.0, 1), ("large_batch_bf16", 0.1, 1),
                                              ("multi_shard_stress", 1.0 / 16.0, 2)])
def test_named_configurations_with_epilogue(name, scale, group, out_dtype):
    check_scaled(wl.make(name), scale, out_dtype, group=group)


@pytest.mark.parametrize("out_dtype", [ts.TS_OUT_FP32, ts.TS_OUT_BF16])
@pytest.mark.parametrize("ids", ["zipf", "single", "distinct"])
def test_small_integer_values_and_power_of_two_scale_are_bit_exact(ids, out_dtype):
    n = [900, 800] if ids == "distinct" else [9000, 8000]
    w = wl.make_custom(V=2000, d=260, n_list=n, ids=ids, seed=71, integer_values=True)
    check_scaled(w, 0.125, out_dtype, exact_bits=True)
    check_scaled(w, -2.0, out_dtype, exact_bits=True)


def test_scale_one_fp32_is_ts_densify_multi_bit_for_bit():
    w = wl.make_custom(V=3000, d=512, n_list=[20000, 3000], seed=72)
    got, _ = run_scaled(w, 1.0, ts.TS_OUT_FP32)
    V, d = w.V, w.d
    ws = ts.Workspace(w.n_total, d, V, DEV)
    try:
        out = torch.empty((V, d), dtype=torch.float32, device=DEV)
        ts.ts_densify_multi([to_dev(i) for i in w.ids], [to_dev(r) for r in w.rows], w.row_dtype, d, V,
                            to_dev(w.dense_in), out)
        ref = out.cpu().numpy()
    finally:
        ws.close()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("V,d,n_list", [(1, 4, [10]), (7, 4, [0]), (1025, 260, [999]), (333, 1028, [5000, 1]),
                                        (5000, 264, [40000, 30000]), (64, 8, [100000]),
                                        (300, 2052, [4000]), (150, 4100, [25000, 5000])])
def test_ragged_shapes_both_outputs(V, d, n_list):
    w = wl.make_custom(V=V, d=d, n_list=n_list, seed=73)
    check_scaled(w, 0.3, ts.TS_OUT_FP32)
    check_scaled(w, 0.3, ts.TS_OUT_BF16)


def test_bf16_rows_to_bf16_output_narrow_and_wide():
    for d in (260, 264):
        w = wl.make_custom(V=700, d=d, n_list=[3000], seed=74, row_dtype=wl.ROW_BF16)
        check_scaled(w, 0.25, ts.TS_OUT_BF16)
        check_scaled(w, 0.7, ts.TS_OUT_FP32)


def test_in_place_no_dense_operand_and_fusion_buffer_offsets():
    w = wl.make_custom(V=3000, d=256, n_list=[5000, 1000], seed=75)
    check_scaled(w, 0.5, ts.TS_OUT_FP32, in_place=True)
    check_scaled(w, 0.3, ts.TS_OUT_FP32, dense=False)
    check_scaled(w, 0.3, ts.TS_OUT_BF16, dense=False)
    cap = 134217728
    off, used = ts.ts_fusion_place(cap, 1000, w.d, w.V, ts.TS_OUT_FP32)
    check_scaled(w, 0.25, ts.TS_OUT_FP32, buffer_offset=off)
    off2, _ = ts.ts_fusion_place(cap, used + 3, w.d, w.V, ts.TS_OUT_BF16)
    assert off2 % 256 == 0 and off2 >= used
    check_scaled(w, 0.25, ts.TS_OUT_BF16, buffer_offset=off2)


def test_many_pairs_on_few_rows_two_level_combine_with_epilogue():
    w = wl.make_custom(V=50, d=512, n_list=[150000], ids="zipf", zipf_s=1.5, seed=76)
    check_scaled(w, 1.0 / 8.0, ts.TS_OUT_BF16)
    check_scaled(w, 1.0 / 7.0, ts.TS_OUT_FP32)


def test_special_values_in_untouched_rows():
    w = wl.make_custom(V=100, d=64, n_list=[30], ids="distinct", seed=77)
    bits = w.dense_in.view(np.uint32)
    u = np.setdiff1d(np.arange(w.V), w.ids[0])
    bits[u, 0] = 0x80000000         # -0.0
    bits[u, 1] = 0xFF800000         # -inf
    bits[u, 2] = 0x00000001         # smallest subnormal
    bits[u, 3] = 0x7F7FFFFF         # largest finite: rounds to +inf in bf16
    check_scaled(w, 0.5, ts.TS_OUT_FP32)
    check_scaled(w, 1.0, ts.TS_OUT_BF16)
    check_scaled(w, -1.5, ts.TS_OUT_BF16)


def test_runs_with_epilogue_are_bit_identical():
    w = wl.make("transformer_base")
    a, _ = run_scaled(w, 0.2, ts.TS_OUT_BF16)
    b, _ = run_scaled(w, 0.2, ts.TS_OUT_BF16)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_scales_and_outputs(seed):
    rng = np.random.default_rng(3000 + seed)
    V = int(rng.choice([1, 3, 64, 513, 2048, 5000, 40000]))
    d = int(rng.choice([4, 8, 12, 256, 260, 264, 1024, 1100]))
    k = int(rng.choice([1, 1, 2, 5]))
    top = int(rng.choice([0, 10, 1000, 20000, 40000]))
    n_list = [int(x) for x in rng.integers(0, top + 1, size=k)]
    exact = seed % 2 == 0
    w = wl.make_custom(V=V, d=d, n_list=n_list, ids=["zipf", "uniform", "single"][seed % 3],
                       zipf_s=float(rng.choice([1.05, 1.3, 2.0])), seed=3000 + seed,
                       row_dtype=wl.ROW_BF16 if seed % 4 == 1 else wl.ROW_FP32, integer_values=exact)
    scale = float(rng.choice([0.5, -2.0, 0.0625])) if exact else float(rng.choice([1.0 / 3.0, -0.7, 1e-3, 1.0]))
    out_dtype = ts.TS_OUT_BF16 if seed % 3 != 2 else ts.TS_OUT_FP32
    check_scaled(w, scale, out_dtype, exact_bits=exact, dense=(seed % 5 != 0),
                 in_place=(out_dtype == ts.TS_OUT_FP32 and seed % 5 != 0 and seed % 2 == 1))
    check_scaled(w, scale, ts.TS_OUT_FP32, exact_bits=exact, dense=(seed % 5 != 0))


def test_scaled_and_range_calls_can_be_captured_in_a_hip_graph():
    # both enqueue kernels only; every replay must give the eager call's bits, also with eager
    # calls through the same workspace between the replays
    from paper_1905_04035_amd import binding
    w = wl.make_custom(V=6000, d=512, n_list=[60000, 5000], zipf_s=1.3, seed=91)      # two sort launches
    ids_d = [to_dev(i) for i in w.ids]
    rows_d = [to_dev(r) for r in w.rows]
    dn = to_dev(w.dense_in)
    v0, v1 = 1000, 4500
    dn_slice = dn[v0:v1].contiguous()
    ws = ts.Workspace(w.n_total, w.d, w.V, DEV)
    try:
        eager_s = torch.empty((w.V, w.d), dtype=torch.int16, device=DEV)
        eager_r = torch.empty_like(dn_slice)
        ts.ts_densify_scaled(ids_d, rows_d, w.row_dtype, w.d, w.V, dn, eager_s, 0.125)
        ts.ts_densify_range(ids_d, rows_d, w.row_dtype, w.d, w.V, v0, v1, dn_slice, eager_r)
        torch.cuda.synchronize()
        out_s = torch.zeros_like(eager_s)
        out_r = torch.zeros_like(eager_r)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ts.ts_densify_scaled(ids_d, rows_d, w.row_dtype, w.d, w.V, dn, out_s, 0.125)
            ts.ts_densify_range(ids_d, rows_d, w.row_dtype, w.d, w.V, v0, v1, dn_slice, out_r)
        for rep in range(3):
            out_s.zero_()
            out_r.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out_s, eager_s), f"scaled: replay {rep} differs from the eager call"
            assert torch.equal(out_r, eager_r), f"range: replay {rep} differs from the eager call"
            other = torch.empty_like(dn)
            binding.ts_densify_multi([ids_d[1][: 100 * (rep + 1)]], [rows_d[1][: 100 * (rep + 1)]], w.row_dtype,
                                     w.d, w.V, dn, other)
            torch.cuda.synchronize()
    finally:
        ws.close()
