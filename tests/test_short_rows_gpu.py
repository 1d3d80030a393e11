"""GPU parity of the two ways in which output rows with few pairs are added up: by the pieces
that hold their pairs, or row by row by the wavefront that would otherwise copy the row.  The
library chooses by the number of pairs; here each way is forced on the same inputs, compared
with the CPU checker, and the two are compared with each other bit for bit (both add a row's
pairs in sorted order and dense_in last)."""
import numpy as np
import pytest

import oracle
from paper_1905_04035_amd import binding as ts
from paper_1905_04035_amd import workloads as wl

from parity import check, run_gpu, run_oracle
from test_epilogue_gpu import check_scaled, run_scaled
from test_range_gpu import check_range

pytestmark = pytest.mark.gpu


@pytest.fixture(params=[0, 1], ids=["in_the_pieces", "row_by_row"])
def short_rows(request):
    ts.ts_set_short_rows(request.param)
    yield request.param
    ts.ts_set_short_rows(-1)


def _case(w, **kw):
    dense = kw.pop("dense", True)
    exact_bits = kw.pop("exact_bits", False)
    g = run_gpu(w, dense=dense, **kw)
    r = run_oracle(w, dense=dense)
    return check(g, r, w, exact_bits=exact_bits), g, r


def _counts_workload(counts, V, d, seed, row_dtype=wl.ROW_FP32):
    """Rows 2, 5, 8, ... receive exactly counts[0], counts[1], ... pairs, in shuffled input
    order; small-integer values, so that every bit is fixed."""
    ids = np.concatenate([np.full(c, 2 + 3 * i, dtype=np.int32) for i, c in enumerate(counts)])
    rng = np.random.default_rng(seed)
    ids = ids[rng.permutation(len(ids))]
    rows = rng.integers(-4, 5, size=(len(ids), d)).astype(np.float32)
    if row_dtype == wl.ROW_BF16:
        rows = wl.fp32_to_bf16_bits(rows)
    dense = rng.integers(-4, 5, size=(V, d)).astype(np.float32)
    return wl.Workload(spec=wl.Spec("custom", -1, V, d, 1, 0, "zipf", row_dtype=row_dtype), ids=[ids], rows=[rows],
                       dense_in=dense)


def test_named_configurations(short_rows):
    _case(wl.make("tiny"))
    _case(wl.make("transformer_base"), mode="multi")
    _case(wl.make("transformer_big"), mode="single")
    _case(wl.make("large_batch_bf16"), mode="single")


@pytest.mark.parametrize("V,d,n", [(1, 4, 10), (7, 4, 0), (1000, 64, 2048), (1025, 260, 999), (63, 1028, 5000),
                                   (4097, 2052, 3000), (301, 4100, 9000), (70, 8192, 2000)])
def test_ragged_shapes(short_rows, V, d, n):
    w = wl.make_custom(V=V, d=d, n_list=[n // 2, n - n // 2], seed=V + d + n, integer_values=True)
    _case(w, mode="multi", exact_bits=True)
    _case(w, mode="single", exact_bits=True, dense=False)


@pytest.mark.parametrize("V,d,n", [(700, 260, 3000), (700, 264, 3000), (64, 8, 500), (3000, 1536, 40000)])
def test_bf16_rows_narrow_and_wide_loads(short_rows, V, d, n):
    w = wl.make_custom(V=V, d=d, n_list=[n], seed=n + d, row_dtype=wl.ROW_BF16, integer_values=True)
    _case(w, exact_bits=True)
    _case(wl.make_custom(V=V, d=d, n_list=[n], seed=n + d + 1, row_dtype=wl.ROW_BF16))


@pytest.mark.parametrize("piece", [8, 16, 32])
def test_rows_just_below_at_and_above_the_limit_between_the_two_ways(short_rows, piece):
    ts.ts_set_piece_tokens(piece)
    try:
        counts = [piece - 1, piece, piece + 1, 1, 2 * piece, 2, piece, piece + 1, 4 * piece + 1, piece - 1, 1, 1,
                  3, 17 * 4 * piece, piece]
        for dt in (wl.ROW_FP32, wl.ROW_BF16):
            w = _counts_workload(counts, V=3 * len(counts) + 5, d=520, seed=piece, row_dtype=dt)
            worst, g, r = _case(w, exact_bits=True)
            assert int(r.count.max()) == 17 * 4 * piece
    finally:
        ts.ts_set_piece_tokens(0)


@pytest.mark.parametrize("ids", ["distinct", "single", "uniform", "zipf"])
def test_kinds_of_ids_with_and_without_dense_operand_and_in_place(short_rows, ids):
    n = [900, 800] if ids == "distinct" else [9000, 8000]
    w = wl.make_custom(V=2000, d=260, n_list=n, ids=ids, seed=91, integer_values=True)
    _case(w, mode="multi", exact_bits=True)
    _case(w, mode="multi", exact_bits=True, dense=False)
    _case(w, mode="multi", exact_bits=True, in_place=True)
    _case(w, mode="single", exact_bits=True, in_place=True)


def test_out_of_range_ids_and_empty_shards(short_rows):
    w = wl.make_custom(V=500, d=64, n_list=[4000, 0, 100, 0], seed=92)
    w.ids[0][::7] = -1
    w.ids[0][3::11] = 500
    worst, g, r = _case(w, mode="multi")
    assert g["n_bad"] > 0


def test_several_slices_and_the_overlapped_copy(short_rows):
    w = wl.make_custom(V=5000, d=256, n_list=[70000, 30000], zipf_s=1.3, seed=93)
    for mib in (0, 4):
        ts.ts_set_overlap_bytes(mib << 20)
        try:
            _case(w, mode="multi")
        finally:
            ts.ts_set_overlap_bytes(-1)


@pytest.mark.parametrize("out_dtype", [ts.TS_OUT_FP32, ts.TS_OUT_BF16])
def test_with_the_write_back_epilogue(short_rows, out_dtype):
    w = wl.make_custom(V=2000, d=260, n_list=[9000, 8000], seed=94, integer_values=True)
    check_scaled(w, 0.125, out_dtype, exact_bits=True)
    check_scaled(w, -2.0, out_dtype, exact_bits=True, in_place=(out_dtype == ts.TS_OUT_FP32))
    check_scaled(wl.make("transformer_base"), 1.0 / 3.0, out_dtype)
    check_scaled(wl.make_custom(V=3000, d=512, n_list=[50000, 30000], seed=95, row_dtype=wl.ROW_BF16), 0.1, out_dtype)


def test_ranges_of_rows(short_rows):
    w = wl.make_custom(V=3001, d=260, n_list=[9000, 30000], seed=96, integer_values=True)
    r = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    for v0, v1 in [(0, 1), (1, 1000), (1000, 3000), (3000, 3001), (0, 3001)]:
        check_range(w, r, v0, v1, exact_bits=True)
        check_range(w, r, v0, v1, exact_bits=True, in_place=True)


def _run_bits(w, way, **kw):
    ts.ts_set_short_rows(way)
    try:
        return run_gpu(w, **kw)["out"].view(np.uint32)
    finally:
        ts.ts_set_short_rows(-1)


@pytest.mark.parametrize("name", ["transformer_base", "transformer_big", "large_batch_bf16", "multi_shard_stress"])
def test_both_ways_give_the_same_bits(name):
    w = wl.make(name)
    a = _run_bits(w, 0, mode="multi")
    b = _run_bits(w, 1, mode="multi")
    assert np.array_equal(a, b)


def test_both_ways_give_the_same_bits_with_epilogue_and_on_normal_data():
    w = wl.make_custom(V=4000, d=1028, n_list=[30000, 30000], zipf_s=1.2, seed=97, row_dtype=wl.ROW_BF16)
    outs = []
    for mode in (0, 1):
        ts.ts_set_short_rows(mode)
        try:
            outs.append(run_scaled(w, 1.0 / 7.0, ts.TS_OUT_BF16)[0])
        finally:
            ts.ts_set_short_rows(-1)
    assert np.array_equal(outs[0], outs[1])


def test_the_library_chooses_by_the_number_of_pairs():
    # below and above the limit (which depends on the rows' width and type) the results have the
    # bits of the forced runs
    # (d, type, pairs, expected: 0 in the pieces, 1 row by row with lone wavefronts, 2 row by row with
    # pieces of 32 positions in work-groups)
    for d, dt, n, form in [(1024, wl.ROW_FP32, 20000, 0), (1024, wl.ROW_FP32, 60000, 1), (1024, wl.ROW_BF16, 30000, 1),
                           (1024, wl.ROW_BF16, 20000, 0), (512, wl.ROW_FP32, 70000, 1), (512, wl.ROW_FP32, 60000, 0),
                           (256, wl.ROW_FP32, 70000, 0), (64, wl.ROW_BF16, 70000, 0), (2048, wl.ROW_FP32, 21000, 1),
                           (1024, wl.ROW_FP32, 100000, 2), (1024, wl.ROW_BF16, 100000, 1)]:
        w = wl.make_custom(V=3000, d=d, n_list=[n], zipf_s=1.2, seed=n, row_dtype=dt)
        g = run_gpu(w)
        assert g["info"]["short_rows"] == form, (d, dt, n, g["info"])
        auto = g["out"].view(np.uint32)
        assert np.array_equal(auto, _run_bits(w, 0)) and np.array_equal(auto, _run_bits(w, 1))


def test_the_entry_point_with_the_built_in_workspace_row_by_row_and_over_several_slices():
    import torch
    w = wl.make_custom(V=8000, d=1024, n_list=[60000], zipf_s=1.2, seed=98)     # four slices, short rows row by row
    assert ts.ts_workspace_bytes(w.n_total, w.d, w.V) <= ts.TS_STATIC_SCRATCH_BYTES
    ids_h, rows_h = w.concatenated()
    ids, rows, dn = (torch.from_numpy(a).to("cuda:0") for a in (ids_h, rows_h, w.dense_in))
    want = torch.empty_like(dn)
    ws = ts.Workspace(w.n_total, w.d, w.V, "cuda:0")
    ts.ts_densify(ids, rows, w.d, w.V, dn, want)
    torch.cuda.synchronize()
    assert ts.ts_last_launch_info()["sort_slices"] == 4
    ws.close()
    got = torch.full_like(dn, float("nan"))
    ts.ts_densify_static(ids, rows, w.d, w.V, dn, got)
    torch.cuda.synchronize()
    assert torch.equal(want.view(torch.int32), got.view(torch.int32))
    r = run_oracle(w)
    err = np.abs(got.cpu().numpy().astype(np.float64) - r.exact)
    assert (err <= 1e-5 * r.abs_sum).all()
