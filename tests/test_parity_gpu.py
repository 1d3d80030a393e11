"""GPU parity: the HIP path (through the C ABI) against the CPU checker, element by element,
on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_1905_04035_amd import binding as ts
from paper_1905_04035_amd import workloads as wl

from parity import TOL, check, error_bound, run_gpu, run_oracle, to_dev, DEV

pytestmark = pytest.mark.gpu


def _case(w, **kw):
    dense = kw.pop("dense", True)
    exact_bits = kw.pop("exact_bits", False)
    g = run_gpu(w, dense=dense, **kw)
    r = run_oracle(w, dense=dense)
    return check(g, r, w, exact_bits=exact_bits), g, r


# ------------------------------------------------------------- the named configurations
def test_tiny_config():
    worst, g, r = _case(wl.make("tiny"))
    assert len(g["unique_ids"]) > 800
    assert worst < TOL


def test_transformer_base_share_single_and_multi():
    w = wl.make("transformer_base")
    _case(w, mode="single")
    _case(w, mode="multi")


def test_transformer_big_share():
    w = wl.make("transformer_big")
    worst, g, r = _case(w, mode="single")
    assert g["count"].max() > 1500          # the hot row is cut into many pieces
    _case(w, mode="multi")


def test_large_batch_bf16_rows():
    w = wl.make("large_batch_bf16")
    _case(w, mode="multi")


def test_large_batch_bf16_rows_through_the_single_buffer_entry_point():
    # the call the benchmark times for this workload: ts_densify_bf16 on the contributions laid end to end
    w = wl.make("large_batch_bf16")
    worst, g, r = _case(w, mode="single")
    assert g["count"].max() > 15000


def test_read_views_refuses_arrays_sized_for_fewer_rows():
    w = wl.make("tiny")
    ids, rows = w.concatenated()
    dn = to_dev(w.dense_in)
    ws = ts.Workspace(w.n_total, w.d, w.V, DEV)
    try:
        ts.ts_densify(to_dev(ids), to_dev(rows), w.d, w.V, dn, torch.empty_like(dn))
        with pytest.raises(ts.TsError) as e:
            ts.ts_read_views(w.V - 1, w.n_total)          # the last call had V rows
        assert e.value.status == ts.TS_ERR_CAPACITY
        with pytest.raises(ts.TsError) as e:
            ts.ts_read_views(w.V, w.n_total - 1)          # and n_total valid pairs
        assert e.value.status == ts.TS_ERR_CAPACITY
        assert ts.ts_read_views(w.V, w.n_total)[3] == w.n_total
    finally:
        ws.close()


def test_multi_shard_stress_and_buffer_bytes():
    w = wl.make("multi_shard_stress")
    worst, g, r = _case(w, mode="multi", group=2)        # 16 shards of encoder + decoder rows
    assert g["count"].max() > 0.3 * w.n_total             # one row takes about 38 % of the pairs
    top10 = np.sort(g["count"])[-10:].sum() / w.n_total
    assert top10 > 0.7
    gathered, dense = ts.ts_buffer_bytes(16, 2 * 8192, w.d, w.V)
    assert (gathered, dense) == (1074790400, 134217728)
    assert (gathered, dense) == oracle.buffer_bytes(16, 2 * 8192, w.d, w.V)


# ------------------------------------------------------------- exact pins on the GPU path
@pytest.mark.parametrize("name", ["distinct", "zipf", "single"])
def test_small_integer_values_are_bit_exact(name):
    n = {"distinct": 3000, "zipf": 20000, "single": 5000}[name]
    w = wl.make_custom(V=5000, d=256, n_list=[n], ids=name, zipf_s=1.3, seed=21, integer_values=True)
    _case(w, exact_bits=True)


def test_all_distinct_ids_bit_exact_on_normal_data():
    w = wl.make_custom(V=4096, d=512, n_list=[3000], ids="distinct", seed=22)
    _case(w, exact_bits=True)


def test_one_row_takes_every_pair_across_slices():
    # 40000 pairs: more than one sort slice, every pair on one row, 1250+ pieces to combine
    w = wl.make_custom(V=3000, d=128, n_list=[25000, 15000], ids="single", seed=23, integer_values=True)
    _case(w, exact_bits=True, mode="multi")
    wf = wl.make_custom(V=3000, d=128, n_list=[25000, 15000], ids="single", seed=23)
    _case(wf, mode="multi")
    # 300000 pairs on one row: 9375 pieces, 37 segments for the second combine launch
    wb = wl.make_custom(V=50, d=16, n_list=[300000], ids="single", seed=24, integer_values=True)
    _case(wb, exact_bits=True)


# ------------------------------------------------------------- shapes and edges
@pytest.mark.parametrize("V,d,n", [(1, 4, 10), (7, 4, 0), (1000, 64, 2048), (1025, 260, 999),
                                   (2049, 1024, 65), (33000, 8, 70000), (300, 2048, 513)])
def test_ragged_shapes(V, d, n):
    w = wl.make_custom(V=V, d=d, n_list=[n], ids="zipf", zipf_s=1.2, seed=V + d + n)
    _case(w)


def test_more_than_a_million_pairs_walks_each_slice_in_several_rounds():
    # above 64 slices of 16384 pairs the slices grow, and a wavefront walks its share in
    # several rounds of 1024 pairs
    w = wl.make_custom(V=5000, d=8, n_list=[700001, 500000], zipf_s=1.2, seed=51, integer_values=True)
    _case(w, mode="multi", exact_bits=True)


def test_sixty_four_ragged_shards():
    rng = np.random.default_rng(52)
    n_list = [int(x) for x in rng.integers(0, 700, size=64)]
    n_list[5] = 0
    n_list[63] = 1
    w = wl.make_custom(V=2000, d=64, n_list=n_list, zipf_s=1.1, seed=52)
    _case(w, mode="multi")
    # one shard more than the library accepts
    dn = to_dev(w.dense_in)
    with pytest.raises(ts.TsError) as e:
        ts.ts_densify_multi([to_dev(w.ids[0])] * 65, [to_dev(w.rows[0])] * 65, wl.ROW_FP32, w.d, w.V, dn,
                            torch.empty_like(dn))
    assert e.value.status == ts.TS_ERR_SHAPE


def test_huge_vocabulary_few_pairs_and_wide_rows():
    _case(wl.make_custom(V=1000003, d=4, n_list=[50000], zipf_s=1.05, seed=53))
    _case(wl.make_custom(V=37, d=8192, n_list=[300], zipf_s=1.3, seed=54))


@pytest.mark.parametrize("V,d,n", [(700, 260, 3000), (700, 264, 3000), (64, 8, 500), (3000, 1536, 40000)])
def test_bf16_rows_narrow_and_wide_loads(V, d, n):
    # d % 8 == 0 takes 16-byte row loads, otherwise 8-byte ones
    w = wl.make_custom(V=V, d=d, n_list=[n // 2, n - n // 2], zipf_s=1.3, seed=V + d, row_dtype=wl.ROW_BF16)
    _case(w, mode="multi")
    wi = wl.make_custom(V=V, d=d, n_list=[n], zipf_s=1.3, seed=V + d + 1, row_dtype=wl.ROW_BF16,
                        integer_values=True)
    _case(wi, mode="single", exact_bits=True)


@pytest.mark.parametrize("piece", [8, 16, 32])
def test_piece_sizes_and_exact_boundaries(piece):
    ts.ts_set_piece_tokens(piece)
    try:
        # rows with exactly piece-1, piece, piece+1 and 2*piece pairs, at shifting offsets
        V, d = 64, 256
        counts = [piece - 1, piece, piece + 1, 2 * piece, 1, 2 * piece + 1, 3, piece]
        ids = np.concatenate([np.full(c, 5 + 3 * i, dtype=np.int32) for i, c in enumerate(counts)])
        rng = np.random.default_rng(piece)
        ids = ids[rng.permutation(len(ids))]
        rows = rng.integers(-4, 5, size=(len(ids), d)).astype(np.float32)
        dense = rng.integers(-4, 5, size=(V, d)).astype(np.float32)
        w = wl.Workload(spec=wl.Spec("custom", -1, V, d, 1, 0, "zipf"), ids=[ids], rows=[rows], dense_in=dense)
        _case(w, exact_bits=True)
        _case(wl.make_custom(V=2000, d=512, n_list=[9000], zipf_s=1.4, seed=31))
    finally:
        ts.ts_set_piece_tokens(0)


@pytest.mark.parametrize("shift", [0, 1, 37])
@pytest.mark.parametrize("piece", [16, 32])
def test_rows_at_the_boundaries_of_work_groups_and_of_the_combine_tree(piece, shift):
    # A reduce work-group takes 4 pieces; a row inside one work-group is finished there, a longer
    # one leaves a share per work-group, and shares are added up 16 at a time, level by level.
    # Rows of exactly those sizes, one pair less and one more, starting `shift` sorted positions
    # after a work-group boundary; small-integer values, so every bit must match.
    ts.ts_set_piece_tokens(piece)
    try:
        G = 4 * piece                       # sorted positions of one work-group
        counts = [shift] if shift else []
        for c in (G - 1, G, G + 1, 2 * G, 16 * G - 1, 16 * G, 16 * G + 1, 17 * G, 2, piece + 1, 256 * G + 3, 5):
            counts.append(c)
        V, d = 3 * len(counts) + 8, 260      # one full column block and a ragged one
        ids = np.concatenate([np.full(c, 2 + 3 * i, dtype=np.int32) for i, c in enumerate(counts)])
        rng = np.random.default_rng(100 * piece + shift)
        ids = ids[rng.permutation(len(ids))]
        rows = rng.integers(-4, 5, size=(len(ids), d)).astype(np.float32)
        dense = rng.integers(-4, 5, size=(V, d)).astype(np.float32)
        w = wl.Workload(spec=wl.Spec("custom", -1, V, d, 1, 0, "zipf"), ids=[ids], rows=[rows], dense_in=dense)
        worst, g, r = _case(w, exact_bits=True)
        assert g["info"]["combine_levels"] >= 3 and int(r.count.max()) == 256 * G + 3
    finally:
        ts.ts_set_piece_tokens(0)


def test_a_workspace_of_exactly_the_bytes_a_call_uses_is_enough_and_one_byte_less_is_not():
    w = wl.make_custom(V=5000, d=256, n_list=[70000, 30000], zipf_s=1.3, seed=71)     # a multi-slice call
    ids, rows = w.concatenated()
    ids_d, rows_d, dn = to_dev(ids), to_dev(rows), to_dev(w.dense_in)
    need = ts.ts_call_workspace_bytes(w.n_total, ts.TS_ROW_FP32, w.d, w.V)
    assert need <= ts.ts_workspace_bytes(w.n_total, w.d, w.V)
    buf = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = torch.empty_like(dn)
    try:
        assert ts.lib().ts_bind_workspace(buf.data_ptr(), need - 1) == ts.TS_OK
        with pytest.raises(ts.TsError) as e:
            ts.ts_densify(ids_d, rows_d, w.d, w.V, dn, out)
        assert e.value.status == ts.TS_ERR_WORKSPACE
        assert ts.lib().ts_bind_workspace(buf.data_ptr(), need) == ts.TS_OK
        ts.ts_densify(ids_d, rows_d, w.d, w.V, dn, out)
        torch.cuda.synchronize()
        r = run_oracle(w)
        err = np.abs(out.cpu().numpy().astype(np.float64) - r.exact)
        assert np.all(err <= TOL * r.abs_sum)
    finally:
        ts.ts_bind_workspace(None)


@pytest.mark.parametrize("part", [64, 512, 2048])
@pytest.mark.parametrize("ids", ["single", "zipf", "uniform"])
def test_sort_part_sizes_and_lists_of_owned_pairs(part, ids):
    # parts of 2048 ids leave LDS for short lists of owned pairs only: a wavefront that owns more
    # (one id taking every pair is the extreme) flushes its list and rebuilds it when it ranks
    ts.ts_set_sort_part(part)
    try:
        # one slice; several slices; more than 64 slices' worth, so several rounds per wavefront
        for n_list in ([5000], [20000, 30000], [1200000]):
            w = wl.make_custom(V=3000, d=8, n_list=n_list, ids=ids, zipf_s=1.4, seed=part + len(n_list),
                               integer_values=True)
            _case(w, mode="multi", exact_bits=True)
    finally:
        ts.ts_set_sort_part(0)


@pytest.mark.parametrize("mib", [0, 1, 4096])
def test_result_does_not_depend_on_the_overlapped_copy(mib):
    w = wl.make_custom(V=5000, d=512, n_list=[6000, 3000], seed=46)
    ref = run_gpu(w, mode="multi")
    ts.ts_set_overlap_bytes(mib << 20)
    try:
        _case(w, mode="multi")
        got = run_gpu(w, mode="multi")
        _case(w, mode="multi", dense=False)
        wb = wl.make_custom(V=3000, d=256, n_list=[70000], seed=47)      # two sort launches
        _case(wb)
    finally:
        ts.ts_set_overlap_bytes(-1)
    assert np.array_equal(ref["out"].view(np.uint32), got["out"].view(np.uint32))


def test_no_dense_operand_and_in_place():
    w = wl.make_custom(V=3000, d=256, n_list=[5000, 1000], seed=41)
    _case(w, dense=False)                     # Listing 1 alone: untouched rows are +0.0
    _case(w, in_place=True)                   # dense_out == dense_in


def test_out_of_range_ids_are_skipped_and_counted():
    w = wl.make_custom(V=500, d=64, n_list=[4000], seed=42)
    ids = w.ids[0]
    ids[::7] = -1
    ids[3::11] = 500
    ids[5::13] = np.iinfo(np.int32).max
    ids[6::17] = np.iinfo(np.int32).min
    worst, g, r = _case(w)
    assert g["n_bad"] == r.n_bad > 1000


def test_untouched_rows_keep_special_bit_patterns():
    w = wl.make_custom(V=100, d=64, n_list=[30], ids="distinct", seed=43)
    bits = w.dense_in.view(np.uint32)
    bits[:, 0] = 0x80000000
    bits[:, 1] = 0x7FC12345
    bits[:, 2] = 0xFF800000
    g = run_gpu(w)
    r = run_oracle(w)
    untouched = r.count == 0
    assert np.array_equal(g["out"][untouched].view(np.uint32), w.dense_in[untouched].view(np.uint32))
    assert np.array_equal(np.isnan(g["out"]), np.isnan(r.out))


def test_empty_and_ragged_shards():
    w = wl.make_custom(V=900, d=128, n_list=[0, 70, 0, 1, 64, 129, 0], seed=44)
    _case(w, mode="multi")
    # pointers into one buffer == the buffer itself
    ids, rows = w.concatenated()
    a = run_gpu(w, mode="multi")
    b = run_gpu(w, mode="single")
    assert np.array_equal(a["out"].view(np.uint32), b["out"].view(np.uint32))
    assert np.array_equal(a["perm"], b["perm"])


def test_runs_are_bit_identical():
    w = wl.make("transformer_base")
    a = run_gpu(w, mode="single")
    b = run_gpu(w, mode="single")
    c = run_gpu(w, mode="multi")
    assert np.array_equal(a["out"].view(np.uint32), b["out"].view(np.uint32))
    assert np.array_equal(a["out"].view(np.uint32), c["out"].view(np.uint32))


def test_back_to_back_calls_on_one_workspace_keep_their_bits():
    # Long rows are finished inside the reduce launch by whichever work-group brings a row's last
    # share, which reads the other work-groups' shares from scratch memory that the previous call
    # used for other data.  Two different inputs alternate on one workspace, back to back without
    # host synchronisation; every output must have the bits of its first, synchronised run (a share
    # read stale from a cache, or before it was written, would show here).
    wa = wl.make("multi_shard_stress")                       # hottest row: 788 shares, three tree levels
    wb = wl.make_custom(V=32768, d=1024, n_list=[40000, 30000], zipf_s=1.3, seed=49)
    dev = []
    for w in (wa, wb):
        ids, rows = w.concatenated()
        dev.append((w, to_dev(ids), to_dev(rows), to_dev(w.dense_in)))
    ws = ts.Workspace(max(wa.n_total, wb.n_total), 1024, 32768, DEV)
    try:
        want = []
        for w, ids_d, rows_d, dn in dev:
            out = torch.empty_like(dn)
            ts.ts_densify(ids_d, rows_d, w.d, w.V, dn, out)
            torch.cuda.synchronize()
            want.append(out)
        r = run_oracle(wa)
        err = np.abs(want[0].cpu().numpy().astype(np.float64) - r.exact)
        assert np.all(err <= TOL * r.abs_sum)
        outs = [[torch.empty_like(dev[0][3]) for _ in range(4)] for _ in range(2)]
        for rep in range(12):
            for k, (w, ids_d, rows_d, dn) in enumerate(dev):
                ts.ts_densify(ids_d, rows_d, w.d, w.V, dn, outs[k][rep % 4])
            if rep % 4 == 3:
                torch.cuda.synchronize()
                for k in range(2):
                    for o in outs[k]:
                        assert torch.equal(o.view(torch.int32), want[k].view(torch.int32)), (rep, k)
                        o.fill_(float("nan"))
    finally:
        ws.close()


def test_a_call_can_be_captured_in_a_hip_graph_and_replayed():
    # the call enqueues kernels only (no allocation, no host synchronisation, no memset), so it
    # can be recorded once and replayed; every replay must give the eager call's bits
    w = wl.make_custom(V=6000, d=512, n_list=[9000, 5000], zipf_s=1.3, seed=48)
    ids, rows = w.concatenated()
    ids_d, rows_d, dn = to_dev(ids), to_dev(rows), to_dev(w.dense_in)
    eager = torch.empty_like(dn)
    out = torch.zeros_like(dn)
    ws = ts.Workspace(w.n_total, w.d, w.V, DEV)
    try:
        ts.ts_densify(ids_d, rows_d, w.d, w.V, dn, eager)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ts.ts_densify(ids_d, rows_d, w.d, w.V, dn, out)
        for rep in range(3):
            out.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager), f"replay {rep} differs from the eager call"
            # eager work between replays, through the same workspace
            other = torch.empty_like(dn)
            ts.ts_densify(ids_d[: 100 * (rep + 1)], rows_d[: 100 * (rep + 1)], w.d, w.V, dn, other)
            torch.cuda.synchronize()
        r = run_oracle(w)
        assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - r.exact) <= TOL * r.abs_sum)
    finally:
        ws.close()


def test_dense_gradient_fed_as_slices():
    w = wl.make_custom(V=700, d=64, n_list=[1500], seed=45)
    fused = run_gpu(w)
    w2 = wl.Workload(spec=w.spec, ids=[np.arange(w.V, dtype=np.int32)] + w.ids,
                     rows=[w.dense_in] + w.rows, dense_in=w.dense_in)
    sliced = run_gpu(w2, mode="multi", dense=False)
    r = run_oracle(w)
    assert np.all(np.abs(sliced["out"].astype(np.float64) - r.exact) <= TOL * r.abs_sum)
    assert np.array_equal(sliced["count"], fused["count"] + 1)


def test_error_codes_from_the_host_checks():
    V, d = 16, 8
    out = torch.zeros((V, d), dtype=torch.float32, device=DEV)
    ids = torch.zeros(4, dtype=torch.int32, device=DEV)
    rows = torch.zeros((4, d), dtype=torch.float32, device=DEV)
    ts.ts_bind_workspace(None)
    assert ts.ts_densify_raw(ids.data_ptr(), rows.data_ptr(), 4, d, V, None, out.data_ptr()) == ts.TS_ERR_WORKSPACE
    ws = ts.Workspace(4, d, V, DEV)
    try:
        assert ts.ts_densify_raw(ids.data_ptr(), rows.data_ptr(), 4, d, V, None, out.data_ptr()) == ts.TS_OK
        assert ts.ts_densify_raw(ids.data_ptr(), rows.data_ptr(), 100000, d, V, None, out.data_ptr()) == ts.TS_ERR_WORKSPACE
        assert ts.ts_densify_raw(None, rows.data_ptr(), 4, d, V, None, out.data_ptr()) == ts.TS_ERR_NULL
        assert ts.ts_densify_raw(ids.data_ptr(), rows.data_ptr(), 4, d, V, None, None) == ts.TS_ERR_NULL
        assert ts.ts_densify_raw(ids.data_ptr(), rows.data_ptr(), -1, d, V, None, out.data_ptr()) == ts.TS_ERR_SHAPE
        assert ts.ts_densify_raw(ids.data_ptr(), rows.data_ptr(), 4, 6, V, None, out.data_ptr()) == ts.TS_ERR_SHAPE
        assert ts.ts_densify_raw(ids.data_ptr(), rows.data_ptr() + 4, 4, d, V, None, out.data_ptr()) == ts.TS_ERR_ALIGN
        torch.cuda.synchronize()
    finally:
        ws.close()


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_and_options(seed):
    """Seeded random draws of V, d, shard lengths, skew, row type, dense operand and placement."""
    rng = np.random.default_rng(1000 + seed)
    V = int(rng.choice([1, 2, 63, 64, 65, 127, 500, 1023, 1024, 1025, 4097, 20000]))
    d = int(rng.choice([4, 8, 12, 60, 64, 252, 256, 260, 512, 1028]))
    k = int(rng.integers(1, 6))
    scale = int(rng.choice([0, 1, 10, 100, 1000, 20000]))
    n_list = [int(x) for x in rng.integers(0, scale + 1, size=k)]
    row_dtype = wl.ROW_BF16 if seed % 3 == 0 else wl.ROW_FP32
    kind = ["zipf", "uniform", "single", "zipf"][seed % 4]
    exact = seed % 2 == 0
    w = wl.make_custom(V=V, d=d, n_list=n_list, ids=kind, zipf_s=float(rng.choice([1.05, 1.3, 2.0])),
                       seed=2000 + seed, row_dtype=row_dtype, integer_values=exact)
    if seed % 5 == 0 and w.n_total:
        bad = rng.integers(0, len(w.ids[0]) + 1, size=3)
        for b in bad[bad < len(w.ids[0])]:
            w.ids[0][b] = V + int(rng.integers(0, 5))
    mode = "multi" if (k > 1 or seed % 2) else "single"
    _case(w, mode=mode, dense=(seed % 7 != 0), in_place=(seed % 6 == 1), exact_bits=exact)


def test_kernel_timing_events_for_benchmarks():
    w = wl.make_custom(V=4000, d=256, n_list=[9000], seed=61)
    ids_d, rows_d, dn = to_dev(w.ids[0]), to_dev(w.rows[0]), to_dev(w.dense_in)
    out = torch.empty_like(dn)
    ws = ts.Workspace(w.n_total, w.d, w.V, DEV)
    try:
        ts.ts_profile_begin(3)
        for _ in range(5):                      # only the first three calls are timed
            ts.ts_densify(ids_d, rows_d, w.d, w.V, dn, out)
        torch.cuda.synchronize()
        ms = ts.ts_profile_end(3)
        assert len(ms) == 3 and all(0.0 < x < 10.0 for x in ms)
        ts.ts_densify(ids_d, rows_d, w.d, w.V, dn, out)      # recording has stopped
        torch.cuda.synchronize()
        assert ts.ts_profile_end(3) == []
        r = run_oracle(w)
        assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - r.exact) <= TOL * r.abs_sum)
    finally:
        ws.close()


@pytest.mark.parametrize("n", [16385, 20000, 40000, 57344, 57345])
@pytest.mark.parametrize("ids", ["zipf", "single"])
def test_sizes_around_the_one_launch_sort_limit(n, ids):
    # up to 57344 pairs one launch sorts everything, a wavefront walking its share in several rounds
    # of 1024 pairs and keeping its list of owned pairs from round to round ('single': the list of
    # the owning work-group overflows and the share is walked again); one pair more takes two launches
    w = wl.make_custom(V=4000, d=8, n_list=[n], ids=ids, zipf_s=1.3, seed=n, integer_values=True)
    worst, g, r = _case(w, mode="single", exact_bits=True)
    assert g["info"]["sort_slices"] == (1 if n <= 57344 else 4)


@pytest.mark.parametrize("name,group", [("transformer_big", 1), ("large_batch_bf16", 1), ("multi_shard_stress", 2)])
def test_measured_error_stays_under_the_a_priori_bound(name, group):
    # fp32 sums in the library's fixed order: the worst |err| / sum|terms| of a call must not
    # exceed the first-order bound for its longest chain, which itself lies under the tolerance
    w = wl.make(name)
    worst, g, r = _case(w, mode="multi", group=group)
    bound = error_bound(int(r.count.max()), g["info"]["piece_tokens"])
    assert bound < TOL
    assert worst <= bound, (worst, bound)


def test_no_pairs_is_a_pass_through():
    # Section 3, Algorithm 1: with nothing to accumulate the gradient passes through
    w = wl.make_custom(V=777, d=132, n_list=[0], seed=62)
    g = run_gpu(w)
    assert np.array_equal(g["out"].view(np.uint32), w.dense_in.view(np.uint32))
    assert g["n_valid"] == 0 and g["n_bad"] == 0 and len(g["unique_ids"]) == 0 and not g["count"].any()
    z = run_gpu(w, dense=False)
    assert np.array_equal(z["out"].view(np.uint32), np.zeros((777, 132), dtype=np.uint32))


def test_twenty_million_pairs():
    # 64 slices of 312,500 pairs: every wavefront walks its share in 20 rounds; 625,000 pieces
    w = wl.make_custom(V=3000, d=4, n_list=[12_000_000, 8_000_000], ids="zipf", zipf_s=1.2, seed=63,
                       integer_values=True)
    worst, g, r = _case(w, mode="multi")
    assert g["info"]["sort_slices"] == 64 and g["info"]["pieces"] == 625000
    assert int(r.count.max()) > 1_000_000
