"""Pins for the CPU checker (oracle/): it is compared with things other than
itself -- hand-worked values, a brute-force triple loop, library scatter-adds,
closed forms and invariants -- so that a dropped term, a wrong sign or index or
a transposed operand in it fails at least one test here."""
import glob
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1905_04035_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _load(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


# ---------------------------------------------------------------- hand-worked values
@pytest.mark.parametrize("name", ["worked_case_shared_embedding.json", "worked_case_convert_only.json",
                                  "worked_case_bf16_rows.json"])
def test_hand_worked_cases(name):
    g = _load(name)
    V, d = g["V"], g["d"]
    ids = np.array(g["ids"], dtype=np.int32)
    if "rows_bf16_hex" in g:
        rows = np.array([[int(x, 16) for x in r] for r in g["rows_bf16_hex"]], dtype=np.uint16)
        dt = wl.ROW_BF16
    else:
        rows = np.array(g["rows"], dtype=np.float32)
        dt = wl.ROW_FP32
    dense = None if g["dense_in"] is None else np.array(g["dense_in"], dtype=np.float32)
    r = oracle.densify([ids], [rows], d, V, dense, dt)
    assert np.array_equal(r.out, np.array(g["expected_out"], dtype=np.float32))
    assert r.count.tolist() == g["expected_count"]
    assert r.unique_ids.tolist() == g["expected_unique_ids"]
    assert r.n_bad == g["expected_n_bad"]


def test_every_golden_file_has_a_citation():
    files = glob.glob(os.path.join(GOLDEN, "*.json"))
    assert files
    for f in files:
        with open(f) as fh:
            assert len(json.load(fh)["citation"]) > 40


# ---------------------------------------------------------------- brute force
def _triple_loop(ids, rows, d, V, dense):
    acc = [[0.0] * d for _ in range(V)]
    cnt = [0] * V
    for t in range(len(ids)):
        v = int(ids[t])
        if v < 0 or v >= V:
            continue
        cnt[v] += 1
        for c in range(d):
            acc[v][c] = acc[v][c] + float(rows[t][c])
    out = [[0.0] * d for _ in range(V)]
    for v in range(V):
        for c in range(d):
            base = 0.0 if dense is None else float(dense[v][c])
            out[v][c] = base if cnt[v] == 0 else acc[v][c] + base
    return np.array(out, dtype=np.float64).reshape(V, d), cnt


@pytest.mark.parametrize("seed", range(12))
def test_brute_force_tiny(seed):
    rng = np.random.default_rng(seed)
    V = int(rng.integers(1, 9))
    d = int(rng.integers(1, 9))
    n = int(rng.integers(0, 17))
    ids = rng.integers(-1, V + 1, size=n).astype(np.int32)      # includes out-of-range ids
    rows = rng.standard_normal((n, d)).astype(np.float32)
    dense = None if seed % 3 == 0 else rng.standard_normal((V, d)).astype(np.float32)
    r = oracle.densify([ids], [rows], d, V, dense)
    want, cnt = _triple_loop(ids, rows, d, V, dense)
    assert np.array_equal(r.exact, want)                        # same float64 order => same bits
    assert np.array_equal(r.out, want.astype(np.float32))
    assert r.count.tolist() == cnt
    assert r.n_bad == int(((ids < 0) | (ids >= V)).sum())


# ---------------------------------------------------------------- the one-shot form (the one that is timed)
def _golden_inputs(g):
    ids = np.array(g["ids"], dtype=np.int32)
    if "rows_bf16_hex" in g:
        rows = np.array([[int(x, 16) for x in r] for r in g["rows_bf16_hex"]], dtype=np.uint16)
        dt = wl.ROW_BF16
    else:
        rows = np.array(g["rows"], dtype=np.float32)
        dt = wl.ROW_FP32
    dense = None if g["dense_in"] is None else np.array(g["dense_in"], dtype=np.float32)
    return ids, rows, dt, dense


@pytest.mark.parametrize("name", ["worked_case_shared_embedding.json", "worked_case_convert_only.json",
                                  "worked_case_bf16_rows.json"])
def test_one_shot_form_on_the_hand_worked_cases(name):
    # oracle_densify (own float64 array, one call) is the form whose time is reported as the
    # CPU baseline: it must give the hand-worked values (Section 4, Listing 1; Section 6,
    # Algorithm 2) as well.
    g = _load(name)
    ids, rows, dt, dense = _golden_inputs(g)
    out, count, n_bad = oracle.densify_one_shot(ids, rows, g["d"], g["V"], dense, dt)
    assert np.array_equal(out, np.array(g["expected_out"], dtype=np.float32))
    assert count.tolist() == g["expected_count"]
    assert n_bad == g["expected_n_bad"]


@pytest.mark.parametrize("seed", range(12))
def test_one_shot_form_brute_force_tiny(seed):
    rng = np.random.default_rng(100 + seed)
    V = int(rng.integers(1, 9))
    d = int(rng.integers(1, 9))
    n = int(rng.integers(0, 17))
    ids = rng.integers(-1, V + 1, size=n).astype(np.int32)      # includes out-of-range ids
    rows = rng.standard_normal((n, d)).astype(np.float32)
    dense = None if seed % 3 == 0 else rng.standard_normal((V, d)).astype(np.float32)
    out, count, n_bad = oracle.densify_one_shot(ids, rows, d, V, dense)
    want, cnt = _triple_loop(ids, rows, d, V, dense)
    assert np.array_equal(out, want.astype(np.float32))
    assert count.tolist() == cnt
    assert n_bad == int(((ids < 0) | (ids >= V)).sum())


@pytest.mark.parametrize("row_dtype", [wl.ROW_FP32, wl.ROW_BF16])
@pytest.mark.parametrize("with_dense", [True, False])
def test_one_shot_form_on_workload_tiny_with_bad_ids(row_dtype, with_dense):
    # library scatter-add in float64 as the third opinion, then bit equality with the
    # shard-by-shard form the parity tests use
    w = wl.make_custom(V=1000, d=64, n_list=[2048], ids="uniform", seed=21, row_dtype=row_dtype)
    ids, rows = w.concatenated()
    ids = ids.copy()
    ids[[3, 500, 2047]] = [-1, w.V, np.iinfo(np.int32).max]
    dense = w.dense_in if with_dense else None
    out, count, n_bad = oracle.densify_one_shot(ids, rows, w.d, w.V, dense, row_dtype)
    ok = (ids >= 0) & (ids < w.V)
    wide = wl.bf16_bits_to_fp32(rows) if row_dtype == wl.ROW_BF16 else rows
    a = np.zeros((w.V, w.d), dtype=np.float64)
    np.add.at(a, ids[ok], wide[ok].astype(np.float64))
    base = np.zeros((w.V, w.d)) if dense is None else dense.astype(np.float64)
    assert np.array_equal(count, np.bincount(ids[ok], minlength=w.V))
    assert n_bad == 3
    touched = count > 0
    np.testing.assert_allclose(out[touched].astype(np.float64), (a + base)[touched], rtol=1e-6, atol=1e-30)
    want_untouched = np.zeros((w.V, w.d), dtype=np.float32) if dense is None else dense
    assert np.array_equal(out[~touched].view(np.uint32), want_untouched[~touched].view(np.uint32))
    r = oracle.densify([ids], [rows], w.d, w.V, dense, row_dtype)
    assert np.array_equal(out.view(np.uint32), r.out.view(np.uint32))
    assert np.array_equal(count, r.count) and n_bad == r.n_bad


def test_one_shot_form_transposed_rows_would_be_caught():
    ids = np.array([0, 1, 0], dtype=np.int32)
    rows = np.array([[1, 10], [100, 1000], [10000, 100000]], dtype=np.float32)
    out, count, n_bad = oracle.densify_one_shot(ids, rows, 2, 2, None)
    assert out.tolist() == [[10001.0, 100010.0], [100.0, 1000.0]]
    assert count.tolist() == [2, 1] and n_bad == 0


# ---------------------------------------------------------------- library scatter-adds
def test_against_numpy_add_at_and_torch_index_add():
    w = wl.make("tiny")
    ids, rows = w.concatenated()
    r = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    a = np.zeros((w.V, w.d), dtype=np.float64)
    np.add.at(a, ids, rows.astype(np.float64))
    touched = np.bincount(ids, minlength=w.V) > 0
    want = np.where(touched[:, None], a + w.dense_in.astype(np.float64), w.dense_in.astype(np.float64))
    np.testing.assert_allclose(r.exact, want, rtol=0, atol=1e-12)
    t = torch.zeros((w.V, w.d), dtype=torch.float64)
    t.index_add_(0, torch.from_numpy(ids.astype(np.int64)), torch.from_numpy(rows.astype(np.float64)))
    t += torch.from_numpy(w.dense_in.astype(np.float64))
    np.testing.assert_allclose(r.exact, t.numpy(), rtol=0, atol=1e-12)
    assert np.array_equal(r.count, np.bincount(ids, minlength=w.V))
    assert np.array_equal(r.unique_ids, np.unique(ids))
    assert len(r.unique_ids) > 800      # ~871 expected of 1000 for 2048 uniform draws


def test_transposed_rows_would_be_caught():
    # rows are [n, d] row-major: pair t owns elements t*d .. t*d+d-1.  A checker that
    # read them as [d, n] would give a different answer on this asymmetric case.
    ids = np.array([0, 1, 0], dtype=np.int32)
    rows = np.array([[1, 10], [100, 1000], [10000, 100000]], dtype=np.float32)
    r = oracle.densify([ids], [rows], 2, 2, None)
    assert r.out.tolist() == [[10001.0, 100010.0], [100.0, 1000.0]]


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("name,scale", [("tiny", 1.0), ("transformer_base", 0.25)])
def test_invariants_column_sums_untouched_rows_counts(name, scale):
    w = wl.make(name, scale_rows=scale)
    ids, rows = w.concatenated()
    r = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    col = w.dense_in.astype(np.float64).sum(axis=0) + rows.astype(np.float64).sum(axis=0)
    np.testing.assert_allclose(r.exact.sum(axis=0), col, rtol=1e-9, atol=1e-9)
    untouched = r.count == 0
    assert untouched.any()
    assert np.array_equal(r.out[untouched].view(np.uint32), w.dense_in[untouched].view(np.uint32))
    assert int(r.count.sum()) == len(ids) - r.n_bad == len(ids)
    assert np.array_equal(r.unique_ids, np.flatnonzero(r.count > 0))


def test_untouched_rows_keep_negative_zero_and_nan_payload():
    V, d = 6, 4
    dense = np.zeros((V, d), dtype=np.float32)
    bits = dense.view(np.uint32)
    bits[1, :] = 0x80000000            # -0.0
    bits[3, 0] = 0x7FC12345            # NaN with a payload
    bits[3, 1] = 0xFF800000            # -inf
    ids = np.array([0, 2, 2], dtype=np.int32)
    rows = np.ones((3, d), dtype=np.float32)
    r = oracle.densify([ids], [rows], d, V, dense)
    assert np.array_equal(r.out[[1, 3, 4, 5]].view(np.uint32), bits[[1, 3, 4, 5]])
    assert r.out[2].tolist() == [2.0] * d


def test_permutation_of_pairs_changes_nothing_that_is_unique():
    w = wl.make("tiny")
    ids, rows = w.concatenated()
    r0 = oracle.densify([ids], [rows], w.d, w.V, w.dense_in)
    p = np.random.default_rng(7).permutation(len(ids))
    r1 = oracle.densify([ids[p]], [rows[p]], w.d, w.V, w.dense_in)
    assert np.array_equal(r0.count, r1.count)
    assert np.array_equal(r0.unique_ids, r1.unique_ids)
    np.testing.assert_allclose(r0.exact, r1.exact, rtol=0, atol=1e-12)
    np.testing.assert_allclose(r0.abs_sum, r1.abs_sum, rtol=1e-12)


# ---------------------------------------------------------------- exact special cases
def test_all_distinct_ids_is_one_fp32_add_per_element():
    w = wl.make_custom(V=512, d=32, n_list=[300], ids="distinct", seed=3)
    ids, rows = w.concatenated()
    r = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    want = w.dense_in.copy()
    want[ids] = w.dense_in[ids] + rows           # fp32 add, once per element
    assert np.array_equal(r.out.view(np.uint32), want.view(np.uint32))


def test_small_integer_data_is_exact_whatever_the_order():
    w = wl.make_custom(V=64, d=16, n_list=[5000], ids="zipf", zipf_s=1.5, seed=11, integer_values=True)
    ids, rows = w.concatenated()
    r = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    a = np.zeros((w.V, w.d), dtype=np.int64)
    np.add.at(a, ids, rows.astype(np.int64))
    a += w.dense_in.astype(np.int64)
    assert np.array_equal(r.out, a.astype(np.float32))
    assert np.array_equal(r.exact, a.astype(np.float64))
    assert r.count.max() > 1000                                  # one row takes a large share


def test_single_hot_row_takes_every_pair():
    w = wl.make_custom(V=10, d=8, n_list=[777], ids="single", seed=5, integer_values=True)
    ids, rows = w.concatenated()
    r = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    v = int(ids[0])
    assert r.count[v] == 777 and r.count.sum() == 777
    assert np.array_equal(r.out[v], rows.sum(axis=0, dtype=np.float64).astype(np.float32) + w.dense_in[v])


@pytest.mark.parametrize("k", [-3, 5])
def test_power_of_two_scaling_is_exact(k):
    w = wl.make("tiny")
    s = np.float32(2.0 ** k)
    r0 = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    r1 = oracle.densify(w.ids, [x * s for x in w.rows], w.d, w.V, w.dense_in * s)
    assert np.array_equal(r1.out, r0.out * s)
    assert np.array_equal(r1.exact, r0.exact * float(s))


# ---------------------------------------------------------------- decomposition
def test_shards_in_order_equal_their_concatenation():
    w = wl.make_custom(V=200, d=12, n_list=[50, 0, 131, 7], seed=2)
    ids, rows = w.concatenated()
    a = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    b = oracle.densify([ids], [rows], w.d, w.V, w.dense_in)
    assert np.array_equal(a.exact, b.exact) and np.array_equal(a.count, b.count)


def test_two_calls_chain_like_one():
    w = wl.make_custom(V=100, d=8, n_list=[300, 200], seed=9, integer_values=True)
    both = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    first = oracle.densify(w.ids[:1], w.rows[:1], w.d, w.V, w.dense_in)
    second = oracle.densify(w.ids[1:], w.rows[1:], w.d, w.V, first.out)
    assert np.array_equal(both.out, second.out)                  # integer data: exact
    assert np.array_equal(both.count, first.count + second.count)
    wf = wl.make_custom(V=100, d=8, n_list=[300, 200], seed=9)
    both = oracle.densify(wf.ids, wf.rows, wf.d, wf.V, wf.dense_in)
    first = oracle.densify(wf.ids[:1], wf.rows[:1], wf.d, wf.V, wf.dense_in)
    second = oracle.densify(wf.ids[1:], wf.rows[1:], wf.d, wf.V, first.out)
    assert np.all(np.abs(second.exact - both.exact) <= 1e-6 * both.abs_sum + 1e-30)


def test_dense_gradient_fed_as_slices_gives_the_same_tensor():
    # Section 3: under the gather strategy the dense gradient is itself turned into
    # indexed slices, one per vocabulary row.  Densifying those V extra pairs must
    # give what adding the dense tensor gives.
    w = wl.make_custom(V=150, d=8, n_list=[400], seed=4)
    fused = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    all_ids = [np.arange(w.V, dtype=np.int32)] + w.ids
    all_rows = [w.dense_in] + w.rows
    sliced = oracle.densify(all_ids, all_rows, w.d, w.V, None)
    np.testing.assert_allclose(sliced.exact, fused.exact, rtol=0, atol=1e-12)
    assert np.array_equal(sliced.count, fused.count + 1)


def test_bf16_rows_are_widened_exactly():
    w = wl.make_custom(V=300, d=16, n_list=[900], seed=6, row_dtype=wl.ROW_BF16)
    a = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in, wl.ROW_BF16)
    wide = [wl.bf16_bits_to_fp32(r) for r in w.rows]
    b = oracle.densify(w.ids, wide, w.d, w.V, w.dense_in, wl.ROW_FP32)
    assert np.array_equal(a.exact, b.exact) and np.array_equal(a.abs_sum, b.abs_sum)


def test_abs_sum_is_the_sum_of_magnitudes():
    w = wl.make_custom(V=40, d=4, n_list=[200], seed=8)
    ids, rows = w.concatenated()
    r = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    a = np.abs(w.dense_in.astype(np.float64))
    np.add.at(a, ids, np.abs(rows.astype(np.float64)))
    np.testing.assert_allclose(r.abs_sum, a, rtol=1e-12)
    assert np.all(np.abs(r.exact) <= r.abs_sum * (1 + 1e-12))


# ---------------------------------------------------------------- byte counts
def test_buffer_bytes_closed_forms():
    g, dn = oracle.buffer_bytes(16, 16384, 1024, 32768)
    assert g == 16 * 16384 * (4 + 4 * 1024) == 1074790400
    assert dn == 4 * 32768 * 1024 == 134217728
    g2, dn2 = oracle.buffer_bytes(32, 16384, 1024, 32768)
    assert g2 == 2 * g and dn2 == dn                      # gather grows with workers, reduce does not
    gb, _ = oracle.buffer_bytes(2, 65536, 1024, 32768, wl.ROW_BF16)
    assert gb == 2 * 65536 * (4 + 2 * 1024)


def test_buffer_bytes_reproduce_the_papers_figures():
    p = _load("paper_accumulate_sizes.json")
    d = p["d_model"]
    V = round(p["dense_MB"] * 1e6 / (4 * d))
    N = V + 2 * p["tokens_per_batch"]       # dense gradient as V slices + encoder + decoder tokens
    g, dn = oracle.buffer_bytes(p["workers"], N, d, V)
    assert abs(dn / 1e6 - p["dense_MB"]) / p["dense_MB"] < 0.001
    assert abs(g / 1e9 - p["gathered_GB"]) / p["gathered_GB"] < 0.02
    assert abs(g / dn - p["ratio"]) / p["ratio"] < 0.02
