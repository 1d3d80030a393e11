"""Shared by the GPU parity tests: run a workload through the C-ABI library and compare
with the CPU checker element by element."""
import numpy as np
import torch

import oracle
from paper_1905_04035_amd import binding as ts
from paper_1905_04035_amd import workloads as wl

# fp32 outputs must satisfy |gpu - exact| <= TOL * (sum of |terms| of that element).
# The library adds at most C <= 32 rows in sequence inside a piece, the 4 pieces of a
# work-group in sequence, then the work-groups' shares of a long row in a tree with a fan-in
# of 16, and dense_in last; with fp32 unit round-off 2^-24
# the first-order bound is (depth - 1) * 2^-24 * sum|terms|, below 1e-5 for any row of
# fewer than 16^8 pieces (see error_depth and error_bound below).
TOL = 1e-5
DEV = "cuda:0"


def to_dev(a, row_dtype=None):
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def run_gpu(w: wl.Workload, mode="auto", group=1, in_place=False, dense=True):
    """mode: 'single' (concatenate, ts_densify / ts_densify_bf16), 'multi' (ts_densify_multi on
    the contributions, `group` of them merged per shard)."""
    V, d = w.V, w.d
    dn_host = w.dense_in if dense else None
    dn = to_dev(dn_host)
    out = dn if (in_place and dn is not None) else torch.full((V, d), float("nan"), dtype=torch.float32, device=DEV)
    if mode == "auto":
        mode = "single" if len(w.ids) == 1 else "multi"
    ws = ts.Workspace(max(w.n_total, 1), d, V, DEV)
    try:
        if mode == "single":
            ids, rows = w.concatenated()
            ids_d, rows_d = to_dev(ids), to_dev(rows)
            if w.row_dtype == wl.ROW_BF16:
                ts.ts_densify_bf16(ids_d, rows_d, d, V, dn, out)
            else:
                ts.ts_densify(ids_d, rows_d, d, V, dn, out)
        else:
            ids_k, rows_k = w.grouped(group)
            ids_d = [to_dev(i) for i in ids_k]
            rows_d = [to_dev(r) for r in rows_k]
            ts.ts_densify_multi(ids_d, rows_d, w.row_dtype, d, V, dn, out)
        torch.cuda.synchronize()
        count, row_start, perm, n_valid, n_bad = ts.ts_read_views(V, w.n_total)
        uniq = ts.ts_unique_ids(min(max(w.n_total, 1), V))
        out_h = out.cpu().numpy()
        info = ts.ts_last_launch_info()
    finally:
        ws.close()
    return dict(info=info, out=out_h, count=count.numpy(), row_start=row_start.numpy(), perm=perm.numpy(),
                n_valid=n_valid, n_bad=n_bad, unique_ids=uniq.numpy())


def run_oracle(w: wl.Workload, dense=True):
    return oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in if dense else None, w.row_dtype)


def check(g, r: oracle.OracleResult, w: wl.Workload, exact_bits=False):
    ids, _ = w.concatenated()
    # integer work: bit-exact
    assert np.array_equal(g["count"], r.count), "per-row counts differ"
    assert np.array_equal(g["unique_ids"], r.unique_ids), "unique-id sets differ"
    assert g["n_bad"] == r.n_bad
    assert g["n_valid"] == len(ids) - r.n_bad
    rs = np.concatenate([[0], np.cumsum(r.count)]).astype(np.int32)
    assert np.array_equal(g["row_start"], rs), "row_start is not the exclusive prefix of count"
    # the sort is stable: positions ordered by (id, input position), ids outside [0, V) dropped
    ok = (ids >= 0) & (ids < w.V)
    want_perm = np.flatnonzero(ok)[np.argsort(ids[ok], kind="stable")].astype(np.int32)
    assert np.array_equal(g["perm"], want_perm), "sorted order is not (id, input position)"
    # rows without pairs: bit copies of dense_in
    out = g["out"]
    untouched = r.count == 0
    assert np.array_equal(out[untouched].view(np.uint32), r.out[untouched].view(np.uint32)), \
        "a row that received no pair is not a bit copy of dense_in"
    # fp32 sums
    if exact_bits:
        assert np.array_equal(out.view(np.uint32), r.out.view(np.uint32)), "outputs differ in bits"
        return 0.0
    err = np.abs(out.astype(np.float64) - r.exact)
    bound = TOL * r.abs_sum
    bad = err > bound
    assert not bad.any(), (f"{int(bad.sum())} elements outside {TOL} * sum|terms|; worst ratio "
                           f"{float(np.max(err[bad] / np.maximum(r.abs_sum[bad], 1e-300)))}")
    assert not np.isnan(out).any()
    scale = np.maximum(r.abs_sum, 1e-300)
    return float(np.max(err / scale))


def error_depth(count_max: int, C: int) -> int:
    """Additions on the longest chain a term of the fullest row can take: C inside a piece; the
    4 pieces of a work-group in sequence; then, per level of the tree in which the shares of a
    row that spans several work-groups are added up (fan-in 16: one level up to 16 work-groups,
    two up to 256, ...), a balanced tree over a batch of shares followed by the batches in
    sequence: 3 + 2 for two batches of 8 (fp32 rows), 2 + 4 for four batches of 4 (bf16 rows read
    16 bytes per lane); dense_in last."""
    if count_max <= C:
        return count_max + 1
    groups = -(-count_max // (4 * C)) + 1
    levels = 1
    while 16 ** levels < groups:
        levels += 1
    return C + 3 + 6 * levels + 1


def error_bound(count_max: int, C: int) -> float:
    """First-order bound on |err| / sum|terms| for fp32 sums in that order."""
    return (error_depth(count_max, C) - 1) * 2.0 ** -24
