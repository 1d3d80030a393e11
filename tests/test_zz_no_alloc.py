"""ts_densify_static, the entry point that allocates nothing: its output is compared with
ts_densify's (same kernels, a workspace built into the library instead of a bound one), bit
for bit, on two calls in a row, the second smaller than the first."""
import numpy as np
import pytest
import torch

from paper_1905_04035_amd import binding as ts
from paper_1905_04035_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(w):
    ids_h, rows_h = w.concatenated()
    ids = torch.from_numpy(ids_h).to(DEV)
    rows = torch.from_numpy(rows_h).to(DEV)
    dn = torch.from_numpy(w.dense_in).to(DEV)
    want = torch.empty_like(dn)
    ws = ts.Workspace(w.n_total, w.d, w.V, DEV)
    ts.ts_densify(ids, rows, w.d, w.V, dn, want)
    torch.cuda.synchronize()
    want_views = ts.ts_read_views(w.V, w.n_total)
    ws.close()                                   # nothing is bound from here on
    got = torch.full_like(dn, float("nan"))
    ts.ts_densify_static(ids, rows, w.d, w.V, dn, got)
    torch.cuda.synchronize()
    got_views = ts.ts_read_views(w.V, w.n_total)
    return want, got, want_views, got_views


def test_static_scratch_matches_the_bound_workspace_twice_in_a_row():
    big = wl.make("transformer_big")                                           # 16384 pairs, V=32768, d=1024
    small = wl.make_custom(V=5000, d=256, n_list=[700, 300], zipf_s=1.3, seed=77)   # then a smaller call
    for w in (big, small):
        assert ts.ts_workspace_bytes(w.n_total, w.d, w.V) <= ts.TS_STATIC_SCRATCH_BYTES
        want, got, wv, gv = _both(w)
        assert torch.equal(want.view(torch.int32), got.view(torch.int32))     # every bit
        assert torch.equal(wv[0], gv[0]) and torch.equal(wv[1], gv[1]) and torch.equal(wv[2], gv[2])
        assert wv[3:] == gv[3:]


def test_static_scratch_rejects_what_does_not_fit():
    V, d, n = 32768, 1024, 200000
    assert ts.ts_workspace_bytes(n, d, V) > ts.TS_STATIC_SCRATCH_BYTES
    ids = torch.zeros(n, dtype=torch.int32, device=DEV)
    rows = torch.empty((1, d), dtype=torch.float32, device=DEV)        # never read: the call must refuse first
    dn = torch.zeros((8, d), dtype=torch.float32, device=DEV)
    lib = ts.lib()
    rc = lib.ts_densify_static(ids.data_ptr(), rows.data_ptr(), n, d, V, dn.data_ptr(), dn.data_ptr(), None)
    assert rc == ts.TS_ERR_CAPACITY
