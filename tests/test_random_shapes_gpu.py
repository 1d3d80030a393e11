"""GPU parity on seeded random shapes: vocabulary size, row width, number of pairs, number of
shards, row type, id distribution, with and without the dense operand, in place or not, drawn
from ranges that cross the library's switch points.  Small-integer values, so every bit of the
result is fixed whatever the order of additions; counts, unique ids and the sorted order are
compared as everywhere else."""
import numpy as np
import pytest

from paper_1905_04035_amd import workloads as wl

from parity import check, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


def _draw(seed):
    rng = np.random.default_rng(1000 + seed)
    V = int(rng.choice([1, 2, 63, 64, 65, 700, 1023, 1025, 3000, 8191, 20000]))
    d = 4 * int(rng.choice([1, 2, 15, 16, 63, 64, 65, 128, 255, 256, 257, 513]))
    budget = 24_000_000 // d                                 # keeps the CPU checker to well under a second
    n = int(min(budget, rng.choice([0, 1, 63, 64, 65, 1000, 4097, 16384, 16385, 30000, 57344, 57345, 70000, 100000])))
    k = int(rng.integers(1, 6))
    cuts = np.sort(rng.integers(0, n + 1, size=k - 1))
    n_list = np.diff(np.concatenate([[0], cuts, [n]])).astype(int).tolist()
    ids = str(rng.choice(["zipf", "zipf", "uniform", "single", "distinct"]))
    if ids == "distinct" and n > V:
        ids = "zipf"
    return dict(V=V, d=d, n_list=n_list, ids=ids, zipf_s=float(rng.choice([0.8, 1.1, 1.5, 2.0])),
                row_dtype=int(rng.choice([wl.ROW_FP32, wl.ROW_BF16])), seed=seed), rng


@pytest.mark.parametrize("seed", range(160))
def test_random_shape(seed):
    kw, rng = _draw(seed)
    w = wl.make_custom(integer_values=True, **kw)
    if w.n_total > 0 and rng.random() < 0.3:                  # a few ids outside the vocabulary
        bad = rng.integers(0, len(w.ids[0]) + 1, size=3)
        for j, b in enumerate(bad):
            if b < len(w.ids[0]):
                w.ids[0][b] = (-1, w.V, 2**31 - 1)[j]
    dense = bool(rng.random() < 0.8)
    in_place = dense and bool(rng.random() < 0.3)
    mode = "multi" if rng.random() < 0.6 else "single"
    g = run_gpu(w, mode=mode, dense=dense, in_place=in_place)
    check(g, run_oracle(w, dense=dense), w, exact_bits=True)
