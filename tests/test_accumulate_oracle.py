"""Pins for the accumulation-rule checker (oracle/accumulate.py): the branch tables worked by
hand from Algorithms 1 and 2, the gather's size against the paper's figures, sums against
math.fsum, and the equivalence the paper's argument rests on (gather then densify == reduce)."""
import json
import math
import os

import numpy as np

import oracle
from oracle import accumulate as acc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _grads(rng, V, d, spec):
    out = []
    for kind, n in spec:
        if kind == "dense":
            out.append(("dense", rng.standard_normal((V, d)).astype(np.float32)))
        else:
            out.append(("slices", rng.integers(0, V, size=n).astype(np.int32),
                        rng.standard_normal((n, d)).astype(np.float32)))
    return out


def test_branch_tables_worked_by_hand():
    g = json.load(open(os.path.join(GOLDEN, "accumulation_rules.json")))
    for case in g["cases"]:
        assert acc.strategy(case["kinds"], acc.RULE_TF) == case["algorithm_1"], case
        assert acc.strategy(case["kinds"], acc.RULE_PROPOSED) == case["algorithm_2"], case
    # the two rules differ exactly when dense and sparse gradients are mixed
    for case in g["cases"]:
        mixed = len(case["kinds"]) >= 2 and len(set(case["kinds"])) == 2
        assert (case["algorithm_1"] != case["algorithm_2"]) == mixed


def test_gather_is_concatenation_with_the_dense_gradient_as_V_slices():
    rng = np.random.default_rng(1)
    V, d = 7, 3
    grads = _grads(rng, V, d, [("slices", 4), ("dense", 0), ("slices", 2)])
    r = acc.accumulate(grads, acc.RULE_TF, d, V)
    assert r.strategy == acc.GATHER
    assert r.ids.tolist() == grads[0][1].tolist() + list(range(V)) + grads[2][1].tolist()
    assert r.rows.shape == (4 + V + 2, d)
    assert np.array_equal(r.rows[4:4 + V], grads[1][1])
    assert np.array_equal(r.rows[:4], grads[0][2]) and np.array_equal(r.rows[4 + V:], grads[2][2])


def test_gather_size_matches_the_papers_accumulate_buffer():
    p = json.load(open(os.path.join(GOLDEN, "paper_accumulate_sizes.json")))
    d = p["d_model"]
    V = round(p["dense_MB"] * 1e6 / (4 * d))
    # one worker: encoder slices + decoder slices + the dense gradient as V slices; the ids and
    # value rows of what Algorithm 1 gathers are what buffer_bytes prices, for 64 workers
    per_worker = V + 2 * p["tokens_per_batch"]
    kinds = ["slices", "slices", "dense"]
    assert acc.strategy(kinds, acc.RULE_TF) == acc.GATHER and acc.strategy(kinds, acc.RULE_PROPOSED) == acc.DENSIFY_REDUCE
    gathered, dense = oracle.buffer_bytes(p["workers"], per_worker, d, V)
    assert abs(gathered / 1e9 - p["gathered_GB"]) / p["gathered_GB"] < 0.02
    assert abs(gathered / dense - p["ratio"]) / p["ratio"] < 0.02


def test_reduce_against_fsum_and_order_independence():
    rng = np.random.default_rng(2)
    V, d = 5, 4
    grads = _grads(rng, V, d, [("dense", 0)] * 4)
    r = acc.accumulate(grads, acc.RULE_TF, d, V)
    assert r.strategy == acc.REDUCE
    for v in range(V):
        for c in range(d):
            assert abs(r.exact[v, c] - math.fsum(float(g[1][v, c]) for g in grads)) < 1e-15
    r2 = acc.accumulate(grads[::-1], acc.RULE_PROPOSED, d, V)
    np.testing.assert_allclose(r2.exact, r.exact, rtol=0, atol=1e-15)


def test_densifying_what_algorithm_1_gathers_gives_what_algorithm_2_reduces():
    rng = np.random.default_rng(3)
    V, d = 50, 6
    grads = _grads(rng, V, d, [("slices", 200), ("slices", 120), ("dense", 0)])
    gathered = acc.accumulate(grads, acc.RULE_TF, d, V)
    reduced = acc.accumulate(grads, acc.RULE_PROPOSED, d, V)
    assert gathered.strategy == acc.GATHER and reduced.strategy == acc.DENSIFY_REDUCE
    again = oracle.densify([gathered.ids], [gathered.rows], d, V, None)
    np.testing.assert_allclose(again.exact, reduced.exact, rtol=0, atol=1e-12)
    # and it is the hot path's result: slices densified onto the dense gradient
    hot = oracle.densify([grads[0][1], grads[1][1]], [grads[0][2], grads[1][2]], d, V, grads[2][1])
    np.testing.assert_allclose(hot.exact, reduced.exact, rtol=0, atol=1e-12)


def test_pass_through_returns_the_single_gradient():
    rng = np.random.default_rng(4)
    V, d = 9, 2
    (g,) = _grads(rng, V, d, [("slices", 5)])
    r = acc.accumulate([g], acc.RULE_PROPOSED, d, V)
    assert r.strategy == acc.PASS_THROUGH and np.array_equal(r.ids, g[1]) and np.array_equal(r.rows, g[2])
    (g,) = _grads(rng, V, d, [("dense", 0)])
    r = acc.accumulate([g], acc.RULE_TF, d, V)
    assert r.strategy == acc.PASS_THROUGH and np.array_equal(r.dense, g[1])
