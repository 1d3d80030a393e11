"""CPU checker for the two accumulation rules of the paper.  TEST INFRASTRUCTURE ONLY.

Algorithm 1 (Section 3) is TensorFlow's rule: fewer than two gradients pass through; if every
gradient is a dense tensor they are summed (reduce); otherwise every gradient is turned into
indexed slices and the slices are concatenated (gather).  A dense [V, d] tensor turned into
slices is V slices, one per row, with ids 0 .. V-1 (Section 3: the dense projection gradient is
converted to slices as well, although it holds a value for every row).

Algorithm 2 (Section 6) adds one branch before the gather: if at least one gradient is a dense
tensor, every gradient is converted to a dense tensor and the dense tensors are summed.

Each gradient is ("dense", array[V, d]) or ("slices", ids[n], rows[n, d]).  Everything here is
written out from those two statements with numpy: concatenation is numpy.concatenate, sums are
float64.  The conversion of slices to dense is the plain-C checker in densify_oracle.c.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import reference

RULE_TF = 1          # Algorithm 1
RULE_PROPOSED = 2    # Algorithm 2

PASS_THROUGH = 0
REDUCE = 1
DENSIFY_REDUCE = 2
GATHER = 3


def strategy(kinds: Sequence[str], rule: int) -> int:
    """Which branch the rule takes for gradients of these kinds, in the paper's order of tests."""
    if len(kinds) < 2:
        return PASS_THROUGH
    if all(k == "dense" for k in kinds):
        return REDUCE
    if rule == RULE_PROPOSED and any(k == "dense" for k in kinds):
        return DENSIFY_REDUCE
    return GATHER


@dataclass
class AccumulateResult:
    strategy: int
    dense: Optional[np.ndarray] = None        # float32 [V, d] (float64 sum rounded once)
    exact: Optional[np.ndarray] = None        # float64 [V, d]
    abs_sum: Optional[np.ndarray] = None      # float64 [V, d] sum of |terms|
    ids: Optional[np.ndarray] = None          # int32 [total]   (gather / pass-through of slices)
    rows: Optional[np.ndarray] = None         # float32 [total, d]


def as_slices(grad, V: int) -> Tuple[np.ndarray, np.ndarray]:
    if grad[0] == "dense":
        return np.arange(V, dtype=np.int32), np.asarray(grad[1], dtype=np.float32)
    return np.asarray(grad[1], dtype=np.int32), np.asarray(grad[2], dtype=np.float32)


def accumulate(grads: List[tuple], rule: int, d: int, V: int) -> AccumulateResult:
    kinds = [g[0] for g in grads]
    st = strategy(kinds, rule)
    if st == PASS_THROUGH:
        g = grads[0]
        if g[0] == "dense":
            a = np.asarray(g[1], dtype=np.float32)
            return AccumulateResult(st, dense=a.copy(), exact=a.astype(np.float64),
                                    abs_sum=np.abs(a.astype(np.float64)))
        return AccumulateResult(st, ids=np.asarray(g[1], dtype=np.int32).copy(),
                                rows=np.asarray(g[2], dtype=np.float32).copy())
    if st == REDUCE:
        exact = np.zeros((V, d), dtype=np.float64)
        abs_sum = np.zeros((V, d), dtype=np.float64)
        for g in grads:
            exact += np.asarray(g[1], dtype=np.float64)
            abs_sum += np.abs(np.asarray(g[1], dtype=np.float64))
        return AccumulateResult(st, dense=exact.astype(np.float32), exact=exact, abs_sum=abs_sum)
    if st == DENSIFY_REDUCE:
        # convert every gradient to a dense tensor, then sum the dense tensors: in float64 the
        # sum of the converted slices and of the dense tensors is one scatter-add over all of
        # them, the dense ones taken as V slices each
        ids_k, rows_k = zip(*[as_slices(g, V) for g in grads])
        r = reference.densify(list(ids_k), list(rows_k), d, V, None)
        return AccumulateResult(st, dense=r.out, exact=r.exact, abs_sum=r.abs_sum)
    ids_k, rows_k = zip(*[as_slices(g, V) for g in grads])
    return AccumulateResult(st, ids=np.concatenate(ids_k), rows=np.concatenate(rows_k, axis=0))
