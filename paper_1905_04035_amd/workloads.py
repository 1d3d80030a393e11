"""Seeded synthetic inputs for the densify path.

This module only *draws* inputs: token ids, value rows and the dense projection
gradient.  It holds none of the method's arithmetic (no counting, no summing),
so both the GPU path's tests and the CPU checker's tests may feed from it.

The paper trains on sub-word batches of a translation corpus (Section 5); the
corpus is not available here, so token ids are drawn from a bounded Zipf law
over the vocabulary with a random rank -> id permutation, which reproduces the
property that matters for this path: a few very hot rows and a long tail of
rows that are hit once or never.  Value rows and the dense gradient are
independent normal draws.

Every workload is a list of *contributions* (the encoder and the decoder
embedding-lookup gradients of one worker; several workers' pairs for the
gathered case), each an `(ids int32[n_j], rows[n_j, d])` pair, plus one dense
`[V, d]` fp32 gradient of the shared projection weight (Section 3).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

SEED_BASE = 190504035

ROW_FP32 = 0
ROW_BF16 = 1


@dataclass(frozen=True)
class Spec:
    name: str
    index: int              # position in the list of benchmark configurations
    V: int
    d: int
    contributions: int      # number of (ids, rows) pairs
    rows_per_contribution: int
    ids: str                # "uniform" or "zipf"
    zipf_s: float = 0.0
    sigma_rows: float = 1.0
    sigma_dense: float = 1.0
    row_dtype: int = ROW_FP32


SPECS = {
    s.name: s
    for s in [
        Spec("tiny", 0, V=1000, d=64, contributions=1, rows_per_contribution=2048,
             ids="uniform", sigma_rows=1.0, sigma_dense=1.0),
        Spec("transformer_base", 1, V=32768, d=512, contributions=2, rows_per_contribution=4096,
             ids="zipf", zipf_s=1.1, sigma_rows=0.01, sigma_dense=0.01),
        Spec("transformer_big", 2, V=32768, d=1024, contributions=2, rows_per_contribution=8192,
             ids="zipf", zipf_s=1.1, sigma_rows=0.01, sigma_dense=0.01),
        Spec("large_batch_bf16", 3, V=32768, d=1024, contributions=2, rows_per_contribution=65536,
             ids="zipf", zipf_s=1.1, sigma_rows=0.01, sigma_dense=0.01, row_dtype=ROW_BF16),
        Spec("multi_shard_stress", 4, V=32768, d=1024, contributions=32, rows_per_contribution=8192,
             ids="zipf", zipf_s=1.5, sigma_rows=0.01, sigma_dense=0.01),
    ]
}


@dataclass
class Workload:
    spec: Spec
    ids: List[np.ndarray]            # int32 [n_j]
    rows: List[np.ndarray]           # float32 [n_j, d]  or  uint16 [n_j, d] (bf16 bit patterns)
    dense_in: Optional[np.ndarray]   # float32 [V, d]
    seed: int = 0

    @property
    def V(self) -> int:
        return self.spec.V

    @property
    def d(self) -> int:
        return self.spec.d

    @property
    def row_dtype(self) -> int:
        return self.spec.row_dtype

    @property
    def n_total(self) -> int:
        return int(sum(len(i) for i in self.ids))

    def concatenated(self):
        """All contributions laid end to end, in contribution order."""
        return np.concatenate(self.ids), np.concatenate(self.rows, axis=0)

    def grouped(self, per_group: int):
        """Contributions merged `per_group` at a time (a worker's encoder and
        decoder pair laid end to end is one shard of a gathered buffer)."""
        ids, rows = [], []
        for a in range(0, len(self.ids), per_group):
            ids.append(np.concatenate(self.ids[a:a + per_group]))
            rows.append(np.concatenate(self.rows[a:a + per_group], axis=0))
        return ids, rows


def fp32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even narrowing of fp32 to bf16, returned as uint16 bit
    patterns.  Inputs here are finite normal draws, so NaN handling is not needed."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_fp32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32 (for building test inputs)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def zipf_ids(rng: np.random.Generator, n: int, V: int, s: float, rank_to_id: np.ndarray) -> np.ndarray:
    """n draws from p(r) ~ r^-s, r = 1..V (bounded support, inverse-CDF
    sampling), mapped through a rank -> id permutation."""
    p = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(p)
    cdf /= cdf[-1]
    u = rng.random(n)
    r = np.searchsorted(cdf, u, side="left")
    r = np.minimum(r, V - 1)
    return rank_to_id[r].astype(np.int32)


def make(name: str, *, scale_rows: float = 1.0, seed: Optional[int] = None,
         with_dense: bool = True) -> Workload:
    """Build one of the named workloads.  `scale_rows` shrinks (or grows) the
    number of rows per contribution, keeping everything else."""
    spec = SPECS[name]
    seed = SEED_BASE + spec.index if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))
    n_j = max(0, int(round(spec.rows_per_contribution * scale_rows)))
    rank_to_id = rng.permutation(spec.V)
    dense = None
    if with_dense:
        dense = (rng.standard_normal((spec.V, spec.d), dtype=np.float32) * np.float32(spec.sigma_dense))
    ids, rows = [], []
    for _ in range(spec.contributions):
        if spec.ids == "uniform":
            i = rng.integers(0, spec.V, size=n_j, dtype=np.int32)
        else:
            i = zipf_ids(rng, n_j, spec.V, spec.zipf_s, rank_to_id)
        r = rng.standard_normal((n_j, spec.d), dtype=np.float32) * np.float32(spec.sigma_rows)
        if spec.row_dtype == ROW_BF16:
            r = fp32_to_bf16_bits(r)
        ids.append(i)
        rows.append(r)
    return Workload(spec=spec, ids=ids, rows=rows, dense_in=dense, seed=seed)


def make_custom(V: int, d: int, n_list, *, ids: str = "zipf", zipf_s: float = 1.1, seed: int = 1,
                sigma_rows: float = 1.0, sigma_dense: float = 1.0, row_dtype: int = ROW_FP32,
                with_dense: bool = True, integer_values: bool = False) -> Workload:
    """Free-form workload for edge-case tests: any V, d and ragged row counts.

    `integer_values` draws rows and the dense gradient from the integers
    -4..4, so every partial sum is exactly representable and any summation
    order gives the same bits."""
    spec = Spec("custom", -1, V=V, d=d, contributions=len(n_list), rows_per_contribution=0,
                ids=ids, zipf_s=zipf_s, sigma_rows=sigma_rows, sigma_dense=sigma_dense,
                row_dtype=row_dtype)
    rng = np.random.Generator(np.random.PCG64(seed))
    rank_to_id = rng.permutation(V)

    def values(shape, sigma):
        if integer_values:
            return rng.integers(-4, 5, size=shape).astype(np.float32)
        return rng.standard_normal(shape, dtype=np.float32) * np.float32(sigma)

    dense = values((V, d), sigma_dense) if with_dense else None
    ids_l, rows_l = [], []
    for n_j in n_list:
        if ids == "uniform":
            i = rng.integers(0, V, size=n_j, dtype=np.int32)
        elif ids == "distinct":
            i = rng.permutation(V)[:n_j].astype(np.int32)
        elif ids == "single":
            i = np.full(n_j, int(rank_to_id[0]), dtype=np.int32)
        else:
            i = zipf_ids(rng, n_j, V, zipf_s, rank_to_id)
        r = values((n_j, d), sigma_rows)
        if row_dtype == ROW_BF16:
            r = fp32_to_bf16_bits(r)
        ids_l.append(i)
        rows_l.append(r)
    return Workload(spec=spec, ids=ids_l, rows=rows_l, dense_in=dense, seed=seed)
