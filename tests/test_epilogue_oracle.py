"""Pins for the CPU checker's finish step with a write-back epilogue
(out = cast(scale * sum), fp32 or bf16): hand-worked values, a library conversion,
the defining property of round-to-nearest, exact power-of-two scaling, the average of
equal contributions, linearity."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import reference as R
from paper_1905_04035_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16_value(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_hand_worked_average_in_fp32_and_bf16():
    with open(os.path.join(GOLDEN, "worked_case_average_bf16.json")) as f:
        g = json.load(f)
    V, d = g["V"], g["d"]
    ids = np.array(g["ids"], dtype=np.int32)
    rows = np.array(g["rows"], dtype=np.float32)
    dense = np.array(g["dense_in"], dtype=np.float32)
    want32 = np.array([[int(x, 16) for x in r] for r in g["expected_out_fp32_hex"]], dtype=np.uint32)
    want16 = np.array([[int(x, 16) for x in r] for r in g["expected_out_bf16_hex"]], dtype=np.uint16)
    r32 = oracle.densify([ids], [rows], d, V, dense, scale=g["scale"], out_dtype=R.OUT_FP32)
    assert np.array_equal(r32.out.view(np.uint32), want32)
    assert r32.count.tolist() == g["expected_count"]
    r16 = oracle.densify([ids], [rows], d, V, dense, scale=g["scale"], out_dtype=R.OUT_BF16)
    assert r16.out.dtype == np.uint16 and np.array_equal(r16.out, want16)


def test_bf16_rounding_matches_the_library_conversion_of_fp32_values():
    rng = np.random.default_rng(5)
    f = rng.standard_normal(400000).astype(np.float32)
    f *= np.float32(10.0) ** rng.integers(-44, 38, f.size).astype(np.float32)     # subnormals to near overflow
    special = np.array([0.0, -0.0, np.inf, -np.inf, 3.3895314e38, 3.4e38, -3.4e38, 1e-45, 2 ** -126, 2 ** -133,
                        2 ** -134, 1.5 * 2 ** -133], dtype=np.float32)
    f = np.concatenate([f, special])
    lib = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(R.bf16_round(f.astype(np.float64)), lib)


def test_bf16_rounding_hand_cases_ties_and_one_step_rounding():
    x = np.array([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -40, 1 + 2.0 ** -8 - 2.0 ** -40,
                  -(1 + 2.0 ** -7), 255.5, 2.0 ** 128, float("nan")])
    got = R.bf16_round(x).tolist()
    # 1 + 2^-8 + 2^-40 is above the halfway point: one rounding step goes up, although
    # rounding to fp32 first would land on the tie and then go down to the even neighbour
    assert got == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0x3F80, 0xBF81, 0x4380, 0x7F80, 0x7FC0]


def test_bf16_output_is_the_nearest_bf16_value_of_the_exact_result():
    w = wl.make("tiny")
    r = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in, scale=1.0 / 3.0, out_dtype=R.OUT_BF16)
    touched = r.count > 0
    assert touched.any() and (~touched).any()
    bits = r.out[touched].astype(np.int32)
    e = r.exact[touched]
    err = np.abs(bf16_value(bits) - e)
    # no neighbouring bit pattern is nearer (patterns of one sign are ordered like their magnitudes)
    for nb in (bits - 1, bits + 1):
        ok = ((nb & 0x7FFF) <= 0x7F80) & ((nb & 0x8000) == (bits & 0x8000))
        other = np.abs(bf16_value(np.where(ok, nb, bits).astype(np.uint16)) - e)
        assert (err <= other).all()
    assert (err <= np.abs(e) * 2.0 ** -8).all()
    # untouched rows: the fp32 product, then the library's fp32 -> bf16 conversion
    y = np.float32(1.0 / 3.0) * w.dense_in[~touched]
    lib = torch.from_numpy(y).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(r.out[~touched], lib)


@pytest.mark.parametrize("k", [-3, 1, 6])
def test_power_of_two_scale_is_exact(k):
    w = wl.make("tiny")
    plain = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    scaled = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in, scale=2.0 ** k)
    assert np.array_equal(scaled.out.view(np.uint32), (plain.out * np.float32(2.0 ** k)).view(np.uint32))
    assert np.array_equal(scaled.exact, plain.exact * 2.0 ** k)
    assert np.array_equal(scaled.abs_sum, plain.abs_sum * 2.0 ** k)
    assert np.array_equal(scaled.count, plain.count)


def test_average_of_equal_contributions_is_the_contribution():
    rng = np.random.default_rng(11)
    V, d, n, k = 50, 8, 20, 4
    ids = rng.permutation(V)[:n].astype(np.int32)
    rows = rng.standard_normal((n, d)).astype(np.float32)
    r = oracle.densify([ids] * k, [rows] * k, d, V, None, scale=1.0 / k)
    want = np.zeros((V, d), dtype=np.float32)
    want[ids] = rows
    assert np.array_equal(r.out.view(np.uint32), want.view(np.uint32))
    assert r.count.sum() == k * n


def test_scale_one_is_the_plain_finish_bit_for_bit():
    w = wl.make("tiny")
    dense = w.dense_in.copy()
    untouched = np.flatnonzero(np.bincount(np.concatenate(w.ids), minlength=w.V) == 0)
    dense.view(np.uint32)[untouched[0], 0] = 0x7FA12345      # a signalling NaN with a payload
    dense.view(np.uint32)[untouched[0], 1] = 0x80000000      # -0.0
    plain = oracle.densify(w.ids, w.rows, w.d, w.V, dense)
    one = oracle.densify(w.ids, w.rows, w.d, w.V, dense, scale=1.0)
    assert np.array_equal(one.out.view(np.uint32), plain.out.view(np.uint32))


def test_any_scale_is_linear_and_untouched_rows_are_fp32_products():
    w = wl.make("tiny")
    s = np.float32(0.3)
    plain = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in)
    scaled = oracle.densify(w.ids, w.rows, w.d, w.V, w.dense_in, scale=float(s))
    np.testing.assert_allclose(scaled.exact, plain.exact * float(s), rtol=1e-15, atol=0)
    untouched = plain.count == 0
    assert np.array_equal(scaled.out[untouched].view(np.uint32), (s * w.dense_in[untouched]).view(np.uint32))
    t = ~untouched
    assert np.array_equal(scaled.out[t], (plain.exact[t] * float(s)).astype(np.float32))
    # without a dense operand untouched rows are zeros
    z = oracle.densify(w.ids, w.rows, w.d, w.V, None, scale=float(s), out_dtype=R.OUT_BF16)
    assert (z.out[untouched] == 0).all()
