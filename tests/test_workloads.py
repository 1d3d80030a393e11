"""The synthetic input recipe: seeded, bounded Zipf, shapes of the five configurations."""
import numpy as np

from paper_1905_04035_amd import workloads as wl


def test_same_seed_same_inputs():
    a, b = wl.make("tiny"), wl.make("tiny")
    assert all(np.array_equal(x, y) for x, y in zip(a.ids, b.ids))
    assert all(np.array_equal(x, y) for x, y in zip(a.rows, b.rows))
    assert np.array_equal(a.dense_in, b.dense_in)
    c = wl.make("tiny", seed=1)
    assert not np.array_equal(a.ids[0], c.ids[0])


def test_shapes_of_the_named_configurations():
    for name, n, V, d in [("tiny", 2048, 1000, 64), ("transformer_base", 8192, 32768, 512),
                          ("transformer_big", 16384, 32768, 1024)]:
        w = wl.make(name, with_dense=(name == "tiny"))
        assert (w.n_total, w.V, w.d) == (n, V, d)
        assert all(i.dtype == np.int32 and i.min() >= 0 and i.max() < V for i in w.ids)
        assert all(r.dtype == np.float32 and r.shape == (len(i), d) for i, r in zip(w.ids, w.rows))
    s = wl.SPECS["large_batch_bf16"]
    assert (s.contributions * s.rows_per_contribution, s.row_dtype) == (131072, wl.ROW_BF16)
    s = wl.SPECS["multi_shard_stress"]
    assert s.contributions * s.rows_per_contribution == 16 * 2 * 8192 and s.zipf_s == 1.5


def test_zipf_is_bounded_and_skewed_as_expected():
    w = wl.make("transformer_big", with_dense=False)
    ids, _ = w.concatenated()
    cnt = np.bincount(ids, minlength=w.V)
    p = np.arange(1, w.V + 1, dtype=np.float64) ** -1.1
    p /= p.sum()
    # hottest row: analytic share p(1) ~ 14 %; unique ids ~ sum(1 - (1-p)^n)
    assert abs(cnt.max() / len(ids) - p[0]) < 0.02
    expect_unique = np.sum(1.0 - (1.0 - p) ** len(ids))
    assert abs((cnt > 0).sum() - expect_unique) / expect_unique < 0.05
    # the encoder and the decoder contribution share the hot tokens
    assert np.bincount(w.ids[0], minlength=w.V).argmax() == np.bincount(w.ids[1], minlength=w.V).argmax()


def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], dtype=np.float32)   # 1+2^-8 ties to even
    b = wl.fp32_to_bf16_bits(x)
    y = wl.bf16_bits_to_fp32(b)
    assert y.tolist() == [1.0, 1.0, 1.015625, -2.5, 0.0]
    w = wl.make_custom(V=50, d=8, n_list=[10], row_dtype=wl.ROW_BF16)
    assert w.rows[0].dtype == np.uint16


def test_grouping_into_shards():
    w = wl.make_custom(V=50, d=4, n_list=[3, 5, 2, 7])
    ids, rows = w.grouped(2)
    assert [len(i) for i in ids] == [8, 9] and rows[1].shape == (9, 4)
    ci, cr = w.concatenated()
    assert np.array_equal(np.concatenate(ids), ci) and np.array_equal(np.concatenate(rows), cr)
