"""GPU parity at the numbers of pairs where the library changes its form: one sort launch or
slices, pieces of 16 or 32 sorted positions, short rows in the pieces or row by row (a limit that
depends on the rows' width and type), long rows by work-groups or by lone wavefronts.  One pair
below, at and above each limit, small-integer values so that every bit is fixed."""
import numpy as np
import pytest

from paper_1905_04035_amd import workloads as wl

from parity import check, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


def _case(V, d, n, dt, seed, **kw):
    w = wl.make_custom(V=V, d=d, n_list=[n - n // 3, n // 3], zipf_s=1.2, seed=seed, row_dtype=dt, integer_values=True)
    g = run_gpu(w, **kw)
    check(g, run_oracle(w), w, exact_bits=True)
    return g


@pytest.mark.parametrize("d,dt,limit", [(1024, wl.ROW_BF16, 24576), (1024, wl.ROW_FP32, 40960), (2052, wl.ROW_FP32, 20440),
                                        (4096, wl.ROW_BF16, 6144),
                                        (512, wl.ROW_FP32, 65536), (1020, wl.ROW_BF16, 65536), (256, wl.ROW_BF16, 393216),
                                        (508, wl.ROW_FP32, 393216)])
def test_around_the_limit_between_the_two_ways_of_short_rows(d, dt, limit):
    for n in (limit - 1, limit, limit + 1):
        _case(3000, d, n, dt, seed=d + n, mode="multi")


@pytest.mark.parametrize("dt", [wl.ROW_FP32, wl.ROW_BF16])
def test_around_the_limit_between_one_sort_launch_and_slices(dt):
    for n in (57343, 57344, 57345):
        g = _case(5000, 1024, n, dt, seed=n, mode="single")
        assert g["info"]["sort_slices"] == (1 if n <= 57344 else 4)


def test_around_the_limit_between_pieces_of_16_and_of_32_positions():
    for n in (96255, 96256, 96257):
        g = _case(5000, 1024, n, wl.ROW_FP32, seed=n, mode="single")
        assert g["info"]["piece_tokens"] == (16 if n <= 96256 else 32)
        g = _case(5000, 1024, n, wl.ROW_BF16, seed=n, mode="single")       # 16-byte loads of bf16 rows: always 16
        assert g["info"]["piece_tokens"] == 16
        g = _case(5000, 516, n, wl.ROW_BF16, seed=n, mode="single")        # 8-byte loads: as fp32
        assert g["info"]["piece_tokens"] == (16 if n <= 96256 else 32)


@pytest.mark.parametrize("k", [1, 2, 5])
def test_around_whole_numbers_of_slices(k):
    for n in (4 * 16384 * k - 1, 4 * 16384 * k, 4 * 16384 * k + 1):
        g = _case(9000, 256, n, wl.ROW_FP32, seed=n, mode="multi")
        assert g["info"]["sort_slices"] == (n + 16383) // 16384


@pytest.mark.parametrize("V,d,dt", [(131072, 1024, wl.ROW_FP32), (16384, 8192, wl.ROW_BF16)])
def test_a_dense_operand_of_half_a_gigabyte(V, d, dt):
    # there short rows go row by row at any number of pairs; the rows copied, all the rest checked bit for bit
    for n in (3000, 20000):
        g = _case(V, d, n, dt, seed=V + n, mode="multi")
        assert g["info"]["sort_slices"] == 1


@pytest.mark.parametrize("share", [0.5, 0.9])
def test_a_dominating_id_in_a_one_launch_sort_of_several_rounds(share):
    # half of the pairs on one id: every wavefront's list of owned pairs still holds them; nine
    # tenths: the list overflows and the wavefront walks its share a second time
    w = wl.make_custom(V=32768, d=64, n_list=[30000, 21200], zipf_s=1.1, seed=77, integer_values=True)
    rng = np.random.default_rng(78)
    for a in w.ids:
        a[rng.random(len(a)) < share] = 12345
    g = run_gpu(w, mode="multi")
    assert g["info"]["sort_slices"] == 1 and g["info"]["sort_part"] == 512
    r = run_oracle(w)
    assert int(r.count[12345]) > share * 0.9 * w.n_total
    check(g, r, w, exact_bits=True)
