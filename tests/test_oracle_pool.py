"""Pins for the pooling oracle (Section 6 of the paper): checked against the convolution oracle, against the loop nest
written out, and against special cases whose answer is known without computing anything."""
import numpy as np
import pytest

from oracle import conv as oconv
from oracle import pool as opool
from oracle import lower_bound as olb


def small_int_image(p, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(-4, 5, size=p.image_shape).astype(np.float64)


SHAPES = [
    oconv.Problem(3, 4, 4, 5, 4, 3, 2, 1, 1),
    oconv.Problem(2, 3, 3, 4, 3, 3, 3, 2, 2),
    oconv.Problem(1, 2, 2, 3, 5, 2, 4, 3, 1),   # stride larger than the window in w
]


@pytest.mark.parametrize("p", SHAPES)
def test_average_pooling_is_a_convolution_with_a_diagonal_filter(p):
    """R*S * avgpool = conv with Filter[k][r][s][c] = [k == c]: integers, so both sides are exact."""
    img = small_int_image(p, 1)
    flt = np.zeros(p.filter_shape)
    for k in range(p.K):
        flt[k, :, :, k] = 1.0
    conv, _ = oconv.conv_fp64(p, img, flt)
    assert np.array_equal(opool.pool_fp64(p, img, "avg") * (p.R * p.S), conv)


@pytest.mark.parametrize("p", SHAPES)
@pytest.mark.parametrize("mode", opool.MODES)
def test_vectorised_oracle_equals_the_loop_nest(p, mode):
    img = small_int_image(p, 2)
    assert np.array_equal(opool.pool_fp64(p, img, mode), opool.pool_loops(p, img, mode))


@pytest.mark.parametrize("mode", opool.MODES)
def test_one_by_one_window_is_the_transposed_image(mode):
    """R = S = 1, unit strides: Out[c][h][w][b] = Image[w][h][c][b] (W != H so a swapped axis pair cannot pass)."""
    p = oconv.Problem(2, 3, 3, 5, 4, 1, 1, 1, 1)
    img = small_int_image(p, 3)
    assert np.array_equal(opool.pool_fp64(p, img, mode), img.transpose(2, 1, 0, 3))


def test_max_of_an_increasing_image_is_the_far_corner_of_the_window():
    p = oconv.Problem(1, 2, 2, 4, 3, 3, 2, 2, 1)
    x = np.arange(p.IW)[:, None, None, None]
    y = np.arange(p.IH)[None, :, None, None]
    c = np.arange(p.C)[None, None, :, None]
    img = (100.0 * x + y + 1000.0 * c) * np.ones(p.image_shape)
    out = opool.pool_fp64(p, img, "max")
    for k in range(p.K):
        for h in range(p.H):
            for w in range(p.W):
                assert out[k, h, w, 0] == 100.0 * (p.sigma_w * w + p.R - 1) + (p.sigma_h * h + p.S - 1) + 1000.0 * k


@pytest.mark.parametrize("mode", opool.MODES)
def test_constant_image_pools_to_the_constant(mode):
    p = oconv.Problem(2, 2, 2, 3, 3, 3, 3, 2, 2)
    assert np.array_equal(opool.pool_fp64(p, np.full(p.image_shape, 2.5), mode), np.full(p.out_shape, 2.5))


def test_max_is_not_below_average_and_both_are_within_the_window_range():
    p = oconv.Problem(2, 3, 3, 4, 4, 3, 3, 1, 1)
    img = small_int_image(p, 4)
    mx, av = opool.pool_fp64(p, img, "max"), opool.pool_fp64(p, img, "avg")
    assert np.all(mx >= av) and np.all(mx <= img.max()) and np.all(av >= img.min())


def test_k_must_equal_c():
    p = oconv.Problem(1, 2, 3, 2, 2, 2, 2, 1, 1)
    with pytest.raises(ValueError):
        opool.pool_fp64(p, np.zeros(p.image_shape), "avg")


def test_pooling_bound_has_the_three_printed_terms():
    """Section 6: max(BKWH, sw*sh*BCWH, BCKWHRS/M); the third term takes over exactly when C*R*S > M (vs the first)."""
    b = olb.pooling_lower_bound(4, 8, 8, 10, 10, 3, 3, 2, 2, 64.0)
    assert b.terms == [4 * 8 * 10 * 10, 4 * 4 * 8 * 10 * 10, 4 * 8 * 8 * 10 * 10 * 9 / 64.0]
    assert b.bound == max(b.terms)
    assert olb.pooling_lower_bound(4, 8, 8, 10, 10, 3, 3, 1, 1, 8 * 9 - 1.0).argmax == 2
    assert olb.pooling_lower_bound(4, 8, 8, 10, 10, 3, 3, 1, 1, 8 * 9 + 1.0).argmax == 0
