"""Pins for the convolution oracle (paper Section 2, Eq. (1)).  None of these re-type the oracle's own
formula: they are an independent scatter-form derivation, a library cross-correlation, library matrix
products for the 1x1 special case (Section 3), closed forms and algebraic invariants."""
import numpy as np
import pytest
from scipy.signal import correlate2d

import cacnn_inputs as ci
from oracle import conv


def _ints(shape, seed, lo=-3, hi=4):
    return np.random.default_rng(seed).integers(lo, hi, size=shape).astype(np.float32)


ASYM = conv.Problem(B=2, C=3, K=4, W=5, H=3, R=2, S=4, sigma_w=2, sigma_h=3)   # nothing is symmetric


def scatter_form(p, image, filt):
    """Independent derivation: walk over Image elements and push each one to every output it feeds.
    An Image element at first-axis position x feeds output column w through filter tap r iff
    x - r is a non-negative multiple of sigma_w with quotient < W (same for the second axis)."""
    out = np.zeros(p.out_shape)
    for x in range(p.IW):
        for y in range(p.IH):
            taps_w = [(r, (x - r) // p.sigma_w) for r in range(p.R)
                      if x - r >= 0 and (x - r) % p.sigma_w == 0 and (x - r) // p.sigma_w < p.W]
            taps_h = [(s, (y - s) // p.sigma_h) for s in range(p.S)
                      if y - s >= 0 and (y - s) % p.sigma_h == 0 and (y - s) // p.sigma_h < p.H]
            for c in range(p.C):
                for b in range(p.B):
                    v = float(image[x, y, c, b])
                    for r, w in taps_w:
                        for s, h in taps_h:
                            out[:, h, w, b] += v * filt[:, r, s, c].astype(np.float64)
    return out


def test_c_matches_python_loops_on_asymmetric_shape():
    img, flt = _ints(ASYM.image_shape, 1), _ints(ASYM.filter_shape, 2)
    o_py, a_py = conv.conv_loops(ASYM, img, flt)
    o_c, a_c = conv.conv_fp64(ASYM, img, flt)
    assert np.array_equal(o_py, o_c)
    assert np.array_equal(a_py, a_c)


@pytest.mark.parametrize("p", [ASYM, conv.Problem(1, 2, 3, 4, 6, 3, 2, 1, 2), conv.Problem(3, 1, 2, 2, 2, 5, 1, 3, 1)])
def test_scatter_form_agrees(p):
    img, flt = _ints(p.image_shape, 3), _ints(p.filter_shape, 4)
    o_c, _ = conv.conv_fp64(p, img, flt)
    assert np.array_equal(scatter_form(p, img, flt), o_c)   # integer data: exact


@pytest.mark.parametrize("sw,sh", [(1, 1), (2, 1), (1, 3), (2, 3)])
def test_single_channel_is_library_cross_correlation(sw, sh):
    """B=C=K=1: Out(h,w) = sum_rs Image(r+sw*w, s+sh*h) Filter(r,s) is the 'valid' 2-D cross-correlation of
    Image with Filter, sub-sampled by the strides, and transposed (Out is indexed (h,w), Image (w-axis,h-axis))."""
    p = conv.Problem(1, 1, 1, 6, 4, 3, 5, sw, sh)
    img, flt = _ints(p.image_shape, 5), _ints(p.filter_shape, 6)
    o_c, _ = conv.conv_fp64(p, img, flt)
    full = correlate2d(img[:, :, 0, 0].astype(np.float64), flt[0, :, :, 0].astype(np.float64), mode="valid")
    want = full[::sw, ::sh][: p.W, : p.H].T
    assert np.array_equal(o_c[0, :, :, 0], want)


def test_multi_channel_is_sum_of_library_cross_correlations():
    p = conv.Problem(2, 3, 2, 4, 5, 3, 2, 2, 1)
    img, flt = _ints(p.image_shape, 7), _ints(p.filter_shape, 8)
    o_c, _ = conv.conv_fp64(p, img, flt)
    for b in range(p.B):
        for k in range(p.K):
            acc = np.zeros((p.W, p.H))
            for c in range(p.C):
                acc += correlate2d(img[:, :, c, b].astype(np.float64), flt[k, :, :, c].astype(np.float64),
                                   mode="valid")[:: p.sigma_w, :: p.sigma_h][: p.W, : p.H]
            assert np.array_equal(o_c[k, :, :, b], acc.T)


def test_1x1_filter_single_pixel_is_matrix_multiply():
    """Section 3: with R=S=W=H=1 the nest is Out[KxB] = Filter[KxC] * Image[CxB]."""
    p = conv.Problem(B=7, C=5, K=6, W=1, H=1, R=1, S=1)
    img, flt = _ints(p.image_shape, 9), _ints(p.filter_shape, 10)
    o_c, _ = conv.conv_fp64(p, img, flt)
    want = flt.reshape(p.K, p.C).astype(np.float64) @ img.reshape(p.C, p.B).astype(np.float64)
    assert np.array_equal(o_c.reshape(p.K, p.B), want)


def test_1x1_filter_is_per_pixel_matrix_multiply_with_stride():
    p = conv.Problem(B=3, C=4, K=5, W=4, H=3, R=1, S=1, sigma_w=2, sigma_h=3)
    img, flt = _ints(p.image_shape, 11), _ints(p.filter_shape, 12)
    o_c, _ = conv.conv_fp64(p, img, flt)
    fm = flt.reshape(p.K, p.C).astype(np.float64)
    for w in range(p.W):
        for h in range(p.H):
            assert np.array_equal(o_c[:, h, w, :], fm @ img[2 * w, 3 * h].astype(np.float64))


def test_delta_filter_is_strided_crop():
    p = ASYM
    img = _ints(p.image_shape, 13)
    k0, r0, s0, c0 = 2, 1, 3, 1
    flt = np.zeros(p.filter_shape, np.float32)
    flt[k0, r0, s0, c0] = 1.0
    o_c, a_c = conv.conv_fp64(p, img, flt)
    crop = img[r0:: p.sigma_w, s0:: p.sigma_h, c0, :][: p.W, : p.H]          # [w,h,b]
    assert np.array_equal(o_c[k0], np.transpose(crop, (1, 0, 2)).astype(np.float64))
    mask = np.ones(p.K, bool)
    mask[k0] = False
    assert not o_c[mask].any()
    assert np.array_equal(a_c[k0], np.abs(o_c[k0]))


def test_all_ones_counts_the_contraction():
    p = ASYM
    o_c, a_c = conv.conv_fp64(p, np.ones(p.image_shape, np.float32), np.ones(p.filter_shape, np.float32))
    assert np.all(o_c == p.C * p.R * p.S)
    assert np.all(a_c == p.C * p.R * p.S)


def test_bilinearity_exact_on_integers():
    p = ASYM
    i1, i2 = _ints(p.image_shape, 14), _ints(p.image_shape, 15)
    f1, f2 = _ints(p.filter_shape, 16), _ints(p.filter_shape, 17)
    a = 3.0
    lhs, _ = conv.conv_fp64(p, a * i1 + i2, f1)
    assert np.array_equal(lhs, a * conv.conv_fp64(p, i1, f1)[0] + conv.conv_fp64(p, i2, f1)[0])
    lhs, _ = conv.conv_fp64(p, i1, a * f1 + f2)
    assert np.array_equal(lhs, a * conv.conv_fp64(p, i1, f1)[0] + conv.conv_fp64(p, i1, f2)[0])


def test_abs_dominates_and_matches_on_nonnegative_data():
    p = ASYM
    img, flt = _ints(p.image_shape, 18), _ints(p.filter_shape, 19)
    o, a = conv.conv_fp64(p, img, flt)
    assert np.all(a >= np.abs(o))
    o2, a2 = conv.conv_fp64(p, np.abs(img), np.abs(flt))
    assert np.array_equal(o2, a2) and np.array_equal(a2, a)


def test_sampled_outputs_match_full():
    cfg = ci.custom("t", 4, 5, 6, 7, 5, 3, 2, 2, 1, dist="normal", seed=21)
    p = conv.Problem(*cfg.dims)
    img, flt = ci.make_inputs(cfg)
    o, a = conv.conv_fp64(p, img, flt)
    rng = np.random.default_rng(0)
    coords = np.stack([rng.integers(0, n, 50) for n in p.out_shape], axis=1)
    v, va = conv.conv_fp64_at(p, img, flt, coords)
    assert np.allclose(v, o[tuple(coords.T)], rtol=0, atol=1e-14)
    assert np.allclose(va, a[tuple(coords.T)], rtol=0, atol=1e-14)


def test_thread_count_does_not_change_result():
    cfg = ci.custom("t", 3, 4, 5, 6, 5, 3, 3, dist="normal", seed=22)
    p = conv.Problem(*cfg.dims)
    img, flt = ci.make_inputs(cfg)
    assert np.array_equal(conv.conv_fp64(p, img, flt, threads=1)[0], conv.conv_fp64(p, img, flt, threads=4)[0])


def test_rejects_wrong_shapes():
    p = ASYM
    with pytest.raises(ValueError):
        conv.conv_fp64(p, np.zeros((1, 1, 1, 1), np.float32), np.zeros(p.filter_shape, np.float32))


def test_input_generator_is_deterministic_and_bf16_exact():
    cfg = ci.CONFIGS["c1"]
    a, b = ci.make_inputs(cfg)
    a2, b2 = ci.make_inputs(cfg)
    assert np.array_equal(a, a2) and np.array_equal(b, b2)
    assert a.shape == (18, 18, 3, 1) and b.shape == (8, 3, 3, 3)
    assert np.abs(a).max() <= 1.0
    x = np.array([1.0, 1.00390625, 1.01171875, -3.1415927, 1e-30], np.float32)
    r = ci.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.015625)   # ties go to even
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    assert ci.bf16_bits(r).dtype == np.uint16
