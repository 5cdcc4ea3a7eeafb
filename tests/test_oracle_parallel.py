"""Pins for the Section 7 oracle (parallel bound, work division): what the paper and arithmetic fix."""
import itertools
import math

import pytest

from oracle import lower_bound as olb
from oracle import parallel as opar

SHAPES = [(8, 64, 64, 56, 56, 3, 3, 1, 1), (32, 3, 64, 112, 112, 7, 7, 2, 2), (256, 512, 512, 7, 7, 3, 3, 1, 1),
          (8, 1024, 1024, 7, 7, 3, 3, 1, 1), (1, 3, 8, 16, 16, 3, 3, 1, 1), (4, 5, 6, 7, 8, 3, 2, 4, 1)]


@pytest.mark.parametrize("dims", SHAPES)
def test_one_block_is_theorem_1(dims):
    """a = (1,1,1,1): one processor's block is the whole problem, so the expression is Theorem 1's."""
    for M in (1000.0, 40960.0, 1e7):
        got = opar.parallel_bound(*dims, M, 1, 1, 1, 1)
        ref = olb.lower_bound(*dims, M)
        assert got.terms == ref.terms and got.bound == ref.bound and got.argmax == ref.argmax


@pytest.mark.parametrize("dims", SHAPES)
def test_bound_is_p_times_theorem_1_of_a_block(dims):
    """The paper derives the expression as p times Theorem 1 for the block B/a_B x K/a_K x W/a_W x H/a_H with
    p = a_B a_K a_W a_H.  For divisions that divide the dimensions this identity must hold term by term."""
    B, C, K, W, H, R, S, sw, sh = dims
    M = 4096.0
    for a_b, a_k, a_w, a_h in itertools.product((1, 2, 4), (1, 2), (1, 7), (1, 2, 7)):
        if B % a_b or K % a_k or W % a_w or H % a_h:
            continue
        p = a_b * a_k * a_w * a_h
        blk = olb.lower_bound(B // a_b, C, K // a_k, W // a_w, H // a_h, R, S, sw, sh, M)
        got = opar.parallel_bound(*dims, M, a_b, a_k, a_w, a_h)
        for t_par, t_blk in zip(got.terms, blk.terms):
            assert t_par == pytest.approx(p * t_blk, rel=1e-12)


def test_worked_numbers():
    """B=2 C=3 K=4 W=5 H=6 R=S=2 sigma=1 M=16, a=(2,2,1,3): terms by hand.
    T1 = 2*4*5*6 = 240; T2 = a_K * BCWH = 2*180 = 360; T3 = a_B a_W a_H * CKRS = 6*48 = 288;
    T4 = 2*3*4*5*6*4/16 = 180; T5 = 720 * sqrt(4/16) = 360.  Maximum 360, first reached by term 2."""
    got = opar.parallel_bound(2, 3, 4, 5, 6, 2, 2, 1, 1, 16.0, 2, 2, 1, 3)
    assert got.terms == [240.0, 360.0, 288.0, 180.0, 360.0]
    assert got.bound == 360.0 and got.argmax == 1


def test_terms_scale_with_the_division_as_printed():
    base = opar.parallel_bound(8, 16, 32, 14, 14, 3, 3, 1, 1, 512.0, 1, 1, 1, 1)
    got = opar.parallel_bound(8, 16, 32, 14, 14, 3, 3, 1, 1, 512.0, 2, 4, 7, 2)
    assert got.terms[0] == base.terms[0] and got.terms[3] == base.terms[3] and got.terms[4] == base.terms[4]
    assert got.terms[1] == 4 * base.terms[1]             # Image: a_K
    assert got.terms[2] == 2 * 7 * 2 * base.terms[2]     # Filter: a_B a_W a_H


def test_rejects_blocks_below_one_element_and_bad_arguments():
    with pytest.raises(ValueError):
        opar.parallel_bound(2, 3, 4, 5, 6, 2, 2, 1, 1, 16.0, 3, 1, 1, 1)
    with pytest.raises(ValueError):
        opar.parallel_bound(2, 3, 4, 5, 6, 2, 2, 1, 1, 16.0, 1, 1, 0, 1)
    with pytest.raises(ValueError):
        opar.work_division(2, 3, 4, 5, 6, 2, 2, 1, 1, 16.0, 0)


@pytest.mark.parametrize("dims", SHAPES)
def test_division_is_a_minimiser_and_never_beats_theorem_1(dims):
    B, C, K, W, H = dims[:5]
    M = 40960.0
    seq = olb.lower_bound(*dims, M).bound
    for p in (1, 2, 8, 12):
        d = opar.work_division(*dims, M, p)
        a_b, a_k, a_w, a_h = d.a
        assert a_b * a_k * a_w * a_h <= p and a_b <= B and a_k <= K and a_w <= W and a_h <= H
        assert d.bound.bound >= seq                      # replication only adds traffic
        if p == 1:
            assert d.a == (1, 1, 1, 1) and d.bound.bound == seq
        # no admissible division over as many processors does better (independent enumeration order)
        cands = [a for a in itertools.product(range(1, p + 1), repeat=4)
                 if math.prod(a) <= p and a[0] <= B and a[1] <= K and a[2] <= W and a[3] <= H]
        most = max(math.prod(a) for a in cands)
        assert a_b * a_k * a_w * a_h == most
        for a in cands:
            if math.prod(a) != most:
                continue
            other = opar.parallel_bound(*dims, M, *a)
            assert other.bound >= d.bound.bound
            if other.bound == d.bound.bound:
                assert other.terms[1] + other.terms[2] >= d.replicated_words


def test_a_dimension_of_size_one_cannot_be_split():
    d = opar.work_division(1, 4, 1, 1, 3, 1, 1, 1, 1, 64.0, 8)
    assert d.a == (1, 1, 1, 3)          # only H can be divided, and only three ways


def test_filter_heavy_layers_split_k_and_image_heavy_ones_do_not():
    """With eight processors: a layer whose Filter dwarfs its Image should give every processor its own output
    channels (Image replicated, Filter read once), a layer whose Image dwarfs its Filter should split b, w or h."""
    late = opar.work_division(8, 1024, 1024, 7, 7, 3, 3, 1, 1, 40960.0, 8)
    assert late.a[1] == 8 and late.a[0] * late.a[2] * late.a[3] == 1
    early = opar.work_division(32, 3, 64, 112, 112, 7, 7, 2, 2, 40960.0, 8)
    assert early.a[1] == 1 and early.a[0] * early.a[2] * early.a[3] == 8
