"""Pins for the lower-bound oracle (Theorem 1) and the tiling-LP oracle (Section 5, Appendix A):
the values the paper prints for its AlexNet example, the matmul special case of Section 3, the
term-4/term-5 crossover stated after Theorem 1, the optimality statement of Section 5.2 (LP cost = max of
the five terms whenever that is at least M) and the per-case tile volumes of Appendix A."""
import math
import os

import numpy as np
import pytest

from oracle import lower_bound as lb
from oracle import lp_tiling as lp

FIVE = {
    "c1": (1, 3, 8, 16, 16, 3, 3, 1, 1),
    "c2": (8, 64, 64, 56, 56, 3, 3, 1, 1),
    "c3": (32, 3, 64, 112, 112, 7, 7, 2, 2),
    "c4": (64, 256, 256, 14, 14, 3, 3, 1, 1),
    "c5": (256, 512, 512, 7, 7, 3, 3, 1, 1),
}


def read_golden(path):
    vals = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split()
            vals[k] = float(v)
    return vals


@pytest.fixture(scope="module")
def alex(golden_dir):
    g = read_golden(os.path.join(golden_dir, "alexnet_conv1_bound.txt"))
    dims = tuple(int(g[k]) for k in ("B", "C", "K", "W", "H", "R", "S", "sigma_w", "sigma_h"))
    return g, dims


def test_alexnet_term5_tight_up_to_17k_words(alex):
    g, dims = alex
    M = g["term5_tight_up_to_words"]
    b = lb.lower_bound(*dims, M)
    assert b.terms[4] == pytest.approx(b.terms[0], rel=1e-12)        # crossover with the Out-size term
    assert b.terms[0] == 1000 * 96 * 55 * 55 == 290400000
    below = lb.lower_bound(*dims, M / 2)
    above = lb.lower_bound(*dims, M * 2)
    assert below.argmax == 4 and above.argmax == 0                   # tight below, not above


def test_alexnet_matmul_reuse_needs_11_over_4_more(alex):
    g, dims = alex
    for M in (256.0, 1024.0, 4096.0):
        b = lb.lower_bound(*dims, M)
        ratio = lb.matmul_reuse_cost(*dims[:7], M) / b.terms[4]
        assert ratio == pytest.approx(g["matmul_over_term5"], rel=1e-12)


def test_alexnet_lp_volume_and_printed_tiling(alex):
    g, dims = alex
    M = g["M_tiling"]
    r = lp.solve_lp(*dims, M)
    B, C, K, W, H, R, S, sw, sh = dims
    G_closed = M ** 1.5 * math.sqrt(R * S / (sw * sh))               # Lemma of Section 4.3
    assert G_closed == pytest.approx(90112.0)
    assert r.volume == pytest.approx(G_closed, rel=1e-6)
    assert r.cost == pytest.approx(lb.lower_bound(*dims, M).terms[4], rel=1e-6)
    # the tiling printed in the caption is feasible for the LP and has the same volume
    t = {k: g[k] for k in ("b_b", "b_c", "b_k", "b_w", "b_h", "b_r1", "b_r2", "b_s1", "b_s2")}
    vol = np.prod(list(t.values()))
    assert vol == pytest.approx(G_closed, rel=1e-5)
    assert t["b_b"] * t["b_k"] * t["b_w"] * t["b_h"] <= M * (1 + 1e-6)
    assert t["b_c"] * t["b_k"] * t["b_r1"] * t["b_r2"] * t["b_s1"] * t["b_s2"] <= M * (1 + 1e-6)
    for a in ("b_w", "b_r1"):
        for bb in ("b_h", "b_s1"):
            assert t["b_b"] * t["b_c"] * t[a] * t[bb] * t["b_r2"] * t["b_s2"] <= M * (1 + 1e-6)
    assert sw * t["b_r1"] <= R and sh * t["b_s1"] <= S and t["b_r2"] <= sw and t["b_s2"] <= sh


def test_matmul_special_case():
    """R=S=W=H=1, strides 1: the five terms are BK, BC, CK, BCK/M, BCK/sqrt(M) -- Section 3's
    max(n^2, n^2 k / sqrt(M)) for n x n times n x k."""
    n, k, M = 512, 64, 1024.0
    b = lb.lower_bound(k, n, n, 1, 1, 1, 1, 1, 1, M)
    assert b.terms[:3] == [k * n, k * n, n * n]
    assert b.terms[4] == pytest.approx(n * n * k / math.sqrt(M))
    assert b.bound == pytest.approx(max(n * n, n * n * k / math.sqrt(M)))


def test_term5_exceeds_term4_iff_small_filter():
    rng = np.random.default_rng(3)
    for _ in range(300):
        B, C, K, W, H = (int(x) for x in rng.integers(1, 50, 5))
        sw, sh = (int(x) for x in rng.integers(1, 4, 2))
        R, S = int(rng.integers(sw, 40)), int(rng.integers(sh, 40))
        M = float(rng.integers(2, 2000))
        b = lb.lower_bound(B, C, K, W, H, R, S, sw, sh, M)
        if R * S == M * sw * sh:
            continue
        assert (b.terms[4] > b.terms[3]) == (R * S < M * sw * sh)


def test_gain_over_matmul_reuse_is_min_sqrtM_sqrt_rs_over_sigma():
    """Section 1: against F/sqrt(M) the bound's M-dependent part max(T4,T5) is smaller by
    min(sqrt(M), sqrt(RS/(sigma sigma)))."""
    for dims, M in (((4, 8, 8, 10, 10, 3, 3, 1, 1), 64.0), ((4, 8, 8, 10, 10, 9, 9, 1, 1), 16.0),
                    ((4, 8, 8, 10, 10, 8, 8, 2, 2), 4.0)):
        b = lb.lower_bound(*dims, M)
        R, S, sw, sh = dims[5:]
        gain = lb.matmul_reuse_cost(*dims[:7], M) / max(b.terms[3], b.terms[4])
        assert gain == pytest.approx(min(math.sqrt(M), math.sqrt(R * S / (sw * sh))))


def test_clamps_stride_larger_than_filter():
    a = lb.lower_bound(2, 3, 4, 5, 6, 1, 2, 3, 5, 100.0)
    b = lb.lower_bound(2, 3, 4, 5, 6, 1, 2, 1, 2, 100.0)
    assert a.terms == b.terms


def test_rejects_bad_parameters():
    with pytest.raises(ValueError):
        lb.lower_bound(0, 1, 1, 1, 1, 1, 1, 1, 1, 10.0)
    with pytest.raises(ValueError):
        lb.lower_bound(1, 1, 1, 1, 1, 1, 1, 1, 1, 0.0)


@pytest.mark.parametrize("name", list(FIVE))
@pytest.mark.parametrize("M", [40960.0, 81920.0, 172032.0])
def test_lp_cost_equals_bound_on_benchmark_shapes(name, M):
    dims = FIVE[name]
    b = lb.lower_bound(*dims, M)
    r = lp.solve_lp(*dims, M)
    if b.bound >= M:
        assert r.cost == pytest.approx(b.bound, rel=1e-6)
    else:
        assert r.cost >= b.bound * (1 - 1e-9)      # everything fits: the formula charges M per round


def test_lp_cost_never_below_any_term_and_attains_max_when_bound_at_least_M():
    rng = np.random.default_rng(11)
    checked = 0
    for _ in range(400):
        sw, sh = (int(x) for x in rng.integers(1, 4, 2))
        R, S = int(rng.integers(sw, 12)), int(rng.integers(sh, 12))
        W = int(rng.integers(max(1, -(-R // sw)), 40))
        H = int(rng.integers(max(1, -(-S // sh)), 40))
        B, C, K = (int(x) for x in rng.integers(1, 300, 3))
        M = float(2 ** rng.integers(4, 16))
        b = lb.lower_bound(B, C, K, W, H, R, S, sw, sh, M)
        r = lp.solve_lp(B, C, K, W, H, R, S, sw, sh, M)
        assert r.cost >= b.bound * (1 - 1e-7)
        if b.bound >= M:
            assert r.cost == pytest.approx(b.bound, rel=1e-6)
            checked += 1
    assert checked > 100


def test_lp_tiles_are_feasible():
    dims, M = FIVE["c4"], 40960.0
    t = lp.solve_lp(*dims, M).tiles
    B, C, K, W, H, R, S, sw, sh = dims
    eps = 1 + 1e-7
    assert t["b"] * t["k"] * t["w"] * t["h"] <= M * eps
    assert t["c"] * t["k"] * t["r1"] * t["r2"] * t["s1"] * t["s2"] <= M * eps
    assert t["b"] * t["c"] * t["w"] * t["h"] * t["r2"] * t["s2"] <= M * eps
    for nm, hi in (("b", B), ("c", C), ("k", K), ("w", W), ("h", H), ("r2", sw), ("s2", sh)):
        assert 1 - 1e-9 <= t[nm] <= hi * eps


@pytest.mark.parametrize("name,case", [("c1", "1.1"), ("c2", "1.6"), ("c4", "2.2.2.1"), ("c5", "2.2.2.1")])
def test_appendix_a_case_of_benchmark_shapes(name, case):
    dims = FIVE[name]
    M = 40960.0
    label, alb, G = lp.appendix_a_case(*dims[:7], M)
    assert label == case
    b = lb.lower_bound(*dims, M)
    assert alb == pytest.approx(b.bound, rel=1e-12)           # Theorem 2: the attainable bound is Theorem 1's max
    if case != "1.1":
        F = np.prod([float(x) for x in dims[:7]])
        assert F * M / G == pytest.approx(alb, rel=1e-12)
        assert lp.solve_lp_sigma1(*dims[:7], M).volume == pytest.approx(G, rel=1e-6)
        assert lp.solve_lp(*dims, M).volume == pytest.approx(G, rel=1e-6)


def test_appendix_a_other_leaves():
    # 2.1: huge filter RS >= M: G = M^2, cost F/M
    dims = (4, 4, 4, 64, 64, 32, 32)
    M = 512.0
    label, alb, G = lp.appendix_a_case(*dims, M)
    assert label == "2.1" and G == M * M
    assert lp.solve_lp_sigma1(*dims, M).volume == pytest.approx(G, rel=1e-6)
    assert alb == pytest.approx(lb.lower_bound(*dims, 1, 1, M).bound)
    # 2.2.1: M*RS >= (BHW)^2 with nothing fitting: cost KCRS
    dims = (1, 512, 512, 8, 8, 3, 3)
    M = 1024.0
    label, alb, G = lp.appendix_a_case(*dims, M)
    assert label == "2.2.1" and alb == 512 * 512 * 9
    assert lp.solve_lp_sigma1(*dims, M).cost == pytest.approx(alb, rel=1e-6)
    assert alb == pytest.approx(lb.lower_bound(*dims, 1, 1, M).bound)
    # 2.2.2.2: thin channel count
    dims = (32, 3, 64, 112, 112, 7, 7)
    M = 4096.0
    label, alb, G = lp.appendix_a_case(*dims, M)
    assert label == "2.2.2.2" and alb == 64 * 112 * 112 * 32 and G == 3 * 49 * M
    assert lp.solve_lp_sigma1(*dims, M).cost == pytest.approx(alb, rel=1e-6)


def test_array_that_fits_caps_the_cost():
    """Section 5.3: if one of the three arrays fits in cache some tiling costs no more than the largest array."""
    rng = np.random.default_rng(5)
    n = 0
    for _ in range(300):
        R, S = (int(x) for x in rng.integers(1, 6, 2))
        W, H = int(rng.integers(R, 30)), int(rng.integers(S, 30))
        B, C, K = (int(x) for x in rng.integers(1, 100, 3))
        M = float(2 ** rng.integers(8, 15))
        sizes = (B * K * W * H, B * C * W * H, C * K * R * S)
        if min(sizes) <= M < max(sizes):
            r = lp.solve_lp(B, C, K, W, H, R, S, 1, 1, M)
            assert r.cost <= max(max(sizes), M) * (1 + 1e-6)
            n += 1
    assert n > 30


def test_pooling_bound_and_lp():
    """Section 6: the pooling bound has three terms, and its last paragraph says the bound is tight and always
    attainable: the Section 5 LP without the Filter row costs exactly the maximum of the three terms whenever that
    is at least M.  Keeping the Filter row (no row dropped) must fail this on some shapes, otherwise the test would
    not notice which row is dropped."""
    dims, M = (16, 32, 32, 28, 28, 3, 3, 2, 2), 1024.0
    assert len(lb.pooling_lower_bound(*dims, M).terms) == 3
    rng = np.random.default_rng(7)
    checked = with_filter_row_differs = 0
    for _ in range(300):
        R, S = (int(x) for x in rng.integers(1, 8, 2))
        sw, sh = int(rng.integers(1, R + 1)), int(rng.integers(1, S + 1))
        W, H = int(rng.integers(-(-R // sw), 40)), int(rng.integers(-(-S // sh), 40))
        B, C, K = (int(x) for x in rng.integers(1, 200, 3))
        M = float(2 ** rng.integers(4, 16))
        b = lb.pooling_lower_bound(B, C, K, W, H, R, S, sw, sh, M)
        r = lp.solve_lp(B, C, K, W, H, R, S, sw, sh, M, filter_constraint=False)
        assert r.cost >= b.bound * (1 - 1e-7)
        if b.bound >= M:
            assert r.cost == pytest.approx(b.bound, rel=1e-6), (B, C, K, W, H, R, S, sw, sh, M)
            checked += 1
            if lp.solve_lp(B, C, K, W, H, R, S, sw, sh, M).cost > b.bound * (1 + 1e-3):
                with_filter_row_differs += 1
    assert checked > 200 and with_filter_row_differs > 20


# Appendix A, Case 1: one shape per sub-case of the lemma's proof (which of Image CHWB, Filter KCRS, Out KHWB exceed M)
CASE1 = {
    "1.2": ((64, 8, 2, 4, 4, 2, 2), 4096.0),
    "1.3": ((64, 2, 8, 4, 4, 2, 2), 4096.0),
    "1.4": ((2, 8, 8, 4, 4, 8, 8), 1024.0),
    "1.5": ((2, 40, 40, 4, 4, 3, 3), 1500.0),
    "1.6": ((64, 4, 4, 8, 8, 3, 3), 1024.0),
    "1.7": ((1, 64, 32, 4, 4, 3, 3), 700.0),
    "1.8": ((4, 64, 8, 4, 4, 3, 3), 700.0),
    "1.9": ((1, 32, 64, 4, 4, 3, 3), 700.0),
    "1.10": ((4, 8, 64, 4, 4, 3, 3), 700.0),
}


@pytest.mark.parametrize("case", sorted(CASE1))
def test_appendix_a_case_1_leaves(case):
    """Every sub-case of Appendix A's Case 1: the leaf's tile volume is the optimum of the appendix's own
    seven-variable LP, its cost F*M/G is the attainable bound the lemma states, and that is Theorem 1's maximum."""
    dims, M = CASE1[case]
    B, C, K, W, H, R, S = dims
    label, alb, G = lp.appendix_a_case(*dims, M)
    assert label == case
    F = float(np.prod([float(x) for x in dims]))
    assert F * M / G == pytest.approx(alb, rel=1e-12)
    assert lp.solve_lp_sigma1(*dims, M).volume == pytest.approx(G, rel=1e-6)
    assert alb == pytest.approx(lb.lower_bound(*dims, 1, 1, M).bound, rel=1e-12)
    assert alb == max(x for x in (C * H * W * B, K * C * R * S, K * H * W * B))


def test_appendix_a_tree_agrees_with_its_lp_everywhere():
    """Random stride-1 shapes over every leaf of the tree: the leaf's volume equals the seven-variable LP's optimum
    (the appendix's bR <= bW, bS <= bH rows included) whenever the bound is at least M."""
    rng = np.random.default_rng(21)
    seen = set()
    for _ in range(1500):
        R, S = (int(x) for x in rng.integers(1, 6, 2))
        W, H = int(rng.integers(R, 20)), int(rng.integers(S, 20))
        B, C, K = (int(2 ** rng.integers(0, 8)) for _ in range(3))
        M = float(2 ** rng.integers(6, 14))
        label, alb, G = lp.appendix_a_case(B, C, K, W, H, R, S, M)
        if label == "1.1" or alb < M:
            continue
        r = lp.solve_lp_sigma1(B, C, K, W, H, R, S, M)
        assert r.volume == pytest.approx(G, rel=1e-6), (label, B, C, K, W, H, R, S, M)
        seen.add(label)
    # (1.5 and 1.9 need K*C or C large against a tiny H*W*B and are rare in this sample: the test above has them)
    assert {"1.2", "1.3", "1.4", "1.6", "1.7", "1.8", "1.10", "2.2.1", "2.2.2.1", "2.2.2.2"} <= seen, seen


def _brute_footprint(t, R, S, sw, sh):
    """Words of the three arrays one tile touches, by listing the tile's iterations (not by formula)."""
    out, flt, img = set(), set(), set()
    for b in range(t["b"]):
        for c in range(t["c"]):
            for k in range(t["k"]):
                for w in range(t["w"]):
                    for h in range(t["h"]):
                        for r1 in range(t["r1"]):
                            for r2 in range(t["r2"]):
                                for s1 in range(t["s1"]):
                                    for s2 in range(t["s2"]):
                                        r, s = sw * r1 + r2, sh * s1 + s2
                                        if r >= R or s >= S:
                                            continue
                                        out.add((k, h, w, b))
                                        flt.add((k, r, s, c))
                                        img.add((r + sw * w, s + sh * h, c, b))
    return len(out) + len(flt) + len(img)


def test_integer_tiles_against_brute_force():
    """integer_tiles is this oracle's own rounding (Section 5 leaves it open).  On tiny problems every integer tiling
    is enumerated: the returned one fits M by brute-force footprints, and needs at most twice the outer-loop
    iterations of the best tiling that fits (measured: worst 1.67, mean 1.1)."""
    import itertools
    rng = np.random.default_rng(11)
    worst, ratios = 1.0, []
    for _ in range(40):
        B, C, K = (int(x) for x in rng.integers(1, 5, 3))
        R, S = (int(x) for x in rng.integers(1, 4, 2))
        sw, sh = int(rng.integers(1, R + 1)), int(rng.integers(1, S + 1))
        W, H = int(rng.integers(max(1, R // sw), 6)), int(rng.integers(max(1, S // sh), 6))
        dims = (B, C, K, W, H, R, S, sw, sh)
        M = int(rng.integers(12, 200))
        t = lp.integer_tiles(lp.solve_lp(*dims, M / 3.0).tiles, *dims, M)
        cap = {"b": B, "c": C, "k": K, "w": W, "h": H, "r1": -(-R // sw), "r2": sw, "s1": -(-S // sh), "s2": sh}
        assert all(1 <= t[x] <= cap[x] for x in cap)
        assert _brute_footprint(t, R, S, sw, sh) == lp.tile_footprint(t, R, S, sw, sh) <= M
        names, best = list(cap), None
        for combo in itertools.product(*(range(1, cap[n] + 1) for n in names)):
            u = dict(zip(names, combo))
            if lp.tile_footprint(u, R, S, sw, sh) <= M:
                n = int(np.prod([-(-cap[x] // u[x]) for x in names]))
                best = n if best is None else min(best, n)
        mine = int(np.prod([-(-cap[x] // t[x]) for x in names]))
        assert mine == lp.outer_iterations(t, *dims)
        ratios.append(mine / best)
    assert max(ratios) <= 2.0 and np.mean(ratios) <= 1.25, (max(ratios), np.mean(ratios))
