"""Pins for the data-movement simulators (paper Section 4 memory model, Section 5 blocked schedule,
Appendix A cost model): exact counts where a closed form exists, a word-granular LRU run as a second
opinion, and the paper's claim itself: the tiled schedule moves at least the closed-form bound and no more
than a small constant times it."""
import math

import pytest

from oracle import cachesim as cs
from oracle import lower_bound as lb
from oracle import lp_tiling as lp


def whole(dims):
    B, C, K, W, H, R, S, sw, sh = dims
    return {"b": B, "c": C, "k": K, "w": W, "h": H, "r1": -(-R // sw), "r2": sw, "s1": -(-S // sh), "s2": sh}


def test_everything_fits_moves_each_array_once():
    dims = (1, 3, 8, 16, 16, 3, 3, 1, 1)                      # benchmark shape c1
    w = cs.tiled_schedule_words(*dims, whole(dims))
    assert (w.loads_image, w.loads_filter, w.loads_out, w.stores_out) == (18 * 18 * 3, 216, 0, 2048)
    assert w.total == 3236


def test_everything_fits_with_strides_counts_touched_image_extent():
    dims = (2, 3, 4, 5, 6, 7, 3, 2, 3)
    B, C, K, W, H, R, S, sw, sh = dims
    w = cs.tiled_schedule_words(*dims, whole(dims))
    assert w.loads_image == B * C * (sw * (W - 1) + R) * (sh * (H - 1) + S)
    assert w.loads_filter == C * K * R * S and w.stores_out == B * K * W * H and w.loads_out == 0


def test_1x1_case_is_textbook_tiled_matmul_traffic():
    """Section 3: Out[KxB] = Filter[KxC] Image[CxB]; with tiles tm x tk and tk x tn and the contraction loop
    innermost, traffic is mnk(1/tn + 1/tm) + mn."""
    m, n, k = 24, 30, 32          # K, B, C
    tm, tn, tk = 6, 5, 8
    dims = (n, k, m, 1, 1, 1, 1, 1, 1)
    tiles = {"b": tn, "c": tk, "k": tm, "w": 1, "h": 1, "r1": 1, "r2": 1, "s1": 1, "s2": 1}
    w = cs.tiled_schedule_words(*dims, tiles, outer_order=("k", "b", "w", "h", "r1", "r2", "s1", "s2", "c"))
    assert w.loads_filter == m * k * (n // tn)
    assert w.loads_image == k * n * (m // tm)
    assert w.loads_out == 0 and w.stores_out == m * n
    assert w.total == m * n * k * (1 / tn + 1 / tm) + m * n
    # contraction loop outermost instead: every Out tile is stored, and re-loaded on every later visit
    w2 = cs.tiled_schedule_words(*dims, tiles, outer_order=("c", "k", "b", "w", "h", "r1", "r2", "s1", "s2"))
    assert w2.stores_out == m * n * (k // tk) and w2.loads_out == m * n * (k // tk - 1)


def test_lru_agrees_when_everything_fits():
    dims = (2, 2, 3, 3, 2, 2, 2, 1, 2)
    B, C, K, W, H, R, S, sw, sh = dims
    M = 10_000
    w = cs.lru_words(cs.iteration_order_naive(*dims[:7]), sw, sh, M)
    t = cs.tiled_schedule_words(*dims, whole(dims))
    assert (w.loads_image, w.loads_filter, w.loads_out, w.stores_out) == \
           (t.loads_image, t.loads_filter, 0, t.stores_out)


def test_lru_tiled_order_beats_printed_order_and_tile_count_is_an_upper_estimate():
    # the output plane (16x16) is larger than the cache, so the printed loop order thrashes
    dims = (1, 4, 8, 16, 16, 3, 3, 1, 1)
    B, C, K, W, H, R, S, sw, sh = dims
    M = 192
    real = lp.solve_lp(*dims, M / 3).tiles
    tiles = lp.integer_tiles(real, *dims, M)
    order = ("b", "k", "w", "h", "c", "r1", "r2", "s1", "s2")
    tiled_lru = cs.lru_words(cs.iteration_order_tiled(*dims, tiles, order), sw, sh, M)
    naive_lru = cs.lru_words(cs.iteration_order_naive(*dims[:7]), sw, sh, M)
    tiled_cnt = cs.tiled_schedule_words(*dims, tiles, order)
    compulsory = (sw * (W - 1) + R) * (sh * (H - 1) + S) * C * B + C * K * R * S + B * K * W * H
    assert compulsory <= tiled_lru.total <= naive_lru.total
    # a tile's three footprints fit in M together, so an LRU cache never does worse than reloading per tile
    assert tiled_lru.total <= tiled_cnt.total
    # both orders execute exactly the F iterations
    assert sum(1 for _ in cs.iteration_order_tiled(*dims, tiles, order)) == B * C * K * W * H * R * S


def test_lifted_order_with_stride_visits_every_iteration_once():
    dims = (1, 2, 2, 3, 2, 5, 3, 2, 2)         # R=5, sigma_w=2: R/sigma_w is not an integer
    tiles = {"b": 1, "c": 1, "k": 2, "w": 2, "h": 1, "r1": 2, "r2": 1, "s1": 1, "s2": 2}
    seen = list(cs.iteration_order_tiled(*dims, tiles))
    B, C, K, W, H, R, S, sw, sh = dims
    assert len(seen) == len(set(seen)) == B * C * K * W * H * R * S


SHAPES = {
    "c2_quarter": (8, 64, 64, 28, 28, 3, 3, 1, 1),
    "c3_small": (8, 3, 64, 56, 56, 7, 7, 2, 2),
    "c4": (64, 256, 256, 14, 14, 3, 3, 1, 1),
    "c5_half": (128, 512, 256, 7, 7, 3, 3, 1, 1),
    "alexnet_b16": (16, 3, 96, 55, 55, 11, 11, 4, 4),
}


@pytest.mark.parametrize("name,M", [("c2_quarter", 40960), ("c3_small", 40960), ("c4", 40960), ("c5_half", 40960),
                                    ("c4", 8192), ("alexnet_b16", 1024), ("alexnet_b16", 4096)])
def test_tiled_schedule_is_between_bound_and_small_multiple(name, M):
    """The paper's claim (Sections 4 and 5): the LP tiling moves Theta(max of the five terms) words.  The
    schedule keeps all three tiles resident, so the LP is solved for M/3 (Section 3 uses the same M/3) and
    rounded to integers (integer_tiles, pinned by brute force in test_oracle_bound_lp.py).  Three arrays of up to
    M/3 words per outer iteration at a tile volume computed for M/3 already cost 3*sqrt(3) = 5.2 times the M-word
    expression; the Image halo and the integer sizes add the rest.  Measured constants: c2_quarter 6.5, c3_small
    1.4, c4 5.8 (7.7 at M = 8192), c5_half 5.6, AlexNet conv1 7.9 (M = 1024) and 8.0 (M = 4096); asserted: at most 8.5."""
    dims = SHAPES[name]
    bound = lb.lower_bound(*dims, float(M)).bound
    real = lp.solve_lp(*dims, M / 3.0).tiles
    tiles = lp.integer_tiles(real, *dims, M)
    best = None
    for order in (("b", "k", "w", "h", "c", "r1", "r2", "s1", "s2"),      # Out tile stays put
                  ("c", "k", "r1", "r2", "s1", "s2", "b", "w", "h"),      # Filter tile stays put
                  ("b", "c", "w", "h", "r1", "r2", "s1", "s2", "k")):     # Image tile stays put
        w = cs.tiled_schedule_words(*dims, tiles, order)
        best = w.total if best is None else min(best, w.total)
    assert best >= bound
    assert best <= 8.5 * bound, (best / bound, tiles)
