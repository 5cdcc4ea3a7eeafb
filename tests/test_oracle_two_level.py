"""Pins for the two-level oracle (paper Section 4.1: any level of the hierarchy as the fast memory; Section 7: processors
with a memory of their own): degenerate cases that must reduce to the pinned single-level simulators, the word-granular
run with two LRU caches, and the per-processor cache count against the replicated terms Section 7 prints."""
import numpy as np
import pytest

from oracle import cachesim as cs
from oracle import parallel as par
from oracle import two_level as tl


def whole(dims):
    B, C, K, W, H, R, S, sw, sh = dims
    return {"b": B, "c": C, "k": K, "w": W, "h": H}


def test_outer_tile_is_the_whole_problem():
    dims = (4, 6, 8, 9, 7, 3, 3, 1, 1)
    inner = {"b": 2, "c": 3, "k": 4, "w": 3, "h": 7}
    slow, mid = tl.nested_schedule_words(*dims, whole(dims), inner)
    B, C, K, W, H, R, S, sw, sh = dims
    assert (slow.loads_image, slow.loads_filter, slow.loads_out, slow.stores_out) == \
           ((W - 1 + R) * (H - 1 + S) * C * B, C * K * R * S, 0, B * K * W * H)       # every array moves once
    full = dict(inner, r1=3, r2=1, s1=3, s2=1)
    assert mid == cs.tiled_schedule_words(*dims, full)                                # the single-level count


def test_equal_tiles_move_the_same_words_at_both_levels():
    dims = (4, 6, 8, 10, 6, 3, 2, 2, 1)
    t = {"b": 2, "c": 3, "k": 4, "w": 5, "h": 3}
    slow, mid = tl.nested_schedule_words(*dims, t, t)
    # inside an outer tile the inner schedule is one tile: it loads its Image and Filter footprints once, like the outer
    # level; its Out tile goes down to the large cache at the end of every outer tile (once per c-tile: C / 3 = 2 times),
    # where the outer level keeps it resident across the c-tiles and stores it once
    assert mid.loads_image == slow.loads_image and mid.loads_filter == slow.loads_filter
    B, C, K, W, H = dims[:5]
    assert slow.stores_out == B * K * W * H and mid.stores_out == 2 * B * K * W * H


def test_lru2_with_a_huge_large_cache_is_the_single_level_run():
    dims = (2, 2, 3, 4, 3, 2, 2, 1, 2)
    B, C, K, W, H, R, S, sw, sh = dims
    M1 = 24
    slow, mid = tl.lru2_words(cs.iteration_order_naive(*dims[:7]), sw, sh, M1, 10 ** 6)
    one = cs.lru_words(cs.iteration_order_naive(*dims[:7]), sw, sh, M1)
    assert (mid.loads_image, mid.loads_filter, mid.loads_out, mid.stores_out) == \
           (one.loads_image, one.loads_filter, one.loads_out, one.stores_out)
    IW, IH = sw * (W - 1) + R, sh * (H - 1) + S
    assert (slow.loads_image, slow.loads_filter, slow.loads_out, slow.stores_out) == (IW * IH * C * B, K * R * S * C, 0, K * H * W * B)


def test_nested_tiling_bounds_the_two_level_lru_run():
    """Tiles whose footprints fit their cache: an LRU cache never does worse than reloading every tile, at either
    level; and the large cache never moves more than the small one asks of it."""
    dims = (1, 4, 8, 12, 12, 3, 3, 1, 1)
    B, C, K, W, H, R, S, sw, sh = dims
    outer = {"b": 1, "c": 4, "k": 8, "w": 6, "h": 6}       # 8*36 + 4*8*9 + 4*64 = 832 words
    inner = {"b": 1, "c": 2, "k": 4, "w": 3, "h": 3}       # 4*9 + 2*4*9 + 2*25 = 158 words
    M2, M1 = 900, 170
    order_o = ("b", "k", "w", "h", "c", "r1", "r2", "s1", "s2")
    slow_t, mid_t = tl.nested_schedule_words(*dims, outer, inner, order_o, order_o)

    def nested_order():
        for k0 in range(0, K, outer["k"]):
            for w0 in range(0, W, outer["w"]):
                for h0 in range(0, H, outer["h"]):
                    for c0 in range(0, C, outer["c"]):
                        sub = (1, min(outer["c"], C - c0), min(outer["k"], K - k0), min(outer["w"], W - w0), min(outer["h"], H - h0))
                        full = dict(inner, r1=3, r2=1, s1=3, s2=1)
                        for (b, c, k, w, h, r, s) in cs.iteration_order_tiled(*sub, R, S, sw, sh, full, order_o):
                            yield (b, c0 + c, k0 + k, w0 + w, h0 + h, r, s)

    assert sum(1 for _ in nested_order()) == B * C * K * W * H * R * S
    slow_l, mid_l = tl.lru2_words(nested_order(), sw, sh, M1, M2)
    compulsory = (W - 1 + R) * (H - 1 + S) * C * B + C * K * R * S + B * K * W * H
    assert compulsory <= slow_l.total <= slow_t.total
    assert mid_l.total <= mid_t.total
    assert slow_l.loads_image + slow_l.loads_filter <= mid_l.loads_image + mid_l.loads_filter


def test_processor_caches_reproduce_the_replicated_terms_of_section_7():
    """1 x 1 filters (no halo), p = 8 processors that divide the output evenly, caches that hold a processor's whole
    share: the Image is fetched a_K times and the Filter a_B a_W a_H times, the second and third terms of Section 7's
    expression."""
    B, C, K, W, H = 8, 6, 16, 8, 4
    KT, TB, TW, TH = 4, 2, 4, 2          # 4 k-tiles x 4 b-tiles x 2 x 2 = 64 tiles, 8 per processor
    for a_k in (1, 2, 4):
        rounds, words = tl.launch_rounds(B, C, K, W, H, 1, 1, 1, 1, KT, TB, TW, TH, a_k, 0, 8, 64)
        got = tl.processor_cache_words(rounds, words, 10 ** 9)
        a_pos = 8 // a_k
        bound = par.parallel_bound(B, C, K, W, H, 1, 1, 1, 1, 1e9, a_pos, a_k, 1, 1)
        assert got == a_k * B * C * W * H + a_pos * C * K == bound.terms[1] + bound.terms[2]


def test_processor_cache_capacity_and_walk_order():
    """More tiles than a processor holds at once: with the k-tiles fastest the Filter is streamed once per round unless
    the cache keeps it; with the positions fastest the Image is."""
    B, C, K, W, H, R, S = 4, 8, 32, 16, 16, 1, 1
    KT, TB, TW, TH = 4, 4, 2, 2          # 8 k-tiles x 64 position tiles
    img, flt = B * C * W * H, C * K
    for walk in (0, 1):
        rounds, words = tl.launch_rounds(B, C, K, W, H, R, S, 1, 1, KT, TB, TW, TH, 1, walk, 1, 8)
        assert sum(len(r) for r in rounds) == 64
        big = tl.processor_cache_words(rounds, words, 10 ** 9)
        assert big == img + flt                                   # everything once
        tiny = tl.processor_cache_words(rounds, words, 1)         # keeps only the last atom
        if walk == 0:
            # a round = all 8 k-tiles of one position tile: the whole Filter again in every round, each Image tile once
            assert tiny == img + 64 * flt
        else:
            # a round = 8 position tiles of one k-tile: the Image again for every k-tile, a Filter row group per round
            assert tiny == 8 * img + 64 * (flt // 8)


def test_halo_between_position_tiles_shared_or_not():
    """3 x 3 filter, one processor whose cache holds everything: with every Image column an atom the overlap of
    neighbouring position tiles is fetched once (the Image once in all); with a position tile's footprint as one atom
    every tile fetches its own (TW + 2)(TH + 2) columns."""
    B, C, K, W, H, R, S = 4, 5, 8, 8, 6, 3, 3
    KT, TB, TW, TH = 8, 4, 4, 2
    IW, IH = W + R - 1, H + S - 1
    rounds, words = tl.launch_rounds(B, C, K, W, H, R, S, 1, 1, KT, TB, TW, TH, 1, 0, 1, 2, halo_shared=True)
    assert tl.processor_cache_words(rounds, words, 10 ** 9) == IW * IH * C * B + K * R * S * C
    rounds, words = tl.launch_rounds(B, C, K, W, H, R, S, 1, 1, KT, TB, TW, TH, 1, 0, 1, 2, halo_shared=False)
    n_pos = (W // TW) * (H // TH)
    assert tl.processor_cache_words(rounds, words, 10 ** 9) == n_pos * (TW + 2) * (TH + 2) * C * B + K * R * S * C
