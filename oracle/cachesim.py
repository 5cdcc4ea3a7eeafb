"""Oracle for data movement: two simulators of the paper's two-level memory model (Section 4: a slow
memory holding everything and a cache of M words; the cost is the number of words loaded plus stored).

TEST INFRASTRUCTURE ONLY.

  tiled_schedule_words -- runs the lifted, blocked nine-loop schedule of Section 5 tile by tile for given
                          integer tile sizes and an order of the outer (tile) loops, with explicit,
                          software-managed residency: one tile of each array is resident; when the next
                          outer iteration needs the same tile of an array nothing moves for that array.
                          Footprints are exact (clipped to the loop bounds; the Image footprint is the set
                          of indices r'' + sigma_w*(r'+w) actually touched, Section 5 item 3).
                          Cost model: Appendix A ("the three submatrices are each read or written once
                          per iteration of the outer loops").
  lru_words            -- executes an iteration order word by word against a fully associative LRU cache of
                          M words with write-back of dirty Out words (tiny shapes only): a second opinion
                          that does not trust the tile-residency bookkeeping.

Readings: r' runs over ceil(R/sigma_w) values and iterations with sigma_w*r'+r'' >= R are skipped (the
paper writes R/sigma_w as if it divided); same for s.
"""
from collections import OrderedDict
from itertools import product
from typing import Dict, Iterable, List, NamedTuple, Sequence, Tuple

OUTER_DEFAULT = ("b", "k", "w", "h", "c", "r1", "r2", "s1", "s2")


class Words(NamedTuple):
    loads_image: int
    loads_filter: int
    loads_out: int
    stores_out: int

    @property
    def total(self) -> int:
        return self.loads_image + self.loads_filter + self.loads_out + self.stores_out


def _blocks(extent: int, tile: int) -> List[Tuple[int, int]]:
    return [(lo, min(lo + tile, extent)) for lo in range(0, extent, tile)]


def _ceil_div(a, b):
    return -(-a // b)


def _axis_footprint(w_rng, r1_rng, r2_rng, sigma, R):
    """Distinct Image indices r2 + sigma*(r1+w) with r = sigma*r1 + r2 < R."""
    seen = set()
    for r1 in range(*r1_rng):
        for r2 in range(*r2_rng):
            if sigma * r1 + r2 >= R:
                continue
            for w in range(*w_rng):
                seen.add(r2 + sigma * (r1 + w))
    return len(seen)


def _axis_filter_count(r1_rng, r2_rng, sigma, R):
    return sum(1 for r1 in range(*r1_rng) for r2 in range(*r2_rng) if sigma * r1 + r2 < R)


def tiled_schedule_words(B, C, K, W, H, R, S, sigma_w, sigma_h, tiles: Dict[str, int],
                         outer_order: Sequence[str] = OUTER_DEFAULT) -> Words:
    """Words moved by the blocked schedule of Section 5 with integer tile sizes tiles[x], x in
    (b,c,k,w,h,r1,r2,s1,s2), outer loops nested in outer_order (first = outermost)."""
    ext = {"b": B, "c": C, "k": K, "w": W, "h": H,
           "r1": _ceil_div(R, sigma_w), "r2": min(sigma_w, R),
           "s1": _ceil_div(S, sigma_h), "s2": min(sigma_h, S)}
    if sorted(outer_order) != sorted(ext):
        raise ValueError("outer_order must be a permutation of the nine loop names")
    for nm in ext:
        if not (1 <= tiles[nm]):
            raise ValueError(f"tile {nm} must be >= 1")
    blk = {nm: _blocks(ext[nm], min(tiles[nm], ext[nm])) for nm in ext}
    li = lf = lo = so = 0
    res_img = res_flt = res_out = None
    out_started = set()
    out_dirty = False
    out_size_res = 0
    for combo in product(*(blk[nm] for nm in outer_order)):
        t = dict(zip(outer_order, combo))
        nr = _axis_filter_count(t["r1"], t["r2"], sigma_w, R)
        ns = _axis_filter_count(t["s1"], t["s2"], sigma_h, S)
        if nr == 0 or ns == 0:
            continue  # tile holds no valid (r,s): nothing executes
        nb = t["b"][1] - t["b"][0]
        nc = t["c"][1] - t["c"][0]
        nk = t["k"][1] - t["k"][0]
        nw = t["w"][1] - t["w"][0]
        nh = t["h"][1] - t["h"][0]
        id_out = (t["b"], t["k"], t["w"], t["h"])
        id_flt = (t["c"], t["k"], t["r1"], t["r2"], t["s1"], t["s2"])
        id_img = (t["b"], t["c"], t["w"], t["r1"], t["r2"], t["h"], t["s1"], t["s2"])
        if id_img != res_img:
            fx = _axis_footprint(t["w"], t["r1"], t["r2"], sigma_w, R)
            fy = _axis_footprint(t["h"], t["s1"], t["s2"], sigma_h, S)
            li += nb * nc * fx * fy
            res_img = id_img
        if id_flt != res_flt:
            lf += nc * nk * nr * ns
            res_flt = id_flt
        if id_out != res_out:
            if res_out is not None and out_dirty:
                so += out_size_res
            size = nb * nk * nw * nh
            if id_out in out_started:
                lo += size          # partial sums come back from slow memory
            out_started.add(id_out)
            res_out = id_out
            out_size_res = size
        out_dirty = True
    if res_out is not None and out_dirty:
        so += out_size_res
    return Words(li, lf, lo, so)


def iteration_order_tiled(B, C, K, W, H, R, S, sigma_w, sigma_h, tiles: Dict[str, int],
                          outer_order: Sequence[str] = OUTER_DEFAULT) -> Iterable[Tuple[int, ...]]:
    """Yield (b,c,k,w,h,r,s) in the order the blocked schedule of Section 5 executes them."""
    ext = {"b": B, "c": C, "k": K, "w": W, "h": H,
           "r1": _ceil_div(R, sigma_w), "r2": min(sigma_w, R),
           "s1": _ceil_div(S, sigma_h), "s2": min(sigma_h, S)}
    blk = {nm: _blocks(ext[nm], min(tiles[nm], ext[nm])) for nm in ext}
    for combo in product(*(blk[nm] for nm in outer_order)):
        t = dict(zip(outer_order, combo))
        for b, c, k, w, h, r1, r2, s1, s2 in product(*(range(*t[nm]) for nm in
                                                        ("b", "c", "k", "w", "h", "r1", "r2", "s1", "s2"))):
            r = sigma_w * r1 + r2
            s = sigma_h * s1 + s2
            if r >= R or s >= S:
                continue
            yield (b, c, k, w, h, r, s)


def iteration_order_naive(B, C, K, W, H, R, S) -> Iterable[Tuple[int, ...]]:
    """The loop nest of Eq. (1) in the order it is printed: b, c, k, w, h, r, s."""
    for b, c, k, w, h, r, s in product(range(B), range(C), range(K), range(W), range(H), range(R), range(S)):
        yield (b, c, k, w, h, r, s)


def lru_words(order: Iterable[Tuple[int, ...]], sigma_w: int, sigma_h: int, M: int) -> Words:
    """Word-granular simulation: fully associative LRU cache of M words; each iteration touches one word of
    Image, Filter and Out (Out is written, so it is stored back when evicted and at the end)."""
    cache: "OrderedDict[Tuple, bool]" = OrderedDict()  # address -> dirty
    li = lf = lo = so = 0
    out_seen = set()

    def touch(addr, write):
        nonlocal li, lf, lo, so
        if addr in cache:
            dirty = cache.pop(addr)
            cache[addr] = dirty or write
            return
        # miss
        if addr[0] == "I":
            li += 1
        elif addr[0] == "F":
            lf += 1
        else:
            if addr in out_seen:
                lo += 1      # partial sum comes back; the first touch starts from zero, no load
            out_seen.add(addr)
        if len(cache) >= M:
            old, dirty = cache.popitem(last=False)
            if dirty:
                so += 1
        cache[addr] = write

    for (b, c, k, w, h, r, s) in order:
        touch(("I", r + sigma_w * w, s + sigma_h * h, c, b), False)
        touch(("F", k, r, s, c), False)
        touch(("O", k, h, w, b), True)
    for addr, dirty in cache.items():
        if dirty:
            so += 1
    return Words(li, lf, lo, so)
