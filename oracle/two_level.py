"""Oracle for two memory levels (paper, Section 4.1: any level of a hierarchy may be taken as the fast memory, with
everything slower as the slow one; Section 5.3 leaves tilings for several levels at once to future work).

TEST INFRASTRUCTURE ONLY.  Three counters:

  nested_schedule_words -- the blocked schedule of Section 5 applied twice: outer tiles sized for the larger cache
                           (the words they move from the slow memory are counted by the single-level tile-granular
                           simulator on the whole problem), and inside every outer tile the same schedule with the
                           inner tiles (the words that move between the two caches are the single-level counts of the
                           outer tiles taken as problems of their own, summed).  Outer tiles take the filter extents
                           whole, so an outer tile is again a convolution of the same form.
  lru2_words            -- word-granular run of an iteration order against two fully associative LRU caches, the
                           small one in front of the large one (tiny shapes only): a second opinion on both levels.
  processor_cache_words -- what p processors with a private cache each fetch from the shared slow memory when every
                           processor works through a list of rounds, a round being the tiles its compute units hold at
                           one time (Section 7's setting, with the caches made explicit): every tile names the
                           "atoms" it reads -- the Filter rows of its output channels as one atom, the Image columns
                           (one input pixel of one image group, all channels) as one atom each, or the whole Image
                           footprint of its position tile as one -- and a processor
                           keeps atoms in an LRU cache of M words.  This is a model of this build's own making (the
                           paper has no such level of detail); it is what the host's two-level plan is compared with.
"""
from collections import OrderedDict
from typing import Dict, Iterable, List, Sequence, Tuple

from oracle import cachesim as cs

WHOLE_FILTER = ("r1", "r2", "s1", "s2")


def nested_schedule_words(B, C, K, W, H, R, S, sigma_w, sigma_h, outer: Dict[str, int], inner: Dict[str, int],
                          outer_order: Sequence[str] = cs.OUTER_DEFAULT,
                          inner_order: Sequence[str] = cs.OUTER_DEFAULT) -> Tuple[cs.Words, cs.Words]:
    """(words between slow memory and the large cache, words between the large and the small cache).
    outer / inner: tile sizes for (b, c, k, w, h); the outer tiles take r and s whole, the inner ones may cut them
    (keys r1, r2, s1, s2 as in cachesim; missing keys mean whole)."""
    sw, sh = min(sigma_w, R), min(sigma_h, S)
    whole = {"r1": -(-R // sw), "r2": sw, "s1": -(-S // sh), "s2": sh}
    o = dict(whole)
    o.update({k: outer[k] for k in ("b", "c", "k", "w", "h")})
    slow = cs.tiled_schedule_words(B, C, K, W, H, R, S, sigma_w, sigma_h, o, outer_order)
    i = dict(whole)
    i.update(inner)
    li = lf = lo = so = 0
    for b0 in range(0, B, o["b"]):
        for c0 in range(0, C, o["c"]):
            for k0 in range(0, K, o["k"]):
                for w0 in range(0, W, o["w"]):
                    for h0 in range(0, H, o["h"]):
                        sub = (min(o["b"], B - b0), min(o["c"], C - c0), min(o["k"], K - k0),
                               min(o["w"], W - w0), min(o["h"], H - h0))
                        wds = cs.tiled_schedule_words(sub[0], sub[1], sub[2], sub[3], sub[4], R, S, sigma_w, sigma_h,
                                                      i, inner_order)
                        li += wds.loads_image
                        lf += wds.loads_filter
                        lo += wds.loads_out
                        so += wds.stores_out
    return slow, cs.Words(li, lf, lo, so)


def lru2_words(order: Iterable[Tuple[int, ...]], sigma_w: int, sigma_h: int, M1: int, M2: int) -> Tuple[cs.Words, cs.Words]:
    """(words between slow memory and the large cache of M2 words, words between it and the small cache of M1 words).
    Both caches are fully associative LRU; a miss in the small cache is looked up in the large one; dirty Out words
    leaving the small cache are written into the large one, and written to slow memory when they leave that."""
    c1: "OrderedDict[Tuple, bool]" = OrderedDict()
    c2: "OrderedDict[Tuple, bool]" = OrderedDict()
    n1 = [0, 0, 0, 0]   # loads image, filter, out; stores out (small <-> large)
    n2 = [0, 0, 0, 0]   # (large <-> slow)
    seen_out = set()

    def kind(addr):
        return 0 if addr[0] == "I" else (1 if addr[0] == "F" else 2)

    def touch2(addr, write, count_load):
        if addr in c2:
            d = c2.pop(addr)
            c2[addr] = d or write
            return
        if count_load:
            n2[kind(addr)] += 1
        if len(c2) >= M2:
            old, dirty = c2.popitem(last=False)
            if dirty:
                n2[3] += 1
        c2[addr] = write

    def touch1(addr, write):
        if addr in c1:
            d = c1.pop(addr)
            c1[addr] = d or write
            return
        first_out = addr[0] == "O" and addr not in seen_out
        if addr[0] == "O":
            seen_out.add(addr)
        if not first_out:
            n1[kind(addr)] += 1       # comes from the large cache (or through it)
            touch2(addr, False, True)
        if len(c1) >= M1:
            old, dirty = c1.popitem(last=False)
            if dirty:
                n1[3] += 1
                touch2(old, True, False)   # a partial sum moves down; it is not loaded from slow memory for that
        c1[addr] = write

    for (b, c, k, w, h, r, s) in order:
        touch1(("I", r + sigma_w * w, s + sigma_h * h, c, b), False)
        touch1(("F", k, r, s, c), False)
        touch1(("O", k, h, w, b), True)
    for addr, dirty in c1.items():
        if dirty:
            n1[3] += 1
            touch2(addr, True, False)
    for addr, dirty in c2.items():
        if dirty:
            n2[3] += 1
    return cs.Words(*n2), cs.Words(*n1)


def processor_cache_words(rounds_per_processor: List[List[List[Tuple]]], atom_words: Dict[Tuple, int], M: int) -> int:
    """Words fetched from the shared slow memory by processors with private LRU caches of M words.
    rounds_per_processor[p][n] is the list of atoms the tiles of processor p's n-th round read (an atom read by several
    tiles of one round is fetched once: they run at the same time); atoms are looked up in sorted order."""
    total = 0
    for rounds in rounds_per_processor:
        cache: "OrderedDict[Tuple, int]" = OrderedDict()
        used = 0
        for atoms in rounds:
            for a in sorted(set(atoms)):
                if a in cache:
                    cache.move_to_end(a)
                    continue
                sz = atom_words[a]
                total += sz
                cache[a] = sz
                used += sz
                while used > M and len(cache) > 1:
                    _, old = cache.popitem(last=False)
                    used -= old
    return total


def launch_rounds(B, C, K, W, H, R, S, sigma_w, sigma_h, KT, TB, TW, TH, a_k: int, walk: int, n_xcd: int, grid: int,
                  b_group: int = 1, halo_shared: bool = False):
    """The rounds of this build's launch, for processor_cache_words: the tile list is a_k blocks of k-tile groups; inside a
    block the tiles are ordered k-tile fastest, then the b_group b-tiles that share cache lines, w, h, the remaining
    b-tile index (walk 0) or positions (same order) fastest and k-tile slowest (walk 1); XCD x owns a contiguous run of the list; workgroup i (XCD i % n_xcd) takes the tiles at places i / n_xcd,
    i / n_xcd + grid / n_xcd, ... of its XCD's run; round n holds every workgroup's n-th tile.
    halo_shared: True makes every Image column an atom of its own, so position tiles that overlap in their halo fetch
    the overlap once; False (what the measured launches do: a cache has turned a line over before the neighbouring
    position tile asks for it) makes the whole Image footprint of a position tile one atom.
    Returns (rounds_per_processor, atom_words)."""
    cdiv = lambda a, b: -(-a // b)
    tk, tb, tw, th = cdiv(K, KT), cdiv(B, TB), cdiv(W, TW), cdiv(H, TH)
    assert tk % a_k == 0
    kpg = tk // a_k
    npos = tb * tw * th
    n_tiles = tk * npos
    IW, IH = sigma_w * (W - 1) + R, sigma_h * (H - 1) + S
    tiles = []
    for kg in range(a_k):
        for t in range(kpg * npos):
            if walk == 0:
                k_l, pos = t % kpg, t // kpg
            else:
                pos, k_l = t % npos, t // npos
            b_lo = pos % b_group
            w_i = (pos // b_group) % tw
            h_i = (pos // (b_group * tw)) % th
            b_i = (pos // (b_group * tw * th)) * b_group + b_lo
            tiles.append((kg * kpg + k_l, b_i, w_i, h_i))
    assert len(tiles) == n_tiles
    atom_words = {}
    q, rem = divmod(n_tiles, n_xcd)
    rounds = [[] for _ in range(n_xcd)]
    per_xcd = max(1, grid // n_xcd)
    for x in range(n_xcd):
        lo = x * q + min(x, rem)
        hi = lo + q + (1 if x < rem else 0)
        run = tiles[lo:hi]
        for n0 in range(0, len(run), per_xcd):
            atoms = []
            for (k_i, b_i, w_i, h_i) in run[n0:n0 + per_xcd]:
                nb = min(TB, B - b_i * TB)
                fa = ("F", k_i)
                atom_words[fa] = min(KT, K - k_i * KT) * R * S * C
                atoms.append(fa)
                xr = range(sigma_w * w_i * TW, min(IW, sigma_w * w_i * TW + sigma_w * (TW - 1) + R))
                yr = range(sigma_h * h_i * TH, min(IH, sigma_h * h_i * TH + sigma_h * (TH - 1) + S))
                if halo_shared:
                    for x_i in xr:
                        for y_i in yr:
                            ia = ("I", b_i, x_i, y_i)
                            atom_words[ia] = nb * C
                            atoms.append(ia)
                else:
                    ia = ("I", b_i, w_i, h_i, "tile")
                    atom_words[ia] = nb * C * len(xr) * len(yr)
                    atoms.append(ia)
            rounds[x].append(atoms)
    return rounds, atom_words
