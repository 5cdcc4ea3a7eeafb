"""Oracle for the paper's optimal-tiling analysis (Section 5 and Appendix A).

TEST INFRASTRUCTURE ONLY.  Three things, each written from the paper's statement of it:

  solve_lp        -- the nine-variable linear program of Section 5: maximise the
                     log (base M) of the tile volume subject to the tile fitting the loop bounds and the three
                     array footprints fitting in M.  scipy's LP solver is the library step.
  solve_lp_sigma1 -- the seven-variable program of Appendix A (strides 1).
  appendix_a_case -- the decision tree of Appendix A, Theorem 2, with the tile volume G each leaf's
                     construction reaches (Case 1 down to its sub-cases 1.1 to 1.10).
  integer_tiles   -- integer tile sizes near the LP's real ones (the paper leaves the rounding open), with
                     tile_footprint and outer_iterations, the two quantities it trades.

Cost of a tiling (the cost expression of Section 5.2, and Appendix A): words moved = F * M / G with
F = BCKWHRS and G the tile volume.

Readings: R/sigma_w need not be an integer (AlexNet: 11/4); the LP is over reals, so that is harmless
here.  If a stride exceeds its filter extent (outside the paper's assumptions) it is clamped to it.
Several optimal tilings exist (Appendix A says so through its f2/f3 helpers), so only the optimal VOLUME is
a well-defined output; the tile vector returned is one optimiser.
"""
import math
from typing import Dict, NamedTuple, Tuple

import numpy as np
from scipy.optimize import linprog

VARS9 = ("b", "c", "k", "w", "h", "r1", "r2", "s1", "s2")  # r = sigma_w*r1 + r2, s = sigma_h*s1 + s2


class LPResult(NamedTuple):
    tiles: Dict[str, float]   # real-valued tile sizes b_x = M**l_x
    log_volume: float         # sum of l_x (base M)
    volume: float             # G
    cost: float               # F*M/G


def _lg(x, M):
    return math.log(x) / math.log(M)


def solve_lp(B, C, K, W, H, R, S, sigma_w, sigma_h, M, filter_constraint: bool = True) -> LPResult:
    """Section 5 LP.  filter_constraint=False drops the Filter footprint row (Section 6, pooling)."""
    sw = min(sigma_w, R)
    sh = min(sigma_h, S)
    idx = {v: i for i, v in enumerate(VARS9)}
    n = len(VARS9)
    A, ub = [], []

    def row(names, rhs):
        a = np.zeros(n)
        for nm in names:
            a[idx[nm]] += 1.0
        A.append(a)
        ub.append(rhs)

    # tile no larger than its loop bound
    for nm, val in (("b", B), ("c", C), ("k", K), ("w", W), ("h", H)):
        row([nm], _lg(val, M))
    row(["r2"], _lg(sw, M))
    row(["s2"], _lg(sh, M))
    row(["r1"], _lg(R, M) - _lg(sw, M))      # sigma_w * b_r' <= R
    row(["s1"], _lg(S, M) - _lg(sh, M))
    # footprints <= M
    row(["b", "k", "w", "h"], 1.0)                                   # Out
    if filter_constraint:
        row(["c", "k", "r1", "r2", "s1", "s2"], 1.0)                 # Filter
    row(["b", "c", "w", "h", "r2", "s2"], 1.0)                       # Image: (b_w+b_r')(b_h+b_s') expanded
    row(["b", "c", "w", "s1", "r2", "s2"], 1.0)
    row(["b", "c", "r1", "h", "r2", "s2"], 1.0)
    row(["b", "c", "r1", "s1", "r2", "s2"], 1.0)
    res = linprog(c=-np.ones(n), A_ub=np.array(A), b_ub=np.array(ub), bounds=[(0, None)] * n,
                  method="highs")
    if res.status != 0:
        raise RuntimeError(f"LP failed: {res.message}")
    l = res.x
    logv = float(np.sum(l))
    G = M ** logv
    F = float(B) * C * K * W * H * R * S
    tiles = {v: float(M ** l[i]) for i, v in enumerate(VARS9)}
    return LPResult(tiles, logv, G, F * M / G)


def solve_lp_sigma1(B, C, K, W, H, R, S, M) -> LPResult:
    """Appendix A's seven-variable LP (strides 1): variables bB,bK,bH,bW,bR,bS,bC."""
    names = ("b", "k", "h", "w", "r", "s", "c")
    idx = {v: i for i, v in enumerate(names)}
    n = 7
    A, ub = [], []

    def row(coefs, rhs):
        a = np.zeros(n)
        for nm, cf in coefs.items():
            a[idx[nm]] += cf
        A.append(a)
        ub.append(rhs)

    row({"k": 1, "h": 1, "w": 1, "b": 1}, 1.0)     # Out tile
    row({"c": 1, "h": 1, "w": 1, "b": 1}, 1.0)     # Image tile (constant 4 dropped as in the paper)
    row({"k": 1, "r": 1, "s": 1, "c": 1}, 1.0)     # Filter tile
    row({"r": 1, "w": -1}, 0.0)                    # bR <= bW
    row({"s": 1, "h": -1}, 0.0)                    # bS <= bH
    for nm, val in (("b", B), ("k", K), ("h", H), ("w", W), ("r", R), ("s", S), ("c", C)):
        row({nm: 1}, _lg(val, M))
    res = linprog(c=-np.ones(n), A_ub=np.array(A), b_ub=np.array(ub), bounds=[(0, None)] * n,
                  method="highs")
    if res.status != 0:
        raise RuntimeError(f"LP failed: {res.message}")
    logv = float(np.sum(res.x))
    G = M ** logv
    F = float(B) * C * K * W * H * R * S
    return LPResult({v: float(M ** res.x[i]) for i, v in enumerate(names)}, logv, G, F * M / G)


def appendix_a_case(B, C, K, W, H, R, S, M) -> Tuple[str, float, float]:
    """Appendix A, Theorem 2 (strides 1).  Returns (case label, attainable lower bound ALB, tile volume G of
    the leaf's construction).  Case 1 (some array fits in M) is split into the ten sub-cases of the proof of its
    lemma, by which of Image (CHWB), Filter (KCRS) and Out (KHWB) exceed M; where two sub-cases meet (an array of
    exactly M words) the later one is taken, and their constructions agree there."""
    img, flt, out = C * H * W * B, K * C * R * S, K * H * W * B
    hwb = H * W * B
    F = float(B) * C * K * W * H * R * S
    if min(img, flt, out) <= M:
        big_i, big_f, big_o = img > M, flt > M, out > M
        if not (big_i or big_f or big_o):
            return "1.1", float(max(img, flt, out)), F   # unblocked: one tile is the whole nest
        if big_i and not big_f and not big_o:
            return "1.2", float(img), float(K) * R * S * M          # one image, all k, M/(HW) channels
        if big_o and not big_f and not big_i:
            return "1.3", float(out), float(C) * R * S * M          # Case 1.2 with C and K exchanged
        if big_f and not big_i and not big_o:
            # 1.4 (KC <= M: tile r, s) and 1.5 (KC >= M: tile k, c) reach the same volume
            return ("1.4" if K * C <= M else "1.5"), float(flt), float(hwb) * M
        if big_i and big_o:
            return "1.6", float(max(out, img)), float(min(K, C)) * M * R * S
        if big_i and big_f:
            if K >= hwb:
                return "1.7", float(flt), float(hwb) * M
            return "1.8", float(max(img, flt)), min(float(K) * M * R * S, float(hwb) * M)
        # Filter and Out exceed M, Image fits: Cases 1.7 / 1.8 with C and K exchanged
        if C >= hwb:
            return "1.9", float(flt), float(hwb) * M
        return "1.10", float(max(out, flt)), min(float(C) * M * R * S, float(hwb) * M)
    if R * S >= M:
        return "2.1", F / M, float(M) ** 2
    if M * R * S >= (B * H * W) ** 2:
        return "2.2.1", float(flt), float(H * W * B) * M
    if min(C, K) >= math.sqrt(M / (R * S)):
        return "2.2.2.1", float(K) * C * H * W * B * math.sqrt(R * S / M), M ** 1.5 * math.sqrt(R * S)
    return "2.2.2.2", float(max(out, img)), float(min(C, K)) * R * S * M


def _tile_caps(B, C, K, W, H, R, S, sigma_w, sigma_h) -> Dict[str, int]:
    sw, sh = min(sigma_w, R), min(sigma_h, S)
    return {"b": B, "c": C, "k": K, "w": W, "h": H, "r1": -(-R // sw), "r2": sw, "s1": -(-S // sh), "s2": sh}


def tile_footprint(t: Dict[str, int], R, S, sigma_w, sigma_h) -> int:
    """Words one tile of each array occupies together: Out b*k*w*h, Filter c*k*(taps in the tile), Image
    b*c*(distinct first-axis indices)*(distinct second-axis indices), the Image extent per axis being the set
    of indices r'' + sigma*(r' + w) the tile touches (Section 5, item 3)."""
    sw, sh = min(sigma_w, R), min(sigma_h, S)

    def axis(nw, n1, n2, sg, ext):
        taps = sum(1 for r1 in range(n1) for r2 in range(n2) if sg * r1 + r2 < ext)
        idx = {r2 + sg * (r1 + w) for r1 in range(n1) for r2 in range(n2) if sg * r1 + r2 < ext for w in range(nw)}
        return taps, len(idx)

    nr, fx = axis(t["w"], t["r1"], t["r2"], sw, R)
    ns, fy = axis(t["h"], t["s1"], t["s2"], sh, S)
    return t["b"] * t["k"] * t["w"] * t["h"] + t["c"] * t["k"] * nr * ns + t["b"] * t["c"] * fx * fy


def outer_iterations(t: Dict[str, int], B, C, K, W, H, R, S, sigma_w, sigma_h) -> int:
    """Iterations of the nine outer (tile) loops of the blocked schedule: the product of ceil(extent / tile)."""
    cap = _tile_caps(B, C, K, W, H, R, S, sigma_w, sigma_h)
    n = 1
    for x in cap:
        n *= -(-cap[x] // t[x])
    return n


def integer_tiles(real_tiles: Dict[str, float], B, C, K, W, H, R, S, sigma_w, sigma_h, M) -> Dict[str, int]:
    """Turn the LP's real tile sizes into integers whose three exact footprints fit in M words TOGETHER.

    Not from the paper: Section 5 leaves the rounding open and remarks that the exact LP sizes need not perform
    best.  What is minimised here is the number of outer-loop iterations, because Appendix A's cost model charges
    each of them at most M words: start from the floor of the LP sizes, then repeat the single best move among
    "grow one size to x+1 or to the next size that needs fewer tiles along its loop" and the same move paid for by
    shrinking one other size just enough to fit, as long as the iteration count falls (ties: smaller footprint)."""
    cap = _tile_caps(B, C, K, W, H, R, S, sigma_w, sigma_h)
    t = {k: max(1, min(cap[k], int(math.floor(v + 1e-9)))) for k, v in real_tiles.items()}

    def fp(u):
        return tile_footprint(u, R, S, sigma_w, sigma_h)

    def iters(u):
        n = 1
        for x in cap:
            n *= -(-cap[x] // u[x])
        return n

    while fp(t) > M:            # the floor can still overshoot: the LP bounds each array by M alone
        big = max((k for k in t if t[k] > 1), key=lambda k: t[k], default=None)
        if big is None:
            break
        t[big] -= 1
    names = list(t)
    while True:
        n0, best = iters(t), None
        for x in names:
            cur = -(-cap[x] // t[x])
            sizes = set()
            if t[x] < cap[x]:
                sizes.add(t[x] + 1)
            if cur > 1:
                sizes.add(-(-cap[x] // (cur - 1)))
            for nx in sorted(sizes):
                u = dict(t)
                u[x] = nx
                trials = [u] if fp(u) <= M else []
                if not trials:
                    for y in names:
                        if y == x:
                            continue
                        v = dict(u)
                        while v[y] > 1 and fp(v) > M:
                            v[y] -= 1
                        if fp(v) <= M:
                            trials.append(v)
                for v in trials:
                    key = (iters(v), fp(v))
                    if key[0] < n0 and (best is None or key < best[0]):
                        best = (key, v)
        if best is None:
            return t
        t = best[1]
