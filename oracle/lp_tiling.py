"""Oracle for the paper's optimal-tiling analysis (Section 5 and Appendix A).

TEST INFRASTRUCTURE ONLY.  Three things, each written from the paper's statement of it:

  solve_lp        -- the nine-variable linear program of Section 5 (the one labelled eq:mplp): maximise the
                     log (base M) of the tile volume subject to the tile fitting the loop bounds and the three
                     array footprints fitting in M.  scipy's LP solver is the library step.
  solve_lp_sigma1 -- the seven-variable program of Appendix A (strides 1).
  appendix_a_case -- the decision tree of Appendix A, Theorem 2, with the tile volume G each leaf's
                     construction reaches.

Cost of a tiling (Section 5.2, Eq. eq:ccost_tile, and Appendix A): words moved = F * M / G with
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
    the leaf's construction or nan where the appendix gives several sub-constructions)."""
    img, flt, out = C * H * W * B, K * C * R * S, K * H * W * B
    F = float(B) * C * K * W * H * R * S
    if min(img, flt, out) <= M:
        if img > M and out > M and flt <= M:
            G = min(K, C) * M * R * S         # Case 1.6
            return "1.6", float(max(out, img)), float(G)
        if img <= M and flt <= M and out <= M:
            return "1.1", float(max(img, flt, out)), F  # unblocked: one tile is the whole nest
        return "1", float(max(img, flt, out)), float("nan")
    if R * S >= M:
        return "2.1", F / M, float(M) ** 2
    if M * R * S >= (B * H * W) ** 2:
        return "2.2.1", float(flt), float(H * W * B) * M
    if min(C, K) >= math.sqrt(M / (R * S)):
        return "2.2.2.1", float(K) * C * H * W * B * math.sqrt(R * S / M), M ** 1.5 * math.sqrt(R * S)
    return "2.2.2.2", float(max(out, img)), float(min(C, K)) * R * S * M


def integer_tiles(real_tiles: Dict[str, float], B, C, K, W, H, R, S, sigma_w, sigma_h, M) -> Dict[str, int]:
    """Turn the LP's real tile sizes into integers whose three exact footprints fit in M words TOGETHER.

    Not from the paper (it leaves rounding open: "the exact tile sizes may not necessarily give the best
    performance", Section 5): floor every size, then grow sizes one at a time, largest relative gain first,
    while Out + Filter + Image footprints (Image with its exact halo extent) still sum to at most M."""
    sw, sh = min(sigma_w, R), min(sigma_h, S)
    cap = {"b": B, "c": C, "k": K, "w": W, "h": H, "r1": -(-R // sw), "r2": sw, "s1": -(-S // sh), "s2": sh}
    t = {k: max(1, min(cap[k], int(math.floor(v + 1e-9)))) for k, v in real_tiles.items()}

    def footprint(t):
        nr = min(R, sw * (t["r1"] - 1) + t["r2"]) if t["r2"] == sw else t["r1"] * t["r2"]
        ns = min(S, sh * (t["s1"] - 1) + t["s2"]) if t["s2"] == sh else t["s1"] * t["s2"]
        out = t["b"] * t["k"] * t["w"] * t["h"]
        flt = t["c"] * t["k"] * nr * ns
        img = t["b"] * t["c"] * (t["w"] + t["r1"] - 1) * t["r2"] * (t["h"] + t["s1"] - 1) * t["s2"]
        return out + flt + img

    while footprint(t) > M:            # floor can still overshoot because the LP bounds each array by M alone
        big = max((k for k in t if t[k] > 1), key=lambda k: t[k], default=None)
        if big is None:
            break
        t[big] -= 1
    grew = True
    while grew:
        grew = False
        for k in sorted(t, key=lambda k: t[k]):
            if t[k] < cap[k]:
                t[k] += 1
                if footprint(t) <= M:
                    grew = True
                else:
                    t[k] -= 1
    return t
