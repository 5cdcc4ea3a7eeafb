"""Oracle for the communication lower bound (paper, Theorem 1 in Section 4; also stated
in Section 1).

TEST INFRASTRUCTURE ONLY.  The bound is a closed form, so the oracle is that closed form written out:

    W_CNN = Omega(max(T1..T5)),  T1 = BKWH                      (size of Out)
                                 T2 = sigma_w*sigma_h*BCWH      (size of Image, asymptotic form)
                                 T3 = CKRS                      (size of Filter)
                                 T4 = BCKWHRS / M               (HBL bound, Section 4.2)
                                 T5 = BCKWH*sqrt(RS*sigma_w*sigma_h / M)   (small-filter bound, Section 4.3)

Readings: the constant hidden in Omega is taken as 1 and nothing is floored; "words" are elements;
outside the paper's assumption sigma <= filter extent (Section 2) the strides are clamped to the filter
extents in T2 and T5, because only touched Image elements have to move.
"""
import math
from typing import List, NamedTuple


class Bound(NamedTuple):
    terms: List[float]
    bound: float
    argmax: int  # 0-based index of the first largest term


def lower_bound(B, C, K, W, H, R, S, sigma_w, sigma_h, M) -> Bound:
    if min(B, C, K, W, H, R, S, sigma_w, sigma_h) < 1 or not (M > 0):
        raise ValueError("all parameters must be >= 1 and M > 0")
    sw = min(sigma_w, R)
    sh = min(sigma_h, S)
    t1 = float(B) * K * W * H
    t2 = float(sw) * sh * B * C * W * H
    t3 = float(C) * K * R * S
    t4 = float(B) * C * K * W * H * R * S / M
    t5 = float(B) * C * K * W * H * math.sqrt(R * S * sw * sh / M)
    terms = [t1, t2, t3, t4, t5]
    best = max(terms)
    return Bound(terms, best, terms.index(best))


def matmul_reuse_cost(B, C, K, W, H, R, S, M) -> float:
    """Words moved if only matmul-style reuse were available: F / sqrt(M) (Section 1)."""
    return float(B) * C * K * W * H * R * S / math.sqrt(M)


def pooling_lower_bound(B, C, K, W, H, R, S, sigma_w, sigma_h, M) -> Bound:
    """Section 6: pooling has no Filter, so only three terms remain."""
    sw = min(sigma_w, R)
    sh = min(sigma_h, S)
    terms = [float(B) * K * W * H, float(sw) * sh * B * C * W * H,
             float(B) * C * K * W * H * R * S / M]
    best = max(terms)
    return Bound(terms, best, terms.index(best))
