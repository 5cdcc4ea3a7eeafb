"""Oracle for the parallel bound and the work division (paper, Section 7, "Parallel Algorithm").

TEST INFRASTRUCTURE ONLY.  p processors share one memory; each gets one block of the output dimensions,
B' = B/a_B, K' = K/a_K, W' = W/a_W, H' = H/a_H with a_B a_K a_W a_H <= p, and runs the sequential algorithm on
its block.  The total traffic is p times Theorem 1's expression for the block, which the paper writes out as

    max( BKWH,  a_K * sw*sh*BCWH,  a_B a_W a_H * CKRS,  BCKWHRS / M,  BCKWH * sqrt(RS*sw*sh / M) )

(every processor reads the Image block of all channels, so the Image term is replicated a_K times, and the
Filter block of its K' output channels, replicated a_B a_W a_H times), and says to choose the a's that minimise it.
The closed form is written out below; the minimisation is the enumeration of every admissible (a_B, a_K, a_W, a_H).

Readings (the paper leaves them open):
  * each a divides nothing in particular in the paper ("evenly partitioning"); here an a is admissible if it is
    between 1 and the size of its dimension (a block cannot be smaller than one element); the printed side
    conditions "p a_B <= B, etc." are taken as that;
  * the work is divided over all processors: only divisions whose product a_B a_K a_W a_H is the largest admissible
    one (p itself whenever the dimensions allow it) are candidates; the printed "<= p" alone would always be
    minimised by a single block, which divides nothing;
  * the maximum has many ties (terms 1, 4, 5 do not depend on the a's); among minimisers of the maximum the
    division with the least replicated traffic a_K*T2 + a_B a_W a_H*T3 is taken, then the lexicographically
    smallest (a_B, a_K, a_W, a_H);
  * strides above the filter extent are clamped as in Theorem 1's oracle.
"""
import math
from typing import List, NamedTuple, Tuple


class ParallelBound(NamedTuple):
    terms: List[float]
    bound: float
    argmax: int  # 0-based index of the first largest term


def parallel_bound(B, C, K, W, H, R, S, sigma_w, sigma_h, M, a_b, a_k, a_w, a_h) -> ParallelBound:
    if min(B, C, K, W, H, R, S, sigma_w, sigma_h, a_b, a_k, a_w, a_h) < 1 or not (M > 0):
        raise ValueError("all parameters must be >= 1 and M > 0")
    if a_b > B or a_k > K or a_w > W or a_h > H:
        raise ValueError("a block cannot be smaller than one element")
    sw = min(sigma_w, R)
    sh = min(sigma_h, S)
    out_words = float(B) * K * W * H
    image_words = float(sw) * sh * B * C * W * H
    filter_words = float(C) * K * R * S
    macs = float(B) * C * K * W * H * R * S
    terms = [out_words,
             a_k * image_words,
             a_b * a_w * a_h * filter_words,
             macs / M,
             float(B) * C * K * W * H * math.sqrt(R * S * sw * sh / M)]
    best = max(terms)
    return ParallelBound(terms, best, terms.index(best))


class Division(NamedTuple):
    a: Tuple[int, int, int, int]   # (a_B, a_K, a_W, a_H)
    bound: ParallelBound
    replicated_words: float        # a_K * T2 + a_B a_W a_H * T3


def work_division(B, C, K, W, H, R, S, sigma_w, sigma_h, M, p) -> Division:
    """Among the admissible (a_B, a_K, a_W, a_H) with the largest product <= p, the one that minimises the bound, ties
    broken as the module header says.  Plain enumeration: p is a processor count, small."""
    if p < 1:
        raise ValueError("p must be >= 1")
    best = None
    for a_b in range(1, min(B, p) + 1):
        for a_k in range(1, min(K, p // a_b) + 1):
            for a_w in range(1, min(W, p // (a_b * a_k)) + 1):
                for a_h in range(1, min(H, p // (a_b * a_k * a_w)) + 1):
                    pb = parallel_bound(B, C, K, W, H, R, S, sigma_w, sigma_h, M, a_b, a_k, a_w, a_h)
                    rep = pb.terms[1] + pb.terms[2]
                    key = (-(a_b * a_k * a_w * a_h), pb.bound, rep, (a_b, a_k, a_w, a_h))
                    if best is None or key < best[0]:
                        best = (key, Division((a_b, a_k, a_w, a_h), pb, rep))
    return best[1]
