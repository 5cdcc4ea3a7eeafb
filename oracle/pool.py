"""Pooling oracle.

TEST INFRASTRUCTURE ONLY.  The paper's pooling nest (Section 6, "Application to Pooling") is the convolution nest
without the Filter: Out(k,h,w,b) (+)= Image(r + sigma_w*w, s + sigma_h*h, c, b), where (+) adds the element divided by
R*S (average pooling) or takes the maximum (max pooling).  Printed literally the nest also runs over k and c
independently although neither array carries both; it is read here as per-channel pooling, k = c (K must equal C):

    Out[c][h][w][b] = (1/(R*S)) * sum_{r,s} Image[r + sigma_w*w][s + sigma_h*h][c][b]        (average)
    Out[c][h][w][b] = max_{r,s} Image[r + sigma_w*w][s + sigma_h*h][c][b]                    (max)

Layouts as for the convolution: Image[IW, IH, C, B], Out[K = C, H, W, B], numpy C order, computed in fp64.
pool_fp64 takes one strided window view per (r, s) and reduces them in the order r, then s; pool_loops is the same
thing as seven-minus-one plain Python loops for tiny shapes.
"""
import numpy as np

from .conv import Problem

MODES = ("avg", "max")


def _check(p: Problem, image: np.ndarray, mode: str) -> None:
    if mode not in MODES:
        raise ValueError("mode must be 'avg' or 'max'")
    if p.K != p.C:
        raise ValueError("per-channel pooling needs K == C")
    if tuple(image.shape) != p.image_shape:
        raise ValueError("image shape %r, expected %r" % (image.shape, p.image_shape))


def pool_fp64(p: Problem, image: np.ndarray, mode: str) -> np.ndarray:
    """Out[K, H, W, B] in fp64."""
    _check(p, image, mode)
    img = np.asarray(image, dtype=np.float64)
    acc = None
    for r in range(p.R):
        for s in range(p.S):
            win = img[r:r + p.sigma_w * (p.W - 1) + 1:p.sigma_w, s:s + p.sigma_h * (p.H - 1) + 1:p.sigma_h]   # [W, H, C, B]
            if acc is None:
                acc = win.copy()
            elif mode == "avg":
                acc = acc + win
            else:
                acc = np.maximum(acc, win)
    if mode == "avg":
        acc = acc / float(p.R * p.S)
    return np.ascontiguousarray(acc.transpose(2, 1, 0, 3))   # [C, H, W, B]


def pool_loops(p: Problem, image: np.ndarray, mode: str) -> np.ndarray:
    """The loop nest written out (pure Python, tiny shapes)."""
    _check(p, image, mode)
    out = np.zeros(p.out_shape, dtype=np.float64)
    for k in range(p.K):
        for h in range(p.H):
            for w in range(p.W):
                for b in range(p.B):
                    vals = [float(image[r + p.sigma_w * w, s + p.sigma_h * h, k, b])
                            for r in range(p.R) for s in range(p.S)]
                    out[k, h, w, b] = sum(vals) / (p.R * p.S) if mode == "avg" else max(vals)
    return out
