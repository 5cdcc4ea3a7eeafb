"""Python face of the convolution oracle.

TEST INFRASTRUCTURE ONLY.  Two implementations of the paper's Eq. (1) (Section 2, "CNN Model"):

  conv_loops   -- the seven loops literally, in pure Python, fp64 (tiny shapes only);
  conv_fp64    -- the same loop nest in C (conv_fp64.c), fp64, OpenMP over (k,h) (any shape);
  conv_fp64_at -- the same sum for a list of output coordinates, one at a time.

Layouts (reading of the paper, which is silent on storage order): numpy C-order arrays
Image[IW, IH, C, B], Filter[K, R, S, C], Out[K, H, W, B] with IW = sigma_w*(W-1)+R, IH = sigma_h*(H-1)+S.
"""
import ctypes
import os
from typing import NamedTuple, Optional, Tuple

import numpy as np

from . import build as _build


class Problem(NamedTuple):
    """The nine integers of the paper's problem statement (Section 2). W, H are OUTPUT extents."""
    B: int
    C: int
    K: int
    W: int
    H: int
    R: int
    S: int
    sigma_w: int = 1
    sigma_h: int = 1

    @property
    def IW(self) -> int:
        return self.sigma_w * (self.W - 1) + self.R

    @property
    def IH(self) -> int:
        return self.sigma_h * (self.H - 1) + self.S

    @property
    def image_shape(self) -> Tuple[int, int, int, int]:
        return (self.IW, self.IH, self.C, self.B)

    @property
    def filter_shape(self) -> Tuple[int, int, int, int]:
        return (self.K, self.R, self.S, self.C)

    @property
    def out_shape(self) -> Tuple[int, int, int, int]:
        return (self.K, self.H, self.W, self.B)

    @property
    def F(self) -> int:
        """Number of multiply-adds (paper: F = BCKWHRS)."""
        return self.B * self.C * self.K * self.W * self.H * self.R * self.S


class _CProblem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in
                ("B", "C", "K", "W", "H", "R", "S", "sigma_w", "sigma_h")]


_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        lib.oracle_conv_fp64.restype = ctypes.c_int
        lib.oracle_conv_fp64.argtypes = [ctypes.POINTER(_CProblem), ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.oracle_conv_fp64_at.restype = ctypes.c_int
        lib.oracle_conv_fp64_at.argtypes = [ctypes.POINTER(_CProblem), ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the C oracle uses by default (OpenMP's max)."""
    return int(_load().oracle_num_threads())


def _check_inputs(p: Problem, image: np.ndarray, filt: np.ndarray):
    if tuple(image.shape) != p.image_shape:
        raise ValueError(f"image shape {image.shape} != {p.image_shape}")
    if tuple(filt.shape) != p.filter_shape:
        raise ValueError(f"filter shape {filt.shape} != {p.filter_shape}")


def conv_loops(p: Problem, image: np.ndarray, filt: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. (1) as seven Python loops in fp64.  Returns (Out, Abs).  For tiny shapes."""
    _check_inputs(p, image, filt)
    img = np.asarray(image, dtype=np.float64)
    flt = np.asarray(filt, dtype=np.float64)
    out = np.zeros(p.out_shape, dtype=np.float64)
    ab = np.zeros(p.out_shape, dtype=np.float64)
    for b in range(p.B):
        for c in range(p.C):
            for k in range(p.K):
                for w in range(p.W):
                    for h in range(p.H):
                        for r in range(p.R):
                            for s in range(p.S):
                                prod = img[r + p.sigma_w * w, s + p.sigma_h * h, c, b] * flt[k, r, s, c]
                                out[k, h, w, b] += prod
                                ab[k, h, w, b] += abs(prod)
    return out, ab


def conv_fp64(p: Problem, image: np.ndarray, filt: np.ndarray, threads: int = 0,
              want_abs: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Eq. (1) through the C loop nest.  image/filt are float32 arrays (bf16 configs pass bf16-rounded
    values held in float32).  Returns (Out, Abs) as float64 arrays."""
    _check_inputs(p, image, filt)
    img = np.ascontiguousarray(image, dtype=np.float32)
    flt = np.ascontiguousarray(filt, dtype=np.float32)
    out = np.empty(p.out_shape, dtype=np.float64)
    ab = np.empty(p.out_shape, dtype=np.float64) if want_abs else None
    cp = _CProblem(*p)
    rc = _load().oracle_conv_fp64(ctypes.byref(cp), img.ctypes.data, flt.ctypes.data, out.ctypes.data,
                                  ab.ctypes.data if ab is not None else None, int(threads))
    if rc != 0:
        raise ValueError("oracle_conv_fp64 rejected its arguments")
    return out, ab


def conv_fp64_at(p: Problem, image: np.ndarray, filt: np.ndarray,
                 coords: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. (1) for the output coordinates coords[n,4] = (k,h,w,b).  Returns (values, abs) float64[n]."""
    _check_inputs(p, image, filt)
    img = np.ascontiguousarray(image, dtype=np.float32)
    flt = np.ascontiguousarray(filt, dtype=np.float32)
    co = np.ascontiguousarray(coords, dtype=np.int64)
    if co.ndim != 2 or co.shape[1] != 4:
        raise ValueError("coords must be n x 4")
    n = co.shape[0]
    out = np.empty(n, dtype=np.float64)
    ab = np.empty(n, dtype=np.float64)
    cp = _CProblem(*p)
    rc = _load().oracle_conv_fp64_at(ctypes.byref(cp), img.ctypes.data, flt.ctypes.data, co.ctypes.data,
                                     n, out.ctypes.data, ab.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_conv_fp64_at rejected its arguments")
    return out, ab
