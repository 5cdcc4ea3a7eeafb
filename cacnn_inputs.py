"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the convolution itself: only the five benchmark shapes and a
counter-based random generator (splitmix64 -> uniform; Box-Muller -> normal; round-to-nearest-even to
bf16).  Both the CPU oracle and the GPU library are fed the arrays produced here, so the generator cannot
influence parity.

The paper (Section 2) defines the problem by nine integers (B, C, K, W, H, R, S, sigma_w, sigma_h) and uses
no dataset; the shapes below are the synthetic benchmark configurations, with their value distributions.
"""
from typing import Dict, NamedTuple, Tuple

import numpy as np

SEED_BASE = 18020690


class Config(NamedTuple):
    name: str
    B: int
    C: int
    K: int
    W: int          # output width
    H: int          # output height
    R: int          # filter extent paired with w
    S: int          # filter extent paired with h
    sigma_w: int
    sigma_h: int
    dtype: str      # "f32" or "bf16" (bf16 inputs, fp32 accumulate, fp32 Out)
    dist: str       # "uniform" (U[-1,1]) or "normal" (N(0,1)/sqrt(C*R*S))
    seed: int

    @property
    def dims(self) -> Tuple[int, ...]:
        return (self.B, self.C, self.K, self.W, self.H, self.R, self.S, self.sigma_w, self.sigma_h)

    @property
    def IW(self) -> int:
        return self.sigma_w * (self.W - 1) + self.R

    @property
    def IH(self) -> int:
        return self.sigma_h * (self.H - 1) + self.S

    @property
    def image_shape(self):
        return (self.IW, self.IH, self.C, self.B)

    @property
    def filter_shape(self):
        return (self.K, self.R, self.S, self.C)

    @property
    def out_shape(self):
        return (self.K, self.H, self.W, self.B)

    @property
    def macs(self) -> int:
        return self.B * self.C * self.K * self.W * self.H * self.R * self.S


CONFIGS: Dict[str, Config] = {
    "c1": Config("c1", 1, 3, 8, 16, 16, 3, 3, 1, 1, "f32", "uniform", SEED_BASE + 1),
    "c2": Config("c2", 8, 64, 64, 56, 56, 3, 3, 1, 1, "f32", "normal", SEED_BASE + 2),
    "c3": Config("c3", 32, 3, 64, 112, 112, 7, 7, 2, 2, "f32", "uniform", SEED_BASE + 3),
    "c4": Config("c4", 64, 256, 256, 14, 14, 3, 3, 1, 1, "bf16", "normal", SEED_BASE + 4),
    "c5": Config("c5", 256, 512, 512, 7, 7, 3, 3, 1, 1, "bf16", "normal", SEED_BASE + 5),
}


# Pooling workload (the paper's Section 6 names no shape; this is the 3x3 stride-2 pooling that follows a stem layer
# of c3's size): Image 113 x 113 x 64 x 32, Out 64 x 56 x 56 x 32.  The Filter half of make_inputs is unused.
POOL_CONFIGS: Dict[str, Config] = {
    "p1": Config("p1", 32, 64, 64, 56, 56, 3, 3, 2, 2, "f32", "uniform", SEED_BASE + 6),
}

# Work-division workload (Section 7 with the XCDs as processors): a late layer whose Filter (18.9 MB) is larger than
# its Image (10.6 MB), 16 k-tiles.  The paper names no such shape; this is a 3x3 layer of 1024 channels on 7x7 outputs.
DIVISION_CONFIGS: Dict[str, Config] = {
    "d1": Config("d1", 64, 1024, 1024, 7, 7, 3, 3, 1, 1, "bf16", "normal", SEED_BASE + 7),
    # the same layer on four times the images: 448 tiles, more than the compute units hold at once, so an XCD works
    # through its run in two rounds and the order inside the run decides what its L2 still holds in the second
    "d2": Config("d2", 256, 1024, 1024, 7, 7, 3, 3, 1, 1, "bf16", "normal", SEED_BASE + 8),
}


def custom(name, B, C, K, W, H, R, S, sigma_w=1, sigma_h=1, dtype="f32", dist="uniform", seed=1) -> Config:
    """A shape outside the five benchmark ones (edge cases, ragged sizes)."""
    return Config(name, B, C, K, W, H, R, S, sigma_w, sigma_h, dtype, dist, seed)


# ---------------------------------------------------------------------------------------------------------
# counter-based generator
_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(counter: np.ndarray, seed: int) -> np.ndarray:
    """splitmix64 output function applied to (seed + (counter+1)*golden): one 64-bit word per counter."""
    with np.errstate(over="ignore"):
        z = (np.uint64(seed) + (counter.astype(np.uint64) + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15)) & _MASK
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _MASK
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _MASK
        z = z ^ (z >> np.uint64(31))
    return z


def _unit(counter: np.ndarray, seed: int) -> np.ndarray:
    """Uniform doubles in (0,1): top 53 bits, offset by half an ulp so 0 never occurs."""
    return ((_splitmix64(counter, seed) >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def uniform_pm1(n: int, seed: int) -> np.ndarray:
    """n values uniform in (-1,1), float64."""
    return 2.0 * _unit(np.arange(n, dtype=np.uint64), seed) - 1.0


def normal01(n: int, seed: int) -> np.ndarray:
    """n standard normal values (Box-Muller on two independent counter streams), float64."""
    idx = np.arange(n, dtype=np.uint64)
    u1 = _unit(idx * np.uint64(2), seed)
    u2 = _unit(idx * np.uint64(2) + np.uint64(1), seed)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result is float32 holding bf16 values."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already exactly representable in bf16."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    if np.any(bits & np.uint32(0xFFFF)):
        raise ValueError("values are not bf16-representable")
    return (bits >> np.uint32(16)).astype(np.uint16)


def make_inputs(cfg: Config) -> Tuple[np.ndarray, np.ndarray]:
    """(Image, Filter) as float32 arrays of cfg.image_shape / cfg.filter_shape.  For dtype 'bf16' the values
    are already rounded to bf16 (held in float32), so the oracle and the GPU see identical numbers."""
    n_img = int(np.prod(cfg.image_shape))
    n_flt = int(np.prod(cfg.filter_shape))
    if cfg.dist == "uniform":
        img = uniform_pm1(n_img, cfg.seed)
        flt = uniform_pm1(n_flt, cfg.seed ^ 0x5DEECE66D)
    elif cfg.dist == "normal":
        scale = 1.0 / np.sqrt(cfg.C * cfg.R * cfg.S)
        img = normal01(n_img, cfg.seed) * scale
        flt = normal01(n_flt, cfg.seed ^ 0x5DEECE66D) * scale
    elif cfg.dist == "smallint":
        # small integers: every product and partial sum is exact in fp32, bf16 and fp64
        img = np.floor(uniform_pm1(n_img, cfg.seed) * 4.0)
        flt = np.floor(uniform_pm1(n_flt, cfg.seed ^ 0x5DEECE66D) * 4.0)
    else:
        raise ValueError(cfg.dist)
    img = img.astype(np.float32).reshape(cfg.image_shape)
    flt = flt.astype(np.float32).reshape(cfg.filter_shape)
    if cfg.dtype == "bf16":
        img = round_to_bf16(img)
        flt = round_to_bf16(flt)
    return img, flt
