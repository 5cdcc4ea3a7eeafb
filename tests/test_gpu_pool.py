"""GPU parity of cacnn_pool_forward (Section 6 of the paper, per-channel reading) against the pooling oracle, through
the C ABI.  Max pooling must be bit-exact; average pooling sums nine-ish fp32 terms and divides once, so it is held to
the convolution's fp32 tolerance, 1e-5 of the mean absolute window value."""
import sys

import numpy as np
import pytest

import cacnn_inputs as ci
from oracle import conv as oconv
from oracle import pool as opool

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_1802_06905_amd as cc
    assert torch.cuda.is_available(), "these tests need the GPU"
    return cc, torch


def make_image(p, dtype, seed, dist="uniform"):
    cfg = ci.custom("pool", p.B, p.C, p.K, p.W, p.H, p.R, p.S, p.sigma_w, p.sigma_h, dtype=dtype, dist=dist, seed=seed)
    img, _ = ci.make_inputs(cfg)
    return img


def run_pool(cc, torch, p, dtype, mode, img, misalign=0, stream=None):
    if dtype == "bf16":
        host = torch.from_numpy(ci.bf16_bits(img).view(np.int16).reshape(-1))
    else:
        host = torch.from_numpy(np.ascontiguousarray(img, dtype=np.float32).reshape(-1))
    if misalign:
        buf = torch.zeros(host.numel() + misalign, dtype=host.dtype, device="cuda:0")
        buf[misalign:] = host.to("cuda:0")
        d_img = buf[misalign:]
    else:
        d_img = host.to("cuda:0")
    d_out = torch.full((int(np.prod(p.out_shape)),), float("nan"), dtype=torch.float32, device="cuda:0")
    cc.cacnn_pool_forward(tuple(p), 0 if dtype == "f32" else 1, 0 if mode == "avg" else 1, d_img, d_out, stream=stream)
    torch.cuda.synchronize()
    return d_out.cpu().numpy().reshape(p.out_shape)


def check(p, mode, img, out):
    ref = opool.pool_fp64(p, img, mode)
    if mode == "max":
        assert np.array_equal(out.astype(np.float64), ref)
    else:
        scale = opool.pool_fp64(p, np.abs(img), "avg")
        err = np.abs(out.astype(np.float64) - ref)
        assert np.all(err <= 1e-5 * scale + 0.0), float(np.max(err / np.maximum(scale, 1e-300)))
        assert np.all(out[scale == 0] == 0)


SHAPES = [
    # B, C, K, W, H, R, S, sw, sh
    oconv.Problem(32, 16, 16, 9, 7, 3, 3, 2, 2),      # vector path, several workgroups
    oconv.Problem(8, 24, 24, 11, 6, 3, 2, 1, 1),      # overlapping windows, R != S
    oconv.Problem(5, 7, 7, 6, 9, 2, 3, 2, 1),         # B not a multiple of the vector: scalar path
    oconv.Problem(16, 3, 3, 4, 5, 2, 2, 3, 4),        # strides larger than the window
    oconv.Problem(64, 40, 40, 3, 2, 1, 1, 1, 1),      # 1x1 window: a transposed copy
    oconv.Problem(1, 1, 1, 1, 1, 5, 4, 1, 1),         # one output
]


@pytest.mark.parametrize("p", SHAPES, ids=[f"B{p.B}C{p.C}W{p.W}H{p.H}R{p.R}S{p.S}s{p.sigma_w}{p.sigma_h}" for p in SHAPES])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", ["avg", "max"])
def test_pool_matches_the_oracle(env, p, dtype, mode):
    cc, torch = env
    img = make_image(p, dtype, seed=200 + p.B + p.C)
    say(f"[pool] {tuple(p)} {dtype} {mode}")
    check(p, mode, img, run_pool(cc, torch, p, dtype, mode, img))


@pytest.mark.parametrize("mode", ["avg", "max"])
def test_benchmark_pooling_shape_full_array(env, mode):
    cc, torch = env
    cfg = ci.POOL_CONFIGS["p1"]
    p = oconv.Problem(*cfg.dims)
    img, _ = ci.make_inputs(cfg)
    say(f"[pool] p1 {mode}")
    check(p, mode, img, run_pool(cc, torch, p, cfg.dtype, mode, img))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_unaligned_image_takes_the_scalar_path(env, dtype):
    cc, torch = env
    p = oconv.Problem(16, 8, 8, 5, 4, 3, 3, 1, 1)
    img = make_image(p, dtype, seed=77)
    for mode in ("avg", "max"):
        say(f"[pool] unaligned {dtype} {mode}")
        check(p, mode, img, run_pool(cc, torch, p, dtype, mode, img, misalign=1))


def test_small_integers_average_exactly_and_a_side_stream_works(env):
    cc, torch = env
    p = oconv.Problem(8, 4, 4, 6, 5, 2, 2, 2, 2)       # R*S = 4: the division is exact
    img = make_image(p, "f32", seed=5, dist="smallint")
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    out = run_pool(cc, torch, p, "f32", "avg", img, stream=st)
    assert np.array_equal(out.astype(np.float64), opool.pool_fp64(p, img, "avg"))


def test_infinities_stay_in_their_windows(env):
    cc, torch = env
    p = oconv.Problem(8, 2, 2, 6, 6, 2, 2, 2, 2)       # disjoint windows
    img = make_image(p, "f32", seed=9)
    img[4, 6, 1, 3] = np.inf
    out = run_pool(cc, torch, p, "f32", "max", img)
    bad = ~np.isfinite(out)
    assert bad.sum() == 1 and bad[1, 3, 2, 3]
