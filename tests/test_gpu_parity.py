"""GPU parity: the HIP path (through the C ABI) against the fp64 loop-nest oracle, element by element on the same
seeded inputs.  Tolerance (benchmark definition): max|err| / sum|Image*Filter| <= 1e-5 for fp32, <= 1e-2 for bf16
inputs with fp32 accumulation; integer-valued inputs must match exactly."""
import re
import sys

import numpy as np
import pytest

import cacnn_inputs as ci
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_1802_06905_amd as cc
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return cc, torch


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_benchmark_shape_full_array(env, name):
    """The five benchmark shapes at full size, in the launch configuration the benchmark times (planner's choice),
    every output element against the oracle."""
    cc, torch = env
    cfg = ci.CONFIGS[name]
    say(f"[parity] {name} dims={cfg.dims} dtype={cfg.dtype} entry=cacnn_conv_forward")
    img, flt = ci.make_inputs(cfg)
    out = gu.run_gpu(cc, torch, cfg, img, flt)
    ref, ab = gu.oracle_full(cfg, img, flt)
    e = gu.assert_parity(cfg, out, ref, ab, "planner")
    say(f"[parity] {name} max rel err {e:.3e}")


# layers of ordinary networks that the fixed-geometry kernels only take since they mask their Out stores or take strides:
# 13 x 13 outputs with 384 output channels, a strided 1 x 1 layer, a 3 x 3 layer with strides 2, fewer images than a tile
LAYERS = [("bf16", 128, 256, 384, 13, 13, 3, 3, 1, 1), ("bf16", 64, 256, 512, 14, 14, 1, 1, 2, 2),
          ("bf16", 64, 256, 256, 14, 14, 3, 3, 2, 2), ("bf16", 48, 128, 128, 28, 28, 3, 3, 1, 1),
          ("f32", 16, 128, 192, 13, 13, 3, 3, 1, 1), ("f32", 8, 256, 512, 14, 14, 1, 1, 2, 2),
          # filters the kernels compiled for 1 x 1 take one tap at a time: 5 x 5, 1 x 7, fp32 3 x 3 with strides 2
          ("bf16", 64, 96, 128, 13, 13, 5, 5, 1, 1), ("bf16", 32, 128, 128, 17, 17, 1, 7, 1, 1),
          ("f32", 16, 64, 128, 14, 14, 3, 3, 2, 2)]


@pytest.mark.parametrize("layer", LAYERS, ids=["x".join(str(v) for v in l) for l in LAYERS])
def test_whole_layers_on_the_fixed_geometry_kernels(env, layer):
    """Whole layers at ordinary sizes through cacnn_conv_forward: the planner gives them a fixed-geometry kernel, and every
    output element agrees with the oracle (tiles that overhang Out in w, h, k or b; strided staging)."""
    cc, torch = env
    dtype, dims = layer[0], layer[1:]
    cfg = ci.custom("layer", *dims, dtype=dtype, dist="normal", seed=61)
    plan = cc.cacnn_tile_plan(cfg.dims, gu.dtype_code(cfg))
    name = cc.cacnn_variant_name(plan.variant)
    say(f"[parity] layer {layer} planner's kernel '{name}' grid {plan.grid[0]}")
    assert " fx" in name, name
    img, flt = ci.make_inputs(cfg)
    out = gu.run_gpu(cc, torch, cfg, img, flt)
    ref, ab = gu.oracle_full(cfg, img, flt)
    gu.assert_parity(cfg, out, ref, ab, f"layer {layer}")


# shapes that span several tiles with ragged tails in every dimension, strides, asymmetric filters
RAGGED = [
    # name, B, C, K, W, H, R, S, sw, sh
    ("tiny_b1", 1, 3, 8, 16, 16, 3, 3, 1, 1),
    ("ragged_all", 5, 7, 37, 11, 9, 3, 2, 1, 1),
    ("stride_2_3", 3, 5, 33, 9, 7, 5, 4, 2, 3),
    ("stride_gt_filter", 2, 4, 9, 6, 5, 1, 2, 3, 2),
    ("stride_200", 4, 4, 4, 3, 3, 3, 3, 200, 200),       # only a one-position tile's Image range fits the LDS
    ("one_by_one", 9, 19, 40, 5, 6, 1, 1, 1, 1),
    ("matmul", 70, 45, 66, 1, 1, 1, 1, 1, 1),
    ("wide_b", 67, 6, 10, 5, 3, 3, 3, 1, 1),
    ("b_mult8", 16, 24, 70, 9, 10, 3, 3, 1, 1),
    ("c_one", 4, 1, 5, 7, 8, 2, 3, 1, 2),
    ("big_filter", 2, 3, 6, 4, 3, 9, 8, 1, 1),
    ("seven_by_seven", 40, 16, 96, 7, 7, 3, 3, 1, 1),
    # shapes the pipelined persistent kernels accept (16-byte-legal b and c), ragged in k, w, h
    ("pipe_friendly", 64, 24, 70, 9, 5, 3, 3, 1, 1),
    ("pipe_stride", 32, 16, 40, 6, 7, 5, 3, 2, 2),
    ("pipe_many_tiles", 32, 8, 64, 50, 46, 3, 3, 1, 1),      # more tiles than resident workgroups
    ("pipe_resident_filter", 32, 3, 64, 21, 20, 7, 7, 2, 2),  # one Filter tile for the whole grid, odd C
    ("pipe_b8", 8, 16, 64, 13, 12, 3, 3, 1, 1),
    # shapes the fixed-geometry kernels tile exactly (3x3 taps, unit strides), several tiles and several c-slices
    ("fx_w7", 128, 64, 128, 7, 3, 3, 3, 1, 1),
    ("fx_1x1", 64, 96, 128, 14, 4, 1, 1, 1, 1),
    # 1 x 1 filters with strides (2, 3) and (2, 2): the tiles stage the positions their outputs read and nothing between
    ("fx_1x1_strides", 64, 64, 128, 7, 4, 1, 1, 2, 3),
    ("fx_b32_1x1_strides", 32, 32, 64, 14, 5, 1, 1, 2, 2),
    ("fx_b32", 96, 64, 128, 7, 6, 3, 3, 1, 1),
    ("fx_b32_1x1", 32, 96, 64, 14, 2, 1, 1, 1, 1),
    ("fx_w2h2", 64, 96, 192, 4, 6, 3, 3, 1, 1),
    # the bf16 kernels that load the Image straight into LDS mask their Out stores: tiles that overhang Out in w, in h and in
    # k (the second k-tile has 36 channels: one whole 32-row block, then 4 rows of the lanes' first group and none of the second)
    ("fx_overhang", 64, 64, 100, 9, 5, 3, 3, 1, 1),
    ("fx_b32_overhang", 32, 32, 72, 8, 3, 3, 3, 1, 1),
    ("fx_1x1_overhang", 64, 32, 40, 5, 3, 1, 1, 1, 1),
    # ... and in b: 40 images (a 64-image tile's lanes beyond 40 store nothing; the second 32-image tile holds 8), 8 images
    ("fx_b_overhang", 40, 32, 72, 9, 3, 3, 3, 1, 1),
    ("fx_b8_1x1", 8, 32, 64, 7, 2, 1, 1, 1, 1),
    # 3 x 3 filters with strides 2 (the bf16 kernel compiled for them), three tiles along w of which the last overhangs
    ("fx_s2", 64, 64, 128, 5, 6, 3, 3, 2, 2),
    # C a multiple of 8 but not of 32: the instances of the bf16 kernels whose last c-slice is partly filled (48 channels: a
    # whole slice and a half one per filter row; 16 or 8 channels: partly filled slices only; tails of 8 and 24), 3 x 3 and 1 x 1
    ("fx_tail16", 64, 48, 128, 7, 4, 3, 3, 1, 1),
    ("fx_tail16_only", 64, 16, 64, 4, 4, 3, 3, 1, 1),
    ("fx_tail16_1x1", 64, 80, 64, 7, 2, 1, 1, 1, 2),
    ("fx_tail8", 64, 40, 128, 7, 4, 3, 3, 1, 1),
    ("fx_tail8_only", 64, 8, 64, 4, 4, 3, 3, 1, 1),
    ("fx_tail24_1x1", 64, 56, 64, 7, 2, 1, 1, 1, 2),
    # ... and on tiles of 32 images (a chunk holds 16 channels: tails of 8 and 24 end inside one)
    ("fx_b32_tail", 32, 40, 72, 8, 3, 3, 3, 1, 1),
    ("fx_b32_tail_1x1", 96, 24, 64, 14, 2, 1, 1, 1, 1),
    # ... and on 64-channel units (tails of 32, 8 and 56 channels; the last with a 3 x 1 filter, a tap at a time)
    ("fx_c64_tail", 64, 96, 64, 4, 4, 1, 1, 1, 1),
    ("fx_c64_tail8", 64, 72, 64, 4, 2, 1, 1, 2, 1),
    ("fx_c64_tail56", 64, 120, 72, 3, 2, 3, 1, 1, 1),
    # filters other than 1 x 1 on the kernels compiled for 1 x 1 (a unit per tap and c-slice): 5 x 5; 3 x 2 with strides
    # (2, 3) and C = 16 mod 32
    ("fx_taps_5x5", 64, 64, 128, 5, 3, 5, 5, 1, 1),
    ("fx_taps_strides", 64, 48, 64, 5, 4, 3, 2, 2, 3),
    ("fx_w4h4", 64, 32, 128, 8, 12, 3, 3, 1, 1),
    # more tiles than workgroups (a workgroup walks several tiles), and a filter taller than the fixed b_s
    ("fx_many_tiles", 64, 32, 128, 24, 24, 3, 3, 1, 1),
    ("fx_w7_many_tiles", 64, 32, 64, 7, 300, 3, 3, 1, 1),
    ("fx_s6", 64, 32, 64, 4, 4, 3, 6, 1, 1),
    # the fp32 kernel with 16x16 blocks (tiles of 8 images x 2 x 7 positions): two tiles in every dimension and two
    # c-slices; a taller filter with more tiles than workgroups
    ("fx16_two_each", 16, 32, 128, 4, 14, 3, 3, 1, 1),
    ("fx16_1x1", 8, 48, 64, 4, 14, 1, 1, 1, 1),
    # the same kernel with tiles that overhang Out in w (one column of the second tile), h (two rows of seven) and k (36
    # channels in the second k-tile: two waves' sixteen, four of the third wave's first lane group, none of the fourth's)
    ("fx16_overhang", 16, 32, 100, 3, 9, 3, 3, 1, 1),
    ("fx16_1x1_overhang", 8, 32, 72, 3, 9, 1, 1, 1, 1),
    ("fx16_1x1_strides", 8, 32, 64, 4, 9, 1, 1, 2, 3),
    ("fx16_taps", 8, 32, 72, 3, 9, 2, 3, 1, 2),
    # C a multiple of 4 but not of the 16-channel slice: a slice and a half, a quarter slice only, a slice and a quarter with strides
    ("fx16_tail", 8, 24, 64, 4, 14, 3, 3, 1, 1),
    ("fx16_tail_only", 8, 4, 64, 4, 7, 3, 3, 1, 1),
    ("fx16_tail_1x1", 8, 20, 72, 3, 9, 1, 1, 2, 1),
    ("fx16_many_tiles_s6", 8, 16, 64, 46, 42, 3, 6, 1, 1),
    # the stem-layer kernel: 7x7 taps, strides 2, three channels; more tiles than workgroups and three k-tiles, so a
    # workgroup walks several tiles and restages its Filter tile
    ("fx_stem", 32, 3, 192, 28, 16, 7, 7, 2, 2),
    # ... with tiles that overhang Out in w, h, k (72 channels) and b (24 images)
    ("fx_stem_overhang", 24, 3, 72, 27, 15, 7, 7, 2, 2),
]

def is_pipelined(name):
    """Pipelined / wave-specialised variants only accept 16-byte-legal shapes whose slice fits their staging registers;
    fixed-geometry variants only their own contraction tile."""
    return " pipe" in name or " ws" in name or " fx" in name


def variants_for(cc, dtype):
    return [i for i in range(cc.cacnn_variant_count()) if cc.cacnn_variant_name(i).startswith(dtype + " ")]


# the forced contraction tiles; the last two are the ones the fixed-geometry kernels are compiled for
FORCED_TILES = {"f32": ((1 << 20, 1 << 20, 1 << 20), (3, 2, 1), (16, 3, 3), (32, 3, 1), (16, 1, 1)),
                "bf16": ((1 << 20, 1 << 20, 1 << 20), (16, 2, 1), (16, 3, 3), (32, 3, 1), (32, 3, 3), (32, 1, 1), (64, 1, 1))}


def staged_tile_fits(cc, cfg, vi, bc, br, bs):
    """Whether the Image range and the Filter tile that a tile of this variant stages for the forced contraction tile can
    fit the LDS at all (variant names carry the tile as k<KT> b<TB>w<TW>h<TH>)."""
    m = re.search(r" b(\d+)w(\d+)h(\d+)", cc.cacnn_variant_name(vi))
    tb, tw, th = (int(x) for x in m.groups())
    kt = int(re.search(r" k(\d+) ", cc.cacnn_variant_name(vi)).group(1))
    xs = cfg.sigma_w * (tw - 1) + min(br, cfg.R)
    ys = cfg.sigma_h * (th - 1) + min(bs, cfg.S)
    esz = 4 if cfg.dtype == "f32" else 2
    gran = 1 if cfg.dtype == "f32" else 16         # bf16 c-slices are whole 16-channel MFMA steps
    ct = min(-(-bc // gran) * gran, -(-cfg.C // gran) * gran)
    return (xs * ys * tb + kt * min(br, cfg.R) * min(bs, cfg.S)) * ct * esz <= 160 * 1024


def run_every_variant(cc, torch, shape, dtype, ran):
    """Every variant x forced contraction tile on one shape against the oracle; ran[vi] counts the launches that ran."""
    cfg = ci.custom(shape[0], *shape[1:], dtype=dtype, dist="normal", seed=100 + len(shape[0]))
    img, flt = ci.make_inputs(cfg)
    ref, ab = gu.oracle_full(cfg, img, flt)
    for vi in variants_for(cc, dtype):
        for (bc, br, bs) in FORCED_TILES[dtype]:
            plan = cc.Plan()
            plan.variant, plan.b_c, plan.b_r, plan.b_s = vi, bc, br, bs
            say(f"[parity] {shape[0]} {dtype} variant={vi} '{cc.cacnn_variant_name(vi)}' b_c={bc} b_r={br} b_s={bs}")
            try:
                out = gu.run_gpu(cc, torch, cfg, img, flt, plan=plan)
            except cc.CacnnError as e:
                # a forced tile may not fit in LDS, and the pipelined kernels only take 16-byte-legal shapes whose
                # slice fits their staging registers: the library must say so, not launch
                assert e.status == 3 and (bc == 1 << 20 or is_pipelined(cc.cacnn_variant_name(vi)) or
                                          not staged_tile_fits(cc, cfg, vi, bc, br, bs)), (e.status, bc)
                continue
            gu.assert_parity(cfg, out, ref, ab, f"variant {vi} tile ({bc},{br},{bs})")
            ran[vi] = ran.get(vi, 0) + 1


@pytest.mark.parametrize("shape", RAGGED, ids=[s[0] for s in RAGGED])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_every_variant_on_ragged_shapes(env, shape, dtype):
    """Every compiled kernel variant must compute every shape (tiles overhang the arrays in all dimensions), with
    the whole contraction in one tile and with the contraction cut in (c, r, s) tiles."""
    cc, torch = env
    run_every_variant(cc, torch, shape, dtype, {})


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_every_variant_runs_on_some_ragged_shape(env, dtype):
    """No variant is refused everywhere: on a handful of the shapes above (generic, 16-byte-legal, one per
    fixed-geometry family) every variant launches at least once, the generic ones with at least two tilings."""
    cc, torch = env
    ran = {}
    pick = ("ragged_all", "pipe_friendly", "pipe_b8", "fx_w7", "fx_1x1", "fx_1x1_strides", "fx_b32", "fx_b32_1x1", "fx_w2h2", "fx_overhang", "fx_b_overhang", "fx_s2", "fx_tail16", "fx_tail16_1x1", "fx_b32_tail", "fx_b32_tail_1x1", "fx_c64_tail", "fx_w4h4", "fx16_two_each", "fx16_1x1", "fx16_overhang", "fx_stem")
    for shape in RAGGED:
        if shape[0] in pick:
            run_every_variant(cc, torch, shape, dtype, ran)
    for vi in variants_for(cc, dtype):
        name = cc.cacnn_variant_name(vi)
        need = 1 if " fx" in name else 2     # a fixed-geometry kernel accepts one contraction tile only
        assert ran.get(vi, 0) >= need, f"variant {vi} '{name}' ran {ran.get(vi, 0)} times"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_direct_kernels_with_one_to_seven_units_per_workgroup(env, dtype):
    """The staging schedules of the fixed-geometry kernels have separate code for workgroups with one, two, and three
    or more units (tile x contraction slice), different ways out of their loops (odd and even counts) and, in the
    register-staged kernels, a rotation of four or six register sets and buffers: one tile with 1..7 units (with
    3..21 sub-units where an Image unit serves three filter rows), on every such kernel."""
    cc, torch = env
    names = {cc.cacnn_variant_name(i): i for i in variants_for(cc, dtype)}
    fx = [n for n in names if re.search(r" fx(d|d16|r|p\d) ", n)]
    assert len(fx) >= 2
    for name in fx:
        v = names[name]
        tb, tw, th = (int(x) for x in re.search(r" b(\d+)w(\d+)h(\d+) ", name).groups())
        bc, br, bs = (int(x) for x in re.search(r" c(\d+)r(\d+)s(\d+)", name).groups())
        for units in range(1, 8):
            if bs == 3:
                C, S = bc * units, 3          # units c-slices, each with all three filter rows
                if " fxd16 " in name:
                    C -= (0, 4, 8, 12)[units % 4]        # (this kernel takes a partly filled last slice)
            elif name.endswith(" t8"):
                C, S = bc * units - (8, 16, 24)[units % 3], 1     # units c-slices of one filter row, the last one partly filled
            else:
                C, S = bc, units              # one c-slice, units filter rows
            m = re.search(r" s(\d+)$", name)
            stride = int(m.group(1)) if m else 1           # (a kernel compiled for strides 2 says so at the end of its name)
            cfg = ci.custom(f"units{units}", tb, C, 64, tw, th, br, S, stride, stride, dtype=dtype, dist="normal", seed=500 + units)
            img, flt = ci.make_inputs(cfg)
            ref, ab = gu.oracle_full(cfg, img, flt)
            plan = cc.Plan()
            plan.variant, plan.b_c, plan.b_r, plan.b_s = v, bc, br, bs
            say(f"[parity] {units} unit(s) '{name}' dims={cfg.dims}")
            out = gu.run_gpu(cc, torch, cfg, img, flt, plan=plan)
            gu.assert_parity(cfg, out, ref, ab, f"{name}, {units} units")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_integer_inputs_are_exact(env, dtype):
    """Small integers: every product and partial sum is exact in bf16/fp32/fp64, so the result must be bit-exact
    whatever the summation order."""
    cc, torch = env
    cfg = ci.custom("ints", 32, 24, 50, 9, 6, 3, 4, 2, 1, dtype=dtype, dist="smallint", seed=7)
    img, flt = ci.make_inputs(cfg)
    ref, _ = gu.oracle_full(cfg, img, flt)
    say(f"[parity] ints {dtype} planner")
    out = gu.run_gpu(cc, torch, cfg, img, flt)
    assert np.array_equal(out.astype(np.float64), ref)
    for vi in variants_for(cc, dtype):
        plan = cc.Plan()
        plan.variant, plan.b_c, plan.b_r, plan.b_s = vi, 16, 2, 3
        say(f"[parity] ints {dtype} variant={vi}")
        try:
            out = gu.run_gpu(cc, torch, cfg, img, flt, plan=plan)
        except cc.CacnnError as e:
            assert e.status == 3 and is_pipelined(cc.cacnn_variant_name(vi))
            continue
        assert np.array_equal(out.astype(np.float64), ref)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_unaligned_pointers_take_the_scalar_paths(env, dtype):
    cc, torch = env
    cfg = ci.custom("unaligned", 16, 16, 40, 6, 5, 3, 3, 1, 1, dtype=dtype, dist="normal", seed=9)
    img, flt = ci.make_inputs(cfg)
    ref, ab = gu.oracle_full(cfg, img, flt)
    say(f"[parity] unaligned {dtype}")
    out = gu.run_gpu(cc, torch, cfg, img, flt, misalign=1)
    gu.assert_parity(cfg, out, ref, ab, "misaligned by one element")


def test_runs_on_a_side_stream_and_overwrites_out(env):
    cc, torch = env
    cfg = ci.custom("stream", 8, 16, 64, 12, 12, 3, 3, 1, 1, dtype="f32", dist="normal", seed=11)
    img, flt = ci.make_inputs(cfg)
    ref, ab = gu.oracle_full(cfg, img, flt)
    s = torch.cuda.Stream()
    say("[parity] side stream")
    out = gu.run_gpu(cc, torch, cfg, img, flt, stream=s, prefill=123.0)
    gu.assert_parity(cfg, out, ref, ab, "side stream")
    # same launch twice gives identical bits (no atomics, fixed summation order)
    out2 = gu.run_gpu(cc, torch, cfg, img, flt, prefill=-1.0)
    assert np.array_equal(out, out2)


def test_nonfinite_inputs_stay_local(env):
    """An Inf in the Image must reach exactly the outputs whose receptive field holds it (zero-padding inside the
    kernel must not multiply it into other outputs)."""
    cc, torch = env
    for dtype in ("f32", "bf16"):
        cfg = ci.custom("inf", 2, 3, 5, 6, 5, 3, 3, 1, 1, dtype=dtype, dist="normal", seed=13)
        img, flt = ci.make_inputs(cfg)
        img[4, 3, 1, 0] = np.inf
        say(f"[parity] inf {dtype}")
        out = gu.run_gpu(cc, torch, cfg, img, flt)
        bad = ~np.isfinite(out)
        want = np.zeros(cfg.out_shape, bool)
        for w in range(cfg.W):
            for h in range(cfg.H):
                if 0 <= 4 - w < cfg.R and 0 <= 3 - h < cfg.S:
                    want[:, h, w, 0] = True
        assert np.array_equal(bad, want)


def fixed_geometry_case(name):
    """A small shape that a fixed-geometry variant accepts, read off its name
    ('<dtype> fx.. k<KT> b<TB>w<TW>h<TH> ... c<CT>r<BR>s<BS>[ s<stride>]'): two tiles along w and h, two c-slices
    (the stem kernel's three channels are its whole contraction), a filter as high as it is wide."""
    kt = int(re.search(r" k(\d+) ", name).group(1))
    tb, tw, th = (int(x) for x in re.search(r" b(\d+)w(\d+)h(\d+) ", name).groups())
    ct, br, bs = (int(x) for x in re.search(r" c(\d+)r(\d+)s(\d+)", name).groups())
    m = re.search(r" s(\d+)$", name)
    stride = int(m.group(1)) if m else 1
    C = ct if " fxsd " in name else 2 * ct - 24 if name.endswith(" t8") else 2 * ct - 4 if " fxd16 " in name else 2 * ct
    dims = (tb, C, kt, 2 * tw, 2 * th, br, br, stride, stride)
    return dims, (ct, br, bs), (tw, th)


def overhanging(dims, tw, fewer_images):
    """The same shape with the second tile along w one column short, eight output channels more than a k-tile and, for
    the kernels that take it, eight images fewer than a tile."""
    B, C, K, W, H, R, S, sw, sh = dims
    return (B - 8 if fewer_images and B > 8 else B, C, K + 8, 2 * tw - 1, H, R, S, sw, sh)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_nonfinite_inputs_stay_local_in_fixed_geometry_kernels(env, dtype):
    """The fixed-geometry kernels pad inside LDS (odd contraction lengths pair the last index with a zero, the stem
    kernel pairs its missing 22nd slot with the Image row below the window) and stage whole halo planes.  One Inf or
    NaN at a time -- inside a tile, in the last plane and last row of a tile's halo, in the first row below a tile's
    window, in the last channel and image -- must make exactly the outputs non-finite whose receptive field holds it
    (Section 2, Eq. (1)): Out(k,h,w,b) for all k with 0 <= x - sigma_w w < R and 0 <= y - sigma_h h < S."""
    cc, torch = env
    names = {cc.cacnn_variant_name(i): i for i in variants_for(cc, dtype)}
    fx = [n for n in names if " fx" in n]
    assert fx
    cases = [(name, False) for name in fx] + [(name, True) for name in fx if name.startswith(("bf16 fxd ", "f32 fxd16 ", "f32 fxsd "))]
    # (the kernels compiled for 1 x 1 filters on a 2 x 3 filter, which they take one tap at a time, with an overhanging tile)
    cases += [(name, "taps") for name in fx if re.search(r"r1s1( t8)?$", name)]
    for name, ragged in cases:
        dims, (ct, br, bs), (tw, th) = fixed_geometry_case(name)
        if ragged:
            if tw < 2:
                continue
            # (the kernels that mask their Out stores: a tile that overhangs Out)
            dims = overhanging(dims, tw, name.startswith(("bf16 ", "f32 fxsd ")))
        if ragged == "taps":
            dims = dims[:5] + (2, 3) + dims[7:]
        cfg = ci.custom("inf_fx", *dims, dtype=dtype, dist="normal", seed=29)
        img0, flt = ci.make_inputs(cfg)
        assert np.all(flt != 0)
        B, C, K, W, H, R, S, sw, sh = dims
        IW, IH = sw * (W - 1) + R, sh * (H - 1) + S
        spots = [(R, S, 1, 3),                                       # inside the first tile
                 (sw * (tw - 1) + R - 1, sh * (th - 1) + S - 1, C - 1, B - 1),   # last plane, last row of its halo
                 (0, sh * (th - 1) + S, 0, 0),                       # the row directly below the first tile's window
                 (sw * tw, sh * (th - 1) + S, C - 1, 1),             # the same row, second tile along w
                 (IW - 1, IH - 1, 0, B - 1), (0, 0, C - 1, 0)]       # the corners of the Image
        plan = cc.Plan()
        plan.variant, plan.b_c, plan.b_r, plan.b_s = names[name], ct, br, bs
        for n, (x, y, c, b) in enumerate(spots):
            img = img0.copy()
            img[x, y, c, b] = np.inf if n % 2 == 0 else np.nan
            say(f"[parity] non-finite at Image[{x},{y},{c},{b}] '{name}' dims={dims}")
            out = gu.run_gpu(cc, torch, cfg, img, flt, plan=plan)
            want = np.zeros(cfg.out_shape, bool)
            for w in range(W):
                for h in range(H):
                    if 0 <= x - sw * w < R and 0 <= y - sh * h < S:
                        want[:, h, w, b] = True
            assert want.any()
            assert np.array_equal(~np.isfinite(out), want), (name, (x, y, c, b))


def test_error_paths_enqueue_nothing(env):
    cc, torch = env
    cfg = ci.CONFIGS["c1"]
    img, flt = ci.make_inputs(cfg)
    d_img, d_flt = gu.upload(cfg, img, flt, torch)
    d_out = torch.zeros(int(np.prod(cfg.out_shape)), dtype=torch.float32, device="cuda:0")
    with pytest.raises(cc.CacnnError) as e:
        cc.cacnn_conv_forward(cfg.dims, 0, 0, d_flt, d_out)
    assert e.value.status == 1
    with pytest.raises(cc.CacnnError) as e:
        cc.cacnn_conv_forward((1, 3, 8, 16, 0, 3, 3, 1, 1), 0, d_img, d_flt, d_out)
    assert e.value.status == 2
    with pytest.raises(cc.CacnnError) as e:
        cc.cacnn_conv_forward(cfg.dims, 7, d_img, d_flt, d_out)
    assert e.value.status == 3
    plan = cc.Plan()
    plan.variant, plan.b_c, plan.b_r, plan.b_s = 999, 1, 1, 1
    with pytest.raises(cc.CacnnError) as e:
        cc.cacnn_conv_forward_with_plan(cfg.dims, 0, plan, d_img, d_flt, d_out)
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert not d_out.any()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_every_xcd_division_computes_the_same_convolution(env, dtype):
    """Section 7 with the XCDs as processors: the tile order may divide the output channels into 1, 2, 4 or 8 groups.
    and inside a group either the k-tiles of a position tile or the position tiles of a k-tile may be neighbours.
    Every such layout is a permutation of the tile list, so every one must give the oracle's result: on a shape with 8
    k-tiles and several position tiles, for the planner's kernel, a one-tile-per-workgroup one and a fixed-geometry one.  Divisions that do not divide the k-tile count are refused."""
    cc, torch = env
    B, C = (8, 32) if dtype == "f32" else (64, 64)
    cfg = ci.custom("xcd_div", B, C, 512, 8, 4, 3, 3, 1, 1, dtype=dtype, dist="normal", seed=321)
    img, flt = ci.make_inputs(cfg)
    ref, ab = gu.oracle_full(cfg, img, flt)
    base = cc.cacnn_tile_plan(cfg.dims, gu.dtype_code(cfg))
    names = {cc.cacnn_variant_name(i): i for i in variants_for(cc, dtype)}
    picks = {"planner": (base.variant, base.b_c, base.b_r, base.b_s)}
    picks["one tile per workgroup"] = (names[f"{dtype} k64 b8w4h4 w2x2 m1n2"], 16, 3, 3)
    fx = [n for n in names if " fxd " in n and ("b8w4h4" in n or "b64w2h2" in n)]
    assert fx, "no fixed-geometry kernel for this shape"
    picks["fixed"] = (names[fx[0]], 16 if dtype == "f32" else 32, 3, 3 if dtype == "f32" else 1)
    for what, (vi, bc, br, bs) in picks.items():
        for split in (1, 2, 4, 8, 0):
            for walk in ((0,) if split == 0 else (0, 1)):     # walk 1: the position tiles of a k-tile are neighbours
                plan = cc.Plan()
                plan.variant, plan.b_c, plan.b_r, plan.b_s, plan.xcd_split_k, plan.xcd_walk = vi, bc, br, bs, split, walk
                say(f"[xcd division] {dtype} {what} '{cc.cacnn_variant_name(vi)}' a_K={split} walk={walk}")
                out = gu.run_gpu(cc, torch, cfg, img, flt, plan=plan)
                gu.assert_parity(cfg, out, ref, ab, f"{what} a_K={split} walk={walk}")
    plan = cc.Plan()
    plan.variant, plan.b_c, plan.b_r, plan.b_s, plan.xcd_split_k, plan.xcd_walk = base.variant, base.b_c, base.b_r, base.b_s, 2, 2
    with pytest.raises(cc.CacnnError) as e:
        gu.run_gpu(cc, torch, cfg, img, flt, plan=plan)
    assert e.value.status == 2
    for bad in (3, 16, -1):
        plan = cc.Plan()
        plan.variant, plan.b_c, plan.b_r, plan.b_s, plan.xcd_split_k = base.variant, base.b_c, base.b_r, base.b_s, bad
        with pytest.raises(cc.CacnnError) as e:
            gu.run_gpu(cc, torch, cfg, img, flt, plan=plan)
        assert e.value.status == 2
    # an odd number of k-tiles cannot be divided into two groups
    odd = ci.custom("xcd_div_odd", B, C, 192, 4, 4, 3, 3, 1, 1, dtype=dtype, dist="normal", seed=322)
    plan = cc.cacnn_tile_plan(odd.dims, gu.dtype_code(odd))
    assert plan.xcd_split_k == 1
    if (192 // plan.b_k) % 2 == 1:
        plan.xcd_split_k = 2
        i2, f2 = ci.make_inputs(odd)
        with pytest.raises(cc.CacnnError) as e:
            gu.run_gpu(cc, torch, odd, i2, f2, plan=plan)
        assert e.value.status == 2


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_tuned_plan_is_correct(env, dtype):
    """cacnn_tune times every variant that accepts the problem and remembers the fastest: `out` holds a valid result
    afterwards, and later cacnn_conv_forward calls use the remembered plan and still match the oracle.  The two times
    are printed, not asserted: a parity suite must not go red on a noisy clock."""
    cc, torch = env
    cfg = ci.custom("tune", 8, 64, 64, 28, 28, 3, 3, 1, 1, dtype=dtype, dist="normal", seed=77)
    img, flt = ci.make_inputs(cfg)
    ref, ab = gu.oracle_full(cfg, img, flt)
    d_img, d_flt = gu.upload(cfg, img, flt, torch)
    d_out = torch.full((int(np.prod(cfg.out_shape)),), float("nan"), dtype=torch.float32, device="cuda:0")
    dt = gu.dtype_code(cfg)

    def timed():
        for _ in range(20):
            cc.cacnn_conv_forward(cfg.dims, dt, d_img, d_flt, d_out)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(100):
            cc.cacnn_conv_forward(cfg.dims, dt, d_img, d_flt, d_out)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / 100

    planned = cc.cacnn_tile_plan(cfg.dims, dt)
    t_planned = timed()
    tuned = cc.cacnn_tune(cfg.dims, dt, d_img, d_flt, d_out)
    torch.cuda.synchronize()
    gu.assert_parity(cfg, d_out.cpu().numpy().reshape(cfg.out_shape), ref, ab, "out after cacnn_tune")
    say(f"[tune] {dtype}: planned '{cc.cacnn_variant_name(planned.variant)}' {t_planned * 1e3:.1f} us, "
        f"tuned '{cc.cacnn_variant_name(tuned.variant)}' b_c={tuned.b_c} b_r={tuned.b_r} b_s={tuned.b_s}")
    d_out.fill_(float("nan"))
    t_tuned = timed()
    gu.assert_parity(cfg, d_out.cpu().numpy().reshape(cfg.out_shape), ref, ab, "cacnn_conv_forward after cacnn_tune")
    say(f"[tune] {dtype}: tuned plan {t_tuned * 1e3:.1f} us")


def test_launches_can_be_captured_in_a_graph_and_replayed(env):
    """cacnn_conv_forward only enqueues a kernel, so a run of launches can be captured into a HIP graph (what a
    launch-bound caller would do with c1).  Every replay, with eager work and synchronisation between the replays, must
    reproduce the eager result bit for bit."""
    cc, torch = env
    cfg = ci.CONFIGS["c1"]
    img, flt = ci.make_inputs(cfg)
    ref, ab = gu.oracle_full(cfg, img, flt)
    d_img, d_flt = gu.upload(cfg, img, flt, torch)
    n_out = int(np.prod(cfg.out_shape))
    eager = torch.full((n_out,), float("nan"), dtype=torch.float32, device="cuda:0")
    cc.cacnn_conv_forward(cfg.dims, 0, d_img, d_flt, eager)          # also plans and sets the kernel up outside the capture
    torch.cuda.synchronize()
    gu.assert_parity(cfg, eager.cpu().numpy().reshape(cfg.out_shape), ref, ab, "eager")
    outs = [torch.full((n_out,), float("nan"), dtype=torch.float32, device="cuda:0") for _ in range(4)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for o in outs:
                cc.cacnn_conv_forward(cfg.dims, 0, d_img, d_flt, o)
    torch.cuda.synchronize()
    for rep in range(3):
        for o in outs:
            o.fill_(float("nan"))                                    # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, o in enumerate(outs):
            assert torch.equal(o, eager), f"replay {rep}, launch {i}"


def test_planner_picks_on_mid_size_layers(env):
    """cacnn_conv_forward with the planner's own choice on the mid-size and ragged layers the cost model is fitted on
    and judged by (bench.py's two lists): whatever generic kernel and contraction tile the fitted model picks, the
    result is the oracle's."""
    import bench
    cc, torch = env
    picked = set()
    for sh in bench.PLANNER_SHAPES + bench.CALIBRATION_SHAPES:
        dtype, dims = sh[0], sh[1:]
        cfg = ci.custom("mid", *dims, dtype=dtype, dist="normal", seed=21)
        plan = cc.cacnn_tile_plan(dims, 0 if dtype == "f32" else 1)
        vname = cc.cacnn_variant_name(plan.variant)
        say(f"[parity] mid-size {dtype} {dims} -> {vname} [{plan.b_c} {plan.b_r} {plan.b_s}]")
        img, flt = ci.make_inputs(cfg)
        out = gu.run_gpu(cc, torch, cfg, img, flt)
        ref, ab = gu.oracle_full(cfg, img, flt)
        gu.assert_parity(cfg, out, ref, ab, vname)
        picked.add(vname.split()[1] if not vname.split()[1].startswith("k") else "one-tile")
    assert len(picked) >= 3, picked          # the layers exercise several kernel families


def test_planner_path_on_random_shapes(env):
    """Seeded random problems (both dtypes; batch, channel, image and filter sizes from lists that include 1, primes and
    the kernels' tile sizes; strides up to 3) through cacnn_conv_forward with the planner's own choice, against the oracle."""
    import random
    cc, torch = env
    rng = random.Random(20260)
    done, families = 0, set()
    while done < 60:
        dtype = rng.choice(["f32", "bf16"])
        dims = (rng.choice([1, 2, 3, 5, 8, 16, 24, 32, 40, 64, 96, 128]), rng.choice([1, 3, 4, 8, 16, 24, 32, 48, 64, 96, 128, 200, 256]),
                rng.choice([1, 8, 16, 32, 40, 64, 96, 128, 192, 256, 320]), rng.choice([1, 2, 3, 5, 7, 8, 13, 14, 16, 20, 28]),
                rng.choice([1, 2, 3, 5, 7, 8, 13, 14, 16, 20, 28]), rng.choice([1, 1, 2, 3, 3, 3, 5, 7]),
                rng.choice([1, 1, 2, 3, 3, 3, 5, 7]), rng.choice([1, 1, 1, 2, 3]), rng.choice([1, 1, 1, 2, 3]))
        macs = float(np.prod([float(d) for d in dims[:7]]))
        if macs > 6e9 or (done % 2 == 1 and macs < 1e8):      # every other one is a mid-size problem
            continue
        cfg = ci.custom("rnd", *dims, dtype=dtype, dist="normal", seed=3000 + done)
        plan = cc.cacnn_tile_plan(dims, 0 if dtype == "f32" else 1)
        vname = cc.cacnn_variant_name(plan.variant)
        say(f"[parity] random {done} {dtype} {dims} -> {vname} [{plan.b_c} {plan.b_r} {plan.b_s}]")
        img, flt = ci.make_inputs(cfg)
        out = gu.run_gpu(cc, torch, cfg, img, flt)
        ref, ab = gu.oracle_full(cfg, img, flt)
        gu.assert_parity(cfg, out, ref, ab, vname)
        families.add(vname.split()[1] if not vname.split()[1].startswith("k") else "one-tile")
        done += 1
    assert len(families) >= 3, families
