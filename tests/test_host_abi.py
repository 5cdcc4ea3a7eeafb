"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares, and its host-only
entry points (lower bound, tile planner) agree with the oracle.  No GPU compute is called here."""
import ctypes
import os
import re
import subprocess
import tempfile

import numpy as np
import pytest

import cacnn_inputs as ci
import paper_1802_06905_amd as cc
from oracle import lower_bound as olb
from oracle import lp_tiling as olp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "cacnn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(cacnn_[a-z_]+)\s*\(", header))
    assert {"cacnn_lower_bound", "cacnn_tile_plan", "cacnn_conv_forward", "cacnn_conv_forward_with_plan",
            "cacnn_status_string", "cacnn_variant_count", "cacnn_variant_name"} <= names
    lib = ctypes.CDLL(cc.library_path())
    for n in names:
        assert hasattr(lib, n), n


def test_struct_sizes_match_the_header():
    src = r'''
    #include <stdio.h>
    #include "cacnn.h"
    int main(void){ printf("%zu %zu %zu %zu %zu %zu %zu %zu\n", sizeof(cacnn_problem), sizeof(cacnn_bound), sizeof(cacnn_machine), sizeof(cacnn_plan), sizeof(cacnn_pool_bound), sizeof(cacnn_division), sizeof(cacnn_machine_l2), sizeof(cacnn_l2_plan)); return 0; }
    '''
    with tempfile.TemporaryDirectory() as d:
        open(os.path.join(d, "t.c"), "w").write(src)
        subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                        "-o", os.path.join(d, "t"), os.path.join(d, "t.c")], check=True)
        sizes = [int(x) for x in subprocess.run([os.path.join(d, "t")], capture_output=True, text=True,
                                                check=True).stdout.split()]
    assert sizes == [ctypes.sizeof(cc.Problem), ctypes.sizeof(cc.Bound), ctypes.sizeof(cc.Machine),
                     ctypes.sizeof(cc.Plan), ctypes.sizeof(cc.PoolBound), ctypes.sizeof(cc.Division),
                     ctypes.sizeof(cc.MachineL2), ctypes.sizeof(cc.L2Plan)]


def test_fastdiv_is_exact_over_its_domain():
    """The kernels divide staged-tile indices by run-time constants with one multiply-high; check the host-made
    magic numbers against plain division for every divisor up to 4096 over the index range an LDS tile can have."""
    src = r'''
    #include <cstdio>
    #include <cstdint>
    #include "cacnn_internal.h"
    int main(){
      for (uint32_t d = 1; d <= 4096; ++d) {
        cacnn::FastDiv f = cacnn::make_fastdiv(d);
        for (uint32_t n = 0; n < 200000; n += (n < 70000 ? 1 : 7)) {
          uint32_t q = f.mul ? (uint32_t)(((uint64_t)n * f.mul) >> 32) : n;
          if (q != n / d) { printf("bad %u %u\n", n, d); return 1; }
        }
      }
      printf("ok\n"); return 0; }
    '''
    with tempfile.TemporaryDirectory() as d:
        open(os.path.join(d, "t.cpp"), "w").write(src)
        subprocess.run(["g++", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "paper_1802_06905_amd", "csrc"),
                        "-o", os.path.join(d, "t"), os.path.join(d, "t.cpp")], check=True)
        out = subprocess.run([os.path.join(d, "t")], capture_output=True, text=True).stdout
    assert out.strip() == "ok"


def test_lower_bound_matches_oracle():
    rng = np.random.default_rng(0)
    for _ in range(200):
        dims = [int(x) for x in rng.integers(1, 300, 7)] + [int(x) for x in rng.integers(1, 5, 2)]
        M = float(rng.integers(1, 100000))
        got = cc.cacnn_lower_bound(dims, M)
        want = olb.lower_bound(*dims, M)
        assert np.allclose(list(got.term), want.terms, rtol=1e-13)
        assert got.bound == pytest.approx(want.bound, rel=1e-13)
        assert got.argmax == want.argmax


def test_lower_bound_alexnet_example():
    dims = (1000, 3, 96, 55, 55, 11, 11, 4, 4)
    b = cc.cacnn_lower_bound(dims, 17424.0)
    assert b.term[4] == pytest.approx(b.term[0]) and b.term[0] == 290400000.0


def test_lower_bound_errors():
    with pytest.raises(cc.CacnnError) as e:
        cc.cacnn_lower_bound((0, 1, 1, 1, 1, 1, 1, 1, 1), 10.0)
    assert e.value.status == 2
    with pytest.raises(cc.CacnnError) as e:
        cc.cacnn_lower_bound((1, 1, 1, 1, 1, 1, 1, 1, 1), 0.0)
    assert e.value.status == 2
    assert cc.cacnn_status_string(0) == "ok" and "unknown" in cc.cacnn_status_string(99)


@pytest.mark.parametrize("name", list(ci.CONFIGS))
def test_plan_paper_block_matches_oracle(name):
    cfg = ci.CONFIGS[name]
    dtype = 0 if cfg.dtype == "f32" else 1
    plan = cc.cacnn_tile_plan(cfg.dims, dtype)
    M = 160 * 1024 / (4 if dtype == 0 else 2)
    want = olp.solve_lp(*cfg.dims, M)
    assert plan.lp_volume == pytest.approx(want.volume, rel=1e-6)
    assert plan.lp_cost_words == pytest.approx(want.cost, rel=1e-6)
    assert plan.bound_words == pytest.approx(olb.lower_bound(*cfg.dims, M).bound, rel=1e-12)
    assert np.prod(list(plan.lp_tile)) == pytest.approx(plan.lp_volume, rel=1e-9)
    if cfg.sigma_w == 1 and cfg.sigma_h == 1:
        label = olp.appendix_a_case(*cfg.dims[:7], M)[0]
        assert str(plan.paper_case) == label.replace(".", "")
    else:
        assert plan.paper_case == 0


def test_plan_appendix_a_leaf_matches_oracle_on_random_shapes():
    rng = np.random.default_rng(4)
    seen = set()
    for _ in range(400):
        R, S = (int(x) for x in rng.integers(1, 6, 2))
        W, H = int(rng.integers(R, 20)), int(rng.integers(S, 20))
        B, C, K = (int(2 ** rng.integers(0, 8)) for _ in range(3))
        lds = int(2 ** rng.integers(11, 18))
        plan = cc.cacnn_tile_plan((B, C, K, W, H, R, S, 1, 1), 0, cc.Machine(lds, 512 * 1024, 256))
        label = olp.appendix_a_case(B, C, K, W, H, R, S, lds / 4)[0]
        assert str(plan.paper_case) == label.replace(".", ""), (B, C, K, W, H, R, S, lds)
        seen.add(label)
    assert len(seen) >= 10, seen


def test_plan_lp_volume_matches_oracle_on_random_shapes():
    rng = np.random.default_rng(1)
    for _ in range(150):
        sw, sh = (int(x) for x in rng.integers(1, 4, 2))
        R, S = int(rng.integers(1, 12)), int(rng.integers(1, 12))
        W, H = int(rng.integers(1, 60)), int(rng.integers(1, 60))
        B, C, K = (int(x) for x in rng.integers(1, 600, 3))
        lds = int(2 ** rng.integers(11, 18))
        mach = cc.Machine(lds, 512 * 1024, 256)
        dtype = int(rng.integers(0, 2))
        try:
            plan = cc.cacnn_tile_plan((B, C, K, W, H, R, S, sw, sh), dtype, mach)
        except cc.CacnnError as e:
            assert e.status == 2          # nothing fits a tiny LDS
            continue
        M = lds / (4 if dtype == 0 else 2)
        want = olp.solve_lp(B, C, K, W, H, R, S, sw, sh, M)
        assert plan.lp_volume == pytest.approx(want.volume, rel=1e-6)


@pytest.mark.parametrize("name", list(ci.CONFIGS))
def test_plan_gpu_block_is_feasible(name):
    cfg = ci.CONFIGS[name]
    dtype = 0 if cfg.dtype == "f32" else 1
    plan = cc.cacnn_tile_plan(cfg.dims, dtype)
    assert 0 <= plan.variant < cc.cacnn_variant_count()
    assert cc.cacnn_variant_name(plan.variant).startswith(cfg.dtype + " ")
    assert 0 < plan.lds_bytes_used <= 160 * 1024
    cdiv = lambda a, b: -(-a // b)
    tiles = cdiv(cfg.K, plan.b_k) * cdiv(cfg.B, plan.b_b) * cdiv(cfg.W, plan.b_w) * cdiv(cfg.H, plan.b_h)
    if any(f in cc.cacnn_variant_name(plan.variant) for f in (" pipe", " ws", " fx")):
        assert 1 <= plan.grid[0] <= min(tiles, 2 * 256)      # persistent workgroups walk the tiles
    else:
        assert plan.grid[0] == tiles
    assert plan.block in (64, 128, 256, 512)
    assert 1 <= plan.b_r <= cfg.R and 1 <= plan.b_s <= cfg.S and plan.b_c >= 1
    assert plan.b_r2 <= cfg.sigma_w and cfg.sigma_w * (plan.b_r1 - 1) + 1 <= plan.b_r
    # the schedule reads at least each input once and writes Out once
    compulsory = np.prod(cfg.image_shape) + np.prod(cfg.filter_shape) + np.prod(cfg.out_shape)
    assert plan.predicted_words >= compulsory
    assert plan.tile_volume == plan.b_b * plan.b_c * plan.b_k * plan.b_w * plan.b_h * plan.b_r * plan.b_s


def test_plan_fills_the_compute_units_on_the_benchmark_shapes():
    """The four large shapes get one tile per workgroup or an even share of many (the machine has 256 compute units),
    and c2's 56 x 56 x 8 outputs are cut into 224 tiles of 2 x 7 positions rather than 196 of 4 x 4."""
    want = {"c2": (224, 2, 7), "c3": (256, 2, 2), "c4": (196, 2, 2), "c5": (224, 7, 1)}
    for name, (grid, bw, bh) in want.items():
        cfg = ci.CONFIGS[name]
        plan = cc.cacnn_tile_plan(cfg.dims, 0 if cfg.dtype == "f32" else 1)
        assert " fx" in cc.cacnn_variant_name(plan.variant), (name, cc.cacnn_variant_name(plan.variant))
        assert (plan.grid[0], plan.b_w, plan.b_h) == (grid, bw, bh), (name, plan.grid[0], plan.b_w, plan.b_h)


def test_plan_errors():
    with pytest.raises(cc.CacnnError) as e:
        cc.cacnn_tile_plan((1, 1, 1, 1, 1, 1, 1, 1, 0), 0)
    assert e.value.status == 2
    with pytest.raises(cc.CacnnError) as e:
        cc.cacnn_tile_plan((1, 1, 1, 1, 1, 1, 1, 1, 1), 5)
    assert e.value.status == 3
    with pytest.raises(cc.CacnnError) as e:
        cc.cacnn_tile_plan((2 ** 20, 2 ** 20, 4, 4, 4, 1, 1, 1, 1), 0)     # Image has more than 2^31 elements
    assert e.value.status == 2
    assert cc.cacnn_variant_name(-1) is None and cc.cacnn_variant_name(10 ** 6) is None


def test_conv_forward_rejects_null_and_bad_arguments_without_a_gpu():
    lib = ctypes.CDLL(cc.library_path())
    lib.cacnn_conv_forward.restype = ctypes.c_int
    lib.cacnn_conv_forward.argtypes = [ctypes.POINTER(cc.Problem), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p, ctypes.c_void_p]
    p = cc.Problem(1, 3, 8, 16, 16, 3, 3, 1, 1)
    assert lib.cacnn_conv_forward(None, 0, 16, 16, 16, None) == 1
    assert lib.cacnn_conv_forward(ctypes.byref(p), 0, None, 16, 16, None) == 1
    assert lib.cacnn_conv_forward(ctypes.byref(p), 9, 16, 16, 16, None) == 3
    bad = cc.Problem(1, 3, 8, 16, 16, 3, 3, 0, 1)
    assert lib.cacnn_conv_forward(ctypes.byref(bad), 0, 16, 16, 16, None) == 2
    assert lib.cacnn_conv_forward(ctypes.byref(p), 0, 18, 16, 16, None) == 2      # pointer not aligned to a float


def test_conv_forward_without_a_gpu_reports_no_device():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    lib = ctypes.CDLL(cc.library_path())
    lib.cacnn_conv_forward.restype = ctypes.c_int
    lib.cacnn_conv_forward.argtypes = [ctypes.POINTER(cc.Problem), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p, ctypes.c_void_p]
    p = cc.Problem(1, 3, 8, 16, 16, 3, 3, 1, 1)
    assert lib.cacnn_conv_forward(ctypes.byref(p), 0, 4096, 8192, 16384, None) == 5   # never dereferenced


def test_pool_bound_matches_the_oracle_and_rejects_bad_arguments():
    from oracle import lower_bound as olb
    for dims, M in (((4, 8, 8, 10, 10, 3, 3, 2, 2), 64.0), ((32, 64, 64, 56, 56, 3, 3, 2, 2), 40960.0),
                    ((2, 3, 3, 5, 4, 2, 5, 4, 1), 7.0)):
        got = cc.cacnn_pool_lower_bound(dims, M)
        ref = olb.pooling_lower_bound(*dims, M)
        assert list(got.term) == pytest.approx(ref.terms, rel=1e-15)
        assert got.bound == pytest.approx(ref.bound, rel=1e-15) and got.argmax == ref.argmax
    with pytest.raises(cc.CacnnError) as e:
        cc.cacnn_pool_lower_bound((4, 8, 8, 10, 10, 3, 3, 2, 0), 64.0)
    assert e.value.status == 2
    with pytest.raises(cc.CacnnError) as e:
        cc.cacnn_pool_lower_bound((4, 8, 8, 10, 10, 3, 3, 2, 2), 0.0)
    assert e.value.status == 2


def test_pool_forward_rejects_bad_arguments_before_touching_the_gpu():
    ok = (2, 4, 4, 3, 3, 2, 2, 1, 1)
    for dims, dtype, mode, img, out, status in (
            (ok, 0, 0, 0, 16, 1),                      # null image
            (ok, 0, 0, 16, 0, 1),                      # null out
            (ok, 7, 0, 16, 16, 3),                     # unknown dtype
            (ok, 0, 5, 16, 16, 3),                     # unknown mode
            ((2, 4, 5, 3, 3, 2, 2, 1, 1), 0, 0, 16, 16, 2),   # K != C
            ((2, 4, 4, 0, 3, 2, 2, 1, 1), 0, 0, 16, 16, 2),   # W < 1
            ((1 << 20, 4, 4, 1 << 10, 3, 2, 2, 1, 1), 0, 0, 16, 16, 2),   # too many elements
            (ok, 0, 0, 18, 16, 2),                     # image pointer not aligned to its element size
    ):
        with pytest.raises(cc.CacnnError) as e:
            cc.cacnn_pool_forward(dims, dtype, mode, img, out, stream=0)
        assert e.value.status == status, (dims, dtype, mode, img, out)


def test_probes_reject_bad_arguments_before_touching_the_gpu():
    for dtype, ops, sink, iters, status in (
            (0, 0, 16, 10, 1),          # null operands
            (0, 16, 0, 10, 1),          # null sink
            (9, 16, 16, 10, 3),         # unknown dtype
            (0, 16, 16, 0, 2),          # iters < 1
            (0, 16, 16, 1 << 25, 2),    # iters too large
            (1, 24, 16, 10, 2),         # operands not 16-byte aligned
    ):
        with pytest.raises(cc.CacnnError) as e:
            cc.cacnn_probe_mfma(dtype, ops, sink, iters, stream=0)
        assert e.value.status == status, (dtype, ops, sink, iters)
    for src, dst, n, status in ((0, 16, 64, 1), (16, 0, 64, 1), (16, 32, 0, 2), (16, 32, 24, 2), (8, 32, 64, 2)):
        with pytest.raises(cc.CacnnError) as e:
            cc.cacnn_probe_copy(src, dst, n, stream=0)
        assert e.value.status == status, (src, dst, n)


def test_unit_mix_probe_rejects_bad_arguments_before_touching_the_gpu():
    """cacnn_probe_mfma_and_fill_on through the raw C ABI with made-up (never dereferenced) pointers: NULLs, compute-unit
    counts outside 1 .. 256, unknown tile and mode, a barrier with unequal iteration counts, windows that are no power of two or out of range, iteration counts."""
    lib = ctypes.CDLL(cc.library_path())
    f = lib.cacnn_probe_mfma_and_fill_on
    f.restype = ctypes.c_int
    f.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                  ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
    ok = dict(cus=224, tile=0, reads=1, ops=4096, src=8192, window=2 << 20, sink=16384, mi=1, fi=1)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["cus"], a["tile"], a["reads"], a["ops"], a["src"], a["window"], a["sink"], a["mi"], a["fi"], None)

    for kw in (dict(ops=None), dict(src=None), dict(sink=None)):
        assert call(**kw) == 1, kw
    for kw in (dict(cus=0), dict(cus=257), dict(tile=2), dict(tile=-1), dict(reads=4), dict(reads=-1), dict(reads=2, mi=1, fi=2),
               dict(reads=3, mi=5, fi=0), dict(window=3 << 20), dict(window=1 << 15),
               dict(window=64 << 20), dict(mi=-1), dict(mi=0, fi=0), dict(fi=(1 << 20) + 1), dict(ops=4100), dict(src=8200)):
        assert call(**kw) == 2, kw
    import torch
    if not torch.cuda.is_available():
        assert call() == 5          # valid arguments, no device: nothing is launched


PAR_SHAPES = [(8, 64, 64, 56, 56, 3, 3, 1, 1), (32, 3, 64, 112, 112, 7, 7, 2, 2), (256, 512, 512, 7, 7, 3, 3, 1, 1),
              (8, 1024, 1024, 7, 7, 3, 3, 1, 1), (1, 3, 8, 16, 16, 3, 3, 1, 1), (4, 5, 6, 7, 8, 3, 2, 4, 1),
              (1, 4, 1, 1, 3, 1, 1, 1, 1)]


@pytest.mark.parametrize("dims", PAR_SHAPES)
def test_parallel_bound_and_work_division_match_the_oracle(dims):
    from oracle import parallel as opar
    for M in (16.0, 40960.0, 1e7):
        for a in ((1, 1, 1, 1), (1, dims[2], 1, 1), (dims[0], 1, dims[3], dims[4])):
            got = cc.cacnn_parallel_bound(dims, M, a)
            ref = opar.parallel_bound(*dims, M, *a)
            assert list(got.term) == ref.terms and got.bound == ref.bound and got.argmax == ref.argmax
        for p in (1, 2, 3, 8, 12, 64, 256):
            a, b = cc.cacnn_work_division(dims, M, p)
            ref = opar.work_division(*dims, M, p)
            assert a == ref.a, (dims, M, p)
            assert list(b.term) == ref.bound.terms and b.bound == ref.bound.bound and b.argmax == ref.bound.argmax


def test_parallel_entry_points_reject_bad_arguments():
    ok = (2, 3, 4, 5, 6, 2, 2, 1, 1)
    for dims, M, a, status in ((ok, 16.0, (3, 1, 1, 1), 2), (ok, 16.0, (1, 1, 0, 1), 2), (ok, 0.0, (1, 1, 1, 1), 2),
                               ((2, 3, 0, 5, 6, 2, 2, 1, 1), 16.0, (1, 1, 1, 1), 2)):
        with pytest.raises(cc.CacnnError) as e:
            cc.cacnn_parallel_bound(dims, M, a)
        assert e.value.status == status
    for p in (0, -3, 4097):
        with pytest.raises(cc.CacnnError) as e:
            cc.cacnn_work_division(ok, 16.0, p)
        assert e.value.status == 2


def test_plan_lays_out_an_xcds_run_by_the_two_level_model():
    # Filter 18.9 MB against an Image of 1.3 MB, 16 k-tiles: every XCD should work on its own output channels, which both
    # a_K = 8 and "position tiles of a k-tile are neighbours" (walk 1) achieve; the k-tiles-fastest order with a_K = 1
    # would fetch the Filter into every L2
    dims = (8, 1024, 1024, 7, 7, 3, 3, 1, 1)
    plan, l2 = cc.cacnn_tile_plan(dims, 1), cc.cacnn_two_level_plan(dims, 1)
    cand = {(l2.cand_a_k[i], l2.cand_walk[i]): l2.cand_words[i] for i in range(l2.n_candidates)}
    assert (plan.xcd_split_k, plan.xcd_walk) in ((8, 0), (1, 1), (2, 1), (4, 1), (8, 1))
    assert cand[(plan.xcd_split_k, plan.xcd_walk)] == min(cand.values()) and cand[(1, 0)] > 2 * min(cand.values())
    # the benchmark shapes are Image-heavy (or have one k-tile): positions only, k-tiles fastest
    for name, cfg in ci.CONFIGS.items():
        p = cc.cacnn_tile_plan(cfg.dims, 0 if cfg.dtype == "f32" else 1)
        assert (p.xcd_split_k, p.xcd_walk) == (1, 0), name
    # a layout given to cacnn_conv_forward_with_plan is validated on the host before anything is launched
    p = cc.cacnn_tile_plan(dims, 1)
    assert p.xcd_walk in (0, 1)


def test_tune_rejects_bad_arguments_and_needs_a_gpu():
    ok = (2, 4, 4, 3, 3, 2, 2, 1, 1)
    for dims, dtype, img, flt, out, status in ((ok, 0, 0, 16, 16, 1), (ok, 0, 16, 0, 16, 1), (ok, 0, 16, 16, 0, 1),
                                               (ok, 5, 16, 16, 16, 3), ((2, 4, 4, 0, 3, 2, 2, 1, 1), 0, 16, 16, 16, 2)):
        with pytest.raises(cc.CacnnError) as e:
            cc.cacnn_tune(dims, dtype, img, flt, out, stream=0)
        assert e.value.status == status, (dims, dtype, img, flt, out)
    import torch
    if not torch.cuda.is_available():
        with pytest.raises(cc.CacnnError) as e:
            cc.cacnn_tune(ok, 0, 16, 32, 48, stream=0)
        assert e.value.status == 5


def _plan_vs_simulator(dims, dtype):
    from oracle import cachesim as cs
    B, C, K, W, H, R, S, sw, sh = dims
    plan = cc.cacnn_tile_plan(dims, dtype)
    tiles = {"b": plan.b_b, "c": plan.b_c, "k": plan.b_k, "w": plan.b_w, "h": plan.b_h,
             "r1": plan.b_r1, "r2": plan.b_r2, "s1": plan.b_s1, "s2": plan.b_s2}
    # the kernels' loop order: Out tiles outermost (one per workgroup), the contraction tiles inside, c fastest
    sim = cs.tiled_schedule_words(*dims, tiles, ("k", "b", "w", "h", "r1", "r2", "s1", "s2", "c"))
    cdiv = lambda a, b: -(-a // b)
    slices = cdiv(R, plan.b_r) * cdiv(S, plan.b_s) * cdiv(C, plan.b_c)
    # both count the same words when no tile stays resident from one outer iteration to the next (two or more
    # contraction tiles per Out tile), the contraction tiles divide R and S, and the staged contiguous Image range has
    # no untouched rows (stride <= the tile's filter extent, or a single output column / row per tile)
    same_model = (slices >= 2 and R % plan.b_r == 0 and S % plan.b_s == 0 and
                  (sw <= plan.b_r or plan.b_w == 1) and (sh <= plan.b_s or plan.b_h == 1) and
                  plan.b_r % min(sw, R) == 0 and plan.b_s % min(sh, S) == 0)
    # a fixed-geometry kernel whose tile overhangs Out stages the tile's whole window (what of it lies inside the Image);
    # the simulator only the rows that the tile's outputs inside Out touch
    if " fx" in cc.cacnn_variant_name(plan.variant) and (W % plan.b_w or H % plan.b_h):
        same_model = False
    return plan, sim, same_model


def test_predicted_words_equal_the_cache_simulator_on_the_plans_tile():
    """cacnn_plan.predicted_words against the oracle's tile-granular simulator run with the plan's integer tile and the
    kernels' loop order: equal wherever the two cost models coincide, never below it elsewhere (the simulator keeps
    a tile resident across outer iterations and counts only touched Image rows; a workgroup restages)."""
    from tests.test_gpu_parity import RAGGED
    cases = [(c.dims, 0 if c.dtype == "f32" else 1) for c in ci.CONFIGS.values()]
    cases += [(tuple(s[1:]), d) for s in RAGGED for d in (0, 1)]
    rng = np.random.default_rng(5)
    for _ in range(40):
        sw, sh = (int(x) for x in rng.integers(1, 4, 2))
        R, S = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        W, H = int(rng.integers(1, 30)), int(rng.integers(1, 30))
        B, C, K = (int(x) for x in rng.integers(1, 200, 3))
        cases.append(((B, C, K, W, H, R, S, sw, sh), int(rng.integers(0, 2))))
    equal = 0
    for dims, dtype in cases:
        plan, sim, same_model = _plan_vs_simulator(dims, dtype)
        assert sim.loads_out == 0 and sim.stores_out == dims[0] * dims[2] * dims[3] * dims[4]   # Out moves once
        if same_model:
            assert plan.predicted_words == sim.total, (dims, dtype, cc.cacnn_variant_name(plan.variant))
            equal += 1
        else:
            assert plan.predicted_words >= sim.total, (dims, dtype)
    assert equal >= 25
    # the four large benchmark shapes: c2, c4, c5 are in the common regime; c3's tile holds the whole contraction, its
    # Filter tile is staged once per workgroup and its Image tiles once each, which is the simulator's Image count
    for name in ("c2", "c4", "c5"):
        cfg = ci.CONFIGS[name]
        assert _plan_vs_simulator(cfg.dims, 0 if cfg.dtype == "f32" else 1)[2], name
    c3 = ci.CONFIGS["c3"]
    plan, sim, _ = _plan_vs_simulator(c3.dims, 0)
    assert plan.predicted_words == sim.loads_image + plan.grid[0] * sim.loads_filter + sim.stores_out


def test_large_strides_get_a_tile_that_fits_or_an_error():
    """Strides far above the filter extent: the planner must not size a tile from wrapped 32-bit extents.  Either an
    error, or a tile whose staged Image range sigma*(b-1)+b_r by sigma*(b-1)+b_s really fits the LDS it reports; the
    launch path (dummy pointers, no GPU here) must agree with the planner instead of reaching a kernel launch."""
    shapes = [(4, 4, 4, 2, 2, 3, 3, s, s) for s in (5, 20, 200, 3000, 5000, 8189, 65536)]
    shapes += [(4, 4, 4, 1, 1, 3, 3, 2 ** 31 - 1, 2 ** 31 - 1), (4, 4, 4, 3, 3, 3, 3, 200, 200),
               (2, 8, 8, 5, 4, 2, 3, 1000, 3), (2, 8, 8, 5, 4, 2, 3, 3, 1000)]
    import torch
    no_gpu = not torch.cuda.is_available()      # with a GPU the dummy pointers below must never reach a launch
    lib = ctypes.CDLL(cc.library_path())
    lib.cacnn_conv_forward.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p]
    for dims in shapes:
        for dtype in (0, 1):
            esz = 4 if dtype == 0 else 2
            try:
                plan = cc.cacnn_tile_plan(dims, dtype)
            except cc.CacnnError as e:
                assert e.status in (2, 3), (dims, e.status)
                continue
            assert 0 < plan.lds_bytes_used <= 160 * 1024, (dims, plan.lds_bytes_used)
            xs = dims[7] * (plan.b_w - 1) + plan.b_r
            ys = dims[8] * (plan.b_h - 1) + plan.b_s
            assert xs * ys * plan.b_c * plan.b_b * esz <= plan.lds_bytes_used, (dims, xs, ys, plan.lds_bytes_used)
            # same decision on the launch path: 16-byte-aligned dummy pointers, no device in the CPU test environment
            if no_gpu:
                prob = cc.Problem(*dims)
                rc = lib.cacnn_conv_forward(ctypes.byref(prob), dtype, 4096, 8192, 16384, None)
                assert rc == 5, (dims, rc, cc.cacnn_status_string(rc))      # past every geometry check: no device


def test_binding_refuses_tensors_that_do_not_fit_the_problem():
    """The binding checks element size and element count of tensor arguments before it hands their addresses over."""
    import torch
    dims = (2, 3, 4, 5, 4, 3, 2, 1, 1)          # Image 7 x 5 x 3 x 2, Filter 4 x 3 x 2 x 3, Out 4 x 4 x 5 x 2
    from paper_1802_06905_amd import binding
    prob = binding.Problem(*dims)
    img, flt, out = torch.zeros(210), torch.zeros(72), torch.zeros(160)
    binding._check_operands("t", prob, 0, img, flt, out)
    binding._check_operands("t", prob, 0, 1234, 5678, out)                 # plain addresses are not checked
    with pytest.raises(ValueError, match="out holds 159"):
        binding._check_operands("t", prob, 0, img, flt, torch.zeros(159))
    with pytest.raises(ValueError, match="image holds"):
        binding._check_operands("t", prob, 0, torch.zeros(209), flt, out)
    with pytest.raises(ValueError, match="2-byte"):
        binding._check_operands("t", prob, 1, img, flt, out)               # bf16 call, fp32 tensors
    with pytest.raises(ValueError, match="4-byte"):
        binding._check_operands("t", prob, 0, img.to(torch.int16), flt, out)
    binding._check_operands("t", prob, 1, img.to(torch.int16), flt.to(torch.bfloat16), out)
    with pytest.raises(ValueError, match="float32"):
        binding._check_operands("t", prob, 0, img, flt, out.to(torch.int32))


def _variant_tile(name):
    kt = int(re.search(r" k(\d+) ", name).group(1))
    tb, tw, th = (int(x) for x in re.search(r" b(\d+)w(\d+)h(\d+)", name).groups())
    return kt, tb, tw, th


def test_two_level_plan_matches_the_oracle():
    """cacnn_two_level_plan: the Section 5 LP and Theorem 1 at M = one L2 equal the oracle's, and the modelled words of
    every candidate layout of an XCD's run equal the oracle's per-processor LRU count on the same launch."""
    from oracle import two_level as tl
    shapes = [(c.dims, 0 if c.dtype == "f32" else 1) for c in ci.CONFIGS.values()]
    shapes += [(ci.DIVISION_CONFIGS["d1"].dims, 1), ((256, 256, 512, 7, 7, 3, 3, 1, 1), 1), ((16, 64, 256, 28, 28, 3, 3, 1, 1), 0),
               ((8, 24, 200, 30, 17, 5, 3, 2, 1), 1), ((3, 5, 33, 9, 7, 5, 4, 2, 3), 0)]
    walked = 0
    for dims, dtype in shapes:
        esz = 4 if dtype == 0 else 2
        plan = cc.cacnn_tile_plan(dims, dtype)
        l2 = cc.cacnn_two_level_plan(dims, dtype)
        M = 4 * 1024 * 1024 / esz
        want = olp.solve_lp(*dims, M)
        assert l2.lp_volume == pytest.approx(want.volume, rel=1e-6)
        assert l2.lp_cost_words == pytest.approx(want.cost, rel=1e-6)
        assert l2.bound_words == pytest.approx(olb.lower_bound(*dims, M).bound, rel=1e-12)
        assert (plan.xcd_split_k, plan.xcd_walk) == (l2.a_k, l2.walk)
        kt, tb, tw, th = _variant_tile(cc.cacnn_variant_name(plan.variant))
        assert (kt, tb, tw, th) == (plan.b_k, plan.b_b, plan.b_w, plan.b_h)
        tiles_b = -(-dims[0] // tb)
        b_group = max(d for d in range(1, max(1, 128 // (tb * esz)) + 1) if tiles_b % d == 0)
        assert l2.n_candidates >= 1
        best = None
        for i in range(l2.n_candidates):
            ak, walk = l2.cand_a_k[i], l2.cand_walk[i]
            rounds, words = tl.launch_rounds(*dims, kt, tb, tw, th, ak, walk, 8, plan.grid[0], b_group)
            model = tl.processor_cache_words(rounds, words, int(M)) + dims[0] * dims[2] * dims[3] * dims[4]
            assert l2.cand_words[i] == model, (dims, ak, walk)
            walked += walk
            if best is None or model < 0.97 * best[0]:
                best = (model, ak, walk)
        assert (l2.a_k, l2.walk) == best[1:] and l2.chosen_words == best[0]
        for nm, lo in (("l2_tile_b", plan.b_b), ("l2_tile_k", plan.b_k), ("l2_tile_w", plan.b_w), ("l2_tile_h", plan.b_h)):
            assert getattr(l2, nm) % lo == 0 and getattr(l2, nm) >= lo
    assert walked > 0
    # a smaller L2 and fewer XCDs are taken as given
    small = cc.cacnn_two_level_plan(ci.CONFIGS["c5"].dims, 1, None, cc.MachineL2(1 << 20, 4, 16))
    assert small.bound_words == pytest.approx(olb.lower_bound(*ci.CONFIGS["c5"].dims, (1 << 20) / 2).bound, rel=1e-12)
    assert all(small.cand_a_k[i] <= 4 for i in range(small.n_candidates))
    with pytest.raises(cc.CacnnError):
        cc.cacnn_two_level_plan(ci.CONFIGS["c5"].dims, 1, None, cc.MachineL2(1 << 20, 3, 16))


def test_plan_variant_reports_the_cost_model_per_variant():
    """cacnn_plan_variant: every variant that accepts a shape comes back as itself with a positive estimate whose terms
    are consistent with the plan (tiles per CU from the grid of Out tiles), and on a shape no fixed-geometry kernel
    takes the planner's choice is the variant with the smallest estimate."""
    dims, dt = (20, 40, 72, 17, 19, 3, 3, 1, 1), 0
    chosen = cc.cacnn_tile_plan(dims, dt)
    best = None
    seen = 0
    for vi in range(cc.cacnn_variant_count()):
        name = cc.cacnn_variant_name(vi)
        try:
            plan, us, terms = cc.cacnn_plan_variant(dims, dt, vi, True)
        except cc.CacnnError as e:
            assert e.status == 3                      # other dtype, or the variant does not take the shape
            continue
        seen += 1
        assert plan.variant == vi and name.startswith("f32 ") and us > 0 and len(terms) == 5
        tiles = (-(-dims[2] // plan.b_k)) * (-(-dims[0] // plan.b_b)) * (-(-dims[3] // plan.b_w)) * (-(-dims[4] // plan.b_h))
        assert terms[0] == -(-tiles // 256) and terms[1] > 0 and terms[3] >= 1
        if best is None or us < best[0]:
            best = (us, vi)
    assert seen >= 10 and best[1] == chosen.variant
    with pytest.raises(cc.CacnnError):
        cc.cacnn_plan_variant(dims, dt, cc.cacnn_variant_count())
    with pytest.raises(cc.CacnnError):
        cc.cacnn_plan_variant((20, 40, 0, 17, 19, 3, 3, 1, 1), dt, 1)


def test_lp_tile_at_l2_and_cache_model_agree_on_the_channel_groups():
    """Two routes to the number of output-channel groups a_K the eight XCDs are divided into: the k-extent of the
    Section 5 LP's tile at M = one L2 (K / l2_tile_k, rounded to the nearest admissible power of two in log distance) and
    the per-XCD cache model's cheapest layout.  On the benchmark shapes and the two Filter-heavy workloads they agree."""
    import math
    for name in ("c2", "c3", "c4", "c5", "d1", "d2"):
        cfg = ci.CONFIGS.get(name) or ci.DIVISION_CONFIGS[name]
        dt = 0 if cfg.dtype == "f32" else 1
        plan, l2 = cc.cacnn_tile_plan(cfg.dims, dt), cc.cacnn_two_level_plan(cfg.dims, dt)
        tiles_k = -(-cfg.K // plan.b_k)
        want = cfg.K / l2.l2_tile_k
        admissible = [a for a in (1, 2, 4, 8) if tiles_k % a == 0]
        from_lp = min(admissible, key=lambda a: abs(math.log(a / want)))
        assert from_lp == l2.a_k, (name, want, l2.a_k)


def test_which_shapes_the_fixed_geometry_kernels_accept():
    """The host's legality rules for the kernels that load the Image straight into LDS, without a GPU: channel counts (bf16:
    multiples of 32, or of 8 on the instances whose last c-slice is zero-filled; fp32: multiples of 4), filters other than
    the one a kernel is compiled for (only the 1 x 1 instances walk taps), strides, image counts."""
    names = {cc.cacnn_variant_name(i): i for i in range(cc.cacnn_variant_count())}

    def accepts(name, dims, dt):
        try:
            plan, _ = cc.cacnn_plan_variant(dims, dt, names[name])
        except cc.CacnnError:
            return False
        assert plan.variant == names[name]
        return True

    w7 = "bf16 fxd k64 b64w7h1 w2x2 m1n7 c32r3s1"
    assert accepts(w7, (64, 64, 64, 14, 14, 3, 3, 1, 1), 1)
    assert not accepts(w7, (64, 48, 64, 14, 14, 3, 3, 1, 1), 1)           # C = 16 mod 32: the t8 instance's
    assert accepts(w7 + " t8", (64, 48, 64, 14, 14, 3, 3, 1, 1), 1)
    assert accepts(w7 + " t8", (64, 8, 64, 14, 14, 3, 3, 1, 1), 1)
    assert not accepts(w7 + " t8", (64, 64, 64, 14, 14, 3, 3, 1, 1), 1)   # ... and not the other way round
    assert not accepts(w7 + " t8", (64, 44, 64, 14, 14, 3, 3, 1, 1), 1)   # 16-byte Filter loads need C % 8 == 0
    assert not accepts(w7, (64, 64, 64, 14, 14, 3, 3, 2, 2), 1)           # compiled for strides 1
    assert not accepts(w7, (64, 64, 64, 14, 14, 5, 5, 1, 1), 1)           # compiled for 3 taps along w
    assert not accepts(w7, (60, 64, 64, 14, 14, 3, 3, 1, 1), 1)           # 16-byte Image loads need B % 8 == 0
    assert accepts(w7, (40, 64, 100, 13, 9, 3, 3, 1, 1), 1)               # overhang in b, k, w, h
    one = "bf16 fxd k64 b64w2h2 w2x2 m1n4 c32r1s1"
    assert accepts(one, (64, 64, 64, 14, 14, 1, 1, 3, 2), 1)              # 1 x 1: any strides
    assert accepts(one, (64, 64, 64, 14, 14, 5, 7, 2, 1), 1)              # ... and any filter, a tap at a time
    assert not accepts("bf16 fxd k64 b64w2h2 w2x2 m1n4 c64r1s1", (64, 96, 64, 14, 14, 1, 1, 1, 1), 1)   # 64-channel units
    assert accepts("bf16 fxd k64 b64w2h2 w2x2 m1n4 c64r1s1 t8", (64, 96, 64, 14, 14, 1, 1, 1, 1), 1)
    assert accepts("bf16 fxd k64 b64w2h2 w2x2 m1n4 c32r3s1 s2", (64, 64, 64, 14, 14, 3, 3, 2, 2), 1)
    assert not accepts("bf16 fxd k64 b64w2h2 w2x2 m1n4 c32r3s1 s2", (64, 64, 64, 14, 14, 3, 3, 2, 1), 1)
    f16 = "f32 fxd16 k64 b8w2h7 w4x1 m1n7 c16r3s3"
    assert accepts(f16, (8, 64, 64, 14, 14, 3, 3, 1, 1), 0)
    assert accepts(f16, (8, 20, 70, 13, 9, 3, 3, 1, 1), 0)                # C a multiple of 4, overhang in k, w, h
    assert not accepts(f16, (8, 18, 64, 14, 14, 3, 3, 1, 1), 0)
    assert not accepts(f16, (12, 64, 64, 14, 14, 3, 3, 1, 1), 0)          # whole 8-image tiles
    assert not accepts(f16, (8, 64, 64, 14, 14, 5, 5, 1, 1), 0)
    assert accepts("f32 fxd16 k64 b8w2h7 w4x1 m1n7 c16r1s1", (8, 64, 64, 14, 14, 5, 5, 2, 3), 0)
    stem = "f32 fxsd k64 b32w2h2 w2x2 m1n2 c3r7s7 s2"
    assert accepts(stem, (32, 3, 64, 112, 112, 7, 7, 2, 2), 0)
    assert accepts(stem, (20, 3, 72, 27, 15, 7, 7, 2, 2), 0)              # overhang in b, k, w, h
    assert not accepts(stem, (32, 4, 64, 112, 112, 7, 7, 2, 2), 0)
    assert not accepts(stem, (32, 3, 64, 112, 112, 7, 7, 1, 1), 0)
    assert not accepts(stem, (30, 3, 64, 112, 112, 7, 7, 2, 2), 0)        # 16-byte Image loads need B % 4 == 0
    # and the planner hands such layers to them
    for dims, dt in (((64, 96, 128, 13, 13, 5, 5, 1, 1), 1), ((64, 40, 120, 28, 28, 3, 3, 1, 1), 1),
                     ((16, 24, 96, 56, 56, 3, 3, 1, 1), 0), ((64, 3, 96, 109, 109, 7, 7, 2, 2), 0)):
        assert " fx" in cc.cacnn_variant_name(cc.cacnn_tile_plan(dims, dt).variant), dims
