"""The measurement kernels behind bench.py's machine_sustained figures, through the C ABI: the copy copies, the MFMA
loop computes what its definition says (checked on operands that make every product exact), and both report rates
inside what the hardware can do."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_1802_06905_amd as cc
    assert torch.cuda.is_available(), "these tests need the GPU"
    return cc, torch


def test_copy_probe_copies(env):
    cc, torch = env
    n = (1 << 20) + 16 * 7          # a ragged count of 16-byte words
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros(n + 16, dtype=torch.uint8, device="cuda:0")
    cc.cacnn_probe_copy(src, dst, n)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src) and int(dst[n:].sum()) == 0


@pytest.mark.parametrize("dtype", [0, 1])
def test_mfma_probe_sums_what_it_says(env, dtype):
    """All operands 1: every MFMA adds the contraction length (2 for fp32, 16 for bf16) to each accumulator element;
    a thread owns 7 accumulators x 16 elements and each accumulator receives 3 MFMAs per step, 2 * iters steps."""
    cc, torch = env
    iters = 5
    word = np.float32(1.0).view(np.int32) if dtype == 0 else np.int32(0x3f803f80)
    ops = torch.from_numpy(np.full(4096, word, dtype=np.int32)).cuda()
    sink = torch.zeros(65536, dtype=torch.float32, device="cuda:0")
    n = cc.cacnn_probe_mfma(dtype, ops, sink, iters)
    torch.cuda.synchronize()
    assert n == 256 * 4 * iters * 42
    k = 2 if dtype == 0 else 16
    assert torch.all(sink == float(7 * 16 * 3 * 2 * iters * k))


def test_probe_counts_scale_with_iterations(env):
    """The MFMA count the probe reports (what bench.py divides by the measured time) is linear in the iteration count;
    the rates themselves are reported by bench.py (machine_sustained), not asserted here."""
    cc, torch = env
    ops = torch.zeros(4096, dtype=torch.int32, device="cuda:0")
    sink = torch.zeros(65536, dtype=torch.float32, device="cuda:0")
    for dtype in (0, 1):
        n1 = cc.cacnn_probe_mfma(dtype, ops, sink, 100)
        n4 = cc.cacnn_probe_mfma(dtype, ops, sink, 400)
        torch.cuda.synchronize()
        assert n1 > 0 and n4 == 4 * n1


def test_lds_fill_probe_reads_the_window(env):
    """The LDS-fill loop reports, per thread, one byte of what wave 0 loaded last; with a source whose every byte is its
    chunk number modulo 251 that identifies the chunks, for the shared window and for the divided one.  Bad arguments
    are refused on the host."""
    cc, torch = env
    sink = torch.zeros(65536, dtype=torch.float32, device="cuda:0")
    for window in (1 << 20, 64 << 20):
        chunks = window >> 10
        src = (torch.arange(chunks, device="cuda:0", dtype=torch.int64) % 251).to(torch.uint8).repeat_interleave(1024)
        iters = 3
        moved = cc.cacnn_probe_lds_fill(src, window, sink, iters)
        torch.cuda.synchronize()
        assert moved == 256 * 48 * 1024 * iters
        got = sink.cpu().numpy().reshape(256, 4, 64)          # workgroup, wave, lane
        shared = window < (64 << 20)
        part = chunks if shared else chunks // 256
        step = 48 * 5 + 12 if shared else 48
        # thread t of a workgroup reports LDS byte 16 t: threads 64 q .. 64 q + 63 look into the q-th KiB of wave 0's
        # slots, which holds the q-th chunk of wave 0's last round
        for wg in (0, 1, 17, 255):
            first = ((wg * 53) % chunks) if shared else 0
            first = (first + (iters - 1) * step) % part
            base = 0 if shared else wg * part
            for q in range(4):
                assert np.all(got[wg, q, :] == float((base + (first + q) % part) % 251)), (window, wg, q)
    for bad in (1000, 3 << 20, 1 << 15):
        with pytest.raises((cc.CacnnError, ValueError)):
            cc.cacnn_probe_lds_fill(torch.zeros(4 << 20, dtype=torch.uint8, device="cuda:0"), bad, sink, 1)


def test_mfma_and_fill_probe_sums_and_refuses(env):
    """The combined probe's MFMA half computes what the MFMA probe computes (all-ones operands), with and without the
    fill running next to it; bad arguments are refused on the host."""
    cc, torch = env
    ops = torch.from_numpy(np.full(4096, np.int32(0x3f803f80), dtype=np.int32)).cuda()
    src = torch.zeros(2 << 20, dtype=torch.uint8, device="cuda:0")
    iters = 4
    for fill in (0, 7):
        sink = torch.zeros(65536, dtype=torch.float32, device="cuda:0")
        cc.cacnn_probe_mfma_and_fill(ops, src, 2 << 20, sink, iters, fill)
        torch.cuda.synchronize()
        assert torch.all(sink == float(7 * 16 * 3 * 2 * iters * 16))
    sink = torch.zeros(65536, dtype=torch.float32, device="cuda:0")
    cc.cacnn_probe_mfma_and_fill(ops, src, 2 << 20, sink, 0, 5)      # fill alone: runs, leaves the sink alone
    torch.cuda.synchronize()
    assert float(sink.abs().sum()) == 0.0
    for window, mi, fi in ((3 << 20, 1, 1), (2 << 20, 0, 0), (2 << 20, -1, 1), (64 << 20, 1, 1)):
        with pytest.raises((cc.CacnnError, ValueError)):
            cc.cacnn_probe_mfma_and_fill(ops, torch.zeros(64 << 20, dtype=torch.uint8, device="cuda:0"), window, sink, mi, fi)


def test_mfma_and_fill_probe_on_some_compute_units(env):
    """With fewer workgroups than compute units the probe writes exactly that many workgroups' sums, for both tile
    geometries, with operands in registers and read from the LDS; it refuses counts outside 1 .. 256 and unknown modes."""
    cc, torch = env
    ops = torch.from_numpy(np.full(4096, np.int32(0x3f803f80), dtype=np.int32)).cuda()
    src = torch.zeros(2 << 20, dtype=torch.uint8, device="cuda:0")
    iters = 3
    for tile, blocks in ((0, 7), (1, 4)):
        for cus in (1, 196, 224):
            sink = torch.zeros(65536, dtype=torch.float32, device="cuda:0")
            cc.cacnn_probe_mfma_and_fill_on(cus, tile, 0, ops, src, 2 << 20, sink, iters, 2)
            torch.cuda.synchronize()
            got = sink.reshape(256, 256)
            assert torch.all(got[:cus] == float(blocks * 16 * 3 * 2 * iters * 16))
            assert float(got[cus:].abs().sum()) == 0.0
    for cus in (0, 257, -1):
        with pytest.raises(cc.CacnnError):
            cc.cacnn_probe_mfma_and_fill_on(cus, 0, 0, ops, src, 2 << 20, sink, 1, 1)
    # operands read from the LDS: it starts out as copies of the operand words (bf16 ones) and a window of bf16 ones is
    # filled in, so every fragment read is ones and the sums are the register-only figure, with the fill and without
    ones = torch.from_numpy(np.full(1 << 19, np.int32(0x3f803f80), dtype=np.int32)).cuda()
    # (mode 2 and 3: with a workgroup barrier per iteration, which needs equal iteration counts)
    for tile, blocks in ((0, 7), (1, 4)):
        for mode, fill in ((1, 8), (1, 0), (3, 8), (2, 8)):
            sink = torch.zeros(65536, dtype=torch.float32, device="cuda:0")
            cc.cacnn_probe_mfma_and_fill_on(224, tile, mode, ops, ones, 2 << 20, sink, 8, fill)
            torch.cuda.synchronize()
            assert torch.all(sink.reshape(256, 256)[:224] == float(blocks * 16 * 3 * 2 * 8 * 16))
    for tile, mode, fill in ((0, 4, 1), (2, 0, 1), (-1, 1, 1), (0, 3, 2), (1, 2, 0)):
        with pytest.raises(cc.CacnnError):
            cc.cacnn_probe_mfma_and_fill_on(224, tile, mode, ops, src, 2 << 20, sink, 1, fill)
