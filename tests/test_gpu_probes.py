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


def test_sustained_rates_are_physical(env):
    cc, torch = env
    ops = torch.zeros(4096, dtype=torch.int32, device="cuda:0")
    sink = torch.zeros(65536, dtype=torch.float32, device="cuda:0")
    for dtype, flops, peak in ((0, 4096.0, 157.3e12), (1, 32768.0, 2.5e15)):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            cc.cacnn_probe_mfma(dtype, ops, sink, 400)
        e0.record()
        n = cc.cacnn_probe_mfma(dtype, ops, sink, 400)
        e1.record()
        torch.cuda.synchronize()
        rate = n * flops / (e0.elapsed_time(e1) * 1e-3)
        assert 0.3 * peak < rate < 1.02 * peak, (dtype, rate)
