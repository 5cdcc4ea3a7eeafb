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
