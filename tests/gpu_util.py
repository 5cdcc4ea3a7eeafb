"""Helpers shared by the GPU parity tests: upload the seeded inputs, call the C-ABI through the binding,
compare with the oracle under the tolerance of the benchmark definition."""
import numpy as np

import cacnn_inputs as ci
from oracle import conv as oconv

TOL = {"f32": 1e-5, "bf16": 1e-2}   # max |err| / sum|Image*Filter| per output element


def upload(cfg, img, flt, torch, device="cuda:0", misalign=0):
    """Device tensors for the library: fp32 as is, bf16 as raw 16-bit patterns.  misalign > 0 places the data
    that many elements into a larger buffer so the pointers are not 16-byte aligned."""
    def put(a):
        if cfg.dtype == "bf16":
            host = torch.from_numpy(ci.bf16_bits(a).view(np.int16).reshape(-1))
        else:
            host = torch.from_numpy(np.ascontiguousarray(a).reshape(-1))
        if misalign:
            buf = torch.zeros(host.numel() + misalign, dtype=host.dtype, device=device)
            buf[misalign:] = host.to(device)
            return buf[misalign:]
        return host.to(device)
    return put(img), put(flt)


def dtype_code(cfg):
    return 0 if cfg.dtype == "f32" else 1


def run_gpu(cc, torch, cfg, img, flt, plan=None, stream=None, misalign=0, prefill=float("nan")):
    d_img, d_flt = upload(cfg, img, flt, torch, misalign=misalign)
    n_out = int(np.prod(cfg.out_shape))
    d_out = torch.full((n_out,), prefill, dtype=torch.float32, device="cuda:0")
    if stream is not None:
        stream.wait_stream(torch.cuda.current_stream())
    if plan is None:
        cc.cacnn_conv_forward(cfg.dims, dtype_code(cfg), d_img, d_flt, d_out, stream=stream)
    else:
        cc.cacnn_conv_forward_with_plan(cfg.dims, dtype_code(cfg), plan, d_img, d_flt, d_out, stream=stream)
    if stream is not None:
        stream.synchronize()
    torch.cuda.synchronize()
    return d_out.cpu().numpy().reshape(cfg.out_shape)


def oracle_full(cfg, img, flt):
    return oconv.conv_fp64(oconv.Problem(*cfg.dims), img, flt)


def rel_err(out_gpu, ref, ab):
    """max over outputs of |gpu - oracle| / sum|Image*Filter|; outputs whose denominator is 0 must be exactly 0."""
    out64 = out_gpu.astype(np.float64)
    if not np.all(np.isfinite(out64)):
        return float("inf")
    zero = ab == 0
    if np.any(out64[zero] != 0):
        return float("inf")
    err = np.abs(out64 - ref)
    return float(np.max(np.where(zero, 0.0, err / np.where(zero, 1.0, ab)))) if err.size else 0.0


def assert_parity(cfg, out_gpu, ref, ab, what=""):
    e = rel_err(out_gpu, ref, ab)
    assert e <= TOL[cfg.dtype], f"{cfg.name} {what}: max|err|/sum|prod| = {e:.3e} > {TOL[cfg.dtype]:.0e}"
    return e
