"""ctypes binding with the same names as the C entry points declared in include/cacnn.h.

The shared library must have been built in-tree (python paper_1802_06905_amd/build.py); importing this module without
it raises: there is no CPU fallback.
"""
import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcacnn.so")

CACNN_F32 = 0
CACNN_BF16_F32ACC = 1


class CacnnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {cacnn_status_string(status)} (status {status})")


class Problem(ctypes.Structure):
    """cacnn_problem: B, C, K, W, H (output extents), R, S, sigma_w, sigma_h."""
    _fields_ = [(n, ctypes.c_int64) for n in ("B", "C", "K", "W", "H", "R", "S", "sigma_w", "sigma_h")]

    @property
    def IW(self):
        return self.sigma_w * (self.W - 1) + self.R

    @property
    def IH(self):
        return self.sigma_h * (self.H - 1) + self.S


class Bound(ctypes.Structure):
    _fields_ = [("term", ctypes.c_double * 5), ("bound", ctypes.c_double), ("argmax", ctypes.c_int32)]


class PoolBound(ctypes.Structure):
    _fields_ = [("term", ctypes.c_double * 3), ("bound", ctypes.c_double), ("argmax", ctypes.c_int32)]


CACNN_POOL_AVG = 0
CACNN_POOL_MAX = 1


class Machine(ctypes.Structure):
    _fields_ = [("lds_bytes", ctypes.c_int64), ("vgpr_bytes_per_cu", ctypes.c_int64), ("num_cu", ctypes.c_int64)]


class Plan(ctypes.Structure):
    _fields_ = [
        ("lp_tile", ctypes.c_double * 9), ("lp_volume", ctypes.c_double), ("lp_cost_words", ctypes.c_double),
        ("bound_words", ctypes.c_double), ("paper_case", ctypes.c_int32),
        ("variant", ctypes.c_int32),
        ("b_b", ctypes.c_int32), ("b_c", ctypes.c_int32), ("b_k", ctypes.c_int32), ("b_w", ctypes.c_int32),
        ("b_h", ctypes.c_int32),
        ("b_r1", ctypes.c_int32), ("b_r2", ctypes.c_int32), ("b_s1", ctypes.c_int32), ("b_s2", ctypes.c_int32),
        ("b_r", ctypes.c_int32), ("b_s", ctypes.c_int32),
        ("grid", ctypes.c_int32 * 3), ("block", ctypes.c_int32),
        ("lds_bytes_used", ctypes.c_int64),
        ("tile_volume", ctypes.c_double), ("predicted_words", ctypes.c_double),
        ("xcd_split_k", ctypes.c_int32),
        ("xcd_walk", ctypes.c_int32),
    ]


class MachineL2(ctypes.Structure):
    _fields_ = [("l2_bytes", ctypes.c_int64), ("n_xcd", ctypes.c_int32), ("cu_per_xcd", ctypes.c_int32)]


class L2Plan(ctypes.Structure):
    _fields_ = [
        ("lp_tile", ctypes.c_double * 9), ("lp_volume", ctypes.c_double), ("lp_cost_words", ctypes.c_double),
        ("bound_words", ctypes.c_double),
        ("l2_tile_b", ctypes.c_int32), ("l2_tile_k", ctypes.c_int32), ("l2_tile_w", ctypes.c_int32),
        ("l2_tile_h", ctypes.c_int32),
        ("a_k", ctypes.c_int32), ("walk", ctypes.c_int32), ("n_candidates", ctypes.c_int32),
        ("cand_a_k", ctypes.c_int32 * 8), ("cand_walk", ctypes.c_int32 * 8), ("cand_words", ctypes.c_double * 8),
        ("chosen_words", ctypes.c_double), ("parallel_bound_words", ctypes.c_double),
    ]


class ClosedForm(ctypes.Structure):
    _fields_ = [
        ("region", ctypes.c_int32), ("n_regions", ctypes.c_int32), ("theta", ctypes.c_double * 9),
        ("l", ctypes.c_double * 9), ("tile", ctypes.c_double * 9), ("log_volume", ctypes.c_double),
        ("volume", ctypes.c_double), ("cost_words", ctypes.c_double), ("bound_words", ctypes.c_double),
        ("worst_violation", ctypes.c_double),
    ]


class Division(ctypes.Structure):
    _fields_ = [("a_b", ctypes.c_int32), ("a_k", ctypes.c_int32), ("a_w", ctypes.c_int32), ("a_h", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python paper_1802_06905_amd/build.py` "
                      "(there is no CPU fallback)")

# PyTorch owns the device memory and the streams handed to this library, so both must talk to the SAME HIP runtime:
# import torch first, so that its copy of libamdhip64 (same SONAME) is the one the loader binds libcacnn.so to.
import torch  # noqa: E402,F401

_lib = ctypes.CDLL(_LIB_PATH)
_lib.cacnn_lower_bound.restype = ctypes.c_int
_lib.cacnn_lower_bound.argtypes = [ctypes.POINTER(Problem), ctypes.c_double, ctypes.POINTER(Bound)]
_lib.cacnn_tile_plan.restype = ctypes.c_int
_lib.cacnn_tile_plan.argtypes = [ctypes.POINTER(Problem), ctypes.c_int, ctypes.POINTER(Machine), ctypes.POINTER(Plan)]
_lib.cacnn_conv_forward.restype = ctypes.c_int
_lib.cacnn_conv_forward.argtypes = [ctypes.POINTER(Problem), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_void_p]
_lib.cacnn_conv_forward_with_plan.restype = ctypes.c_int
_lib.cacnn_conv_forward_with_plan.argtypes = [ctypes.POINTER(Problem), ctypes.c_int, ctypes.POINTER(Plan),
                                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
_lib.cacnn_tune.restype = ctypes.c_int
_lib.cacnn_tune.argtypes = [ctypes.POINTER(Problem), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                            ctypes.c_void_p, ctypes.POINTER(Plan)]
_lib.cacnn_parallel_bound.restype = ctypes.c_int
_lib.cacnn_parallel_bound.argtypes = [ctypes.POINTER(Problem), ctypes.c_double, ctypes.POINTER(Division),
                                      ctypes.POINTER(Bound)]
_lib.cacnn_work_division.restype = ctypes.c_int
_lib.cacnn_work_division.argtypes = [ctypes.POINTER(Problem), ctypes.c_double, ctypes.c_int32, ctypes.POINTER(Division),
                                     ctypes.POINTER(Bound)]
_lib.cacnn_closed_form_tiling.restype = ctypes.c_int
_lib.cacnn_closed_form_tiling.argtypes = [ctypes.POINTER(Problem), ctypes.c_double, ctypes.POINTER(ClosedForm)]
_lib.cacnn_plan_variant.restype = ctypes.c_int
_lib.cacnn_plan_variant.argtypes = [ctypes.POINTER(Problem), ctypes.c_int, ctypes.c_int, ctypes.POINTER(Plan),
                                    ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
_lib.cacnn_two_level_plan.restype = ctypes.c_int
_lib.cacnn_two_level_plan.argtypes = [ctypes.POINTER(Problem), ctypes.c_int, ctypes.POINTER(Machine), ctypes.POINTER(MachineL2),
                                      ctypes.POINTER(L2Plan)]
_lib.cacnn_pool_lower_bound.restype = ctypes.c_int
_lib.cacnn_pool_lower_bound.argtypes = [ctypes.POINTER(Problem), ctypes.c_double, ctypes.POINTER(PoolBound)]
_lib.cacnn_pool_forward.restype = ctypes.c_int
_lib.cacnn_pool_forward.argtypes = [ctypes.POINTER(Problem), ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_void_p]
_lib.cacnn_probe_mfma.restype = ctypes.c_int
_lib.cacnn_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                  ctypes.POINTER(ctypes.c_int64), ctypes.c_void_p]
_lib.cacnn_probe_lds_fill.restype = ctypes.c_int
_lib.cacnn_probe_lds_fill.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p,
                                      ctypes.POINTER(ctypes.c_int64)]
_lib.cacnn_probe_mfma_and_fill.restype = ctypes.c_int
_lib.cacnn_probe_mfma_and_fill.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int32,
                                           ctypes.c_int32, ctypes.c_void_p]
_lib.cacnn_probe_mfma_and_fill_on.restype = ctypes.c_int
_lib.cacnn_probe_mfma_and_fill_on.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
_lib.cacnn_probe_copy.restype = ctypes.c_int
_lib.cacnn_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.cacnn_variant_count.restype = ctypes.c_int
_lib.cacnn_variant_name.restype = ctypes.c_char_p
_lib.cacnn_variant_name.argtypes = [ctypes.c_int]
_lib.cacnn_status_string.restype = ctypes.c_char_p
_lib.cacnn_status_string.argtypes = [ctypes.c_int]


def cacnn_status_string(status: int) -> str:
    return _lib.cacnn_status_string(int(status)).decode()


def cacnn_variant_count() -> int:
    return int(_lib.cacnn_variant_count())


def cacnn_variant_name(i: int) -> Optional[str]:
    s = _lib.cacnn_variant_name(int(i))
    return s.decode() if s is not None else None


def _as_problem(problem) -> Problem:
    if isinstance(problem, Problem):
        return problem
    return Problem(*[int(x) for x in problem])


def cacnn_lower_bound(problem, M_words: float) -> Bound:
    """Theorem 1's five terms and their maximum for a cache of M_words words (host only)."""
    out = Bound()
    rc = _lib.cacnn_lower_bound(ctypes.byref(_as_problem(problem)), float(M_words), ctypes.byref(out))
    if rc != 0:
        raise CacnnError(rc, "cacnn_lower_bound")
    return out


def cacnn_tile_plan(problem, dtype: int, machine: Optional[Machine] = None) -> Plan:
    """The paper's tiling LP and the gfx950 tiling the kernel is launched with (host only)."""
    out = Plan()
    rc = _lib.cacnn_tile_plan(ctypes.byref(_as_problem(problem)), int(dtype),
                              ctypes.byref(machine) if machine is not None else None, ctypes.byref(out))
    if rc != 0:
        raise CacnnError(rc, "cacnn_tile_plan")
    return out


def _ptr(t) -> int:
    """Device address of a torch tensor (or a plain int address)."""
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("cacnn_conv_forward takes device tensors")
    if not t.is_contiguous():
        raise ValueError("cacnn_conv_forward takes contiguous tensors")
    return t.data_ptr()


def _check_operands(where: str, problem: Problem, dtype: int, image, filt, out, pooling: bool = False) -> None:
    """Refuse tensors that are too small or of the wrong element size for the problem: the library trusts its pointers,
    so an undersized Out would become an out-of-bounds device write.  Plain integer addresses are taken as they are."""
    if int(dtype) not in (CACNN_F32, CACNN_BF16_F32ACC) or min(getattr(problem, n) for n, _ in Problem._fields_) < 1:
        return                                  # the library reports these itself
    esz = 4 if int(dtype) == CACNN_F32 else 2
    need = (("image", image, problem.IW * problem.IH * problem.C * problem.B, esz),
            ("filter", filt, problem.K * problem.R * problem.S * problem.C, esz),
            ("out", out, (problem.C if pooling else problem.K) * problem.H * problem.W * problem.B, 4))
    for name, t, numel, size in need:
        if t is None or isinstance(t, int):
            continue
        if t.element_size() != size:
            raise ValueError(f"{where}: {name} has {t.element_size()}-byte elements, the call needs {size}-byte ones")
        if name == "out" and not t.dtype.is_floating_point:
            raise ValueError(f"{where}: out must be a float32 tensor")
        if t.numel() < numel:
            raise ValueError(f"{where}: {name} holds {t.numel()} elements, the problem needs {numel}")


def _stream_handle(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def cacnn_conv_forward(problem, dtype: int, image, filt, out, stream=None) -> None:
    """Enqueue Out = conv(Image, Filter) on `stream` (torch stream, raw handle, or None = torch's current stream).
    image/filt/out are device tensors laid out Image[IW,IH,C,B], Filter[K,R,S,C], Out[K,H,W,B] (fp32)."""
    prob = _as_problem(problem)
    _check_operands("cacnn_conv_forward", prob, dtype, image, filt, out)
    rc = _lib.cacnn_conv_forward(ctypes.byref(prob), int(dtype), _ptr(image), _ptr(filt), _ptr(out),
                                 _stream_handle(stream))
    if rc != 0:
        raise CacnnError(rc, "cacnn_conv_forward")


def cacnn_tune(problem, dtype: int, image, filt, out, stream=None) -> Plan:
    """Time every kernel variant that accepts the problem on these buffers (synchronises), remember and return the fastest."""
    plan = Plan()
    _check_operands("cacnn_tune", _as_problem(problem), dtype, image, filt, out)
    rc = _lib.cacnn_tune(ctypes.byref(_as_problem(problem)), int(dtype), _ptr(image), _ptr(filt), _ptr(out),
                         _stream_handle(stream), ctypes.byref(plan))
    if rc != 0:
        raise CacnnError(rc, "cacnn_tune")
    return plan


def cacnn_parallel_bound(problem, M_words: float, a) -> Bound:
    """Section 7: the five terms for the division a = (a_B, a_K, a_W, a_H) (host only)."""
    out = Bound()
    div = a if isinstance(a, Division) else Division(*[int(x) for x in a])
    rc = _lib.cacnn_parallel_bound(ctypes.byref(_as_problem(problem)), float(M_words), ctypes.byref(div), ctypes.byref(out))
    if rc != 0:
        raise CacnnError(rc, "cacnn_parallel_bound")
    return out


def cacnn_work_division(problem, M_words: float, p: int):
    """Section 7: ((a_B, a_K, a_W, a_H), Bound) for p processors (host only)."""
    div, out = Division(), Bound()
    rc = _lib.cacnn_work_division(ctypes.byref(_as_problem(problem)), float(M_words), int(p), ctypes.byref(div),
                                  ctypes.byref(out))
    if rc != 0:
        raise CacnnError(rc, "cacnn_work_division")
    return (div.a_b, div.a_k, div.a_w, div.a_h), out


def cacnn_two_level_plan(problem, dtype: int, machine: Optional[Machine] = None,
                         machine_l2: Optional[MachineL2] = None) -> L2Plan:
    """The Section 5 LP at M = one L2, and the layout of an XCD's run of tiles the two-level model prefers (host only)."""
    out = L2Plan()
    rc = _lib.cacnn_two_level_plan(ctypes.byref(_as_problem(problem)), int(dtype),
                                   ctypes.byref(machine) if machine is not None else None,
                                   ctypes.byref(machine_l2) if machine_l2 is not None else None, ctypes.byref(out))
    if rc != 0:
        raise CacnnError(rc, "cacnn_two_level_plan")
    return out


def cacnn_plan_variant(problem, dtype: int, variant: int, with_terms: bool = False):
    """(plan, model_us[, terms]): the plan if `variant` were the only kernel, the cost model's time estimate and, on
    request, its five terms (host only)."""
    out = Plan()
    us = ctypes.c_double(0.0)
    terms = (ctypes.c_double * 5)()
    rc = _lib.cacnn_plan_variant(ctypes.byref(_as_problem(problem)), int(dtype), int(variant), ctypes.byref(out),
                                 ctypes.byref(us), terms)
    if rc != 0:
        raise CacnnError(rc, "cacnn_plan_variant")
    return (out, us.value, list(terms)) if with_terms else (out, us.value)


def cacnn_closed_form_tiling(problem, M_words: float) -> ClosedForm:
    """The optimal tile logs of the Section 5 LP from the tabulated closed form of Section 5.1 (host only, no LP solve)."""
    out = ClosedForm()
    rc = _lib.cacnn_closed_form_tiling(ctypes.byref(_as_problem(problem)), float(M_words), ctypes.byref(out))
    if rc != 0:
        raise CacnnError(rc, "cacnn_closed_form_tiling")
    return out


def cacnn_pool_lower_bound(problem, M_words: float) -> PoolBound:
    """The three terms of the pooling bound and their maximum (host only)."""
    out = PoolBound()
    rc = _lib.cacnn_pool_lower_bound(ctypes.byref(_as_problem(problem)), float(M_words), ctypes.byref(out))
    if rc != 0:
        raise CacnnError(rc, "cacnn_pool_lower_bound")
    return out


def cacnn_pool_forward(problem, dtype: int, mode: int, image, out, stream=None) -> None:
    """Enqueue per-channel average (mode 0) or max (mode 1) pooling of Image[IW,IH,C,B] into Out[K=C,H,W,B] (fp32)."""
    _check_operands("cacnn_pool_forward", _as_problem(problem), dtype, image, None, out, pooling=True)
    rc = _lib.cacnn_pool_forward(ctypes.byref(_as_problem(problem)), int(dtype), int(mode), _ptr(image), _ptr(out),
                                 _stream_handle(stream))
    if rc != 0:
        raise CacnnError(rc, "cacnn_pool_forward")


def cacnn_probe_mfma(dtype: int, operands, sink, iters: int, stream=None) -> int:
    """Enqueue the register-only MFMA loop (operands: 16 KiB device tensor, sink: 65536 fp32); returns the MFMAs issued."""
    n = ctypes.c_int64(0)
    rc = _lib.cacnn_probe_mfma(int(dtype), _ptr(operands), _ptr(sink), int(iters), ctypes.byref(n), _stream_handle(stream))
    if rc != 0:
        raise CacnnError(rc, "cacnn_probe_mfma")
    return n.value


def cacnn_probe_copy(src, dst, nbytes: int, stream=None) -> None:
    """Enqueue the streaming copy dst[0..nbytes) = src[0..nbytes) (device tensors)."""
    rc = _lib.cacnn_probe_copy(_ptr(src), _ptr(dst), int(nbytes), _stream_handle(stream))
    if rc != 0:
        raise CacnnError(rc, "cacnn_probe_copy")


def cacnn_probe_lds_fill(src, window_bytes: int, sink, iters: int, stream=None) -> int:
    """Enqueue the LDS-fill loop on every CU over the first window_bytes of src; returns the bytes the launch moves."""
    if src.numel() * src.element_size() < int(window_bytes) or sink.numel() * sink.element_size() < 65536 * 4:
        raise ValueError("cacnn_probe_lds_fill: src shorter than the window, or sink shorter than 65536 floats")
    n = ctypes.c_int64(0)
    rc = _lib.cacnn_probe_lds_fill(_ptr(src), int(window_bytes), _ptr(sink), int(iters), _stream_handle(stream), ctypes.byref(n))
    if rc != 0:
        raise CacnnError(rc, "cacnn_probe_lds_fill")
    return n.value


def cacnn_probe_mfma_and_fill(operands, src, window_bytes: int, sink, mfma_iters: int, fill_iters: int, stream=None) -> None:
    """Enqueue the bf16 MFMA loop and the LDS fill side by side on every CU (either iteration count may be 0)."""
    if operands.numel() * operands.element_size() < 16384 or src.numel() * src.element_size() < int(window_bytes) or \
            sink.numel() * sink.element_size() < 65536 * 4:
        raise ValueError("cacnn_probe_mfma_and_fill: operands (16 KiB), src (the window) or sink (65536 floats) too short")
    rc = _lib.cacnn_probe_mfma_and_fill(_ptr(operands), _ptr(src), int(window_bytes), _ptr(sink), int(mfma_iters),
                                        int(fill_iters), _stream_handle(stream))
    if rc != 0:
        raise CacnnError(rc, "cacnn_probe_mfma_and_fill")


def cacnn_probe_mfma_and_fill_on(compute_units: int, tile: int, mode: int, operands, src, window_bytes: int, sink,
                                 mfma_iters: int, fill_iters: int, stream=None) -> None:
    """The same on `compute_units` compute units only (one workgroup each, the others idle); tile 0 / 1: the MFMA loop of
    the kernel with 7 x 1 / 2 x 2 positions per tile; mode bit 0: the MFMA wavefronts read their operands from the LDS
    being filled, as that kernel's multiplying wavefronts do; bit 1: a workgroup barrier per iteration (equal counts)."""
    if operands.numel() * operands.element_size() < 16384 or src.numel() * src.element_size() < int(window_bytes) or \
            sink.numel() * sink.element_size() < 65536 * 4:
        raise ValueError("cacnn_probe_mfma_and_fill_on: operands (16 KiB), src (the window) or sink (65536 floats) too short")
    rc = _lib.cacnn_probe_mfma_and_fill_on(int(compute_units), int(tile), int(mode), _ptr(operands), _ptr(src),
                                           int(window_bytes), _ptr(sink), int(mfma_iters), int(fill_iters), _stream_handle(stream))
    if rc != 0:
        raise CacnnError(rc, "cacnn_probe_mfma_and_fill_on")


def cacnn_conv_forward_with_plan(problem, dtype: int, plan: Plan, image, filt, out, stream=None) -> None:
    """Same as cacnn_conv_forward with a caller-chosen kernel variant and contraction tile."""
    _check_operands("cacnn_conv_forward_with_plan", _as_problem(problem), dtype, image, filt, out)
    rc = _lib.cacnn_conv_forward_with_plan(ctypes.byref(_as_problem(problem)), int(dtype), ctypes.byref(plan),
                                           _ptr(image), _ptr(filt), _ptr(out), _stream_handle(stream))
    if rc != 0:
        raise CacnnError(rc, "cacnn_conv_forward_with_plan")
