"""Thin Python binding of the C-ABI library (argument marshalling only).

Every function has the name and the contract of its C counterpart in
``include/gptq_w4a16.h``; tensors are torch CUDA(HIP) tensors whose device pointers are
handed to the library, and the work is enqueued on torch's current stream.  Nothing is
computed on the host and there is no fallback: if the library has not been built, loading
fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libgptq_w4a16.so")

_lib = None


class GptqError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


class Plan(ctypes.Structure):
    """Mirror of gptq_w4a16_plan_t."""

    _fields_ = [("kernel", ctypes.c_int), ("split_k", ctypes.c_int), ("tile", ctypes.c_int),
                ("flags", ctypes.c_int), ("reserved", ctypes.c_int * 4)]


EXPORTS = ("gptq_w4a16_gemm", "gptq_w4a16_gemm_static", "gptq_w4a16_gemm_plan", "gptq_w4a16_plan_query", "gptq_w4a16_act_order_prepare",
           "gptq_w4a16_gemm_prepared", "gptq_w4a16_shift_zeros", "gptq_w4a16_dequant", "gptq_w4a16_unpack",
           "gptq_w4a16_workspace_bytes", "gptq_w4a16_set_workspace", "gptq_w4a16_strerror", "gptq_w4a16_version",
           "gptq_w4a16_stream_probe", "gptq_w4a16_mfma_probe", "gptq_w4a16_issue_probe")


def load() -> ctypes.CDLL:
    """Load the built library.  Raises if it is missing: build it with ``python -m paper_2511_19438_amd.build``."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: the HIP library must be built first "
            "(python -m paper_2511_19438_amd.build); there is no CPU fallback")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.gptq_w4a16_gemm.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, vp]
    lib.gptq_w4a16_gemm.restype = ci
    lib.gptq_w4a16_gemm_static.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, vp]
    lib.gptq_w4a16_gemm_static.restype = ci
    lib.gptq_w4a16_gemm_plan.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, vp, ctypes.POINTER(Plan)]
    lib.gptq_w4a16_gemm_plan.restype = ci
    lib.gptq_w4a16_plan_query.argtypes = [ci, ci, ci, ci, ci, ctypes.POINTER(Plan), ctypes.POINTER(Plan)]
    lib.gptq_w4a16_plan_query.restype = ci
    lib.gptq_w4a16_act_order_prepare.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp]
    lib.gptq_w4a16_act_order_prepare.restype = ci
    lib.gptq_w4a16_gemm_prepared.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, vp]
    lib.gptq_w4a16_gemm_prepared.restype = ci
    lib.gptq_w4a16_shift_zeros.argtypes = [vp, vp, ci, ci, ci, ci, vp]
    lib.gptq_w4a16_shift_zeros.restype = ci
    lib.gptq_w4a16_dequant.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, vp]
    lib.gptq_w4a16_dequant.restype = ci
    lib.gptq_w4a16_unpack.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp]
    lib.gptq_w4a16_unpack.restype = ci
    lib.gptq_w4a16_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.gptq_w4a16_workspace_bytes.restype = ctypes.c_size_t
    lib.gptq_w4a16_set_workspace.argtypes = [vp, ctypes.c_size_t]
    lib.gptq_w4a16_set_workspace.restype = ci
    lib.gptq_w4a16_strerror.argtypes = [ci]
    lib.gptq_w4a16_strerror.restype = ctypes.c_char_p
    lib.gptq_w4a16_stream_probe.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.gptq_w4a16_stream_probe.restype = ci
    lib.gptq_w4a16_mfma_probe.argtypes = [vp, ctypes.c_size_t, vp, ci, ctypes.POINTER(ctypes.c_double), vp]
    lib.gptq_w4a16_mfma_probe.restype = ci
    lib.gptq_w4a16_issue_probe.argtypes = [vp, ctypes.c_size_t, vp, ci, ci, ci, ctypes.POINTER(ctypes.c_double), vp]
    lib.gptq_w4a16_issue_probe.restype = ci
    lib.gptq_w4a16_version.argtypes = []
    lib.gptq_w4a16_version.restype = ci
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().gptq_w4a16_strerror(int(code)).decode()


def version() -> int:
    return int(load().gptq_w4a16_version())


def _ptr(t: Optional[torch.Tensor], dtype, name: str):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _shapes(qweight, qzeros, scales, g_idx, group_size):
    if qweight.dim() != 2:
        raise ValueError("qweight must be [K/8, N]")
    K, N = qweight.shape[0] * 8, qweight.shape[1]
    if group_size > 0 and K % group_size == 0 and N % 8 == 0:
        G = K // group_size
        if tuple(qzeros.shape) != (G, N // 8):
            raise ValueError(f"qzeros must be [{G}, {N // 8}], got {tuple(qzeros.shape)}")
        if tuple(scales.shape) != (G, N):
            raise ValueError(f"scales must be [{G}, {N}], got {tuple(scales.shape)}")
    if g_idx is not None and tuple(g_idx.shape) != (K,):
        raise ValueError(f"g_idx must be [{K}], got {tuple(g_idx.shape)}")
    return K, N


def gptq_w4a16_gemm_static(x, qweight, qzeros, scales, g_idx, out, group_size: int):
    """gptq_w4a16_gemm on the library's static scratch block: allocates nothing (see the header)."""
    return gptq_w4a16_gemm(x, qweight, qzeros, scales, g_idx, out, group_size, _static=True)


def gptq_w4a16_gemm(x, qweight, qzeros, scales, g_idx, out, group_size: int, plan: Optional[Plan] = None,
                    _static: bool = False):
    """out[M, N] = x[M, K] @ W (see the header).  Shapes are taken from the tensors; `out` is overwritten."""
    K, N = _shapes(qweight, qzeros, scales, g_idx, group_size)
    if x.dim() != 2 or x.shape[1] != K:
        raise ValueError(f"x must be [M, {K}], got {tuple(x.shape)}")
    M = x.shape[0]
    if tuple(out.shape) != (M, N):
        raise ValueError(f"out must be [{M}, {N}], got {tuple(out.shape)}")
    lib = load()
    args = (_ptr(x, torch.float16, "x"), _ptr(qweight, torch.int32, "qweight"), _ptr(qzeros, torch.int32, "qzeros"),
            _ptr(scales, torch.float16, "scales"), _ptr(g_idx, torch.int32, "g_idx"), _ptr(out, torch.float16, "out"),
            M, K, N, int(group_size), _stream())
    if _static:
        rc = lib.gptq_w4a16_gemm_static(*args)
    elif plan is None:
        rc = lib.gptq_w4a16_gemm(*args)
    else:
        rc = lib.gptq_w4a16_gemm_plan(*args, ctypes.byref(plan))
    if rc != 0:
        raise GptqError(rc, "gptq_w4a16_gemm_static" if _static else "gptq_w4a16_gemm")
    return out


def gptq_w4a16_act_order_prepare(qweight, g_idx, qweight_sorted, perm, group_size: int):
    """One-time repack of an act-order checkpoint: fills perm[K] (int32) and qweight_sorted[K/8, N] (int32).  Blocks."""
    K, N = qweight.shape[0] * 8, qweight.shape[1]
    if tuple(g_idx.shape) != (K,) or tuple(perm.shape) != (K,):
        raise ValueError(f"g_idx and perm must be [{K}]")
    if tuple(qweight_sorted.shape) != tuple(qweight.shape):
        raise ValueError("qweight_sorted must have the shape of qweight")
    rc = load().gptq_w4a16_act_order_prepare(_ptr(qweight, torch.int32, "qweight"), _ptr(g_idx, torch.int32, "g_idx"),
                                             _ptr(qweight_sorted, torch.int32, "qweight_sorted"),
                                             _ptr(perm, torch.int32, "perm"), K, N, int(group_size), _stream())
    if rc != 0:
        raise GptqError(rc, "gptq_w4a16_act_order_prepare")
    return qweight_sorted, perm


def gptq_w4a16_gemm_prepared(x, qweight_sorted, qzeros, scales, perm, out, group_size: int):
    """The act-order GEMM on a repacked checkpoint: out = x[:, perm] @ W_sorted."""
    K, N = _shapes(qweight_sorted, qzeros, scales, perm, group_size)
    if x.dim() != 2 or x.shape[1] != K:
        raise ValueError(f"x must be [M, {K}], got {tuple(x.shape)}")
    M = x.shape[0]
    if tuple(out.shape) != (M, N):
        raise ValueError(f"out must be [{M}, {N}], got {tuple(out.shape)}")
    rc = load().gptq_w4a16_gemm_prepared(
        _ptr(x, torch.float16, "x"), _ptr(qweight_sorted, torch.int32, "qweight_sorted"),
        _ptr(qzeros, torch.int32, "qzeros"), _ptr(scales, torch.float16, "scales"), _ptr(perm, torch.int32, "perm"),
        _ptr(out, torch.float16, "out"), M, K, N, int(group_size), _stream())
    if rc != 0:
        raise GptqError(rc, "gptq_w4a16_gemm_prepared")
    return out


def gptq_w4a16_shift_zeros(qzeros_in, qzeros_out, delta: int, group_size: int):
    """qzeros_out = (qzeros_in + delta) mod 16 per zero point (one-time format conversion; may be in place)."""
    G, N8 = qzeros_in.shape
    if tuple(qzeros_out.shape) != (G, N8):
        raise ValueError("qzeros_out must have the shape of qzeros_in")
    rc = load().gptq_w4a16_shift_zeros(_ptr(qzeros_in, torch.int32, "qzeros_in"), _ptr(qzeros_out, torch.int32, "qzeros_out"),
                                       int(delta), G * int(group_size), N8 * 8, int(group_size), _stream())
    if rc != 0:
        raise GptqError(rc, "gptq_w4a16_shift_zeros")
    return qzeros_out


def gptq_w4a16_dequant(qweight, qzeros, scales, g_idx, w_out, group_size: int):
    """w_out[K, N] (fp16) = dequantised weights."""
    K, N = _shapes(qweight, qzeros, scales, g_idx, group_size)
    if tuple(w_out.shape) != (K, N):
        raise ValueError(f"w_out must be [{K}, {N}]")
    rc = load().gptq_w4a16_dequant(_ptr(qweight, torch.int32, "qweight"), _ptr(qzeros, torch.int32, "qzeros"),
                                   _ptr(scales, torch.float16, "scales"), _ptr(g_idx, torch.int32, "g_idx"),
                                   _ptr(w_out, torch.float16, "w_out"), K, N, int(group_size), _stream())
    if rc != 0:
        raise GptqError(rc, "gptq_w4a16_dequant")
    return w_out


def gptq_w4a16_unpack(qweight, q_out, qzeros, z_out, group_size: int):
    """q_out[K, N] (uint8) = 4-bit codes; z_out[K/group, N] (uint8, optional) = zero points."""
    K, N = qweight.shape[0] * 8, qweight.shape[1]
    if tuple(q_out.shape) != (K, N):
        raise ValueError(f"q_out must be [{K}, {N}]")
    if z_out is not None and tuple(z_out.shape) != (K // group_size, N):
        raise ValueError(f"z_out must be [{K // group_size}, {N}]")
    rc = load().gptq_w4a16_unpack(_ptr(qweight, torch.int32, "qweight"), _ptr(q_out, torch.uint8, "q_out"),
                                  _ptr(qzeros, torch.int32, "qzeros"), _ptr(z_out, torch.uint8, "z_out"),
                                  K, N, int(group_size), _stream())
    if rc != 0:
        raise GptqError(rc, "gptq_w4a16_unpack")
    return q_out, z_out


def gptq_w4a16_plan_query(M: int, K: int, N: int, group_size: int, act_order: bool = False,
                          plan: Optional["Plan"] = None) -> "Plan":
    """The plan a GEMM call of this shape resolves to (host only, touches no device)."""
    out = Plan()
    rc = load().gptq_w4a16_plan_query(int(M), int(K), int(N), int(group_size), int(bool(act_order)),
                                      ctypes.byref(plan) if plan is not None else None, ctypes.byref(out))
    if rc != 0:
        raise GptqError(rc, "gptq_w4a16_plan_query")
    return out


def gptq_w4a16_workspace_bytes(M: int, K: int, N: int, group_size: int) -> int:
    return int(load().gptq_w4a16_workspace_bytes(int(M), int(K), int(N), int(group_size)))


def gptq_w4a16_set_workspace(buf: Optional[torch.Tensor]):
    """Hand a caller-owned device buffer (uint8 tensor) to the library as split-K scratch; None returns to library-owned scratch."""
    if buf is None:
        rc = load().gptq_w4a16_set_workspace(None, 0)
    else:
        rc = load().gptq_w4a16_set_workspace(_ptr(buf, torch.uint8, "workspace"), buf.numel())
    if rc != 0:
        raise GptqError(rc, "gptq_w4a16_set_workspace")


def gptq_w4a16_stream_probe(buf: torch.Tensor, sink: torch.Tensor):
    """Plain read of `buf` (any dtype, contiguous): the measurement aid of the header."""
    rc = load().gptq_w4a16_stream_probe(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                        ctypes.c_void_p(sink.data_ptr()), _stream())
    if rc != 0:
        raise GptqError(rc, "gptq_w4a16_stream_probe")


def gptq_w4a16_mfma_probe(operands: torch.Tensor, sink: torch.Tensor, iters: int) -> float:
    """MFMA-only loop on register operands taken from `operands` (fp16); returns the flops of the launch."""
    flops = ctypes.c_double(0.0)
    rc = load().gptq_w4a16_mfma_probe(_ptr(operands, torch.float16, "operands"), operands.numel() * 2,
                                      ctypes.c_void_p(sink.data_ptr()), int(iters), ctypes.byref(flops), _stream())
    if rc != 0:
        raise GptqError(rc, "gptq_w4a16_mfma_probe")
    return float(flops.value)


def gptq_w4a16_issue_probe(operands: torch.Tensor, sink: torch.Tensor, iters: int, valu_per_mfma: int,
                           waves_per_simd: int) -> float:
    """One MFMA + `valu_per_mfma` independent packed-fp16 instructions per group, `waves_per_simd` wavefronts per
    SIMD; returns the number of MFMAs each SIMD executes in the launch."""
    count = ctypes.c_double(0.0)
    rc = load().gptq_w4a16_issue_probe(_ptr(operands, torch.float16, "operands"), operands.numel() * 2,
                                       ctypes.c_void_p(sink.data_ptr()), int(iters), int(valu_per_mfma),
                                       int(waves_per_simd), ctypes.byref(count), _stream())
    if rc != 0:
        raise GptqError(rc, "gptq_w4a16_issue_probe")
    return float(count.value)
