"""Thin Python binding of libquest.so: argument marshalling only.

Every function has the name and the argument order of the C entry point it wraps
(include/quest.h).  Tensors are torch device tensors used purely as device memory; every step of
the path runs in the HIP kernels behind the C ABI, on torch's current stream.  There is no CPU or
eager fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libquest.so")

QUEST_F32, QUEST_BF16 = 0, 1
EXPORTS = ("quest_hadamard_quantize", "quest_hadamard_quantize_pair", "quest_hadamard_quantize_absmax", "quest_hadamard_quantize_fp4", "quest_hadamard_quantize_fp4_pair", "quest_alpha_star_fp4",
           "quest_lowbit_gemm", "quest_lowbit_gemm_workspace_bytes", "quest_lowbit_gemm_static", "quest_lowbit_gemm_fp4", "quest_trust_backward", "quest_trust_backward_pair",
           "quest_grad_gemm", "quest_grad_gemm_workspace_bytes", "quest_grad_gemm_fp4",
           "quest_grad_gemm_fp4_workspace_bytes", "quest_weight_only_gemm", "quest_weight_only_gemm_workspace_bytes",
           "quest_init", "quest_alpha_star", "quest_container_bits", "quest_status_string")

_i64, _i32, _f32, _p = ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p
_lib = None


class QuestError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


def load():
    """dlopen libquest.so (built by __graft_entry__.build()); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = ctypes.CDLL(LIB_PATH)
        lib.quest_hadamard_quantize.argtypes = [_p, _i32, _i64, _i64, _i64, _i32, _i32, _f32, _f32,
                                                _p, _p, _p, _p, _p]
        lib.quest_hadamard_quantize_pair.argtypes = [_p, _i64, _i64, _p, _p, _p, _p, _i64, _i64, _p, _p, _p,
                                                     _i32, _i64, _i32, _i32, _f32, _f32, _p]
        lib.quest_hadamard_quantize_pair.restype = ctypes.c_int
        lib.quest_hadamard_quantize_absmax.argtypes = [_p, _i32, _i64, _i64, _i64, _i32, _i32,
                                                       _p, _p, _p, _p, _p]
        lib.quest_hadamard_quantize_fp4.argtypes = [_p, _i32, _i64, _i64, _i64, _i32, _f32, _p, _p, _p, _p, _p]
        lib.quest_hadamard_quantize_fp4.restype = ctypes.c_int
        lib.quest_hadamard_quantize_fp4_pair.argtypes = [_p, _i64, _i64, _p, _p, _p, _p, _i64, _i64, _p, _p, _p,
                                                         _i32, _i64, _i32, _f32, _p]
        lib.quest_hadamard_quantize_fp4_pair.restype = ctypes.c_int
        lib.quest_alpha_star_fp4.argtypes = []
        lib.quest_alpha_star_fp4.restype = _f32
        lib.quest_lowbit_gemm.argtypes = [_p, _p, _i64, _p, _p, _i64, _i64, _i32, _p, _i64, _p, _p, _i64, _p]
        lib.quest_lowbit_gemm_static.argtypes = [_p, _p, _i64, _p, _p, _i64, _i64, _i32, _p, _i64, _p, _p]
        lib.quest_lowbit_gemm_static.restype = ctypes.c_int
        lib.quest_lowbit_gemm_workspace_bytes.argtypes = [_i64, _i64, _i64, _i32]
        lib.quest_lowbit_gemm_workspace_bytes.restype = _i64
        lib.quest_lowbit_gemm_fp4.argtypes = [_p, _p, _i64, _p, _p, _i64, _i64, _p, _i64, _p, _p]
        lib.quest_lowbit_gemm_fp4.restype = ctypes.c_int
        lib.quest_trust_backward.argtypes = [_p, _i32, _p, _i64, _i64, _i32, _p, _i32, _p]
        lib.quest_trust_backward_pair.argtypes = [_p, _p, _i64, _p, _p, _p, _i64, _p, _i32, _i64, _i32, _i32, _p]
        lib.quest_trust_backward_pair.restype = ctypes.c_int
        lib.quest_grad_gemm.argtypes = [_i32, _p, _p, _p, _i32, _i64, _i64, _i64, _p, _p, _i64, _p]
        lib.quest_weight_only_gemm.argtypes = [_p, _p, _p, _i32, _i64, _i64, _i64, _p, _p, _i64, _p]
        lib.quest_grad_gemm_fp4.argtypes = [_i32, _p, _p, _p, _i64, _i64, _i64, _p, _p, _i64, _p]
        lib.quest_grad_gemm_fp4.restype = ctypes.c_int
        for name in ("quest_grad_gemm_workspace_bytes", "quest_grad_gemm_fp4_workspace_bytes"):
            getattr(lib, name).argtypes = [_i32, _i64, _i64, _i64]
            getattr(lib, name).restype = _i64
        lib.quest_weight_only_gemm_workspace_bytes.argtypes = [_i64, _i64, _i64]
        lib.quest_weight_only_gemm_workspace_bytes.restype = _i64
        lib.quest_init.argtypes = []
        lib.quest_init.restype = ctypes.c_int
        for name in ("quest_hadamard_quantize", "quest_hadamard_quantize_absmax", "quest_lowbit_gemm",
                     "quest_trust_backward", "quest_grad_gemm", "quest_weight_only_gemm"):
            getattr(lib, name).restype = ctypes.c_int
        lib.quest_alpha_star.argtypes = [_i32]
        lib.quest_alpha_star.restype = _f32
        lib.quest_container_bits.argtypes = [_i32]
        lib.quest_container_bits.restype = _i32
        lib.quest_status_string.argtypes = [ctypes.c_int]
        lib.quest_status_string.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return QUEST_F32
    if t.dtype == torch.bfloat16:
        return QUEST_BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t: torch.Tensor | None):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise QuestError(status, where)


def quest_alpha_star(bits: int) -> float:
    return float(load().quest_alpha_star(bits))


def quest_container_bits(bits: int) -> int:
    return int(load().quest_container_bits(bits))


def status_string(status: int) -> str:
    return load().quest_status_string(status).decode()


def quest_hadamard_quantize(x: torch.Tensor, had_block: int, bits: int, alpha: float = 0.0,
                            outer_trust: float = -1.0, *, codes: torch.Tensor,
                            scales: torch.Tensor, mask: torch.Tensor | None = None,
                            xh_out: torch.Tensor | None = None) -> None:
    """x [rows, cols] (row stride x.stride(0)) -> codes, scales, mask, xh_out (caller-allocated)."""
    rows, cols = x.shape
    _check(load().quest_hadamard_quantize(_ptr(x), _dtype_code(x), rows, cols, x.stride(0),
                                          had_block, bits, alpha, outer_trust, _ptr(codes),
                                          _ptr(scales), _ptr(mask), _ptr(xh_out), _stream()),
           "quest_hadamard_quantize")


def quest_hadamard_quantize_pair(x: torch.Tensor, w: torch.Tensor, had_block: int, bits: int, alpha: float = 0.0,
                                 outer_trust: float = -1.0, *, x_codes: torch.Tensor, x_scales: torch.Tensor,
                                 w_codes: torch.Tensor, w_scales: torch.Tensor,
                                 x_mask: torch.Tensor | None = None, w_mask: torch.Tensor | None = None) -> None:
    """Activations x [rows_x, cols] and weights w [rows_w, cols] of one layer quantized by one call."""
    if x.shape[1] != w.shape[1] or x.dtype != w.dtype:
        raise ValueError("the two operands of a pair call share the row length and the dtype")
    _check(load().quest_hadamard_quantize_pair(_ptr(x), x.shape[0], x.stride(0), _ptr(x_codes), _ptr(x_scales),
                                               _ptr(x_mask), _ptr(w), w.shape[0], w.stride(0), _ptr(w_codes),
                                               _ptr(w_scales), _ptr(w_mask), _dtype_code(x), x.shape[1], had_block,
                                               bits, alpha, outer_trust, _stream()),
           "quest_hadamard_quantize_pair")


def quest_hadamard_quantize_absmax(x: torch.Tensor, had_block: int, bits: int, *, codes: torch.Tensor,
                                   scales: torch.Tensor, mask: torch.Tensor | None = None,
                                   xh_out: torch.Tensor | None = None) -> None:
    """As quest_hadamard_quantize, with the grid spanning each row's largest |x_h|."""
    rows, cols = x.shape
    _check(load().quest_hadamard_quantize_absmax(_ptr(x), _dtype_code(x), rows, cols, x.stride(0),
                                                 had_block, bits, _ptr(codes), _ptr(scales), _ptr(mask),
                                                 _ptr(xh_out), _stream()),
           "quest_hadamard_quantize_absmax")


def quest_hadamard_quantize_fp4(x: torch.Tensor, had_block: int, alpha: float = 0.0, *, codes: torch.Tensor,
                                scales: torch.Tensor, mask: torch.Tensor | None = None,
                                xh_out: torch.Tensor | None = None) -> None:
    """As quest_hadamard_quantize, rounding to the scaled E2M1 grid; codes are E2M1 nibbles."""
    rows, cols = x.shape
    _check(load().quest_hadamard_quantize_fp4(_ptr(x), _dtype_code(x), rows, cols, x.stride(0), had_block,
                                              alpha, _ptr(codes), _ptr(scales), _ptr(mask), _ptr(xh_out),
                                              _stream()),
           "quest_hadamard_quantize_fp4")


def quest_hadamard_quantize_fp4_pair(x: torch.Tensor, w: torch.Tensor, had_block: int, alpha: float = 0.0, *,
                                     x_codes: torch.Tensor, x_scales: torch.Tensor, w_codes: torch.Tensor,
                                     w_scales: torch.Tensor, x_mask: torch.Tensor | None = None,
                                     w_mask: torch.Tensor | None = None) -> None:
    """As quest_hadamard_quantize_pair, rounding to the scaled E2M1 grid."""
    if x.shape[1] != w.shape[1] or x.dtype != w.dtype:
        raise ValueError("the two operands of a pair call share the row length and the dtype")
    _check(load().quest_hadamard_quantize_fp4_pair(_ptr(x), x.shape[0], x.stride(0), _ptr(x_codes),
                                                   _ptr(x_scales), _ptr(x_mask), _ptr(w), w.shape[0],
                                                   w.stride(0), _ptr(w_codes), _ptr(w_scales), _ptr(w_mask),
                                                   _dtype_code(x), x.shape[1], had_block, alpha, _stream()),
           "quest_hadamard_quantize_fp4_pair")


def quest_alpha_star_fp4() -> float:
    return float(load().quest_alpha_star_fp4())


def _bytes(t: torch.Tensor | None) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def quest_init() -> None:
    """Optional per-device set-up (kernel attributes); call before capturing graphs."""
    _check(load().quest_init(), "quest_init")


def quest_lowbit_gemm_workspace_bytes(M: int, N: int, K: int, bits: int) -> int:
    return int(load().quest_lowbit_gemm_workspace_bytes(M, N, K, bits))


def quest_lowbit_gemm(a_codes: torch.Tensor, a_scales: torch.Tensor, b_codes: torch.Tensor,
                      b_scales: torch.Tensor, K: int, bits: int, *, y: torch.Tensor | None,
                      acc_out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> None:
    """y[M, N] (bf16) and/or acc_out[M, N] (int32) from packed codes [M, K*cb/8] and [N, K*cb/8]."""
    M, N = a_codes.shape[0], b_codes.shape[0]
    ld_y = y.stride(0) if y is not None else N
    _check(load().quest_lowbit_gemm(_ptr(a_codes), _ptr(a_scales), M, _ptr(b_codes), _ptr(b_scales),
                                    N, K, bits, _ptr(y), ld_y, _ptr(acc_out), _ptr(workspace),
                                    _bytes(workspace), _stream()),
           "quest_lowbit_gemm")


def quest_lowbit_gemm_static(a_codes: torch.Tensor, a_scales: torch.Tensor, b_codes: torch.Tensor,
                             b_scales: torch.Tensor, K: int, bits: int, *, y: torch.Tensor | None,
                             acc_out: torch.Tensor | None = None) -> None:
    """quest_lowbit_gemm with the library's built-in scratch buffer (allocates nothing)."""
    M, N = a_codes.shape[0], b_codes.shape[0]
    ld_y = y.stride(0) if y is not None else N
    _check(load().quest_lowbit_gemm_static(_ptr(a_codes), _ptr(a_scales), M, _ptr(b_codes), _ptr(b_scales),
                                           N, K, bits, _ptr(y), ld_y, _ptr(acc_out), _stream()),
           "quest_lowbit_gemm_static")


def quest_lowbit_gemm_fp4(a_codes: torch.Tensor, a_scales: torch.Tensor, b_codes: torch.Tensor,
                          b_scales: torch.Tensor, K: int, *, y: torch.Tensor | None,
                          acc_out: torch.Tensor | None = None) -> None:
    """y[M, N] (bf16) and/or acc_out[M, N] (fp32) from packed E2M1 codes [M, K/2] and [N, K/2]."""
    M, N = a_codes.shape[0], b_codes.shape[0]
    ld_y = y.stride(0) if y is not None else N
    _check(load().quest_lowbit_gemm_fp4(_ptr(a_codes), _ptr(a_scales), M, _ptr(b_codes), _ptr(b_scales),
                                        N, K, _ptr(y), ld_y, _ptr(acc_out), _stream()),
           "quest_lowbit_gemm_fp4")


def quest_trust_backward(g: torch.Tensor, mask: torch.Tensor | None, had_block: int, *,
                         out: torch.Tensor) -> None:
    """out = IHT(mask (.) g) for contiguous g, out of shape [rows, cols]."""
    rows, cols = g.shape
    _check(load().quest_trust_backward(_ptr(g), _dtype_code(g), _ptr(mask), rows, cols, had_block,
                                       _ptr(out), _dtype_code(out), _stream()),
           "quest_trust_backward")


def quest_trust_backward_pair(g_x: torch.Tensor, mask_x: torch.Tensor | None, g_w: torch.Tensor,
                              mask_w: torch.Tensor | None, had_block: int, *, out_x: torch.Tensor,
                              out_w: torch.Tensor) -> None:
    """out_x = IHT(mask_x (.) g_x) and out_w = IHT(mask_w (.) g_w) by one call (contiguous, same row length)."""
    if g_x.shape[1] != g_w.shape[1] or g_x.dtype != g_w.dtype or out_x.dtype != out_w.dtype:
        raise ValueError("the two gradients of a pair call share the row length and the dtypes")
    _check(load().quest_trust_backward_pair(_ptr(g_x), _ptr(mask_x), g_x.shape[0], _ptr(out_x), _ptr(g_w),
                                            _ptr(mask_w), g_w.shape[0], _ptr(out_w), _dtype_code(g_x),
                                            g_x.shape[1], had_block, _dtype_code(out_x), _stream()),
           "quest_trust_backward_pair")


def quest_grad_gemm_workspace_bytes(which: int, M: int, N: int, K: int) -> int:
    return int(load().quest_grad_gemm_workspace_bytes(which, M, N, K))


def quest_grad_gemm(which: int, dy: torch.Tensor, q_codes: torch.Tensor, q_scales: torch.Tensor,
                    bits: int, M: int, N: int, K: int, *, out: torch.Tensor,
                    workspace: torch.Tensor | None = None) -> None:
    """which = 0: out[M, K] = dy what_h;  which = 1: out[N, K] = dy^T xhat_h (bf16)."""
    _check(load().quest_grad_gemm(which, _ptr(dy), _ptr(q_codes), _ptr(q_scales), bits, M, N, K,
                                  _ptr(out), _ptr(workspace), _bytes(workspace), _stream()),
           "quest_grad_gemm")


def quest_grad_gemm_fp4_workspace_bytes(which: int, M: int, N: int, K: int) -> int:
    return int(load().quest_grad_gemm_fp4_workspace_bytes(which, M, N, K))


def quest_grad_gemm_fp4(which: int, dy: torch.Tensor, q_codes: torch.Tensor, q_scales: torch.Tensor,
                        M: int, N: int, K: int, *, out: torch.Tensor,
                        workspace: torch.Tensor | None = None) -> None:
    """quest_grad_gemm for E2M1 codes (operands from quest_hadamard_quantize_fp4)."""
    _check(load().quest_grad_gemm_fp4(which, _ptr(dy), _ptr(q_codes), _ptr(q_scales), M, N, K, _ptr(out),
                                      _ptr(workspace), _bytes(workspace), _stream()),
           "quest_grad_gemm_fp4")


def quest_weight_only_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load().quest_weight_only_gemm_workspace_bytes(M, N, K))


def quest_weight_only_gemm(x: torch.Tensor, w_codes: torch.Tensor, w_scales: torch.Tensor, bits: int,
                           *, y: torch.Tensor, workspace: torch.Tensor | None = None) -> None:
    """y[M, N] (bf16) = x[M, K] (bf16) times the transposed weights given as packed codes [N, K*cb/8]."""
    M, K = x.shape
    N = w_codes.shape[0]
    _check(load().quest_weight_only_gemm(_ptr(x), _ptr(w_codes), _ptr(w_scales), bits, M, N, K, _ptr(y),
                                         _ptr(workspace), _bytes(workspace), _stream()),
           "quest_weight_only_gemm")
