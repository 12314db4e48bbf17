"""numpy front end of the C oracle (oracle/quest_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py; never by the product package.  It compiles the C file with
gcc on first use (no GPU, no HIP) and exposes each C function on numpy arrays.  It shares
nothing with the HIP path.

Paper passages: see the header of quest_oracle.c.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

from . import alpha_star as _alpha

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "quest_oracle.c")
_LIB = os.path.join(_HERE, "libquest_oracle.so")

_c_i64 = ctypes.c_int64
_c_int = ctypes.c_int
_c_dbl = ctypes.c_double
_p = ctypes.c_void_p


def build(force: bool = False) -> str:
    """Compile the C oracle into oracle/libquest_oracle.so (gcc -O2, OpenMP over rows)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.qo_widen_bf16.argtypes = [_p, _c_i64, _p]
        lib.qo_widen_f32.argtypes = [_p, _c_i64, _p]
        lib.qo_hadamard_entry.argtypes = [ctypes.c_uint32, ctypes.c_uint32]
        lib.qo_hadamard_entry.restype = _c_int
        lib.qo_hadamard_matrix.argtypes = [_c_i64, _p]
        for name in ("qo_hadamard_dense", "qo_hadamard_sylvester"):
            getattr(lib, name).argtypes = [_p, _c_i64, _c_i64, _c_i64, _p]
        lib.qo_row_rms.argtypes = [_p, _c_i64, _c_i64, _p]
        lib.qo_project.argtypes = [_p, _c_i64, _c_i64, _c_int, _c_dbl, _c_dbl, _p, _p, _p, _p, _p]
        lib.qo_project_absmax.argtypes = [_p, _c_i64, _c_i64, _c_int, _p, _p, _p, _p, _p]
        lib.qo_project_fp4.argtypes = [_p, _c_i64, _c_i64, _c_dbl, _p, _p, _p, _p, _p]
        lib.qo_pack_fp4.argtypes = [_p, _c_i64, _c_i64, _p]
        lib.qo_unpack_fp4.argtypes = [_p, _c_i64, _c_i64, _p]
        lib.qo_container_bits.argtypes = [_c_int]
        lib.qo_container_bits.restype = _c_int
        lib.qo_pack_codes.argtypes = [_p, _c_i64, _c_i64, _c_int, _p]
        lib.qo_unpack_odd.argtypes = [_p, _c_i64, _c_i64, _c_int, _p]
        lib.qo_pack_mask.argtypes = [_p, _c_i64, _c_i64, _p]
        lib.qo_unpack_mask.argtypes = [_p, _c_i64, _c_i64, _p]
        lib.qo_gemm_odd.argtypes = [_p, _p, _c_i64, _c_i64, _c_i64, _p]
        lib.qo_gemm_odd.restype = _c_i64
        lib.qo_gemm_fp4.argtypes = [_p, _p, _c_i64, _c_i64, _c_i64, _p]
        lib.qo_dequant.argtypes = [_p, _p, _p, _c_i64, _c_i64, _p]
        lib.qo_trust_backward.argtypes = [_p, _p, _c_i64, _c_i64, _c_i64, _p]
        lib.qo_grad_input.argtypes = [_p, _p, _p, _c_i64, _c_i64, _c_i64, _p]
        lib.qo_weight_only_gemm.argtypes = [_p, _p, _p, _c_i64, _c_i64, _c_i64, _p]
        lib.qo_grad_weight.argtypes = [_p, _p, _p, _c_i64, _c_i64, _c_i64, _p]
        lib.qo_threads.restype = _c_int
        lib.qo_set_threads.argtypes = [_c_int]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray | None):
    return None if a is None else a.ctypes.data_as(_p)


def _c(a: np.ndarray, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def threads() -> int:
    return int(_load().qo_threads())


def set_threads(count: int) -> None:
    """Number of threads for the row loops from now on (for timing; results do not depend on it)."""
    _load().qo_set_threads(int(count))


def container_bits(bits: int) -> int:
    cb = int(_load().qo_container_bits(bits))
    if cb == 0:
        raise ValueError(f"unsupported bit width {bits}")
    return cb


def widen(x: np.ndarray) -> np.ndarray:
    """Exact widening of the stored input to double.  uint16 arrays are bf16 bit patterns."""
    x = np.ascontiguousarray(x)
    out = np.empty(x.shape, dtype=np.float64)
    if x.dtype == np.uint16:
        _load().qo_widen_bf16(_ptr(x), x.size, _ptr(out))
    elif x.dtype == np.float32:
        _load().qo_widen_f32(_ptr(x), x.size, _ptr(out))
    elif x.dtype == np.float64:
        out[...] = x
    else:
        raise TypeError(f"unsupported input dtype {x.dtype}")
    return out


def hadamard_matrix(n: int) -> np.ndarray:
    """The +-1 Sylvester matrix in natural order, entry by entry (int64)."""
    h = np.empty((n, n), dtype=np.int8)
    _load().qo_hadamard_matrix(n, _ptr(h))
    return h.astype(np.int64)


def hadamard(x: np.ndarray, n: int, dense: bool = False) -> np.ndarray:
    """x_h = x (I (x) H_n) / sqrt(n) along the last axis of a [rows, cols] double array."""
    x = _c(x, np.float64)
    rows, cols = x.shape
    if n < 1 or (n & (n - 1)) or cols % n:
        raise ValueError("Hadamard block must be a power of two dividing cols")
    out = np.empty_like(x)
    fn = _load().qo_hadamard_dense if dense else _load().qo_hadamard_sylvester
    fn(_ptr(x), rows, cols, n, _ptr(out))
    return out


def row_rms(xh: np.ndarray) -> np.ndarray:
    xh = _c(xh, np.float64)
    out = np.empty(xh.shape[0], dtype=np.float64)
    _load().qo_row_rms(_ptr(xh), xh.shape[0], xh.shape[1], _ptr(out))
    return out


@dataclass
class Projection:
    """Everything Algorithm 1 derives from one operand."""
    xh: np.ndarray        # [rows, cols] double, Hadamard-domain values
    rms: np.ndarray       # [rows]
    scale: np.ndarray     # [rows]  s = alpha rms / (L - 1)
    k: np.ndarray         # [rows, cols] int32 cell index
    xhat: np.ndarray      # [rows, cols] double, s * (2k + 1)
    trust: np.ndarray     # [rows, cols] uint8, 1 = trusted
    codes: np.ndarray     # [rows, cols*cb/8] uint8 packed c = k + L/2
    mask: np.ndarray      # [rows, cols/8] uint8 bitmap, LSB first
    alpha: float
    bits: int


def project(xh: np.ndarray, bits: int, alpha: float | None = None,
            outer_trust: float = 1.0) -> Projection:
    """RMS-normalise, clip at alpha (default alpha*(bits)), round, and derive the trust mask."""
    xh = _c(xh, np.float64)
    rows, cols = xh.shape
    cb = container_bits(bits)
    if alpha is None:
        alpha = _alpha.alpha_star(bits)
    rms = np.empty(rows, dtype=np.float64)
    scale = np.empty(rows, dtype=np.float64)
    k = np.empty((rows, cols), dtype=np.int32)
    xhat = np.empty((rows, cols), dtype=np.float64)
    trust = np.empty((rows, cols), dtype=np.uint8)
    lib = _load()
    lib.qo_project(_ptr(xh), rows, cols, bits, float(alpha), float(outer_trust), _ptr(rms),
                   _ptr(scale), _ptr(k), _ptr(xhat), _ptr(trust))
    codes = np.empty((rows, cols * cb // 8), dtype=np.uint8)
    lib.qo_pack_codes(_ptr(k), rows, cols, bits, _ptr(codes))
    mask = np.empty((rows, cols // 8), dtype=np.uint8)
    lib.qo_pack_mask(_ptr(trust), rows, cols, _ptr(mask))
    return Projection(xh, rms, scale, k, xhat, trust, codes, mask, float(alpha), bits)


def project_absmax(xh: np.ndarray, bits: int) -> Projection:
    """The AbsMax comparison quantizer (Sec. 4.1): the grid spans the row's largest magnitude.
    In the result `rms` holds that magnitude and `alpha` is 1 (clip = alpha * rms still holds)."""
    xh = _c(xh, np.float64)
    rows, cols = xh.shape
    cb = container_bits(bits)
    amax = np.empty(rows, dtype=np.float64)
    scale = np.empty(rows, dtype=np.float64)
    k = np.empty((rows, cols), dtype=np.int32)
    xhat = np.empty((rows, cols), dtype=np.float64)
    trust = np.empty((rows, cols), dtype=np.uint8)
    lib = _load()
    lib.qo_project_absmax(_ptr(xh), rows, cols, bits, _ptr(amax), _ptr(scale), _ptr(k), _ptr(xhat),
                          _ptr(trust))
    codes = np.empty((rows, cols * cb // 8), dtype=np.uint8)
    lib.qo_pack_codes(_ptr(k), rows, cols, bits, _ptr(codes))
    mask = np.empty((rows, cols // 8), dtype=np.uint8)
    lib.qo_pack_mask(_ptr(trust), rows, cols, _ptr(mask))
    return Projection(xh, amax, scale, k, xhat, trust, codes, mask, 1.0, bits)


@dataclass
class Fp4Projection:
    """What the FP4 variant (Sec. 4.4) derives from one operand."""
    xh: np.ndarray        # [rows, cols] double
    rms: np.ndarray       # [rows]
    scale: np.ndarray     # [rows]  alpha rms / 6: xhat = scale * value
    code: np.ndarray      # [rows, cols] uint8 E2M1 code, bit 3 = sign
    value: np.ndarray     # [rows, cols] double signed E2M1 value of the code
    xhat: np.ndarray      # [rows, cols] double
    trust: np.ndarray     # [rows, cols] uint8
    codes: np.ndarray     # [rows, cols/2] uint8, two codes per byte, low nibble first
    mask: np.ndarray      # [rows, cols/8] uint8 bitmap
    alpha: float


def unpack_fp4(codes: np.ndarray, cols: int) -> np.ndarray:
    codes = _c(codes, np.uint8)
    rows = codes.shape[0]
    value = np.empty((rows, cols), dtype=np.float64)
    _load().qo_unpack_fp4(_ptr(codes), rows, cols, _ptr(value))
    return value


def project_fp4(xh: np.ndarray, alpha: float | None = None) -> Fp4Projection:
    """RMS-normalise, clip at alpha (default alpha*_FP4), round to the scaled E2M1 grid, trust mask."""
    xh = _c(xh, np.float64)
    rows, cols = xh.shape
    if alpha is None:
        alpha = _alpha.alpha_star_fp4()
    rms = np.empty(rows, dtype=np.float64)
    scale = np.empty(rows, dtype=np.float64)
    code = np.empty((rows, cols), dtype=np.uint8)
    xhat = np.empty((rows, cols), dtype=np.float64)
    trust = np.empty((rows, cols), dtype=np.uint8)
    lib = _load()
    lib.qo_project_fp4(_ptr(xh), rows, cols, float(alpha), _ptr(rms), _ptr(scale), _ptr(code), _ptr(xhat),
                       _ptr(trust))
    codes = np.empty((rows, cols // 2), dtype=np.uint8)
    lib.qo_pack_fp4(_ptr(code), rows, cols, _ptr(codes))
    mask = np.empty((rows, cols // 8), dtype=np.uint8)
    lib.qo_pack_mask(_ptr(trust), rows, cols, _ptr(mask))
    return Fp4Projection(xh, rms, scale, code, unpack_fp4(codes, cols), xhat, trust, codes, mask, float(alpha))


def hadamard_quantize_fp4(x: np.ndarray, n: int, alpha: float | None = None, dense: bool = False) -> Fp4Projection:
    """x_h = HT(x), then the FP4 projection."""
    return project_fp4(hadamard(widen(x), n, dense=dense), alpha)


def gemm_fp4(va: np.ndarray, vb: np.ndarray) -> np.ndarray:
    """acc[m, n] = sum_k v_a[m, k] v_b[n, k] of signed E2M1 values: multiples of 1/4, exact in double."""
    va = _c(va, np.float64)
    vb = _c(vb, np.float64)
    M, K = va.shape
    N, K2 = vb.shape
    if K != K2:
        raise ValueError("contraction lengths differ")
    acc = np.empty((M, N), dtype=np.float64)
    _load().qo_gemm_fp4(_ptr(va), _ptr(vb), M, N, K, _ptr(acc))
    return acc


def hadamard_quantize(x: np.ndarray, n: int, bits: int, alpha: float | None = None,
                      outer_trust: float = 1.0, dense: bool = False) -> Projection:
    """Algorithm 1 for one operand: x_h = HT(x), then the projection and the mask."""
    return project(hadamard(widen(x), n, dense=dense), bits, alpha, outer_trust)


def hadamard_quantize_absmax(x: np.ndarray, n: int, bits: int, dense: bool = False) -> Projection:
    """x_h = HT(x) (n = 1: no transform), then the AbsMax projection."""
    return project_absmax(hadamard(widen(x), n, dense=dense), bits)


def unpack_odd(codes: np.ndarray, cols: int, bits: int) -> np.ndarray:
    codes = _c(codes, np.uint8)
    rows = codes.shape[0]
    u = np.empty((rows, cols), dtype=np.int32)
    _load().qo_unpack_odd(_ptr(codes), rows, cols, bits, _ptr(u))
    return u


def unpack_mask(mask: np.ndarray, cols: int) -> np.ndarray:
    mask = _c(mask, np.uint8)
    rows = mask.shape[0]
    trust = np.empty((rows, cols), dtype=np.uint8)
    _load().qo_unpack_mask(_ptr(mask), rows, cols, _ptr(trust))
    return trust


def gemm_odd(ux: np.ndarray, uw: np.ndarray) -> np.ndarray:
    """acc[m, n] = sum_k u_x[m, k] u_w[n, k], exact (int64, asserted to fit int32)."""
    ux = _c(ux, np.int32)
    uw = _c(uw, np.int32)
    M, K = ux.shape
    N, K2 = uw.shape
    if K != K2:
        raise ValueError("contraction lengths differ")
    acc = np.empty((M, N), dtype=np.int64)
    worst = _load().qo_gemm_odd(_ptr(ux), _ptr(uw), M, N, K, _ptr(acc))
    assert worst < 2 ** 31, "accumulator does not fit 32 bits"
    return acc


def dequant(acc: np.ndarray, sx: np.ndarray, sw: np.ndarray) -> np.ndarray:
    acc = _c(acc, np.int64)
    sx = _c(sx, np.float64)
    sw = _c(sw, np.float64)
    M, N = acc.shape
    y = np.empty((M, N), dtype=np.float64)
    _load().qo_dequant(_ptr(acc), _ptr(sx), _ptr(sw), M, N, _ptr(y))
    return y


def trust_backward(g: np.ndarray, trust: np.ndarray | None, n: int) -> np.ndarray:
    """IHT(M (.) g) on a [rows, cols] double array; trust is one byte per element or None."""
    g = _c(g, np.float64)
    rows, cols = g.shape
    if trust is not None:
        trust = _c(trust, np.uint8)
        if trust.shape != g.shape:
            raise ValueError("trust must have one byte per element")
    out = np.empty_like(g)
    _load().qo_trust_backward(_ptr(g), _ptr(trust), rows, cols, n, _ptr(out))
    return out


def grad_input(dy: np.ndarray, uw: np.ndarray, sw: np.ndarray) -> np.ndarray:
    """G_x = dY what, what = s_w u_w  (Algorithm 2, gradient w.r.t. xhat_h)."""
    dy = _c(dy, np.float64)
    uw = _c(uw, np.int32)
    sw = _c(sw, np.float64)
    M, N = dy.shape
    K = uw.shape[1]
    gx = np.empty((M, K), dtype=np.float64)
    _load().qo_grad_input(_ptr(dy), _ptr(uw), _ptr(sw), M, N, K, _ptr(gx))
    return gx


def weight_only_gemm(x: np.ndarray, uw: np.ndarray, sw: np.ndarray) -> np.ndarray:
    """y = x what^T, what = s_w u_w: the forward product with 16-bit activations (Sec. 4.4)."""
    x = _c(x, np.float64)
    uw = _c(uw, np.int32)
    sw = _c(sw, np.float64)
    M, K = x.shape
    N = uw.shape[0]
    y = np.empty((M, N), dtype=np.float64)
    _load().qo_weight_only_gemm(_ptr(x), _ptr(uw), _ptr(sw), M, N, K, _ptr(y))
    return y


def grad_weight(dy: np.ndarray, ux: np.ndarray, sx: np.ndarray) -> np.ndarray:
    """G_w = dY^T xhat, xhat = s_x u_x, shaped [N, K] like the weight (Algorithm 2)."""
    dy = _c(dy, np.float64)
    ux = _c(ux, np.int32)
    sx = _c(sx, np.float64)
    M, N = dy.shape
    K = ux.shape[1]
    gw = np.empty((N, K), dtype=np.float64)
    _load().qo_grad_weight(_ptr(dy), _ptr(ux), _ptr(sx), M, N, K, _ptr(gw))
    return gw
