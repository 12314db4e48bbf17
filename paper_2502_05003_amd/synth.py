"""Seeded synthetic inputs with the shapes and value structure of the paper's workloads.

This module holds NONE of the method's arithmetic (no transform, no quantizer): it only
draws tensors and rounds them once to their storage dtype, so that the HIP path and the CPU
oracle can be fed the very same bytes.  Shapes follow the Llama-2-style layers of the
paper's model table (App. A.4: hidden 1024 and 2048, MLP width 8/3 * hidden padded to 256);
value structure follows what the paper argues from (Sec. 3.1: sub-Gaussian bulk, long
tails, outlier channels).  The datasets and trained weights of the paper are not available
here; these tensors stand in for them.

bf16 tensors are returned as uint16 bit patterns (numpy has no bf16).
"""
from __future__ import annotations

import numpy as np


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round to nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return to_bf16_bits(x)
    raise ValueError(f"unknown storage dtype {dtype!r}")


def gaussian(rows: int, cols: int, std: float, seed: int, dtype: str = "bf16") -> np.ndarray:
    """N(0, std^2) entries (weights: std 0.02; upstream gradients: std sqrt(1e-3))."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(std)
    return _store(x, dtype)


def outlier_activations(rows: int, cols: int, frac: float, gain: float, seed: int,
                        dtype: str = "bf16") -> np.ndarray:
    """N(0,1) activations in which round(frac * cols) whole channels (columns) are scaled by gain."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols), dtype=np.float32)
    count = int(round(frac * cols))
    if count:
        channels = rng.choice(cols, size=count, replace=False)
        x[:, channels] *= np.float32(gain)
    return _store(x, dtype)


def student_t_activations(rows: int, cols: int, nu: float, seed: int,
                          dtype: str = "bf16") -> np.ndarray:
    """Heavy-tailed activations: Student-t with nu degrees of freedom, tensor rescaled to unit RMS."""
    rng = np.random.default_rng(seed)
    z = rng.standard_normal((rows, cols), dtype=np.float32)
    chi2 = rng.chisquare(nu, size=(rows, cols)).astype(np.float32)
    x = z / np.sqrt(chi2 / np.float32(nu))
    x /= np.float32(np.sqrt(np.mean(np.square(x, dtype=np.float64))))
    return _store(x, dtype)


# The workload configurations: name -> dict of recipe parameters.
CONFIGS = {
    "tiny": dict(M=256, K=512, N=512, had_block=512, bits=4, dtype="f32"),
    "mlp_up_100m": dict(M=8192, K=1024, N=4096, had_block=1024, bits=4, dtype="bf16",
                        outlier_frac=0.01, outlier_gain=20.0),
    "bit_sweep_1p6b": dict(M=16384, K=2048, N=5632, had_block=2048, bits=4, dtype="bf16", nu=3.0),
    "mlp_up_1p6b": dict(M=16384, K=2048, N=5632, had_block=2048, bits=4, dtype="bf16",
                        outlier_frac=0.005, outlier_gain=50.0),
    "mlp_down_1p6b": dict(M=16384, K=5632, N=2048, had_block=512, bits=4, dtype="bf16",
                          outlier_frac=0.005, outlier_gain=50.0),
    # the proportionally scaled 7B model of the paper's per-layer runtime figure (hidden 4096, MLP 11008)
    "mlp_up_7b": dict(M=16384, K=4096, N=11008, had_block=4096, bits=4, dtype="bf16",
                      outlier_frac=0.005, outlier_gain=50.0),
    "mlp_down_7b": dict(M=16384, K=11008, N=4096, had_block=256, bits=4, dtype="bf16",
                        outlier_frac=0.005, outlier_gain=50.0),
}


def make_config(name: str, seed: int = 0, rows: int | None = None):
    """Return (X, W, cfg) for a named configuration; `rows` truncates M (same first rows)."""
    cfg = dict(CONFIGS[name])
    M = cfg["M"]
    K, N, dtype = cfg["K"], cfg["N"], cfg["dtype"]
    if name == "tiny":
        x = gaussian(M, K, 1.0, seed, dtype)
    elif name == "bit_sweep_1p6b":
        x = student_t_activations(M, K, cfg["nu"], seed, dtype)
    else:
        x = outlier_activations(M, K, cfg["outlier_frac"], cfg["outlier_gain"], seed, dtype)
    if rows is not None:
        x = np.ascontiguousarray(x[:rows])
        cfg["M"] = rows
    w = gaussian(N, K, 0.02, seed + 1000, dtype)
    return x, w, cfg


def upstream_gradient(M: int, N: int, seed: int = 0, dtype: str = "bf16") -> np.ndarray:
    """dY ~ N(0, 1e-3) (variance), the upstream gradient of the full forward+backward workload."""
    return gaussian(M, N, float(np.sqrt(1e-3)), seed + 2000, dtype)
