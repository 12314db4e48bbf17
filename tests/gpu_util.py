"""Helpers for the GPU parity tests: host <-> device marshalling and the comparison rules."""
from __future__ import annotations

import numpy as np
import torch

from oracle import quest_oracle as qo
from paper_2502_05003_amd import binding as q

DEV = "cuda:0"


def to_device(a: np.ndarray) -> torch.Tensor:
    """numpy -> device tensor; uint16 arrays are bf16 bit patterns."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(DEV)
    return torch.from_numpy(a).to(DEV)


def _scratch(nbytes: int):
    """Caller-owned scratch of at least `nbytes` (None when the call needs none); filled with a pattern."""
    assert nbytes >= 0, "the library does not accept this shape"
    return torch.full((nbytes,), 0xC3, dtype=torch.uint8, device=DEV) if nbytes else None


def grad_ws(which: int, M: int, N: int, K: int, fp4: bool = False):
    query = q.quest_grad_gemm_fp4_workspace_bytes if fp4 else q.quest_grad_gemm_workspace_bytes
    return _scratch(query(which, M, N, K))


def weight_only_ws(M: int, N: int, K: int):
    return _scratch(q.quest_weight_only_gemm_workspace_bytes(M, N, K))


def lowbit_ws(M: int, N: int, K: int, bits: int):
    return _scratch(q.quest_lowbit_gemm_workspace_bytes(M, N, K, bits))


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def gpu_quantize(x_host: np.ndarray, had_block: int, bits: int, alpha: float = 0.0,
                 outer_trust: float = -1.0, want_xh: bool = True, want_mask: bool = True, ld=None,
                 absmax: bool = False, fp4: bool = False):
    """Run quest_hadamard_quantize on a host array; returns host arrays."""
    rows, cols = x_host.shape
    cb = q.quest_container_bits(bits)
    if ld is None:
        x = to_device(x_host)
    else:
        buf = np.zeros((rows, ld), dtype=x_host.dtype)
        buf[:, :cols] = x_host
        x = to_device(buf)[:, :cols]
    codes = torch.full((rows, cols * cb // 8), 0xAA, dtype=torch.uint8, device=DEV)
    scales = torch.full((rows,), -1.0, dtype=torch.float32, device=DEV)
    mask = torch.full((rows, cols // 8), 0x55, dtype=torch.uint8, device=DEV) if want_mask else None
    xh = torch.full((rows, cols), float("nan"), dtype=torch.float32, device=DEV) if want_xh else None
    if fp4:
        q.quest_hadamard_quantize_fp4(x, had_block, alpha, codes=codes, scales=scales, mask=mask, xh_out=xh)
    elif absmax:
        q.quest_hadamard_quantize_absmax(x, had_block, bits, codes=codes, scales=scales, mask=mask, xh_out=xh)
    else:
        q.quest_hadamard_quantize(x, had_block, bits, alpha, outer_trust, codes=codes, scales=scales,
                                  mask=mask, xh_out=xh)
    torch.cuda.synchronize()
    return dict(codes=codes.cpu().numpy(), scales=scales.cpu().numpy(),
                mask=None if mask is None else mask.cpu().numpy(),
                xh=None if xh is None else xh.cpu().numpy(),
                dev=dict(codes=codes, scales=scales, mask=mask))


def compare_quantizer(got: dict, ref: qo.Projection, cols: int, bits: int, outer_trust: float = 1.0):
    """The parity bar for the fused quantizer against the double-precision oracle.

    Hadamard outputs within 1e-5 (relative to max(|x_h|, row rms)); scales within 2e-6 relative;
    packed codes and mask bits identical except for elements within 1e-6 (relative, in RMS units)
    of a rounding boundary / of the trust edge, which must be fewer than 1e-5 of all elements and
    may differ by one level only.  Returns the counts of tolerated differences.
    """
    levels = 1 << bits
    rms = ref.rms[:, None]
    safe = np.where(rms > 0, rms, 1.0)
    if got["xh"] is not None:
        bound = 1e-5 * np.maximum(np.abs(ref.xh), rms) + 1e-30
        assert np.all(np.abs(got["xh"].astype(np.float64) - ref.xh) <= bound), "Hadamard outputs differ"
    assert np.allclose(got["scales"].astype(np.float64), ref.scale, rtol=2e-6, atol=0), "scales differ"

    xn = ref.xh / safe
    step = 2.0 * ref.alpha / (levels - 1)
    u_got = qo.unpack_odd(got["codes"], cols, bits)
    u_ref = 2 * ref.k + 1
    diff = u_got != u_ref
    n_code = int(diff.sum())
    if n_code:
        t = xn[diff] / step
        near = np.abs(t - np.rint(t)) * step <= 1e-6 * np.maximum(np.abs(xn[diff]), 1.0)
        assert np.all(near), "a code differs away from any rounding boundary"
        assert np.all(np.abs(u_got[diff] - u_ref[diff]) == 2), "a code differs by more than one level"
    assert n_code < 1e-5 * diff.size + 1, f"{n_code} codes differ"
    if bits == 3:  # 3-bit codes live in nibbles whose top bit must stay clear
        assert np.all((got["codes"] & 0x88) == 0)

    n_mask = 0
    if got["mask"] is not None:
        t_got = qo.unpack_mask(got["mask"], cols)
        mdiff = t_got != ref.trust
        n_mask = int(mdiff.sum())
        if n_mask:
            edge = ref.alpha * (1.0 + outer_trust / (levels - 1))
            assert np.all(np.abs(np.abs(xn[mdiff]) - edge) <= 1e-6 * edge), "mask differs away from the edge"
        assert n_mask < 1e-5 * mdiff.size + 1, f"{n_mask} mask bits differ"
    return n_code, n_mask


def compare_quantizer_fp4(got: dict, ref, cols: int):
    """Parity bar for the FP4 variant: as compare_quantizer, the rounding boundaries being the
    midpoints between neighbouring E2M1 magnitudes (in units of alpha rms / 6) and zero (the sign bit)."""
    rms = ref.rms[:, None]
    safe = np.where(rms > 0, rms, 1.0)
    if got["xh"] is not None:
        bound = 1e-5 * np.maximum(np.abs(ref.xh), rms) + 1e-30
        assert np.all(np.abs(got["xh"].astype(np.float64) - ref.xh) <= bound), "Hadamard outputs differ"
    assert np.allclose(got["scales"].astype(np.float64), ref.scale, rtol=2e-6, atol=0), "scales differ"
    v_got = qo.unpack_fp4(got["codes"], cols)
    diff = (v_got != ref.value) | (np.signbit(v_got) != np.signbit(ref.value))
    n_code = int(diff.sum())
    if n_code:
        t = np.abs(6.0 * ref.xh / safe / ref.alpha)[diff]
        mids = np.array([0.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
        near = np.min(np.abs(t[:, None] - mids[None, :]), axis=1) <= 1e-6 * np.maximum(t, 1.0)
        assert np.all(near), "a code differs away from any rounding boundary"
        mag = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
        step = np.abs(np.searchsorted(mag, np.abs(v_got[diff])) - np.searchsorted(mag, np.abs(ref.value[diff])))
        assert np.all(step <= 1), "a code differs by more than one level"
    assert n_code < 1e-5 * diff.size + 1, f"{n_code} codes differ"
    n_mask = 0
    if got["mask"] is not None:
        mdiff = qo.unpack_mask(got["mask"], cols) != ref.trust
        n_mask = int(mdiff.sum())
        if n_mask:
            edge = ref.alpha * (1.0 + 1.0 / 6.0)
            xn = ref.xh / safe
            assert np.all(np.abs(np.abs(xn[mdiff]) - edge) <= 1e-6 * edge), "mask differs away from the edge"
        assert n_mask < 1e-5 * mdiff.size + 1
    return n_code, n_mask


BF16_HALF_ULP = 2.0 ** -8      # largest relative error of one round-to-nearest bf16 rounding


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def check_gemm_output(y: torch.Tensor, ref_acc: np.ndarray, sa: np.ndarray, sb: np.ndarray):
    """Dequantized bf16 output against the oracle accumulators and scales.

    (i) bit-exact against the same fp32 expression evaluated on the host,
    bf16((float(acc) * s_a) * s_b); (ii) every element within one bf16 rounding (2^-8 relative) of
    the double-precision product; (iii) norm-wise relative error below 2e-3.
    """
    from paper_2502_05003_amd import synth
    mirror = (ref_acc.astype(np.float32) * sa.astype(np.float32)[:, None]) * sb.astype(np.float32)[None, :]
    assert np.array_equal(bf16_bits(y), synth.to_bf16_bits(mirror)), "bf16 output bits differ from the fp32 mirror"
    if np.issubdtype(ref_acc.dtype, np.integer):
        ref = qo.dequant(ref_acc, sa.astype(np.float64), sb.astype(np.float64))
    else:   # FP4 accumulators: multiples of 1/4, held in double
        ref = ref_acc * sa.astype(np.float64)[:, None] * sb.astype(np.float64)[None, :]
    got = to_host_f64(y)
    assert np.all(np.abs(got - ref) <= BF16_HALF_ULP * (1 + 1e-5) * np.abs(ref) + 1e-38)
    assert np.linalg.norm(got - ref) <= 2e-3 * np.linalg.norm(ref)
    return got
