#!/usr/bin/env python3
"""Benchmark of the QuEST W4A4 linear-layer hot path on one MI355X.

A step is one pass of the whole path over one batch of the 1.6B-model MLP up-projection
(d = 2048, ffn 5632, 16384 tokens; Algorithm 1 + Algorithm 2 of arXiv 2502.05003):
    quantize X and W (one call, one launch), low-bit GEMM with bf16 epilogue,
    two 16-bit gradient GEMMs, both trust-masked inverse transforms (one call, one launch).
Inputs are synthetic, seeded and resident in HBM before the timed region.  Prints ONE JSON line.

After the timed region (never inside it) the same run also measures, unless --no-extra:
  * a plain streaming kernel (what this machine's memory system gives a copy), so that every
    bandwidth-bound kernel is also reported as a fraction of that;
  * the forward-only 100M-model layer (X 8192x1024 with outlier channels, Hadamard blocks 128 and
    1024) and the bit-width sweep b in {1,2,3,4,8} on heavy-tailed activations (quantizer-only
    bandwidth and trust-mask density), the other two benchmark configurations of this build.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-extra]
                    [--workload mlp_down_1p6b] [--grid fp4] [--bits b] [--graph] [--library-gemm]
                    [--only KERNEL]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
INT8_PEAK_TOPS = 5000.0      # dense INT8 MFMA (5.0 POP/s)
BF16_PEAK_TFLOPS = 2500.0    # dense bf16 MFMA
FP4_PEAK_TOPS = 10100.0      # dense FP4 MFMA (--grid fp4)

WORKLOAD = "mlp_up_1p6b"     # the headline: X 16384x2048, W 5632x2048, Hadamard block 2048, b = 4
# down: X 16384x5632, W 2048x5632, block 512; the 7B pair (hidden 4096, MLP width 11008: the model of
# the paper's per-layer runtime figure) is there for context, never the default
WORKLOADS = ("mlp_up_1p6b", "mlp_down_1p6b", "mlp_up_7b", "mlp_down_7b")
# calls of a step: activations and weights are quantized by one call (Algorithm 1 steps 2-5 for both
# operands), and the two masked inverse transforms that end Algorithm 2 are one call as well; --only
# can also launch either operand's quantizer or inverse transform alone
STEP_KERNELS = ("quantize_xw", "lowbit_gemm", "grad_gemm_x", "grad_gemm_w", "trust_backward_xw")
SINGLE_OPERAND_KERNELS = ("quantize_x", "quantize_w", "trust_backward_x", "trust_backward_w")
KERNELS = SINGLE_OPERAND_KERNELS + STEP_KERNELS
FP4_KERNELS = ("quantize_x_fp4", "lowbit_gemm_fp4")   # the FP4 variant of the forward (--only)


# HBM-side traffic per launch on the headline workload, MiB read and MiB written, copied from the
# table in profiles/bench_step_mlp_up_1p6b_hbm_traffic.md (tests/test_repo_contract.py checks that
# the two agree): rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE runs of this script, counter value
# in KiB per dispatch, FETCH_SIZE scaled by the factor by which it under-reads the streaming kernel
# of known size that the same run launches.  A gradient matmul is the sum over the kernels of its call.
MIB = 1 << 20
MEASURED_TRAFFIC_MIB = {
    "quantize_xw": (86.1, 27.2),
    "lowbit_gemm": (126.5, 176.0),
    "grad_gemm_x": (555.7, 102.8),
    "grad_gemm_w": (1005.5, 205.7),
    "trust_backward_xw": (91.5, 86.0),
}


def algorithmic_bytes_quantize(rows, cols, cb=4, in_bytes=2):
    """input + packed codes + mask bitmap + one fp32 scale per row."""
    return rows * cols * in_bytes + rows * cols * cb // 8 + rows * cols // 8 + 4 * rows


def algorithmic_bytes_backward(rows, cols):
    """bf16 gradient in + bitmap + bf16 out."""
    return rows * cols * 2 + rows * cols // 8 + rows * cols * 2


def algorithmic_bytes_gemm(M, N, K, cb=4):
    """packed codes of both operands + their scales + the bf16 output."""
    return (M + N) * K * cb // 8 + 4 * (M + N) + 2 * M * N


class BufferSet:
    """One complete set of device buffers for a step (rotated so that caches cannot serve re-use)."""

    def __init__(self, torch, dev, x_bits, w_bits, dy_bits, cfg, q, fp4=False):
        import numpy as np
        M, N, K = cfg["M"], cfg["N"], cfg["K"]

        def bf16(a):
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(dev)

        u8, f32, b16 = torch.uint8, torch.float32, torch.bfloat16
        self.x, self.w, self.dy = bf16(x_bits), bf16(w_bits), bf16(dy_bits)
        self.x_codes = torch.empty(M, K // 2, dtype=u8, device=dev)
        self.x_scales = torch.empty(M, dtype=f32, device=dev)
        self.x_mask = torch.empty(M, K // 8, dtype=u8, device=dev)
        self.w_codes = torch.empty(N, K // 2, dtype=u8, device=dev)
        self.w_scales = torch.empty(N, dtype=f32, device=dev)
        self.w_mask = torch.empty(N, K // 8, dtype=u8, device=dev)
        self.y = torch.empty(M, N, dtype=b16, device=dev)
        self.g_x = torch.empty(M, K, dtype=b16, device=dev)
        self.g_w = torch.empty(N, K, dtype=b16, device=dev)
        self.dx = torch.empty(M, K, dtype=b16, device=dev)
        self.dw = torch.empty(N, K, dtype=b16, device=dev)
        # scratch of the calls that need it (the library allocates nothing): sized by its host queries
        grad_query = q.quest_grad_gemm_fp4_workspace_bytes if fp4 else q.quest_grad_gemm_workspace_bytes
        self.ws_gx = torch.empty(max(grad_query(0, M, N, K), 16), dtype=u8, device=dev)
        self.ws_gw = torch.empty(max(grad_query(1, M, N, K), 16), dtype=u8, device=dev)
        self.ws_gemm = torch.empty(max(q.quest_lowbit_gemm_workspace_bytes(M, N, K, cfg["bits"]), 16), dtype=u8,
                                   device=dev)


def step_kernels(q, b, cfg, fp4=False):
    """The launches of one step as (name, thunk) pairs, in execution order."""
    M, N, K, n, bits = cfg["M"], cfg["N"], cfg["K"], cfg["had_block"], cfg["bits"]
    if fp4:   # the FP4 variant of the method (Sec. 4.4): E2M1 codes, FP4 matrix instructions
        return [
            ("quantize_xw", lambda: q.quest_hadamard_quantize_fp4_pair(b.x, b.w, n, x_codes=b.x_codes,
                                                                       x_scales=b.x_scales, x_mask=b.x_mask,
                                                                       w_codes=b.w_codes, w_scales=b.w_scales,
                                                                       w_mask=b.w_mask)),
            ("lowbit_gemm", lambda: q.quest_lowbit_gemm_fp4(b.x_codes, b.x_scales, b.w_codes, b.w_scales, K, y=b.y)),
            ("grad_gemm_x", lambda: q.quest_grad_gemm_fp4(0, b.dy, b.w_codes, b.w_scales, M, N, K, out=b.g_x,
                                                          workspace=b.ws_gx)),
            ("grad_gemm_w", lambda: q.quest_grad_gemm_fp4(1, b.dy, b.x_codes, b.x_scales, M, N, K, out=b.g_w,
                                                          workspace=b.ws_gw)),
            ("trust_backward_xw", lambda: q.quest_trust_backward_pair(b.g_x, b.x_mask, b.g_w, b.w_mask, n,
                                                                      out_x=b.dx, out_w=b.dw)),
        ]
    return [
        ("quantize_xw", lambda: q.quest_hadamard_quantize_pair(b.x, b.w, n, bits, x_codes=b.x_codes,
                                                               x_scales=b.x_scales, x_mask=b.x_mask,
                                                               w_codes=b.w_codes, w_scales=b.w_scales,
                                                               w_mask=b.w_mask)),
        ("lowbit_gemm", lambda: q.quest_lowbit_gemm(b.x_codes, b.x_scales, b.w_codes, b.w_scales,
                                                    K, bits, y=b.y, workspace=b.ws_gemm)),
        ("grad_gemm_x", lambda: q.quest_grad_gemm(0, b.dy, b.w_codes, b.w_scales, bits, M, N, K,
                                                  out=b.g_x, workspace=b.ws_gx)),
        ("grad_gemm_w", lambda: q.quest_grad_gemm(1, b.dy, b.x_codes, b.x_scales, bits, M, N, K,
                                                  out=b.g_w, workspace=b.ws_gw)),
        ("trust_backward_xw", lambda: q.quest_trust_backward_pair(b.g_x, b.x_mask, b.g_w, b.w_mask, n,
                                                                  out_x=b.dx, out_w=b.dw)),
    ]


def single_operand_kernels(q, b, cfg, fp4=False):
    """One operand's quantizer or inverse transform by itself (--only): name -> thunk."""
    n, bits = cfg["had_block"], cfg["bits"]
    if fp4:
        def quantize(t, codes, scales, mask):
            return lambda: q.quest_hadamard_quantize_fp4(t, n, codes=codes, scales=scales, mask=mask)
    else:
        def quantize(t, codes, scales, mask):
            return lambda: q.quest_hadamard_quantize(t, n, bits, codes=codes, scales=scales, mask=mask)
    return {
        "quantize_x": quantize(b.x, b.x_codes, b.x_scales, b.x_mask),
        "quantize_w": quantize(b.w, b.w_codes, b.w_scales, b.w_mask),
        "trust_backward_x": lambda: q.quest_trust_backward(b.g_x, b.x_mask, n, out=b.dx),
        "trust_backward_w": lambda: q.quest_trust_backward(b.g_w, b.w_mask, n, out=b.dw),
    }


def cpu_baseline(x_bits, w_bits, dy_bits, cfg):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same step: once
    on all cores and once, on a smaller sample, on a single thread."""
    from oracle import quest_oracle as qo

    M, N, K, n, bits = cfg["M"], cfg["N"], cfg["K"], cfg["had_block"], cfg["bits"]

    def sample(rows_q, rows_g):
        """Quantize rows_q rows of X and all of W; the three matmuls and both masked inverse
        transforms on rows_g token rows.  Returns seconds."""
        t0 = time.perf_counter()
        px = qo.hadamard_quantize(x_bits[:rows_q], n, bits)
        pw = qo.hadamard_quantize(w_bits, n, bits)
        ux, uw = qo.unpack_odd(px.codes[:rows_g], K, bits), qo.unpack_odd(pw.codes, K, bits)
        acc = qo.gemm_odd(ux, uw)
        qo.dequant(acc, px.scale[:rows_g], pw.scale)
        dy = qo.widen(dy_bits[:rows_g])
        gx = qo.grad_input(dy, uw, pw.scale)
        qo.trust_backward(gx, px.trust[:rows_g], n)
        gw = qo.grad_weight(dy, ux, px.scale[:rows_g])
        qo.trust_backward(gw, pw.trust, n)
        return time.perf_counter() - t0

    cores = qo.threads()
    rows_g = 2048
    seconds = sample(M, rows_g)
    # the three matmuls dominate the step's operation count; the sample ran rows_g of M rows of each
    result = {"value": 6.0 * rows_g * N * K / seconds / 1e12, "unit": "TOPS", "cores": cores, "kind": "oracle",
              "sample": (f"quantize {M} of {M} X rows and all of W; forward matmul, both gradient "
                         f"matmuls and both masked inverse transforms on {rows_g} of {M} token rows; "
                         f"{seconds:.1f} s; value = 6*{rows_g}*N*K ops / time")}
    rows_one = 128
    qo.set_threads(1)
    try:
        seconds_one = sample(1024, rows_one)
    finally:
        qo.set_threads(cores)
    result["single_thread"] = {"value": 6.0 * rows_one * N * K / seconds_one / 1e12, "unit": "TOPS", "cores": 1,
                               "sample": (f"quantize 1024 of {M} X rows and all of W; the matmuls and inverse "
                                          f"transforms on {rows_one} token rows; {seconds_one:.1f} s")}
    return result


def library_gemm_us(torch, dev, M, N, K, reps=20):
    """Context for the matmul rooflines, not part of the step: the vendor library on the step's three
    products with operands already in its own format: int8 matrices for the forward product (no
    widening from nibbles), bf16 matrices for the gradient products (no expansion of codes).  Mean
    microseconds per call, launched back to back."""
    a8 = torch.randint(-15, 16, (M, K), device=dev, dtype=torch.int8)
    b8 = torch.randint(-15, 16, (N, K), device=dev, dtype=torch.int8)
    dy = torch.randn(M, N, device=dev, dtype=torch.bfloat16)
    w = torch.randn(N, K, device=dev, dtype=torch.bfloat16)
    x = torch.randn(M, K, device=dev, dtype=torch.bfloat16)
    cases = {"int8_forward": lambda: torch._int_mm(a8, b8.t()),
             "bf16_grad_x": lambda: torch.matmul(dy, w),
             "bf16_grad_w": lambda: torch.matmul(dy.t(), x)}
    out = {}
    for name, f in cases.items():
        for _ in range(5):
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            f()
        torch.cuda.synchronize()
        out[name] = (time.perf_counter() - t0) * 1e6 / reps
    return out


def time_launches(torch, launches, batch=200, batches=5, warmup=20):
    """Median over `batches` of the mean time per launch, microseconds: each batch is `batch`
    launches back to back between one pair of HIP events on the current stream, rotating over
    `launches` (one thunk per buffer set, so that more than a cache's worth of other data lies
    between two uses of a buffer)."""
    import numpy as np
    for i in range(warmup):
        launches[i % len(launches)]()
    torch.cuda.synchronize()
    samples = []
    for _ in range(batches):
        start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for i in range(batch):
            launches[i % len(launches)]()
        end.record()
        torch.cuda.synchronize()
        samples.append(start.elapsed_time(end) * 1e3 / batch)
    return float(np.median(samples))


def streaming_rate(torch, dev):
    """A plain streaming kernel, 2^30 bytes in and 2^30 bytes out per launch (one elementwise kernel
    of the tensor library): GB/s of read + write.  Also the yardstick for the traffic counters."""
    src = torch.ones(1 << 28, dtype=torch.int32, device=dev)
    dst = torch.empty_like(src)
    us = time_launches(torch, [lambda: torch.add(src, 1, out=dst)], batch=5, batches=5, warmup=2)
    del src, dst
    torch.cuda.empty_cache()
    return 2.0 * (1 << 30) / (us * 1e-6) / 1e9


def mfma_loop_rates(torch, dev, codes, lib_dir):
    """What the matrix pipes sustain on this machine with nothing else to do: the register-only loop
    of include/quest_probe.h on operand data shaped like the method's, taken from quantizer output
    (`codes`: packed 4-bit codes): signed bytes 8 u for the INT8 instruction, bf16 values s u for
    the bf16 one.  Six launches of a few milliseconds back to back; the chip is power-limited, so
    the first (best) and the last (sustained) differ.  Returns T(FL)OP/s."""
    import ctypes
    lib = ctypes.CDLL(os.path.join(lib_dir, "libquest_probe.so"))
    lib.quest_probe_mfma_loop.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                          ctypes.c_int32, ctypes.c_void_p]
    lib.quest_probe_mfma_loop.restype = ctypes.c_int32
    workgroups, iterations = 512, 12000                      # two waves per SIMD
    count = workgroups * 256 * 32                            # operand bytes
    u = (codes.reshape(-1)[:count] & 0xF).to(torch.int16) * 2 - 15          # odd integers of the 4-bit grid
    operands = {0: (u * 8).to(torch.int8).contiguous(),
                1: (u[:count // 2].to(torch.float32) * 0.17).to(torch.bfloat16).contiguous()}
    sink = torch.empty(workgroups * 256, dtype=torch.int32, device=dev)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    out = {}
    for kind, name, macs in ((0, "int8", 32768.0), (1, "bf16", 16384.0)):
        ops = 2.0 * workgroups * 4 * iterations * 8 * macs
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(6)]
        for start, end in pairs:
            start.record()
            status = lib.quest_probe_mfma_loop(kind, ctypes.c_void_p(operands[kind].data_ptr()),
                                               ctypes.c_void_p(sink.data_ptr()), workgroups, iterations, stream)
            end.record()
            if status != 0:
                raise RuntimeError(f"quest_probe_mfma_loop: status {status}")
        torch.cuda.synchronize()
        rates = [ops / (a.elapsed_time(b) * 1e-3) / 1e12 for a, b in pairs]
        out[name] = {"sustained": rates[-1], "best": max(rates)}
    return out


def bf16_tensor(torch, bits, dev):
    return torch.from_numpy(bits.view("int16")).to(dev).view(torch.bfloat16)


def untrusted_fraction(torch, mask):
    """Share of zero bits in a trust bitmap (elements outside the trust region)."""
    table = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int64, device=mask.device)
    ones = int(table[mask.reshape(-1).long()].sum().item())
    return 1.0 - ones / (mask.numel() * 8)


def relative_error(torch, q, x, codes, scales, n, bits):
    """||xhat_h - x_h|| / ||x_h|| of a quantized operand: x_h from the library's own transform output,
    xhat_h = s (2 c - (L - 1)) decoded from the packed 4-bit codes with tensor-library bit operations."""
    assert bits == 4
    rows, cols = x.shape
    xh = torch.empty(rows, cols, dtype=torch.float32, device=x.device)
    scratch_c, scratch_s = torch.empty_like(codes), torch.empty_like(scales)
    q.quest_hadamard_quantize(x, n, bits, codes=scratch_c, scales=scratch_s, xh_out=xh)
    lo = (codes & 0xF).to(torch.float32)
    hi = (codes >> 4).to(torch.float32)
    u = torch.stack((lo, hi), dim=2).reshape(rows, cols) * 2.0 - 15.0
    xhat = u * scales[:, None]
    return float(((xhat - xh).double().norm() / xh.double().norm()).item())


def extra_config_100m(torch, q, synth, dev, streaming):
    """Forward only, 100M-model MLP up-projection: quantizer at Hadamard blocks 128 and 1024, GEMM."""
    x_bits, w_bits, cfg = synth.make_config("mlp_up_100m", seed=0)
    M, N, K, bits = cfg["M"], cfg["N"], cfg["K"], cfg["bits"]
    n_sets = 48                                       # 22 MB per set: > 1 GiB between two uses of a set
    x0, w = bf16_tensor(torch, x_bits, dev), bf16_tensor(torch, w_bits, dev)
    xs = [x0.clone() for _ in range(n_sets)]
    codes = [torch.empty(M, K // 2, dtype=torch.uint8, device=dev) for _ in range(n_sets)]
    scales = [torch.empty(M, dtype=torch.float32, device=dev) for _ in range(n_sets)]
    masks = [torch.empty(M, K // 8, dtype=torch.uint8, device=dev) for _ in range(n_sets)]
    w_codes = torch.empty(N, K // 2, dtype=torch.uint8, device=dev)
    w_scales = torch.empty(N, dtype=torch.float32, device=dev)
    out = {"workload": f"mlp_up_100m: X {M}x{K} bf16 N(0,1) with 1% of channels x20, W {N}x{K} bf16 N(0,0.02^2), "
                       f"b={bits}, forward only", "quantize_x": {}}
    nbytes = algorithmic_bytes_quantize(M, K)
    for block in (128, 1024):
        us = time_launches(torch, [(lambda i=i: q.quest_hadamard_quantize(xs[i], block, bits, codes=codes[i],
                                                                          scales=scales[i], mask=masks[i]))
                                   for i in range(n_sets)])
        gbs = nbytes / (us * 1e-6) / 1e9
        out["quantize_x"][f"block_{block}"] = {
            "us": us, "GBps": gbs, "frac": gbs / HBM_PEAK_GBS, "frac_of_streaming": gbs / streaming,
            "algorithmic": nbytes,
            "relative_error": relative_error(torch, q, xs[0], codes[0], scales[0], block, bits)}
    # both operands of the layer by one call (the weights are quantized anew in every training step)
    ws = [w.clone() for _ in range(n_sets)]
    w_masks = torch.empty(N, K // 8, dtype=torch.uint8, device=dev)
    pair_bytes = nbytes + algorithmic_bytes_quantize(N, K)
    out["quantize_xw"] = {}
    for block in (128, 1024):
        us = time_launches(torch, [(lambda i=i: q.quest_hadamard_quantize_pair(
            xs[i], ws[i], block, bits, x_codes=codes[i], x_scales=scales[i], x_mask=masks[i], w_codes=w_codes,
            w_scales=w_scales, w_mask=w_masks)) for i in range(n_sets)])
        gbs = pair_bytes / (us * 1e-6) / 1e9
        out["quantize_xw"][f"block_{block}"] = {"us": us, "GBps": gbs, "frac": gbs / HBM_PEAK_GBS,
                                                "frac_of_streaming": gbs / streaming, "algorithmic": pair_bytes}
    del ws
    q.quest_hadamard_quantize(w, 1024, bits, codes=w_codes, scales=w_scales)
    for i in range(n_sets):
        q.quest_hadamard_quantize(xs[i], 1024, bits, codes=codes[i], scales=scales[i])
    ys = [torch.empty(M, N, dtype=torch.bfloat16, device=dev) for _ in range(12)]   # 64 MiB each
    us = time_launches(torch, [(lambda i=i: q.quest_lowbit_gemm(codes[i], scales[i], w_codes, w_scales, K, bits,
                                                                y=ys[i])) for i in range(12)],
                       batch=100)
    tops = 2.0 * M * N * K / (us * 1e-6) / 1e12
    out["lowbit_gemm"] = {"us": us, "TOPS": tops, "frac": tops / INT8_PEAK_TOPS, "ops": 2.0 * M * N * K}
    return out


def extra_config_bit_sweep(torch, q, synth, dev, streaming):
    """Bit-width sweep on heavy-tailed activations: quantizer-only bandwidth and mask density per b."""
    x_bits, w_bits, cfg = synth.make_config("bit_sweep_1p6b", seed=0)
    M, N, K, n = cfg["M"], cfg["N"], cfg["K"], cfg["had_block"]
    n_sets = 12
    x0, w0 = bf16_tensor(torch, x_bits, dev), bf16_tensor(torch, w_bits, dev)
    xs = [x0.clone() for _ in range(n_sets)]
    ws = [w0.clone() for _ in range(n_sets)]
    out = {"workload": f"bit_sweep_1p6b: X {M}x{K} bf16 Student-t(nu=3) at unit RMS, W {N}x{K} bf16 N(0,0.02^2), "
                       f"Hadamard block {n}, quantizer only", "bits": {}}
    for bits in (1, 2, 3, 4, 8):
        cb = q.quest_container_bits(bits)
        entry = {}
        for name, tensors, rows in (("x", xs, M), ("w", ws, N)):
            codes = [torch.empty(rows, K * cb // 8, dtype=torch.uint8, device=dev) for _ in range(n_sets)]
            scales = [torch.empty(rows, dtype=torch.float32, device=dev) for _ in range(n_sets)]
            masks = [torch.empty(rows, K // 8, dtype=torch.uint8, device=dev) for _ in range(n_sets)]
            us = time_launches(torch, [(lambda i=i: q.quest_hadamard_quantize(tensors[i], n, bits, codes=codes[i],
                                                                              scales=scales[i], mask=masks[i]))
                                       for i in range(n_sets)])
            nbytes = algorithmic_bytes_quantize(rows, K, cb)
            gbs = nbytes / (us * 1e-6) / 1e9
            entry[name] = {"us": us, "GBps": gbs, "frac": gbs / HBM_PEAK_GBS, "frac_of_streaming": gbs / streaming,
                           "algorithmic": nbytes, "untrusted_fraction": untrusted_fraction(torch, masks[0])}
            if bits == 1 and name == "x":   # the narrower outer trust region of the 1-bit case (Sec. 3.3)
                q.quest_hadamard_quantize(tensors[0], n, bits, 0.0, 0.30, codes=codes[0], scales=scales[0],
                                          mask=masks[0])
                entry[name]["untrusted_fraction_outer_trust_0.30"] = untrusted_fraction(torch, masks[0])
            del codes, scales, masks
        out["bits"][str(bits)] = entry
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip what is measured after the timed region: the streaming kernel, the 100M-model "
                         "forward layer and the bit-width sweep")
    ap.add_argument("--streaming-only", action="store_true",
                    help="of the measurements after the timed region keep only the streaming kernel (the "
                         "yardstick of the rocprofv3 traffic counters)")
    ap.add_argument("--workload", choices=WORKLOADS, default=WORKLOAD,
                    help="layer shape; the default is the one the headline metric is quoted on")
    ap.add_argument("--grid", choices=("int4", "fp4"), default="int4",
                    help="int4: the headline path (Eq. 1 grid, INT8 matrix cores); fp4: the FP4 variant of "
                         "Sec. 4.4 end to end (E2M1 codes, FP4 matrix instructions)")
    ap.add_argument("--bits", type=int, choices=(1, 2, 3, 4), default=None,
                    help="bit width b of the integer grid for both operands (default: the workload's, 4); the "
                         "paper trains at 1 to 4 bits, the matrix cores see signed bytes at every width")
    ap.add_argument("--only", choices=KERNELS + FP4_KERNELS, default=None,
                    help="profiling aid: launch just this kernel --warmup + --steps times back to back "
                         "(outputs of a whole step prepared once) and print its mean time; no benchmark line")
    ap.add_argument("--library-gemm", action="store_true",
                    help="also time the vendor library (torch.matmul bf16, torch._int_mm int8) on this "
                         "workload's three matrix products, operands already in the library's own format: "
                         "context for the kernels' rooflines, not part of the step")
    ap.add_argument("--graph", action="store_true",
                    help="also replay the step from HIP graphs (one per buffer set, captured after the timed "
                         "region) and report that step time as ms_per_step_graph: the same kernels without "
                         "event pairs and host launch gaps")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (one MI355X per box); run with --gpus 1")

    import numpy as np
    import torch

    from paper_2502_05003_amd import binding as q
    from paper_2502_05003_amd import synth

    if not os.path.exists(q.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    q.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    x_bits, w_bits, cfg = synth.make_config(args.workload, seed=0)
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    if args.bits is not None:
        if args.grid == "fp4" and args.bits != 4:
            sys.exit("bench.py: the FP4 grid has 4-bit codes")
        cfg["bits"] = args.bits
    cb = q.quest_container_bits(cfg["bits"])
    dy_bits = synth.upstream_gradient(M, N, seed=0)
    n_sets = 3   # ~0.7 GiB per set: > 1 GiB of other traffic between two uses of any buffer
    q.quest_init()
    sets = [BufferSet(torch, dev, x_bits, w_bits, dy_bits, cfg, q, args.grid == "fp4") for _ in range(n_sets)]
    torch.cuda.synchronize()

    if args.only:
        # one whole step first, so that every input of the chosen kernel exists
        for b in sets:
            for _, launch in step_kernels(q, b, cfg, args.grid == "fp4"):
                launch()
        if args.only in FP4_KERNELS:
            n = cfg["had_block"]
            for b in sets:
                q.quest_hadamard_quantize_fp4(b.x, n, codes=b.x_codes, scales=b.x_scales, mask=b.x_mask)
                q.quest_hadamard_quantize_fp4(b.w, n, codes=b.w_codes, scales=b.w_scales, mask=b.w_mask)
        torch.cuda.synchronize()

        def chosen(b):
            if args.only == "quantize_x_fp4":
                return lambda: q.quest_hadamard_quantize_fp4(b.x, cfg["had_block"], codes=b.x_codes,
                                                             scales=b.x_scales, mask=b.x_mask)
            if args.only == "lowbit_gemm_fp4":
                return lambda: q.quest_lowbit_gemm_fp4(b.x_codes, b.x_scales, b.w_codes, b.w_scales, K, y=b.y)
            if args.only in SINGLE_OPERAND_KERNELS:
                return single_operand_kernels(q, b, cfg, args.grid == "fp4")[args.only]
            return dict(step_kernels(q, b, cfg, args.grid == "fp4"))[args.only]

        launches = [chosen(b) for b in sets]
        for i in range(args.warmup):
            launches[i % n_sets]()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            launches[i % n_sets]()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / args.steps
        print(json.dumps({"only": args.only, "workload": args.workload, "launches": args.steps,
                          "us_per_launch_back_to_back": us}))
        return

    # Every kernel launch is bracketed by a pair of HIP events on the stream it is launched on
    # (torch's current stream), in the warm-up and in the timed region alike, so that the per-kernel
    # durations behind the rooflines come from the very steps that `value` is computed from.  An
    # event pair around a single launch also counts the idle gaps at both ends, a few microseconds;
    # half the duration of an empty pair (one is recorded per step) is subtracted, which brings the
    # figures to within a few percent of the rocprofv3 kernel durations of this same command
    # (profiles/).  The pairs cost the step about 2 % against launching the kernels back to back.
    def event_pair():
        return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    step_names = STEP_KERNELS
    events = [{k: event_pair() for k in step_names} for _ in range(args.steps)]
    empty = [event_pair() for _ in range(args.steps)]
    scratch_pair = event_pair()

    def timed_step(i, pairs, gap_pair):
        for name, launch in step_kernels(q, sets[i % n_sets], cfg, args.grid == "fp4"):
            start, end = pairs[name] if pairs else scratch_pair
            start.record()
            launch()
            end.record()
        gap_pair[0].record()
        gap_pair[1].record()

    for i in range(args.warmup):
        timed_step(i, None, scratch_pair)
    torch.cuda.synchronize()

    # Timed region: exactly `steps` whole steps, host clock, synchronised on both sides.
    t0 = time.perf_counter()
    for i in range(args.steps):
        timed_step(i, events[i], empty[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    gap_ms = 0.5 * float(np.median([a.elapsed_time(b) for a, b in empty]))
    ms = {k: max(float(np.mean([e[k][0].elapsed_time(e[k][1]) for e in events])) - gap_ms, 1e-6)
          for k in step_names}
    ms_per_step = elapsed * 1e3 / args.steps
    gemm_ops = 2.0 * M * N * K
    step_ops = 3.0 * gemm_ops

    streaming = None if args.no_extra else streaming_rate(torch, dev)

    def traffic(name):   # measured for the headline workload only: bytes read + written beyond the L2s
        headline = args.workload == WORKLOAD and args.grid == "int4" and cfg["bits"] == 4
        return sum(MEASURED_TRAFFIC_MIB[name]) * MIB if headline else None

    def hbm(name, nbytes):
        gbs = nbytes / (ms[name] * 1e-3) / 1e9
        return {"kernel": name, "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": gbs / HBM_PEAK_GBS, "frac_of_streaming": gbs / streaming if streaming else None,
                "traffic": traffic(name), "algorithmic": nbytes, "ms": ms[name]}

    def mfma(name, peak, nbytes):
        t = gemm_ops / (ms[name] * 1e-3) / 1e12
        return {"kernel": name, "bound": "mfma", "achieved": t, "peak": peak,
                "unit": "TFLOP/s" if peak == BF16_PEAK_TFLOPS else "TOP/s", "frac": t / peak,
                "traffic": traffic(name), "algorithmic": nbytes, "ms": ms[name]}

    grad_x_bytes = 2 * M * N + N * K * cb // 8 + 4 * N + 2 * M * K     # dY + weight codes + scales + G_x
    grad_w_bytes = 2 * M * N + M * K * cb // 8 + 4 * M + 2 * N * K     # dY + activation codes + scales + G_w
    rooflines = {"quantize_xw": hbm("quantize_xw", algorithmic_bytes_quantize(M, K, cb) +
                                    algorithmic_bytes_quantize(N, K, cb))}
    quantize_ms = ms["quantize_xw"]
    rooflines.update({
        "lowbit_gemm": mfma("lowbit_gemm", FP4_PEAK_TOPS if args.grid == "fp4" else INT8_PEAK_TOPS,
                            algorithmic_bytes_gemm(M, N, K, cb)),
        "grad_gemm_x": mfma("grad_gemm_x", BF16_PEAK_TFLOPS, grad_x_bytes),
        "grad_gemm_w": mfma("grad_gemm_w", BF16_PEAK_TFLOPS, grad_w_bytes),
        "trust_backward_xw": hbm("trust_backward_xw", algorithmic_bytes_backward(M, K) +
                                 algorithmic_bytes_backward(N, K)),
    })

    result = {
        "metric": f"W{cfg['bits']}A{cfg['bits']} QuEST-linear TOPS at d={min(K, N)} "
                  "(forward + backward step; quantizer GB/s in kernels)",
        "value": step_ops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("fp4" if args.grid == "fp4" else "int8") + " (forward matmul) / bf16 (gradient matmuls) / f32 (transform, quantizer)",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: X {M}x{K} bf16 N(0,1) + 0.5% outlier channels x50, "
                               f"W {N}x{K} bf16 N(0,0.02^2), dY {M}x{N} bf16, Hadamard block "
                               f"{cfg['had_block']}, b={cfg['bits']}, forward+backward",
                   "grid": args.grid, "M": M, "N": N, "K": K, "had_block": cfg["had_block"], "bits": cfg["bits"],
                   "buffer_sets": n_sets, "event_gap_us_subtracted": gap_ms * 1e3},
        "quantizer_GBps": rooflines["quantize_xw"]["achieved"],
        "gemm_TOPS": rooflines["lowbit_gemm"]["achieved"],
        "forward_TOPS": gemm_ops / ((quantize_ms + ms["lowbit_gemm"]) * 1e-3) / 1e12,
        "roofline": dict(rooflines["lowbit_gemm"]),
        "kernels": rooflines,
    }
    if streaming:
        # what a plain streaming kernel reaches on this machine, next to the 8 TB/s of the datasheet
        result["streaming_kernel_GBps"] = streaming
    if args.graph:
        capture_stream = torch.cuda.Stream()
        graphs = []
        for b in sets:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.stream(capture_stream):
                with torch.cuda.graph(g, stream=capture_stream):
                    for _, launch in step_kernels(q, b, cfg, args.grid == "fp4"):
                        launch()
            graphs.append(g)
        for i in range(args.warmup):
            graphs[i % n_sets].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[i % n_sets].replay()
        torch.cuda.synchronize()
        result["ms_per_step_graph"] = (time.perf_counter() - t0) * 1e3 / args.steps
    if args.library_gemm:
        result["library_gemm_us"] = library_gemm_us(torch, dev, M, N, K)
    if not args.no_extra and not args.streaming_only:
        loop = mfma_loop_rates(torch, dev, sets[0].x_codes, os.path.dirname(q.LIB_PATH))
        result["mfma_loop"] = {"int8_TOPS": loop["int8"], "bf16_TFLOPS": loop["bf16"],
                               "what": "register-only matrix-instruction loop on operand data shaped like the "
                                       "method's, 6 launches back to back: first (best) and last (sustained)"}
        for name in ("lowbit_gemm", "grad_gemm_x", "grad_gemm_w"):
            ceiling = loop["bf16" if name.startswith("grad") else "int8"]["sustained"]
            if not (name == "lowbit_gemm" and args.grid == "fp4"):
                rooflines[name]["frac_of_mfma_loop"] = rooflines[name]["achieved"] / ceiling
        result["roofline"] = dict(rooflines["lowbit_gemm"])
        del sets
        torch.cuda.empty_cache()
        result["forward_100m"] = extra_config_100m(torch, q, synth, dev, streaming)
        torch.cuda.empty_cache()
        result["bit_sweep"] = extra_config_bit_sweep(torch, q, synth, dev, streaming)
    if not args.no_cpu_baseline and args.grid == "int4":   # the oracle leg times the headline (integer-grid) path
        result["cpu_baseline"] = cpu_baseline(x_bits, w_bits, dy_bits, cfg)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
