#!/usr/bin/env python3
"""Benchmark of the QuEST W4A4 linear-layer hot path on one MI355X.

A step is one pass of the whole path over one batch of the 1.6B-model MLP up-projection
(d = 2048, ffn 5632, 16384 tokens; Algorithm 1 + Algorithm 2 of arXiv 2502.05003):
    quantize X, quantize W, low-bit GEMM with bf16 epilogue,
    two 16-bit gradient GEMMs, two trust-masked inverse transforms.
Inputs are synthetic, seeded and resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--workload mlp_down_1p6b]
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
# down: X 16384x5632, W 2048x5632, block 512; the 7B pair: 4096 -> 11008 (block 4096) and back (block 256)
WORKLOADS = ("mlp_up_1p6b", "mlp_down_1p6b", "mlp_up_7b", "mlp_down_7b")
KERNELS = ("quantize_x", "quantize_w", "lowbit_gemm", "grad_gemm_x", "grad_gemm_w",
           "trust_backward_x", "trust_backward_w")
FP4_KERNELS = ("quantize_x_fp4", "lowbit_gemm_fp4")   # the FP4 variant of the forward (--only)


# HBM-side traffic per launch on this workload, bytes, from rocprofv3 --pmc FETCH_SIZE and
# --pmc WRITE_SIZE runs of this script (profiles/bench_step_mlp_up_1p6b_hbm_traffic.md): counter
# value in KiB per dispatch times 1024, FETCH_SIZE also times 2.0 -- the factor by which it
# under-reads the plain streaming kernel of --copy-calibration (2^30 bytes in, 2^30 out); WRITE_SIZE
# reads that kernel exactly.  A gradient matmul is the sum over the kernels of its call.
MIB = 1 << 20
MEASURED_TRAFFIC = {
    "quantize_x": (2 * 32.1 + 20.1) * MIB,
    "quantize_w": (2 * 11.0 + 6.9) * MIB,
    "lowbit_gemm": (2 * 64.0 + 176.0) * MIB,
    "grad_gemm_x": (2 * (2.9 + 273.0) + 22.0 + 88.5) * MIB,
    "grad_gemm_w": (2 * (8.3 + 441.0 + 52.0) + 64.0 + 120.4 + 22.0) * MIB,
    "trust_backward_x": (2 * 34.1 + 64.0) * MIB,
    "trust_backward_w": (2 * 11.8 + 22.0) * MIB,
}


def algorithmic_bytes_quantize(rows, cols, cb=4, in_bytes=2):
    """input + packed codes + mask bitmap + one fp32 scale per row."""
    return rows * cols * in_bytes + rows * cols * cb // 8 + rows * cols // 8 + 4 * rows


def algorithmic_bytes_backward(rows, cols):
    """bf16 gradient in + bitmap + bf16 out."""
    return rows * cols * 2 + rows * cols // 8 + rows * cols * 2


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
    """The seven launches of one step as (name, thunk) pairs, in execution order."""
    M, N, K, n, bits = cfg["M"], cfg["N"], cfg["K"], cfg["had_block"], cfg["bits"]
    if fp4:   # the FP4 variant of the method (Sec. 4.4): E2M1 codes, FP4 matrix instructions
        return [
            ("quantize_x", lambda: q.quest_hadamard_quantize_fp4(b.x, n, codes=b.x_codes, scales=b.x_scales,
                                                                 mask=b.x_mask)),
            ("quantize_w", lambda: q.quest_hadamard_quantize_fp4(b.w, n, codes=b.w_codes, scales=b.w_scales,
                                                                 mask=b.w_mask)),
            ("lowbit_gemm", lambda: q.quest_lowbit_gemm_fp4(b.x_codes, b.x_scales, b.w_codes, b.w_scales, K, y=b.y)),
            ("grad_gemm_x", lambda: q.quest_grad_gemm_fp4(0, b.dy, b.w_codes, b.w_scales, M, N, K, out=b.g_x,
                                                          workspace=b.ws_gx)),
            ("grad_gemm_w", lambda: q.quest_grad_gemm_fp4(1, b.dy, b.x_codes, b.x_scales, M, N, K, out=b.g_w,
                                                          workspace=b.ws_gw)),
            ("trust_backward_x", lambda: q.quest_trust_backward(b.g_x, b.x_mask, n, out=b.dx)),
            ("trust_backward_w", lambda: q.quest_trust_backward(b.g_w, b.w_mask, n, out=b.dw)),
        ]
    return [
        ("quantize_x", lambda: q.quest_hadamard_quantize(b.x, n, bits, codes=b.x_codes,
                                                         scales=b.x_scales, mask=b.x_mask)),
        ("quantize_w", lambda: q.quest_hadamard_quantize(b.w, n, bits, codes=b.w_codes,
                                                         scales=b.w_scales, mask=b.w_mask)),
        ("lowbit_gemm", lambda: q.quest_lowbit_gemm(b.x_codes, b.x_scales, b.w_codes, b.w_scales,
                                                    K, bits, y=b.y, workspace=b.ws_gemm)),
        ("grad_gemm_x", lambda: q.quest_grad_gemm(0, b.dy, b.w_codes, b.w_scales, bits, M, N, K,
                                                  out=b.g_x, workspace=b.ws_gx)),
        ("grad_gemm_w", lambda: q.quest_grad_gemm(1, b.dy, b.x_codes, b.x_scales, bits, M, N, K,
                                                  out=b.g_w, workspace=b.ws_gw)),
        ("trust_backward_x", lambda: q.quest_trust_backward(b.g_x, b.x_mask, n, out=b.dx)),
        ("trust_backward_w", lambda: q.quest_trust_backward(b.g_w, b.w_mask, n, out=b.dw)),
    ]


def cpu_baseline(x_bits, w_bits, dy_bits, cfg):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same step."""
    import numpy as np
    from oracle import quest_oracle as qo

    M, N, K, n, bits = cfg["M"], cfg["N"], cfg["K"], cfg["had_block"], cfg["bits"]
    rows_q = M             # rows of X through HT + projection (W is done whole)
    rows_g = 2048          # rows of X through the forward matmul and the backward pass
    qo.threads()
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
    seconds = time.perf_counter() - t0
    # the three matmuls dominate the step's operation count; the sample ran rows_g of M rows of each
    ops = 6.0 * rows_g * N * K
    return {"value": ops / seconds / 1e12, "unit": "TOPS", "cores": qo.threads(), "kind": "oracle",
            "sample": (f"quantize {rows_q} of {M} X rows and all of W; forward matmul, both gradient "
                       f"matmuls and both masked inverse transforms on {rows_g} of {M} token rows; "
                       f"{seconds:.1f} s; value = 6*{rows_g}*N*K ops / time")}


def library_gemm_us(torch, dev, M, N, K, reps=20):
    """The vendor library on the step's three products, with ready-made operands: int8 codes for
    the forward product (no widening from nibbles), bf16 matrices for the gradient products (no
    expansion of codes).  Mean microseconds per call, launched back to back."""
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


# Linear layers of the 1.6B model the paper trained and of the proportionally scaled 7B model its
# per-layer figure also shows (Sec. 5, "Runtime Results"): name, K (inputs), N (outputs).
SWEEP_LAYERS = [("1.6B attention 2048->2048", 2048, 2048), ("1.6B up/gate 2048->5632", 2048, 5632),
                ("1.6B down 5632->2048", 5632, 2048), ("7B attention 4096->4096", 4096, 4096),
                ("7B up/gate 4096->11008", 4096, 11008), ("7B down 11008->4096", 11008, 4096)]


def layer_sweep(torch, q, synth, dev, tokens, reps=10):
    """Per-layer forward time of the 4-bit path against the 16-bit product (the paper's per-layer
    speedup figure, Sec. 5): activations quantized per call with and without the Hadamard transform
    (no mask: inference form), weights quantized beforehand, the vendor library's bf16 product as
    the baseline.  Microseconds per launch, launched back to back over rotating buffer sets."""
    # A millisecond of other GPU work goes first, so that the host has queued all timed launches
    # before the first of them starts: short kernels are then timed back to back on the GPU, not
    # at the rate the host can issue them.
    filler = [torch.zeros(8192, 8192, dtype=torch.bfloat16, device=dev) for _ in range(3)]
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(launches):
        for f in launches:
            f()
        torch.cuda.synchronize()
        torch.matmul(filler[0], filler[1], out=filler[2])
        start.record()
        for i in range(reps):
            launches[i % len(launches)]()
        end.record()
        torch.cuda.synchronize()
        return start.elapsed_time(end) * 1e3 / reps

    out = []
    for name, K, N in SWEEP_LAYERS:
        n = K & -K                                  # widest power-of-two block that divides the row
        n_sets = max(2, min(4, int(1.5e9 // (tokens * (K + N) * 2))))
        w_bits = synth.gaussian(N, K, 0.02, seed=1)
        w = torch.from_numpy(w_bits.view("int16")).to(dev).view(torch.bfloat16)
        w_codes = torch.empty(N, K // 2, dtype=torch.uint8, device=dev)
        w_scales = torch.empty(N, dtype=torch.float32, device=dev)
        q.quest_hadamard_quantize(w, n, 4, codes=w_codes, scales=w_scales)
        x_bits = synth.outlier_activations(tokens, K, 0.005, 50.0, seed=0)
        xs = [torch.from_numpy(x_bits.view("int16")).to(dev).view(torch.bfloat16) for _ in range(n_sets)]
        codes = [torch.empty(tokens, K // 2, dtype=torch.uint8, device=dev) for _ in range(n_sets)]
        scales = [torch.empty(tokens, dtype=torch.float32, device=dev) for _ in range(n_sets)]
        ys = [torch.empty(tokens, N, dtype=torch.bfloat16, device=dev) for _ in range(n_sets)]

        def quantize(i, block):
            return lambda: q.quest_hadamard_quantize(xs[i], block, 4, codes=codes[i], scales=scales[i])

        t_q = timed([quantize(i, n) for i in range(n_sets)])
        t_q_plain = timed([quantize(i, 1) for i in range(n_sets)])
        for i in range(n_sets):
            quantize(i, n)()
        t_gemm = timed([(lambda i=i: q.quest_lowbit_gemm(codes[i], scales[i], w_codes, w_scales, K, 4, y=ys[i]))
                        for i in range(n_sets)])
        t_bf16 = timed([(lambda i=i: torch.matmul(xs[i], w.t(), out=ys[i])) for i in range(n_sets)])
        out.append({"layer": name, "tokens": tokens, "K": K, "N": N, "had_block": n,
                    "quantize_us": t_q, "quantize_no_transform_us": t_q_plain, "gemm_int4_us": t_gemm,
                    "matmul_bf16_library_us": t_bf16,
                    "speedup_with_transform": t_bf16 / (t_q + t_gemm),
                    "speedup_without_transform": t_bf16 / (t_q_plain + t_gemm)})
        del xs, codes, scales, ys, w, w_codes, w_scales
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain streaming kernel of known size (reads and writes 1 GiB each), "
                         "the yardstick for the rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--graph", action="store_true",
                    help="also replay the step from HIP graphs (one per buffer set, captured after the timed "
                         "region) and report that step time as ms_per_step_graph: the same kernels without "
                         "event pairs and host launch gaps")
    ap.add_argument("--library-gemm", action="store_true",
                    help="also time the vendor library (torch.matmul bf16, torch._int_mm int8) on this "
                         "workload's three matrix products, operands already in the library's own format: "
                         "context for the kernels' rooflines, not part of the step")
    ap.add_argument("--layer-sweep", action="store_true",
                    help="instead of the benchmark step: forward time of the 4-bit path per linear-layer "
                         "shape of the 1.6B and 7B models against the library's bf16 product (the paper's "
                         "per-layer speedup figure); prints one JSON line of its own")
    ap.add_argument("--tokens", type=int, default=16384, help="rows of the activations in --layer-sweep")
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

    if args.layer_sweep:
        print(json.dumps({"layer_sweep": layer_sweep(torch, q, synth, dev, args.tokens)}))
        return

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
            n, bits = cfg["had_block"], cfg["bits"]
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

    events = [{k: event_pair() for k in KERNELS} for _ in range(args.steps)]
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
          for k in KERNELS}
    ms_per_step = elapsed * 1e3 / args.steps
    gemm_ops = 2.0 * M * N * K
    step_ops = 3.0 * gemm_ops

    def traffic(name):   # measured for the headline workload only
        headline = args.workload == WORKLOAD and args.grid == "int4" and cfg["bits"] == 4
        return MEASURED_TRAFFIC[name] if headline else None

    def hbm(name, nbytes):
        gbs = nbytes / (ms[name] * 1e-3) / 1e9
        return {"kernel": name, "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": gbs / HBM_PEAK_GBS, "traffic": traffic(name), "algorithmic": nbytes,
                "ms": ms[name]}

    def mfma(name, peak):
        t = gemm_ops / (ms[name] * 1e-3) / 1e12
        return {"kernel": name, "bound": "mfma", "achieved": t, "peak": peak,
                "unit": "TFLOP/s" if peak == BF16_PEAK_TFLOPS else "TOPS", "frac": t / peak,
                "traffic": traffic(name), "ms": ms[name]}

    rooflines = {
        "quantize_x": hbm("quantize_x", algorithmic_bytes_quantize(M, K, cb)),
        "quantize_w": hbm("quantize_w", algorithmic_bytes_quantize(N, K, cb)),
        "lowbit_gemm": mfma("lowbit_gemm", FP4_PEAK_TOPS if args.grid == "fp4" else INT8_PEAK_TOPS),
        "grad_gemm_x": mfma("grad_gemm_x", BF16_PEAK_TFLOPS),
        "grad_gemm_w": mfma("grad_gemm_w", BF16_PEAK_TFLOPS),
        "trust_backward_x": hbm("trust_backward_x", algorithmic_bytes_backward(M, K)),
        "trust_backward_w": hbm("trust_backward_w", algorithmic_bytes_backward(N, K)),
    }
    headline = dict(rooflines["lowbit_gemm"])
    headline["unit"] = "TFLOP/s"   # integer multiply-adds counted as 2 ops each, in units of 1e12/s

    result = {
        "metric": f"W{cfg['bits']}A{cfg['bits']} QuEST-linear TOPS at d={min(K, N) if args.workload.endswith('7b') else 2048} "
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
        "quantizer_GBps": rooflines["quantize_x"]["achieved"],
        "gemm_TOPS": rooflines["lowbit_gemm"]["achieved"],
        "forward_TOPS": gemm_ops / ((ms["quantize_x"] + ms["quantize_w"] + ms["lowbit_gemm"]) * 1e-3) / 1e12,
        "roofline": headline,
        "kernels": rooflines,
    }
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            torch.add(src, 1, out=dst)   # one elementwise kernel: 2^30 bytes in, 2^30 bytes out
        torch.cuda.synchronize()
        # what a plain streaming kernel reaches on this machine, next to the 8 TB/s of the datasheet
        result["streaming_kernel_GBps"] = 3 * 2.0 * (1 << 30) / (time.perf_counter() - t0) / 1e9
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
    if not args.no_cpu_baseline and args.grid == "int4":   # the oracle leg times the headline (integer-grid) path
        result["cpu_baseline"] = cpu_baseline(x_bits, w_bits, dy_bits, cfg)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
