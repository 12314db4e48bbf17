"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs."""
import math

import numpy as np
import pytest
import torch

from oracle import quest_oracle as qo
from paper_2502_05003_amd import binding as q
from paper_2502_05003_amd import synth

from gpu_util import (BF16_HALF_ULP, DEV, check_gemm_output, compare_quantizer, compare_quantizer_fp4, gpu_quantize,
                      grad_ws, lowbit_ws, to_device, to_host_f64, weight_only_ws)

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------ quantizer

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_tiny_config_full_forward(dtype):
    """256x512 activations, 512x512 weights, block 512, W4A4: dense-matrix oracle, all outputs."""
    x, w, cfg = synth.make_config("tiny", seed=0)
    if dtype == "bf16":
        x, w = synth.to_bf16_bits(x), synth.to_bf16_bits(w)
    n, bits, K = cfg["had_block"], cfg["bits"], cfg["K"]
    gx, gw = gpu_quantize(x, n, bits), gpu_quantize(w, n, bits)
    px, pw = qo.hadamard_quantize(x, n, bits, dense=True), qo.hadamard_quantize(w, n, bits, dense=True)
    compare_quantizer(gx, px, K, bits)
    compare_quantizer(gw, pw, K, bits)
    # mask density on Gaussian rows ~ the closed-form Gaussian tail (Sec. 3.2 / App. A.1)
    frac = 1.0 - qo.unpack_mask(gx["mask"], K).mean()
    assert abs(frac - 7.327e-3) < 1.5e-3

    M, N = x.shape[0], w.shape[0]
    y = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    acc = torch.empty(M, N, dtype=torch.int32, device=DEV)
    q.quest_lowbit_gemm(gx["dev"]["codes"], gx["dev"]["scales"], gw["dev"]["codes"], gw["dev"]["scales"],
                        K, bits, y=y, acc_out=acc)
    torch.cuda.synchronize()
    ref_acc = qo.gemm_odd(qo.unpack_odd(gx["codes"], K, bits), qo.unpack_odd(gw["codes"], K, bits))
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), ref_acc)
    got_y = check_gemm_output(y, ref_acc, gx["scales"], gw["scales"])
    # and the whole thing approximates x w^T (Sec. 3.3: the transform is unitary)
    exact = qo.widen(x) @ qo.widen(w).T
    assert np.linalg.norm(got_y - exact) / np.linalg.norm(exact) < 0.2


QUANT_CASES = [
    # rows, cols, block, bits, dtype   (several tiles, ragged row counts, every container width)
    (37, 1024, 128, 4, "bf16"), (37, 1024, 1024, 4, "bf16"), (130, 2048, 2048, 4, "bf16"),
    (70, 5632, 512, 4, "bf16"), (5, 4096, 4096, 4, "bf16"), (3, 16384, 16384, 4, "bf16"),
    (33, 2048, 2048, 1, "bf16"), (33, 2048, 2048, 2, "bf16"), (33, 2048, 2048, 3, "bf16"),
    (33, 2048, 2048, 8, "bf16"), (19, 512, 1, 4, "bf16"), (19, 512, 2, 4, "f32"),
    (19, 512, 4, 2, "f32"), (19, 24, 8, 4, "f32"), (1, 8, 8, 4, "bf16"), (300, 64, 64, 8, "f32"),
    (21, 1536, 512, 3, "f32"), (9, 11008, 256, 4, "bf16"),
    # every bit width on the matrix-core path: rows of 1024, 4096 and 5632 (ends in half a tile)
    (70, 5632, 512, 1, "bf16"), (70, 5632, 512, 2, "bf16"), (70, 5632, 512, 3, "bf16"), (70, 5632, 512, 8, "bf16"),
    (9, 1024, 1024, 1, "bf16"), (9, 1024, 1024, 2, "bf16"), (9, 1024, 1024, 3, "bf16"), (9, 1024, 1024, 8, "bf16"),
    (5, 4096, 4096, 1, "bf16"), (5, 4096, 4096, 2, "bf16"), (5, 4096, 4096, 3, "bf16"), (5, 4096, 4096, 8, "bf16"),
    # fp32 rows on the matrix-core path (fp32 MFMA): rows of 512 .. 5632 with their widest block
    (21, 512, 512, 4, "f32"), (37, 1024, 1024, 4, "f32"), (130, 2048, 2048, 4, "f32"), (9, 4096, 4096, 4, "f32"),
    (70, 5632, 512, 4, "f32"),
    # rows of 11008 = 43 x 256 (the last 1024-element tile is three quarters full)
    (70, 11008, 256, 4, "bf16"), (33, 11008, 128, 4, "bf16"), (33, 11008, 16, 4, "bf16"), (5, 11008, 1, 4, "bf16"),
    # the other hidden and MLP widths of the paper's model family, widest block and none
    (37, 640, 128, 4, "bf16"), (37, 768, 256, 4, "bf16"), (37, 1280, 256, 4, "bf16"), (37, 1664, 128, 4, "bf16"),
    (37, 1792, 256, 4, "bf16"), (37, 2816, 256, 4, "bf16"), (37, 3584, 512, 4, "bf16"), (37, 4608, 512, 4, "bf16"),
    (9, 640, 1, 4, "bf16"), (9, 1664, 32, 4, "bf16"), (9, 2816, 8, 4, "bf16"), (9, 4608, 1, 4, "bf16"),
    (37, 640, 128, 4, "f32"), (37, 768, 256, 4, "f32"), (37, 1280, 256, 4, "f32"), (37, 1664, 128, 4, "f32"),
    (37, 1792, 256, 4, "f32"), (37, 2816, 256, 4, "f32"), (37, 3584, 512, 4, "f32"), (37, 4608, 512, 4, "f32"),
    # blocks that span two of a row's four tiles, and one of them
    (33, 4096, 2048, 4, "bf16"), (33, 4096, 1024, 4, "bf16"), (33, 4096, 512, 4, "bf16"),
    # more rows than waves on the chip (4096): every wave takes several rows, the next one staged through
    # LDS while the current one is quantized, with a ragged last pass; a row count below one pass
    (8229, 1024, 1024, 4, "bf16"), (9001, 2048, 512, 2, "bf16"), (5003, 4096, 4096, 8, "bf16"),
    (4099, 2048, 2048, 4, "bf16"),
]


@pytest.mark.parametrize("rows,cols,n,bits,dtype", QUANT_CASES)
def test_quantizer_matches_oracle(rows, cols, n, bits, dtype):
    x = synth.outlier_activations(rows, cols, 0.01, 20.0, seed=rows + cols + bits, dtype=dtype)
    got = gpu_quantize(x, n, bits)
    ref = qo.hadamard_quantize(x, n, bits, dense=(n <= 512))
    compare_quantizer(got, ref, cols, bits)
    # inference form (no mask, no debug output): another kernel instance, the same codes and scales
    lean = gpu_quantize(x, n, bits, want_mask=False, want_xh=False)
    assert np.array_equal(lean["codes"], got["codes"]) and np.array_equal(lean["scales"], got["scales"])


@pytest.mark.parametrize("cols,n", [(512, 512), (1024, 1024), (2048, 2048), (4096, 4096), (5632, 512)])
def test_fp32_rows_keep_all_24_bits(cols, n):
    """fp32 rows reach the matrix cores as three bf16 pieces: rows whose entries are +-v in the
    pattern of one Hadamard row, with v using all 24 significant bits, must come out as sqrt(n) v at
    that row's index and zero elsewhere, to fp32 rounding (a lost or mis-signed piece is 2^-16 or more)."""
    values = [1.0 + 2.0 ** -8 + 2.0 ** -16 + 2.0 ** -23, 3.0 - 2.0 ** -22, 0.7499999403953552, 1.0 + 2.0 ** -20]
    picks = [0, 1, n - 1, n // 2 + 3, 37 % n, n // 4]
    rows = len(values) * len(picks)
    x = np.empty((rows, cols), dtype=np.float32)
    j = np.arange(cols)
    expect = np.zeros((rows, cols))
    for a, v in enumerate(values):
        for b, r in enumerate(picks):
            parity = np.array([bin(int(r) & int(c % n)).count("1") & 1 for c in j])
            x[a * len(picks) + b] = np.float32(v) * (1.0 - 2.0 * parity)
            expect[a * len(picks) + b, r::n] = np.sqrt(n) * float(np.float32(v))
    got = gpu_quantize(x, n, 4)
    bound = 3e-7 * np.sqrt(n) * np.abs(x[:, :1]).astype(np.float64)
    assert np.all(np.abs(got["xh"].astype(np.float64) - expect) <= bound)


PAIR_CASES = [
    # rows_x, rows_w, cols, block, bits, dtype, with masks
    (130, 70, 2048, 2048, 4, "bf16", True), (4099, 1408, 2048, 2048, 4, "bf16", True),
    (37, 300, 1024, 128, 4, "bf16", False), (70, 33, 5632, 512, 4, "bf16", True), (33, 9, 2048, 2048, 2, "bf16", True),
    (0, 70, 2048, 2048, 4, "bf16", True), (70, 0, 2048, 2048, 4, "bf16", True), (1, 1, 2048, 2048, 4, "bf16", True),
    # shapes the one-launch kernel does not cover: the call falls back to one launch per operand
    (21, 40, 1536, 512, 3, "f32", True), (19, 5, 24, 8, 4, "f32", False), (37, 12, 1024, 1024, 4, "f32", True),
]


@pytest.mark.parametrize("rows_x,rows_w,cols,block,bits,dtype,masks", PAIR_CASES)
def test_pair_call_equals_two_single_calls(rows_x, rows_w, cols, block, bits, dtype, masks):
    """Algorithm 1 for x and w in one call (one launch where the matrix-core kernel covers the shape):
    every output byte equals that of two calls of quest_hadamard_quantize, which the cases above
    compare with the oracle."""
    x = synth.outlier_activations(max(rows_x, 1), cols, 0.01, 20.0, seed=rows_x + cols, dtype=dtype)[:rows_x]
    w = synth.gaussian(max(rows_w, 1), cols, 0.02, seed=rows_w + bits, dtype=dtype)[:rows_w]
    cb = qo.container_bits(bits)
    def outputs(rows):
        return (torch.zeros(rows, cols * cb // 8, dtype=torch.uint8, device=DEV),
                torch.zeros(rows, dtype=torch.float32, device=DEV),
                torch.zeros(rows, cols // 8, dtype=torch.uint8, device=DEV) if masks else None)
    xd, wd = to_device(x), to_device(w)
    single = [outputs(rows_x), outputs(rows_w)]
    for t, (c, s, m) in zip((xd, wd), single):
        if t.shape[0]:
            q.quest_hadamard_quantize(t, block, bits, codes=c, scales=s, mask=m)
    pair = [outputs(rows_x), outputs(rows_w)]
    q.quest_hadamard_quantize_pair(xd, wd, block, bits, x_codes=pair[0][0], x_scales=pair[0][1], x_mask=pair[0][2],
                                   w_codes=pair[1][0], w_scales=pair[1][1], w_mask=pair[1][2])
    torch.cuda.synchronize()
    for a, b in zip(single, pair):
        for u, v in zip(a, b):
            if u is not None:
                assert torch.equal(u.view(torch.uint8) if u.dtype == torch.uint8 else u.view(torch.int32),
                                   v.view(torch.uint8) if v.dtype == torch.uint8 else v.view(torch.int32))


@pytest.mark.parametrize("rows_x,rows_w,cols,block,dtype,masks",
                         [(130, 70, 2048, 2048, "bf16", True), (4099, 1408, 2048, 2048, "bf16", True),
                          (37, 300, 1024, 128, "bf16", False), (70, 33, 5632, 512, "bf16", True),
                          (0, 70, 2048, 2048, "bf16", True), (70, 0, 2048, 2048, "bf16", True),
                          (21, 40, 1536, 512, "f32", True)])
def test_fp4_pair_call_equals_two_single_calls(rows_x, rows_w, cols, block, dtype, masks):
    """The FP4 quantizer (Sec. 4.4) for x and w in one call: every output byte equals that of two calls
    of quest_hadamard_quantize_fp4, which test_fp4_quantizer_matches_oracle compares with the oracle."""
    x = synth.outlier_activations(max(rows_x, 1), cols, 0.01, 20.0, seed=rows_x + cols, dtype=dtype)[:rows_x]
    w = synth.gaussian(max(rows_w, 1), cols, 0.02, seed=rows_w + 4, dtype=dtype)[:rows_w]
    def outputs(rows):
        return (torch.zeros(rows, cols // 2, dtype=torch.uint8, device=DEV),
                torch.zeros(rows, dtype=torch.float32, device=DEV),
                torch.zeros(rows, cols // 8, dtype=torch.uint8, device=DEV) if masks else None)
    xd, wd = to_device(x), to_device(w)
    single = [outputs(rows_x), outputs(rows_w)]
    for t, (c, s, m) in zip((xd, wd), single):
        if t.shape[0]:
            q.quest_hadamard_quantize_fp4(t, block, codes=c, scales=s, mask=m)
    pair = [outputs(rows_x), outputs(rows_w)]
    q.quest_hadamard_quantize_fp4_pair(xd, wd, block, x_codes=pair[0][0], x_scales=pair[0][1], x_mask=pair[0][2],
                                       w_codes=pair[1][0], w_scales=pair[1][1], w_mask=pair[1][2])
    torch.cuda.synchronize()
    for a, b in zip(single, pair):
        for u, v in zip(a, b):
            if u is not None:
                assert torch.equal(u.view(torch.uint8) if u.dtype == torch.uint8 else u.view(torch.int32),
                                   v.view(torch.uint8) if v.dtype == torch.uint8 else v.view(torch.int32))


def test_pair_call_on_strided_operands():
    """Row strides above the row length, a different one per operand: the one-launch kernel takes each
    operand's own stride (a slice of a wider activation buffer next to contiguous weights)."""
    cols, block, bits = 2048, 2048, 4
    wide_x = to_device(synth.outlier_activations(300, cols + 64, 0.01, 20.0, seed=3, dtype="bf16"))
    wide_w = to_device(synth.gaussian(77, cols + 512, 0.02, seed=4, dtype="bf16"))
    xd, wd = wide_x[:, :cols], wide_w[:, :cols]
    assert xd.stride(0) == cols + 64 and wd.stride(0) == cols + 512

    def outputs(rows):
        return (torch.zeros(rows, cols // 2, dtype=torch.uint8, device=DEV),
                torch.zeros(rows, dtype=torch.float32, device=DEV),
                torch.zeros(rows, cols // 8, dtype=torch.uint8, device=DEV))
    single = [outputs(300), outputs(77)]
    for t, (c, s, m) in zip((xd.contiguous(), wd.contiguous()), single):
        q.quest_hadamard_quantize(t, block, bits, codes=c, scales=s, mask=m)
    pair = [outputs(300), outputs(77)]
    q.quest_hadamard_quantize_pair(xd, wd, block, bits, x_codes=pair[0][0], x_scales=pair[0][1], x_mask=pair[0][2],
                                   w_codes=pair[1][0], w_scales=pair[1][1], w_mask=pair[1][2])
    torch.cuda.synchronize()
    for a, b in zip(single, pair):
        for u, v in zip(a, b):
            assert torch.equal(u.view(torch.uint8) if u.dtype == torch.uint8 else u.view(torch.int32),
                               v.view(torch.uint8) if v.dtype == torch.uint8 else v.view(torch.int32))


ABSMAX_CASES = [(37, 1024, 128, 4, "bf16"), (130, 2048, 2048, 4, "bf16"), (70, 5632, 512, 4, "bf16"),
                (33, 2048, 1, 4, "bf16"), (33, 2048, 2048, 2, "bf16"), (33, 2048, 2048, 8, "f32"),
                (19, 512, 1, 3, "f32"), (21, 1536, 512, 1, "f32"), (4100, 256, 256, 4, "bf16"),
                # the matrix-core path, bf16 and fp32 rows
                (21, 512, 512, 4, "bf16"), (37, 1024, 1024, 4, "bf16"), (9, 4096, 4096, 4, "bf16"),
                (21, 512, 512, 4, "f32"), (37, 1024, 1024, 4, "f32"), (130, 2048, 2048, 4, "f32"),
                (9, 4096, 4096, 4, "f32"), (70, 5632, 512, 4, "f32")]


@pytest.mark.parametrize("rows,cols,n,bits,dtype", ABSMAX_CASES)
def test_absmax_quantizer_matches_oracle(rows, cols, n, bits, dtype):
    """The AbsMax comparison quantizer (Sec. 4.1), with and without the transform (block 1 is the
    no-transform ablation); an all-zero row among the inputs."""
    x = synth.outlier_activations(rows, cols, 0.01, 20.0, seed=rows + cols + bits, dtype=dtype)
    x[2] = 0
    got = gpu_quantize(x, n, bits, absmax=True)
    ref = qo.hadamard_quantize_absmax(x, n, bits, dense=(1 < n <= 512))
    compare_quantizer(got, ref, cols, bits)
    assert np.all(got["mask"] == 0xFF)
    assert got["scales"][2] == 0.0
    assert np.all(qo.unpack_odd(got["codes"][2:3], cols, bits) == 1)
    lean = gpu_quantize(x, n, bits, absmax=True, want_mask=False, want_xh=False)
    assert np.array_equal(lean["codes"], got["codes"]) and np.array_equal(lean["scales"], got["scales"])


def test_transform_and_gaussian_clip_each_reduce_the_error():
    """The mechanisms behind Sec. 4.3 (Hadamard ablation) and the AbsMax baseline of Sec. 4.1, on the
    headline activations (outlier channels): relative error of the 4-bit reconstruction from the
    GPU's own codes, for the four combinations of {transform, none} x {Gaussian-fitted clip, AbsMax}."""
    x, _, cfg = synth.make_config("mlp_up_1p6b", seed=0, rows=2048)
    K, bits = cfg["K"], cfg["bits"]
    xd = qo.widen(x)
    err = {}
    for n in (2048, 1):
        target = qo.hadamard(xd, n)
        for absmax in (False, True):
            got = gpu_quantize(x, n, bits, want_xh=False, want_mask=False, absmax=absmax)
            xhat = got["scales"][:, None].astype(np.float64) * qo.unpack_odd(got["codes"], K, bits)
            err[(n, absmax)] = np.linalg.norm(xhat - target) / np.linalg.norm(target)
    print({f"block {n}, {'absmax' if a else 'rms clip'}": round(v, 4) for (n, a), v in err.items()})
    assert err[(2048, False)] < err[(2048, True)] < err[(1, True)]
    assert err[(2048, False)] < err[(1, False)]


@pytest.mark.parametrize("cols,n,dtype", [(2048, 2048, "bf16"), (5632, 512, "bf16"), (1536, 512, "f32"),
                                          (2048, 2048, "f32")])
def test_non_finite_rows_stay_in_their_rows(cols, n, dtype):
    """A row that holds an infinity or a NaN gets a non-finite scale (its codes are unspecified) and
    leaves every other row's outputs as they are without it; the masked inverse transform likewise
    keeps a non-finite gradient row to itself.  (Matrix-core kernels and the general ones.)"""
    rows = 41
    x = synth.outlier_activations(rows, cols, 0.01, 20.0, seed=cols, dtype=dtype)
    clean = gpu_quantize(x, n, 4, want_xh=False)
    bad = x.copy()
    inf_bits, nan_bits = (0x7F80, 0x7FC0) if dtype == "bf16" else (np.float32(np.inf), np.float32(np.nan))
    bad[3, 17] = inf_bits
    bad[29, cols - 1] = nan_bits
    got = gpu_quantize(bad, n, 4, want_xh=False)
    assert not np.isfinite(got["scales"][3]) and not np.isfinite(got["scales"][29])
    keep = np.ones(rows, dtype=bool)
    keep[[3, 29]] = False
    for name in ("codes", "scales", "mask"):
        assert np.array_equal(got[name][keep], clean[name][keep]), name
    if dtype == "bf16":
        g = synth.gaussian(rows, cols, 0.03, seed=1, dtype="bf16")
        out_clean = torch.empty(rows, cols, dtype=torch.bfloat16, device=DEV)
        q.quest_trust_backward(to_device(g), clean["dev"]["mask"], n, out=out_clean)
        g_bad = g.copy()
        g_bad[3, 17], g_bad[29, cols - 1] = inf_bits, nan_bits
        out_bad = torch.empty(rows, cols, dtype=torch.bfloat16, device=DEV)
        q.quest_trust_backward(to_device(g_bad), clean["dev"]["mask"], n, out=out_bad)
        torch.cuda.synchronize()
        keep_t = torch.from_numpy(keep).to(DEV)
        assert torch.equal(out_bad[keep_t].view(torch.int16), out_clean[keep_t].view(torch.int16))


FP4_CASES = [(37, 1024, 128, "bf16", 0.0), (130, 2048, 2048, "bf16", 0.0), (70, 5632, 512, "bf16", 0.0),
             (33, 2048, 1, "bf16", 2.0), (19, 512, 64, "f32", 0.0), (4100, 256, 256, "bf16", 3.5)]


@pytest.mark.parametrize("rows,cols,n,dtype,alpha", FP4_CASES)
def test_fp4_quantizer_matches_oracle(rows, cols, n, dtype, alpha):
    """The FP4 variant of the projection (Sec. 4.4): E2M1 codes, scale alpha rms / 6, trust mask."""
    x = synth.outlier_activations(rows, cols, 0.01, 20.0, seed=rows + cols, dtype=dtype)
    x[2] = 0
    got = gpu_quantize(x, n, 4, alpha=alpha, fp4=True)
    ref = qo.hadamard_quantize_fp4(x, n, alpha=(alpha if alpha > 0 else None), dense=(1 < n <= 512))
    compare_quantizer_fp4(got, ref, cols)
    assert got["scales"][2] == 0.0 and np.all(got["codes"][2] == 0) and np.all(got["mask"][2] == 0xFF)


def test_quantizer_options_and_degenerate_rows():
    rows, cols, n = 16, 1024, 256
    x = synth.student_t_activations(rows, cols, 3.0, seed=4, dtype="bf16")
    x[3] = 0                                  # all-zero row
    x[5] = 0
    x[5, 17] = 0x3F80                         # single 1.0
    x[7] = 0x4000                             # constant row: one nonzero coefficient per block
    for bits, alpha, ot in ((4, 2.9, 0.5), (1, 0.0, 0.30), (1, 0.0, 1.0), (2, 1.3, 2.0), (8, 0.0, 0.0)):
        got = gpu_quantize(x, n, bits, alpha=alpha, outer_trust=ot)
        ref = qo.hadamard_quantize(x, n, bits, alpha=(alpha if alpha > 0 else None), outer_trust=ot)
        compare_quantizer(got, ref, cols, bits, outer_trust=ot)
        L = 1 << bits
        assert got["scales"][3] == 0.0
        assert np.all(qo.unpack_odd(got["codes"][3:4], cols, bits) == 1)        # k = 0 -> u = +1
        assert np.all(got["mask"][3] == 0xFF)
        assert L >= 2
    # leading dimension larger than cols, no mask, no xh
    got = gpu_quantize(x, n, 4, want_xh=False, want_mask=False, ld=cols + 64)
    ref = qo.hadamard_quantize(x, n, 4)
    compare_quantizer(got, ref, cols, 4)


def test_quantizer_full_size_headline_shape():
    """16384 x 2048 bf16 with outlier channels, block 2048, b = 4: whole tensor against the oracle."""
    x, _, cfg = synth.make_config("mlp_up_1p6b", seed=0)
    got = gpu_quantize(x, cfg["had_block"], cfg["bits"], want_xh=False)
    ref = qo.hadamard_quantize(x, cfg["had_block"], cfg["bits"])
    n_code, n_mask = compare_quantizer(got, ref, cfg["K"], cfg["bits"])
    print(f"full size: {n_code} codes and {n_mask} mask bits at a boundary out of {x.size}")


@pytest.mark.parametrize("n", [128, 1024])
def test_quantizer_and_gemm_100m_layer_full_size(n):
    """X 8192 x 1024 with 1 % outlier channels x 20, W 4096 x 1024, Hadamard block 128 and 1024:
    whole tensors against the oracle, the forward GEMM (68.7 GOP) on sampled rows.  The full-width
    transform must also give the smaller quantization error (why Sec. 3.1 transforms whole rows)."""
    x, w, cfg = synth.make_config("mlp_up_100m", seed=0)
    K, bits = cfg["K"], cfg["bits"]
    gx = gpu_quantize(x, n, bits, want_xh=False)
    gw = gpu_quantize(w, n, bits, want_xh=False)
    rx, rw = qo.hadamard_quantize(x, n, bits), qo.hadamard_quantize(w, n, bits)
    counts_x = compare_quantizer(gx, rx, K, bits)
    counts_w = compare_quantizer(gw, rw, K, bits)
    print(f"100M layer, block {n}: X {counts_x[0]} codes / {counts_x[1]} mask bits at a boundary out of {x.size}; "
          f"W {counts_w[0]} / {counts_w[1]} out of {w.size}")
    M, N = x.shape[0], w.shape[0]
    y = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    q.quest_lowbit_gemm(gx["dev"]["codes"], gx["dev"]["scales"], gw["dev"]["codes"], gw["dev"]["scales"],
                        K, bits, y=y)
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(n).choice(M, size=64, replace=False))
    rows[0], rows[-1] = 0, M - 1
    ux, uw = qo.unpack_odd(gx["codes"][rows], K, bits), qo.unpack_odd(gw["codes"], K, bits)
    check_gemm_output(y[torch.from_numpy(rows).to(DEV)], qo.gemm_odd(ux, uw), gx["scales"][rows], gw["scales"])
    # relative quantization error of the GPU's own codes, in the Hadamard domain
    xhat = gx["scales"][:, None].astype(np.float64) * qo.unpack_odd(gx["codes"], K, bits)
    err = np.linalg.norm(xhat - rx.xh) / np.linalg.norm(rx.xh)
    print(f"block {n}: relative error of xhat_h {err:.4f}")
    assert err < (0.16 if n == 1024 else 0.30)


@pytest.mark.parametrize("bits,outer_trust", [(1, 1.0), (1, 0.30), (2, 1.0), (3, 1.0), (4, 1.0), (8, 1.0)])
def test_bit_sweep_student_t_full_size(bits, outer_trust, alpha_table):
    """X 16384 x 2048, Student-t with 3 degrees of freedom at unit RMS, block 2048, every bit width:
    whole tensor against the oracle.  After the transform the rows are close to Gaussian, so the
    share of untrusted elements must be close to the Gaussian tail beyond the trust edge."""
    x, _, cfg = synth.make_config("bit_sweep_1p6b", seed=0)
    K, n = cfg["K"], cfg["had_block"]
    got = gpu_quantize(x, n, bits, outer_trust=outer_trust, want_xh=False)
    ref = qo.hadamard_quantize(x, n, bits, outer_trust=outer_trust)
    n_code, n_mask = compare_quantizer(got, ref, K, bits, outer_trust=outer_trust)
    print(f"bit sweep b={bits} outer_trust={outer_trust}: {n_code} codes / {n_mask} mask bits at a boundary out of {x.size}")
    untrusted = 1.0 - qo.unpack_mask(got["mask"], K).mean()
    levels = 1 << bits
    edge = alpha_table[bits] * (1.0 + outer_trust / (levels - 1))
    gaussian_tail = math.erfc(edge / math.sqrt(2.0))
    print(f"b={bits} outer_trust={outer_trust}: untrusted {untrusted:.5f}, Gaussian tail {gaussian_tail:.5f}")
    assert abs(untrusted - gaussian_tail) < 0.1 * gaussian_tail + 2e-4


# ------------------------------------------------------------------ GEMM

GEMM_CASES = [(256, 512, 512, 4), (130, 200, 1024, 4), (1, 1, 64, 4), (257, 129, 2048, 4),
              (64, 640, 5632, 4), (96, 160, 256, 3), (96, 160, 256, 2), (96, 160, 256, 1),
              # shapes that run the 256 x 128 tile kernel: whole tiles, ragged edges, several steps
              (512, 512, 256, 4), (700, 600, 512, 4), (513, 1025, 1024, 4), (768, 512, 5632, 4),
              # more tiles than the chip holds at once, ragged last tile row and column, one step only
              (4096, 4090, 256, 4), (4096, 4096, 128, 4), (4000, 4100, 384, 4),
              # b = 3 on the tile kernels (one more shift in the widening, products carry 256)
              (700, 600, 512, 3), (768, 512, 5632, 3), (513, 1025, 1024, 3),
              # b = 1, 2 re-coded to nibbles for the tile kernels (and for the wide one at K = 5632)
              (700, 600, 512, 2), (513, 1025, 1024, 1), (768, 512, 5632, 2), (768, 512, 5632, 1),
              (4000, 4100, 384, 1), (512, 256, 128, 2),
              # more 256 x 128 tiles than the chip's workgroup slots, with a remainder and a ragged last tile row
              (4090, 5000, 256, 4), (4090, 5000, 128, 3)]


# every case with caller scratch where the call can use it; the 1- and 2-bit cases that can, also without
GEMM_RUNS = [(*c, True) for c in GEMM_CASES] + [(*c, False) for c in GEMM_CASES if c[3] <= 2 and min(c[0], c[1]) >= 128]


@pytest.mark.parametrize("M,N,K,bits,scratch", GEMM_RUNS)
def test_gemm_accumulators_exact_and_output_close(M, N, K, bits, scratch):
    rng = np.random.default_rng(M * 7 + N * 3 + K + bits)
    L = 1 << bits
    cb = qo.container_bits(bits)
    ka = rng.integers(-L // 2, L // 2, size=(M, K), dtype=np.int32)
    kb = rng.integers(-L // 2, L // 2, size=(N, K), dtype=np.int32)
    ka[0] = L // 2 - 1                      # extreme rows: largest |acc|
    kb[0] = L // 2 - 1
    if N > 1:
        kb[1] = -L // 2
    from oracle.quest_oracle import _load, _ptr
    a_codes = np.empty((M, K * cb // 8), dtype=np.uint8)
    b_codes = np.empty((N, K * cb // 8), dtype=np.uint8)
    _load().qo_pack_codes(_ptr(ka), M, K, bits, _ptr(a_codes))
    _load().qo_pack_codes(_ptr(kb), N, K, bits, _ptr(b_codes))
    sa = (rng.random(M) + 0.5).astype(np.float32)
    sb = ((rng.random(N) + 0.5) * 0.01).astype(np.float32)
    y = torch.full((M, N + 2), 7.0, dtype=torch.bfloat16, device=DEV)   # ld_y > N
    acc = torch.empty(M, N, dtype=torch.int32, device=DEV)
    q.quest_lowbit_gemm(to_device(a_codes), to_device(sa), to_device(b_codes), to_device(sb), K, bits,
                        y=y[:, :N], acc_out=acc, workspace=lowbit_ws(M, N, K, bits) if scratch else None)
    torch.cuda.synchronize()
    ref_acc = qo.gemm_odd(2 * ka + 1, 2 * kb + 1)
    got_acc = acc.cpu().numpy().astype(np.int64)
    assert np.array_equal(got_acc, ref_acc)
    assert got_acc[0, 0] == (L - 1) ** 2 * K
    check_gemm_output(y[:, :N], ref_acc, sa, sb)
    assert torch.all(y[:, N:] == 7.0)       # padding columns untouched


def test_gemm_full_size_sampled_rows():
    """M=16384, N=5632, K=2048 in the launch shape the benchmark times; sampled rows vs the oracle."""
    x, w, cfg = synth.make_config("mlp_up_1p6b", seed=0)
    K, bits, n = cfg["K"], cfg["bits"], cfg["had_block"]
    gx = gpu_quantize(x, n, bits, want_xh=False, want_mask=False)
    gw = gpu_quantize(w, n, bits, want_xh=False, want_mask=False)
    M, N = x.shape[0], w.shape[0]
    y = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    q.quest_lowbit_gemm(gx["dev"]["codes"], gx["dev"]["scales"], gw["dev"]["codes"], gw["dev"]["scales"],
                        K, bits, y=y, acc_out=None)
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    rows = np.sort(rng.choice(M, size=48, replace=False))
    rows[0], rows[-1] = 0, M - 1
    ux = qo.unpack_odd(gx["codes"][rows], K, bits)
    uw = qo.unpack_odd(gw["codes"], K, bits)
    got = check_gemm_output(y[torch.from_numpy(rows).to(DEV)], qo.gemm_odd(ux, uw), gx["scales"][rows], gw["scales"])
    # any-size properties: finite everywhere, and the output approximates x w^T on the sampled rows
    assert torch.isfinite(y.float()).all()
    exact = qo.widen(x[rows]) @ qo.widen(w).T
    assert np.linalg.norm(got - exact) / np.linalg.norm(exact) < 0.25


@pytest.mark.parametrize("M,N,K,bits", [(4000, 4100, 384, 3),      # 256 x 128 tiles, ragged edges
                                        (4090, 3100, 4096, 3), (4090, 3100, 4352, 4),   # 256 x 256 tiles
                                        (3000, 1100, 640, 4), (3000, 1100, 640, 3)])    # 128 x 128 tiles
def test_gemm_kernel_variants_sampled_rows(M, N, K, bits):
    """Every tile size of the matmul at b = 3 and b = 4, ragged last tiles, random codes with extreme
    rows: accumulators of sampled rows (first, last, rows around tile edges) against the oracle."""
    rng = np.random.default_rng(M + N + K + bits)
    L = 1 << bits
    ka = rng.integers(-L // 2, L // 2, size=(M, K), dtype=np.int32)
    kb = rng.integers(-L // 2, L // 2, size=(N, K), dtype=np.int32)
    ka[0] = L // 2 - 1
    kb[0] = L // 2 - 1
    kb[N - 1] = -L // 2
    from oracle.quest_oracle import _load, _ptr
    a_codes = np.empty((M, K // 2), dtype=np.uint8)
    b_codes = np.empty((N, K // 2), dtype=np.uint8)
    _load().qo_pack_codes(_ptr(ka), M, K, bits, _ptr(a_codes))
    _load().qo_pack_codes(_ptr(kb), N, K, bits, _ptr(b_codes))
    sa = (rng.random(M) + 0.5).astype(np.float32)
    sb = ((rng.random(N) + 0.5) * 0.01).astype(np.float32)
    y = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    acc = torch.empty(M, N, dtype=torch.int32, device=DEV)
    q.quest_lowbit_gemm(to_device(a_codes), to_device(sa), to_device(b_codes), to_device(sb), K, bits, y=y, acc_out=acc)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 1, 127, 128, 255, 256, M - 257, M - 129, M - 2, M - 1],
                                     rng.choice(M, size=24, replace=False)]))
    ref_acc = qo.gemm_odd(2 * ka[rows] + 1, 2 * kb + 1)
    pick = torch.from_numpy(rows).to(DEV)
    assert np.array_equal(acc[pick].cpu().numpy().astype(np.int64), ref_acc)
    assert ref_acc[0, 0] == (L - 1) ** 2 * K and ref_acc[0, N - 1] == -(L - 1) ** 2 * K
    check_gemm_output(y[pick], ref_acc, sa[rows], sb)


FP4_GEMM_CASES = [(256, 512, 512), (130, 200, 1024), (1, 1, 128), (257, 129, 2048), (64, 640, 5632),
                  (700, 600, 512), (513, 1025, 1024), (4000, 4100, 384),
                  # long contractions, whole and ragged tiles
                  (768, 512, 5632), (513, 1025, 4096), (1024, 777, 4224)]


# larger outputs with the row pitch equal to N (or a multiple of eight above it): whole tiles, ragged last
# tile row and column, one contraction step and many
FP4_GEMM_LARGE = [(4096, 4096, 128, 0), (3600, 3848, 512, 0), (4090, 3080, 1152, 8), (3585, 3592, 2048, 0)]


@pytest.mark.parametrize("M,N,K,pad", [(*c, 2) for c in FP4_GEMM_CASES] + FP4_GEMM_LARGE)
def test_fp4_gemm_accumulators_exact_and_output_close(M, N, K, pad):
    """E2M1 codes on the FP4 matrix instructions (Sec. 4.4): accumulators equal the exact sums."""
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    a_codes = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    b_codes = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    a_codes[0] = 0x77                       # extreme rows: +6 everywhere, largest |acc| = 36 K
    b_codes[0] = 0x77
    if N > 1:
        b_codes[1] = 0xFF                   # -6 everywhere
    sa = (rng.random(M) + 0.5).astype(np.float32)
    sb = ((rng.random(N) + 0.5) * 0.01).astype(np.float32)
    y = torch.full((M, N + pad), 7.0, dtype=torch.bfloat16, device=DEV)   # ld_y >= N
    acc = torch.empty(M, N, dtype=torch.float32, device=DEV)
    q.quest_lowbit_gemm_fp4(to_device(a_codes), to_device(sa), to_device(b_codes), to_device(sb), K,
                            y=y[:, :N], acc_out=acc)
    torch.cuda.synchronize()
    ref_acc = qo.gemm_fp4(qo.unpack_fp4(a_codes, K), qo.unpack_fp4(b_codes, K))
    got_acc = acc.cpu().numpy().astype(np.float64)
    assert np.array_equal(got_acc, ref_acc)
    assert got_acc[0, 0] == 36.0 * K
    check_gemm_output(y[:, :N], ref_acc, sa, sb)
    assert torch.all(y[:, N:] == 7.0)       # padding columns untouched


def test_fp4_forward_full_size_sampled_rows():
    """FP4 forward at M=16384, N=5632, K=2048: quantizer against the oracle on whole tensors, GEMM on
    sampled rows; and FP4 reconstructs these activations slightly worse than INT4 (Sec. 4.4)."""
    x, w, cfg = synth.make_config("mlp_up_1p6b", seed=0)
    K, n = cfg["K"], cfg["had_block"]
    M, N = x.shape[0], w.shape[0]
    gx = gpu_quantize(x, n, 4, want_xh=False, fp4=True)
    gw = gpu_quantize(w, n, 4, want_xh=False, fp4=True)
    rx = qo.hadamard_quantize_fp4(x, n)
    compare_quantizer_fp4(gx, rx, K)
    compare_quantizer_fp4(gw, qo.hadamard_quantize_fp4(w, n), K)
    y = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    q.quest_lowbit_gemm_fp4(gx["dev"]["codes"], gx["dev"]["scales"], gw["dev"]["codes"], gw["dev"]["scales"],
                            K, y=y)
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(4).choice(M, size=32, replace=False))
    rows[0], rows[-1] = 0, M - 1
    va, vb = qo.unpack_fp4(gx["codes"][rows], K), qo.unpack_fp4(gw["codes"], K)
    got = check_gemm_output(y[torch.from_numpy(rows).to(DEV)], qo.gemm_fp4(va, vb), gx["scales"][rows], gw["scales"])
    exact = qo.widen(x[rows]) @ qo.widen(w).T
    assert np.linalg.norm(got - exact) / np.linalg.norm(exact) < 0.25
    err_fp4 = np.linalg.norm(gx["scales"][:, None] * qo.unpack_fp4(gx["codes"], K) - rx.xh) / np.linalg.norm(rx.xh)
    gi = gpu_quantize(x, n, 4, want_xh=False, want_mask=False)
    err_int4 = np.linalg.norm(gi["scales"][:, None].astype(np.float64) * qo.unpack_odd(gi["codes"], K, 4) - rx.xh) / np.linalg.norm(rx.xh)
    print(f"relative error of xhat_h: FP4 {err_fp4:.4f}, INT4 {err_int4:.4f}")
    assert err_int4 < err_fp4 < 1.2 * err_int4


# ------------------------------------------------------------------ backward

BACK_CASES = [(37, 1024, 128, "bf16", "bf16"), (130, 2048, 2048, "bf16", "bf16"), (70, 5632, 512, "bf16", "f32"),
              (19, 512, 1, "f32", "f32"), (5, 16384, 16384, "bf16", "bf16"), (300, 64, 64, "f32", "bf16"),
              (1, 8, 2, "f32", "f32"), (70, 5632, 512, "bf16", "bf16"), (33, 4096, 4096, "bf16", "bf16"),
              (20, 512, 32, "bf16", "bf16"), (16, 2048, 1, "bf16", "bf16"), (9, 1024, 1024, "bf16", "bf16"),
              (6, 512, 512, "bf16", "bf16"), (11, 2048, 8, "bf16", "bf16"),
              # fp32 on either side of the matrix-core path
              (6, 512, 512, "f32", "f32"), (6, 512, 512, "bf16", "f32"), (6, 512, 512, "f32", "bf16"),
              (37, 1024, 1024, "f32", "f32"), (37, 1024, 1024, "bf16", "f32"), (37, 1024, 1024, "f32", "bf16"),
              (130, 2048, 2048, "f32", "f32"), (130, 2048, 2048, "bf16", "f32"), (130, 2048, 2048, "f32", "bf16"),
              (9, 4096, 4096, "f32", "f32"), (9, 4096, 4096, "bf16", "f32"), (9, 4096, 4096, "f32", "bf16"),
              (70, 5632, 512, "f32", "f32"), (70, 5632, 512, "f32", "bf16"),
              # rows of 11008 = 43 x 256
              (70, 11008, 256, "bf16", "bf16"), (33, 11008, 128, "bf16", "bf16"), (9, 11008, 4, "bf16", "bf16"),
              # the other widths of the paper's model family
              (37, 640, 128, "bf16", "bf16"), (37, 768, 256, "bf16", "bf16"), (37, 1280, 256, "bf16", "bf16"),
              (37, 1664, 128, "bf16", "bf16"), (37, 1792, 256, "bf16", "bf16"), (37, 2816, 256, "bf16", "bf16"),
              (37, 3584, 512, "bf16", "bf16"), (37, 4608, 512, "bf16", "bf16"), (9, 1664, 16, "bf16", "bf16"),
              (37, 640, 128, "bf16", "f32"), (37, 1664, 128, "bf16", "f32"), (37, 2816, 256, "bf16", "f32"),
              (37, 4608, 512, "bf16", "f32"), (21, 11008, 256, "bf16", "f32"),
              # blocks that span two of a row's four tiles, and one of them
              (33, 4096, 2048, "bf16", "bf16"), (33, 4096, 1024, "bf16", "bf16"), (33, 4096, 128, "bf16", "bf16"),
              # more rows than waves on the chip (4096): every wave takes several rows, the next one staged
              # through LDS while the current one is transformed and stored, and the last pass is ragged
              (8229, 1024, 1024, "bf16", "bf16"), (8229, 1024, 128, "bf16", "f32"), (9001, 2048, 2048, "bf16", "f32"),
              (5003, 4096, 4096, "bf16", "bf16")]


@pytest.mark.parametrize("rows,cols,n,gd,od", BACK_CASES)
def test_trust_backward_matches_oracle(rows, cols, n, gd, od):
    g = synth.gaussian(rows, cols, 0.03, seed=rows + cols, dtype=gd)
    rng = np.random.default_rng(cols)
    trust = (rng.random((rows, cols)) < 0.98).astype(np.uint8)
    from oracle.quest_oracle import _load, _ptr
    bitmap = np.empty((rows, cols // 8), dtype=np.uint8)
    _load().qo_pack_mask(_ptr(trust), rows, cols, _ptr(bitmap))
    out = torch.empty(rows, cols, dtype=torch.bfloat16 if od == "bf16" else torch.float32, device=DEV)
    for mask_host, trust_ref in ((bitmap, trust), (None, None)):
        q.quest_trust_backward(to_device(g), None if mask_host is None else to_device(mask_host), n, out=out)
        torch.cuda.synchronize()
        ref = qo.trust_backward(qo.widen(g), trust_ref, n)
        scale = np.sqrt(np.mean(ref * ref, axis=1, keepdims=True))
        tol = (BF16_HALF_ULP if od == "bf16" else 1e-5) * np.abs(ref) + 1e-5 * scale + 1e-30
        assert np.all(np.abs(to_host_f64(out) - ref) <= tol)
    zeros = to_device(np.zeros((rows, cols // 8), dtype=np.uint8))
    q.quest_trust_backward(to_device(g), zeros, n, out=out)
    assert torch.all(out == 0)


BACK_PAIR_CASES = [
    # rows_x, rows_w, cols, block, gradient dtype, output dtype, with masks
    (130, 70, 2048, 2048, "bf16", "bf16", True), (4099, 1408, 2048, 2048, "bf16", "bf16", True),
    (5003, 3001, 1024, 128, "bf16", "f32", True), (37, 300, 1024, 128, "bf16", "bf16", False),
    (70, 33, 5632, 512, "bf16", "bf16", True), (9, 33, 4096, 4096, "bf16", "f32", True),
    (0, 70, 2048, 2048, "bf16", "bf16", True), (70, 0, 2048, 2048, "bf16", "bf16", True),
    (1, 1, 2048, 2048, "bf16", "bf16", True),
    # shapes the one-launch kernel does not cover: the call falls back to one launch per gradient
    (21, 40, 1536, 512, "f32", "f32", True), (19, 5, 24, 8, "f32", "bf16", False), (37, 12, 1024, 1024, "f32", "bf16", True),
]


@pytest.mark.parametrize("rows_x,rows_w,cols,block,gd,od,masks", BACK_PAIR_CASES)
def test_backward_pair_call_equals_two_single_calls(rows_x, rows_w, cols, block, gd, od, masks):
    """The two masked inverse transforms that end Algorithm 2 in one call (one launch where the
    matrix-core kernel covers the shape): every output bit equals that of two calls of
    quest_trust_backward, which the cases above compare with the oracle."""
    rng = np.random.default_rng(rows_x + 3 * rows_w + cols)
    grads = [to_device(synth.gaussian(max(r, 1), cols, 0.03, seed=r + cols + i, dtype=gd)[:r])
             for i, r in enumerate((rows_x, rows_w))]
    bitmaps = [to_device(rng.integers(0, 256, size=(r, cols // 8), dtype=np.uint8) |
                         rng.integers(0, 256, size=(r, cols // 8), dtype=np.uint8)) if masks else None
               for r in (rows_x, rows_w)]
    out_type = torch.bfloat16 if od == "bf16" else torch.float32
    single = [torch.full((r, cols), 7.0, dtype=out_type, device=DEV) for r in (rows_x, rows_w)]
    for g, m, o in zip(grads, bitmaps, single):
        if g.shape[0]:
            q.quest_trust_backward(g, m, block, out=o)
    pair = [torch.full((r, cols), 9.0, dtype=out_type, device=DEV) for r in (rows_x, rows_w)]
    q.quest_trust_backward_pair(grads[0], bitmaps[0], grads[1], bitmaps[1], block, out_x=pair[0], out_w=pair[1])
    torch.cuda.synchronize()
    for a, b in zip(single, pair):
        assert torch.equal(a.view(torch.int16 if od == "bf16" else torch.int32),
                           b.view(torch.int16 if od == "bf16" else torch.int32))


def test_trust_backward_full_size_headline_shape():
    """16384 x 2048 bf16 gradient, block 2048, mask from the quantizer: whole tensor against the oracle."""
    x, _, cfg = synth.make_config("mlp_up_1p6b", seed=0)
    rows, cols, n = x.shape[0], cfg["K"], cfg["had_block"]
    gq = gpu_quantize(x, n, cfg["bits"], want_xh=False)
    g = synth.gaussian(rows, cols, 0.03, seed=77, dtype="bf16")
    out = torch.empty(rows, cols, dtype=torch.bfloat16, device=DEV)
    q.quest_trust_backward(to_device(g), gq["dev"]["mask"], n, out=out)
    torch.cuda.synchronize()
    ref = qo.trust_backward(qo.widen(g), qo.unpack_mask(gq["mask"], cols), n)
    scale = np.sqrt(np.mean(ref * ref, axis=1, keepdims=True))
    assert np.all(np.abs(to_host_f64(out) - ref) <= BF16_HALF_ULP * np.abs(ref) + 1e-5 * scale + 1e-30)


@pytest.mark.parametrize("M,N,K", [(192, 128, 256), (512, 256, 512), (768, 512, 256),
                                   # few tiles, long contraction: tiles split between workgroups,
                                   # evenly (12 steps over 4) and unevenly (128 steps in threes)
                                   (768, 8192, 512), (8192, 768, 512),
                                   # more tiles than CUs, two steps each: whole tiles and halves mixed
                                   (5120, 128, 3840), (128, 5120, 3840),
                                   # outputs that end inside a tile (hidden 640 and 1664 of the paper's models)
                                   (640, 1664, 384), (1664, 640, 896), (320, 192, 448), (4096, 640, 1664)])
@pytest.mark.parametrize("which", [0, 1])
def test_grad_gemm_matches_oracle(which, M, N, K):
    """Small shapes run the 64x64 kernel; outputs of at least half a 256x256 tile each way run the
    main kernel (edge tiles may be partial), which splits tiles between workgroups when whole tiles
    would leave CUs idle."""
    bits, n = 4, min(256, K & -K)
    x = synth.gaussian(M, K, 1.0, 11, "bf16")
    w = synth.gaussian(N, K, 0.02, 12, "bf16")
    dy = synth.upstream_gradient(M, N, 0, "bf16")
    src, C = (w, N) if which == 0 else (x, M)
    gq = gpu_quantize(src, n, bits, want_xh=False)
    rows_out = M if which == 0 else N
    out = torch.empty(rows_out, K, dtype=torch.bfloat16, device=DEV)
    q.quest_grad_gemm(which, to_device(dy), gq["dev"]["codes"], gq["dev"]["scales"], bits, M, N, K, out=out, workspace=grad_ws(which, M, N, K))
    torch.cuda.synchronize()
    u = qo.unpack_odd(gq["codes"], K, bits)
    s = gq["scales"].astype(np.float64)
    dyd = qo.widen(dy)
    # the 16-bit operand the paper's backward multiplies with: bf16(s * u), one rounding
    q16 = qo.widen(synth.to_bf16_bits(gq["scales"][:, None] * u.astype(np.float32)))
    if which == 0:
        ref, mirror = qo.grad_input(dyd, u, s), dyd @ q16
        spread = np.sqrt((dyd ** 2) @ (q16 ** 2))
    else:
        ref, mirror = qo.grad_weight(dyd, u, s), dyd.T @ q16
        spread = np.sqrt((dyd.T ** 2) @ (q16 ** 2))
    got = to_host_f64(out)
    # same operand values on both sides: only fp32 accumulation order and the final bf16 rounding differ
    assert np.all(np.abs(got - mirror) <= BF16_HALF_ULP * 1.001 * np.abs(mirror) + 2e-5 * spread)
    # against the exact oracle: the operand rounding adds about 2^-9 of the spread of the terms
    assert np.all(np.abs(got - ref) <= BF16_HALF_ULP * np.abs(ref) + 2e-2 * spread)
    assert np.linalg.norm(got - ref) <= 4e-3 * np.linalg.norm(ref)


def test_grad_gemm_full_size_sampled_rows():
    """Both gradient matmuls at M=16384, N=5632, K=2048 (the launch shapes the benchmark times, the
    weight gradient with its tiles split over the CUs); sampled output rows against the oracle."""
    x, w, cfg = synth.make_config("mlp_up_1p6b", seed=0)
    K, bits, n = cfg["K"], cfg["bits"], cfg["had_block"]
    M, N = x.shape[0], w.shape[0]
    dy = synth.upstream_gradient(M, N, 3, "bf16")
    gx = gpu_quantize(x, n, bits, want_xh=False, want_mask=False)
    gw = gpu_quantize(w, n, bits, want_xh=False, want_mask=False)
    dyd = to_device(dy)
    g_x = torch.empty(M, K, dtype=torch.bfloat16, device=DEV)
    g_w = torch.empty(N, K, dtype=torch.bfloat16, device=DEV)
    q.quest_grad_gemm(0, dyd, gw["dev"]["codes"], gw["dev"]["scales"], bits, M, N, K, out=g_x, workspace=grad_ws(0, M, N, K))
    q.quest_grad_gemm(1, dyd, gx["dev"]["codes"], gx["dev"]["scales"], bits, M, N, K, out=g_w, workspace=grad_ws(1, M, N, K))
    torch.cuda.synchronize()
    assert torch.isfinite(g_x.float()).all() and torch.isfinite(g_w.float()).all()
    rng = np.random.default_rng(1)
    ux, uw = qo.unpack_odd(gx["codes"], K, bits), qo.unpack_odd(gw["codes"], K, bits)
    sx, sw = gx["scales"].astype(np.float64), gw["scales"].astype(np.float64)
    # G_x rows: one per 256-row tile band at the ends, the rest anywhere
    rows = np.sort(rng.choice(M, size=24, replace=False))
    rows[0], rows[-1] = 0, M - 1
    d = qo.widen(dy[rows])
    ref = qo.grad_input(d, uw, sw)
    q16 = qo.widen(synth.to_bf16_bits(gw["scales"][:, None] * uw.astype(np.float32)))
    spread = np.sqrt((d ** 2) @ (q16 ** 2))
    got = to_host_f64(g_x[torch.from_numpy(rows).to(DEV)])
    assert np.all(np.abs(got - d @ q16) <= BF16_HALF_ULP * 1.001 * np.abs(d @ q16) + 2e-5 * spread)
    assert np.all(np.abs(got - ref) <= BF16_HALF_ULP * np.abs(ref) + 2e-2 * spread)
    # G_w rows (columns of dy), each a contraction over all 16384 tokens
    cols = np.sort(rng.choice(N, size=12, replace=False))
    cols[0], cols[-1] = 0, N - 1
    d = qo.widen(np.ascontiguousarray(dy[:, cols]))
    ref = qo.grad_weight(d, ux, sx)
    q16 = qo.widen(synth.to_bf16_bits(gx["scales"][:, None] * ux.astype(np.float32)))
    mirror = d.T @ q16
    spread = np.sqrt((d.T ** 2) @ (q16 ** 2))
    got = to_host_f64(g_w[torch.from_numpy(cols).to(DEV)])
    assert np.all(np.abs(got - mirror) <= BF16_HALF_ULP * 1.001 * np.abs(mirror) + 2e-5 * spread)
    assert np.all(np.abs(got - ref) <= BF16_HALF_ULP * np.abs(ref) + 2e-2 * spread)


def test_down_projection_full_size():
    """The MLP down-projection (X 16384 x 5632 in blocks of 512, W 2048 x 5632; Sec. 5 singles this
    layer out for its transform overhead): quantizer on the whole activation tensor, forward GEMM,
    both gradient matmuls and the trust backward on sampled rows, all at the full launch shape."""
    x, w, cfg = synth.make_config("mlp_down_1p6b", seed=0)
    K, bits, n = cfg["K"], cfg["bits"], cfg["had_block"]
    M, N = x.shape[0], w.shape[0]
    gx = gpu_quantize(x, n, bits, want_xh=False)
    gw = gpu_quantize(w, n, bits, want_xh=False)
    ref = qo.hadamard_quantize(x, n, bits)
    n_code, n_mask = compare_quantizer(gx, ref, K, bits)
    print(f"down-projection X: {n_code} codes / {n_mask} mask bits at a boundary out of {x.size}")
    del ref
    y = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    q.quest_lowbit_gemm(gx["dev"]["codes"], gx["dev"]["scales"], gw["dev"]["codes"], gw["dev"]["scales"],
                        K, bits, y=y, acc_out=None)
    dy = synth.upstream_gradient(M, N, 5, "bf16")
    dyd = to_device(dy)
    g_x = torch.empty(M, K, dtype=torch.bfloat16, device=DEV)
    g_w = torch.empty(N, K, dtype=torch.bfloat16, device=DEV)
    q.quest_grad_gemm(0, dyd, gw["dev"]["codes"], gw["dev"]["scales"], bits, M, N, K, out=g_x, workspace=grad_ws(0, M, N, K))
    q.quest_grad_gemm(1, dyd, gx["dev"]["codes"], gx["dev"]["scales"], bits, M, N, K, out=g_w, workspace=grad_ws(1, M, N, K))
    dx = torch.empty(M, K, dtype=torch.bfloat16, device=DEV)
    q.quest_trust_backward(g_x, gx["dev"]["mask"], n, out=dx)
    torch.cuda.synchronize()
    rng = np.random.default_rng(2)
    rows = np.sort(rng.choice(M, size=16, replace=False))
    rows[0], rows[-1] = 0, M - 1
    rows_d = torch.from_numpy(rows).to(DEV)
    ux_all = qo.unpack_odd(gx["codes"], K, bits)
    uw = qo.unpack_odd(gw["codes"], K, bits)
    sx, sw = gx["scales"].astype(np.float64), gw["scales"].astype(np.float64)
    # forward GEMM rows
    check_gemm_output(y[rows_d], qo.gemm_odd(ux_all[rows], uw), gx["scales"][rows], gw["scales"])
    # G_x rows, then the masked inverse transform of exactly what the GPU produced for them
    d = qo.widen(dy[rows])
    ref = qo.grad_input(d, uw, sw)
    q16 = qo.widen(synth.to_bf16_bits(gw["scales"][:, None] * uw.astype(np.float32)))
    spread = np.sqrt((d ** 2) @ (q16 ** 2))
    got = to_host_f64(g_x[rows_d])
    assert np.all(np.abs(got - d @ q16) <= BF16_HALF_ULP * 1.001 * np.abs(d @ q16) + 2e-5 * spread)
    assert np.all(np.abs(got - ref) <= BF16_HALF_ULP * np.abs(ref) + 2e-2 * spread)
    ref_dx = qo.trust_backward(got, qo.unpack_mask(gx["mask"][rows], K), n)
    scale = np.sqrt(np.mean(ref_dx * ref_dx, axis=1, keepdims=True))
    assert np.all(np.abs(to_host_f64(dx[rows_d]) - ref_dx) <= BF16_HALF_ULP * np.abs(ref_dx) + 1e-5 * scale + 1e-30)
    # G_w rows (columns of dy)
    cols = np.sort(rng.choice(N, size=8, replace=False))
    cols[0], cols[-1] = 0, N - 1
    d = qo.widen(np.ascontiguousarray(dy[:, cols]))
    ref = qo.grad_weight(d, ux_all, sx)
    q16 = qo.widen(synth.to_bf16_bits(gx["scales"][:, None] * ux_all.astype(np.float32)))
    mirror = d.T @ q16
    spread = np.sqrt((d.T ** 2) @ (q16 ** 2))
    got = to_host_f64(g_w[torch.from_numpy(cols).to(DEV)])
    assert np.all(np.abs(got - mirror) <= BF16_HALF_ULP * 1.001 * np.abs(mirror) + 2e-5 * spread)
    assert np.all(np.abs(got - ref) <= BF16_HALF_ULP * np.abs(ref) + 2e-2 * spread)


@pytest.mark.parametrize("name", ["mlp_up_7b", "mlp_down_7b"])
def test_7b_layers_whole_step_sampled(name):
    """The MLP layers of the 7B model of the paper's per-layer runtime figure (hidden 4096 with one
    block of 4096, MLP width 11008 = 43 x 256 in blocks of 256), 8192 tokens: the step through the
    two-operand calls at these launch shapes (wide-K forward kernel, rows that end inside a tile of the
    quantizer), sampled rows of every stage against the oracle."""
    x, w, cfg = synth.make_config(name, seed=0, rows=8192)
    K, bits, n = cfg["K"], cfg["bits"], cfg["had_block"]
    M, N = x.shape[0], w.shape[0]
    dev = torch.device(DEV)
    u8, f32, b16 = torch.uint8, torch.float32, torch.bfloat16
    xc, xs, xm = (torch.empty(M, K // 2, dtype=u8, device=dev), torch.empty(M, dtype=f32, device=dev),
                  torch.empty(M, K // 8, dtype=u8, device=dev))
    wc, ws, wm = (torch.empty(N, K // 2, dtype=u8, device=dev), torch.empty(N, dtype=f32, device=dev),
                  torch.empty(N, K // 8, dtype=u8, device=dev))
    q.quest_hadamard_quantize_pair(to_device(x), to_device(w), n, bits, x_codes=xc, x_scales=xs, x_mask=xm,
                                   w_codes=wc, w_scales=ws, w_mask=wm)
    y = torch.empty(M, N, dtype=b16, device=dev)
    q.quest_lowbit_gemm(xc, xs, wc, ws, K, bits, y=y)
    dy = synth.upstream_gradient(M, N, 5, "bf16")
    dyd = to_device(dy)
    g_x, g_w = torch.empty(M, K, dtype=b16, device=dev), torch.empty(N, K, dtype=b16, device=dev)
    q.quest_grad_gemm(0, dyd, wc, ws, bits, M, N, K, out=g_x, workspace=grad_ws(0, M, N, K))
    q.quest_grad_gemm(1, dyd, xc, xs, bits, M, N, K, out=g_w, workspace=grad_ws(1, M, N, K))
    dx, dw = torch.empty_like(g_x), torch.empty_like(g_w)
    q.quest_trust_backward_pair(g_x, xm, g_w, wm, n, out_x=dx, out_w=dw)
    torch.cuda.synchronize()

    rng = np.random.default_rng(11)
    rows = np.sort(rng.choice(M, size=16, replace=False))
    rows[0], rows[-1] = 0, M - 1
    w_rows = np.sort(rng.choice(N, size=8, replace=False))
    w_rows[0], w_rows[-1] = 0, N - 1
    rows_d, w_rows_d = torch.from_numpy(rows).to(dev), torch.from_numpy(w_rows).to(dev)
    # quantizer: the sampled rows of both operands
    for src, picked, codes, scales, mask in ((x, rows, xc, xs, xm), (w, w_rows, wc, ws, wm)):
        picked_d = torch.from_numpy(picked).to(dev)
        got = dict(codes=codes[picked_d].cpu().numpy(), scales=scales[picked_d].cpu().numpy(),
                   mask=mask[picked_d].cpu().numpy(), xh=None)
        compare_quantizer(got, qo.hadamard_quantize(src[picked], n, bits), K, bits)
    ux_all, uw = qo.unpack_odd(xc.cpu().numpy(), K, bits), qo.unpack_odd(wc.cpu().numpy(), K, bits)
    sx32, sw32 = xs.cpu().numpy(), ws.cpu().numpy()
    sx, sw = sx32.astype(np.float64), sw32.astype(np.float64)
    # forward rows
    check_gemm_output(y[rows_d], qo.gemm_odd(ux_all[rows], uw), sx32[rows], sw32)
    # G_x rows and their masked inverse transform
    d = qo.widen(dy[rows])
    ref = qo.grad_input(d, uw, sw)
    q16 = qo.widen(synth.to_bf16_bits(sw32[:, None] * uw.astype(np.float32)))
    spread = np.sqrt((d ** 2) @ (q16 ** 2))
    got = to_host_f64(g_x[rows_d])
    assert np.all(np.abs(got - d @ q16) <= BF16_HALF_ULP * 1.001 * np.abs(d @ q16) + 2e-5 * spread)
    assert np.all(np.abs(got - ref) <= BF16_HALF_ULP * np.abs(ref) + 2e-2 * spread)
    ref_dx = qo.trust_backward(got, qo.unpack_mask(xm[rows_d].cpu().numpy(), K), n)
    scale = np.sqrt(np.mean(ref_dx * ref_dx, axis=1, keepdims=True))
    assert np.all(np.abs(to_host_f64(dx[rows_d]) - ref_dx) <= BF16_HALF_ULP * np.abs(ref_dx) + 1e-5 * scale + 1e-30)
    # G_w rows (columns of dy) and their masked inverse transform
    d = qo.widen(np.ascontiguousarray(dy[:, w_rows]))
    ref = qo.grad_weight(d, ux_all, sx)
    q16 = qo.widen(synth.to_bf16_bits(sx32[:, None] * ux_all.astype(np.float32)))
    mirror = d.T @ q16
    spread = np.sqrt((d.T ** 2) @ (q16 ** 2))
    got = to_host_f64(g_w[w_rows_d])
    assert np.all(np.abs(got - mirror) <= BF16_HALF_ULP * 1.001 * np.abs(mirror) + 2e-5 * spread)
    assert np.all(np.abs(got - ref) <= BF16_HALF_ULP * np.abs(ref) + 2e-2 * spread)
    ref_dw = qo.trust_backward(got, qo.unpack_mask(wm[w_rows_d].cpu().numpy(), K), n)
    scale = np.sqrt(np.mean(ref_dw * ref_dw, axis=1, keepdims=True))
    assert np.all(np.abs(to_host_f64(dw[w_rows_d]) - ref_dw) <= BF16_HALF_ULP * np.abs(ref_dw) + 1e-5 * scale + 1e-30)


@pytest.mark.parametrize("M,N,K,bits", [(256, 256, 64, 4), (512, 256, 2048, 4), (256, 768, 320, 2),
                                        (768, 512, 1024, 1), (256, 256, 5632, 3),
                                        (4096, 2304, 128, 4),   # 144 tiles: split over the CUs
                                        (640, 1664, 384, 4), (192, 320, 448, 2)])   # outputs ending inside a tile
def test_weight_only_gemm_matches_oracle(M, N, K, bits):
    """Sec. 4.4: bf16 activations in the Hadamard domain (the transform alone is the trust
    backward without a mask) against 1..4-bit weights expanded on the fly."""
    n = 64
    x = synth.outlier_activations(M, K, 0.01, 20.0, seed=M + K, dtype="bf16")
    w = synth.gaussian(N, K, 0.02, 12, "bf16")
    gw = gpu_quantize(w, n, bits, want_xh=False, want_mask=False)
    xh = torch.empty(M, K, dtype=torch.bfloat16, device=DEV)
    q.quest_trust_backward(to_device(x), None, n, out=xh)
    y = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    q.quest_weight_only_gemm(xh, gw["dev"]["codes"], gw["dev"]["scales"], bits, y=y, workspace=weight_only_ws(M, N, K))
    torch.cuda.synchronize()
    xh_host = to_host_f64(xh)
    ref_xh = qo.hadamard(qo.widen(x), n)
    scale = np.sqrt(np.mean(ref_xh * ref_xh, axis=1, keepdims=True))
    assert np.all(np.abs(xh_host - ref_xh) <= BF16_HALF_ULP * np.abs(ref_xh) + 1e-5 * scale)
    u = qo.unpack_odd(gw["codes"], K, bits)
    ref = qo.weight_only_gemm(xh_host, u, gw["scales"].astype(np.float64))
    w16 = qo.widen(synth.to_bf16_bits(gw["scales"][:, None] * u.astype(np.float32)))   # the 16-bit operand
    mirror = xh_host @ w16.T
    spread = np.sqrt((xh_host ** 2) @ (w16.T ** 2))
    got = to_host_f64(y)
    assert np.all(np.abs(got - mirror) <= BF16_HALF_ULP * 1.001 * np.abs(mirror) + 2e-5 * spread)
    assert np.all(np.abs(got - ref) <= BF16_HALF_ULP * np.abs(ref) + 2e-2 * spread)
    assert np.linalg.norm(got - ref) <= 4e-3 * np.linalg.norm(ref)
    # and the product approximates x w^T (the transform is orthogonal)
    exact = qo.widen(x) @ qo.widen(w).T
    print(f"b={bits}: relative error against x w^T {np.linalg.norm(got - exact) / np.linalg.norm(exact):.3f}")


def test_split_tiles_are_summed_in_a_fixed_order():
    """The weight gradient at the headline shape has its tiles split over the CUs; the partial tiles
    are added in workgroup order, so two runs (with other work in between) agree bit for bit."""
    M, N, K, bits = 8192, 768, 512, 4
    x = synth.gaussian(M, K, 1.0, 1, "bf16")
    dy = to_device(synth.upstream_gradient(M, N, 2, "bf16"))
    gx = gpu_quantize(x, 512, bits, want_xh=False, want_mask=False)
    outs = []
    for rep in range(3):
        out = torch.empty(N, K, dtype=torch.bfloat16, device=DEV)
        q.quest_grad_gemm(1, dy, gx["dev"]["codes"], gx["dev"]["scales"], bits, M, N, K, out=out, workspace=grad_ws(1, M, N, K))
        if rep == 0:   # a call of another shape in between, with scratch of its own
            other = torch.empty(256, 256, dtype=torch.bfloat16, device=DEV)
            q.quest_grad_gemm(0, dy[:256, :256].contiguous(), gx["dev"]["codes"][:256, :128].contiguous(),
                              gx["dev"]["scales"][:256].contiguous(), bits, 256, 256, 256, out=other,
                              workspace=grad_ws(0, 256, 256, 256))
        outs.append(out)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[1], outs[2])


@pytest.mark.parametrize("which,M,N,K", [(1, 8192, 2560, 2304), (0, 2560, 8192, 2304), (1, 4096, 2368, 2560)])
def test_split_tiles_mid_size_alternating_inputs(which, M, N, K):
    """Ninety-odd tiles with a long contraction over 256 CUs: every tile is shared by three or four
    workgroups (the benchmark's weight-gradient situation at a size whose whole output can be
    checked).  The whole output against the fp64 product of the same 16-bit operands, sampled rows
    against the oracle, and runs on alternating inputs over one workspace bit-identical (a stale
    partial tile from the call before would show)."""
    bits, n = 4, 256
    src_rows, out_rows = (N, M) if which == 0 else (M, N)
    ws = grad_ws(which, M, N, K)
    results = {}
    for rep, seed in enumerate((5, 6, 5, 6)):
        src = synth.gaussian(src_rows, K, 1.0 if which else 0.02, seed, "bf16")
        dy = synth.upstream_gradient(M, N, seed + 10, "bf16")
        gq = gpu_quantize(src, n, bits, want_xh=False, want_mask=False)
        out = torch.empty(out_rows, K, dtype=torch.bfloat16, device=DEV)
        q.quest_grad_gemm(which, to_device(dy), gq["dev"]["codes"], gq["dev"]["scales"], bits, M, N, K, out=out,
                          workspace=ws)
        torch.cuda.synchronize()
        if seed in results:
            assert torch.equal(results[seed], out), (rep, seed)
            continue
        results[seed] = out
        u = qo.unpack_odd(gq["codes"], K, bits)
        q16 = qo.widen(synth.to_bf16_bits(gq["scales"][:, None] * u.astype(np.float32)))
        dyd = qo.widen(dy)
        left = dyd if which == 0 else dyd.T
        mirror = left @ q16
        spread = np.sqrt((left ** 2) @ (q16 ** 2))
        got = to_host_f64(out)
        assert np.all(np.abs(got - mirror) <= BF16_HALF_ULP * 1.001 * np.abs(mirror) + 2e-5 * spread)
        rows = np.sort(np.random.default_rng(seed).choice(out_rows, size=8, replace=False))
        rows[0], rows[-1] = 0, out_rows - 1
        s = gq["scales"].astype(np.float64)
        ref = qo.grad_input(dyd[rows], u, s) if which == 0 else qo.grad_weight(np.ascontiguousarray(dyd[:, rows]), u, s)
        assert np.all(np.abs(got[rows] - ref) <= BF16_HALF_ULP * np.abs(ref) + 2e-2 * spread[rows])


@pytest.mark.parametrize("which,M,N,K", [(0, 512, 256, 512), (1, 512, 256, 512), (0, 768, 8192, 512),
                                          (1, 8192, 768, 512),
                                          (0, 640, 1664, 384), (1, 1664, 640, 896)])   # outputs ending inside a tile
def test_fp4_grad_gemm_matches_oracle(which, M, N, K):
    """Backward matmuls of the FP4 variant (Algorithm 2 on E2M1-coded operands), whole and split tiles."""
    n = min(256, K & -K)
    x = synth.gaussian(M, K, 1.0, 11, "bf16")
    w = synth.gaussian(N, K, 0.02, 12, "bf16")
    dy = synth.upstream_gradient(M, N, 0, "bf16")
    gq = gpu_quantize(w if which == 0 else x, n, 4, want_xh=False, fp4=True)
    out = torch.empty(M if which == 0 else N, K, dtype=torch.bfloat16, device=DEV)
    q.quest_grad_gemm_fp4(which, to_device(dy), gq["dev"]["codes"], gq["dev"]["scales"], M, N, K, out=out,
                          workspace=grad_ws(which, M, N, K, fp4=True))
    torch.cuda.synchronize()
    v = qo.unpack_fp4(gq["codes"], K)
    u2 = np.rint(2.0 * v).astype(np.int32)                      # E2M1 values are multiples of 1/2
    s_half = 0.5 * gq["scales"].astype(np.float64)
    dyd = qo.widen(dy)
    q16 = qo.widen(synth.to_bf16_bits((gq["scales"][:, None] * v.astype(np.float32)).astype(np.float32)))
    if which == 0:
        ref, mirror = qo.grad_input(dyd, u2, s_half), dyd @ q16
        spread = np.sqrt((dyd ** 2) @ (q16 ** 2))
    else:
        ref, mirror = qo.grad_weight(dyd, u2, s_half), dyd.T @ q16
        spread = np.sqrt((dyd.T ** 2) @ (q16 ** 2))
    got = to_host_f64(out)
    assert np.all(np.abs(got - mirror) <= BF16_HALF_ULP * 1.001 * np.abs(mirror) + 2e-5 * spread)
    assert np.all(np.abs(got - ref) <= BF16_HALF_ULP * np.abs(ref) + 2e-2 * spread)
    assert np.linalg.norm(got - ref) <= 4e-3 * np.linalg.norm(ref)


def test_full_linear_forward_backward_small():
    """Algorithm 1 + Algorithm 2 end to end through the C ABI on a small layer."""
    M, N, K, bits, n = 128, 192, 512, 4, 512
    x = synth.outlier_activations(M, K, 0.01, 20.0, 5, "bf16")
    w = synth.gaussian(N, K, 0.02, 6, "bf16")
    dy = synth.upstream_gradient(M, N, 7, "bf16")
    gx, gw = gpu_quantize(x, n, bits, want_xh=False), gpu_quantize(w, n, bits, want_xh=False)
    dyd = to_device(dy)
    g_x = torch.empty(M, K, dtype=torch.bfloat16, device=DEV)
    g_w = torch.empty(N, K, dtype=torch.bfloat16, device=DEV)
    q.quest_grad_gemm(0, dyd, gw["dev"]["codes"], gw["dev"]["scales"], bits, M, N, K, out=g_x, workspace=grad_ws(0, M, N, K))
    q.quest_grad_gemm(1, dyd, gx["dev"]["codes"], gx["dev"]["scales"], bits, M, N, K, out=g_w, workspace=grad_ws(1, M, N, K))
    dx = torch.empty(M, K, dtype=torch.float32, device=DEV)
    dw = torch.empty(N, K, dtype=torch.float32, device=DEV)
    q.quest_trust_backward(g_x, gx["dev"]["mask"], n, out=dx)
    q.quest_trust_backward(g_w, gw["dev"]["mask"], n, out=dw)
    torch.cuda.synchronize()
    ux, uw = qo.unpack_odd(gx["codes"], K, bits), qo.unpack_odd(gw["codes"], K, bits)
    sx, sw = gx["scales"].astype(np.float64), gw["scales"].astype(np.float64)
    ref_dx = qo.trust_backward(qo.grad_input(qo.widen(dy), uw, sw), qo.unpack_mask(gx["mask"], K), n)
    ref_dw = qo.trust_backward(qo.grad_weight(qo.widen(dy), ux, sx), qo.unpack_mask(gw["mask"], K), n)
    for got, ref in ((dx, ref_dx), (dw, ref_dw)):
        err = np.linalg.norm(to_host_f64(got) - ref) / np.linalg.norm(ref)
        assert err < 5e-3


def test_whole_step_replayed_from_a_graph_matches_eager_launches():
    """The step's five calls (both operands quantized by one call, both inverse transforms by one
    call) captured into one HIP graph with no eager call before the capture (only quest_init), then
    a larger gradient matmul run eagerly with scratch of its own, then replays on new input contents
    with eager work and synchronisations between them: every replay must reproduce, bit for bit,
    what the step gives when launched eagerly as seven single-operand calls.  Shapes that split tiles
    (second launch, partial tiles in the caller's workspace)."""
    M, N, K, bits, n = 768, 8192, 512, 4, 512
    dev = torch.device(DEV)
    q.quest_init()

    def buffers():
        u8, f32, b16 = torch.uint8, torch.float32, torch.bfloat16
        return dict(xc=torch.empty(M, K // 2, dtype=u8, device=dev), xs=torch.empty(M, dtype=f32, device=dev),
                    xm=torch.empty(M, K // 8, dtype=u8, device=dev), wc=torch.empty(N, K // 2, dtype=u8, device=dev),
                    ws=torch.empty(N, dtype=f32, device=dev), wm=torch.empty(N, K // 8, dtype=u8, device=dev),
                    y=torch.empty(M, N, dtype=b16, device=dev), gx=torch.empty(M, K, dtype=b16, device=dev),
                    gw=torch.empty(N, K, dtype=b16, device=dev), dx=torch.empty(M, K, dtype=b16, device=dev),
                    dw=torch.empty(N, K, dtype=b16, device=dev))

    x = torch.empty(M, K, dtype=torch.bfloat16, device=dev)
    w = torch.empty(N, K, dtype=torch.bfloat16, device=dev)
    dy = torch.empty(M, N, dtype=torch.bfloat16, device=dev)

    def step(b, scratch, paired):
        if paired:
            q.quest_hadamard_quantize_pair(x, w, n, bits, x_codes=b["xc"], x_scales=b["xs"], x_mask=b["xm"],
                                           w_codes=b["wc"], w_scales=b["ws"], w_mask=b["wm"])
        else:
            q.quest_hadamard_quantize(x, n, bits, codes=b["xc"], scales=b["xs"], mask=b["xm"])
            q.quest_hadamard_quantize(w, n, bits, codes=b["wc"], scales=b["ws"], mask=b["wm"])
        q.quest_lowbit_gemm(b["xc"], b["xs"], b["wc"], b["ws"], K, bits, y=b["y"])
        q.quest_grad_gemm(0, dy, b["wc"], b["ws"], bits, M, N, K, out=b["gx"], workspace=scratch[0])
        q.quest_grad_gemm(1, dy, b["xc"], b["xs"], bits, M, N, K, out=b["gw"], workspace=scratch[1])
        if paired:
            q.quest_trust_backward_pair(b["gx"], b["xm"], b["gw"], b["wm"], n, out_x=b["dx"], out_w=b["dw"])
        else:
            q.quest_trust_backward(b["gx"], b["xm"], n, out=b["dx"])
            q.quest_trust_backward(b["gw"], b["wm"], n, out=b["dw"])

    def fill(seed):
        x.copy_(to_device(synth.outlier_activations(M, K, 0.01, 20.0, seed, "bf16")).view(torch.bfloat16))
        w.copy_(to_device(synth.gaussian(N, K, 0.02, seed + 1, "bf16")).view(torch.bfloat16))
        dy.copy_(to_device(synth.upstream_gradient(M, N, seed + 2, "bf16")).view(torch.bfloat16))

    eager, captured = buffers(), buffers()
    eager_scratch = (grad_ws(0, M, N, K), grad_ws(1, M, N, K))
    captured_scratch = (grad_ws(0, M, N, K), grad_ws(1, M, N, K))
    fill(0)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            step(captured, captured_scratch, paired=True)
    torch.cuda.synchronize()
    # a larger shape, eagerly, after the capture: it brings its own scratch and touches nothing of the graph's
    M2, N2, K2 = 2048, 8192, 1024
    big_codes = torch.zeros(M2, K2 // 2, dtype=torch.uint8, device=dev)
    big_scales = torch.ones(M2, dtype=torch.float32, device=dev)
    big_dy = torch.zeros(M2, N2, dtype=torch.bfloat16, device=dev)
    big_out = torch.empty(N2, K2, dtype=torch.bfloat16, device=dev)
    q.quest_grad_gemm(1, big_dy, big_codes, big_scales, bits, M2, N2, K2, out=big_out, workspace=grad_ws(1, M2, N2, K2))
    torch.cuda.synchronize()
    for seed in (10, 20, 30):
        fill(seed)
        step(eager, eager_scratch, paired=False)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in eager:
            assert torch.equal(eager[name].view(torch.uint8), captured[name].view(torch.uint8)), (seed, name)


def test_two_streams_with_two_workspaces_run_concurrently():
    """Two weight-gradient matmuls (split tiles: expanded operand and partial tiles in scratch) issued to
    two streams with a workspace each must give what each gives alone."""
    M, N, K, bits = 8192, 768, 512, 4
    dev = torch.device(DEV)
    jobs = []
    for seed in (1, 2):
        gx = gpu_quantize(synth.gaussian(M, K, 1.0, seed, "bf16"), 512, bits, want_xh=False, want_mask=False)
        jobs.append(dict(dy=to_device(synth.upstream_gradient(M, N, seed + 10, "bf16")), codes=gx["dev"]["codes"],
                         scales=gx["dev"]["scales"], ws=grad_ws(1, M, N, K),
                         alone=torch.empty(N, K, dtype=torch.bfloat16, device=dev),
                         together=torch.empty(N, K, dtype=torch.bfloat16, device=dev)))
    for j in jobs:
        q.quest_grad_gemm(1, j["dy"], j["codes"], j["scales"], bits, M, N, K, out=j["alone"], workspace=j["ws"])
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(4):
        for j, st in zip(jobs, streams):
            with torch.cuda.stream(st):
                q.quest_grad_gemm(1, j["dy"], j["codes"], j["scales"], bits, M, N, K, out=j["together"],
                                  workspace=j["ws"])
    torch.cuda.synchronize()
    for j in jobs:
        assert torch.equal(j["alone"], j["together"])
    assert not torch.equal(jobs[0]["alone"], jobs[1]["alone"])
