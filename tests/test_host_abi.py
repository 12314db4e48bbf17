"""Host-side checks of the C-ABI library: it loads, exports what include/quest.h declares, its
constant table matches the oracle's derivation, and invalid arguments are turned into status
codes before anything is launched (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2502_05003_amd import binding as q

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x10000)          # 16-byte aligned, never dereferenced: validation fails first


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(q.LIB_PATH):
        from paper_2502_05003_amd import build
        build.build_library()
    return q.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "quest.h")).read()
    declared = set(re.findall(r"\b(quest_[a-z_0-9]+)\s*\(", header))
    assert declared == set(q.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_builtin_alpha_table_matches_the_oracle(lib, alpha_table):
    for bits, alpha in alpha_table.items():
        assert q.quest_alpha_star(bits) == pytest.approx(alpha, rel=3e-7)
    assert q.quest_alpha_star(5) == 0.0
    from oracle import alpha_star
    assert q.quest_alpha_star_fp4() == pytest.approx(alpha_star.alpha_star_fp4(), rel=3e-7)
    assert [q.quest_container_bits(b) for b in (1, 2, 3, 4, 8, 5)] == [1, 2, 4, 4, 8, 0]
    from oracle import quest_oracle as qo
    assert all(q.quest_container_bits(b) == qo.container_bits(b) for b in (1, 2, 3, 4, 8))


def _hq(lib, x=FAKE, dtype=1, rows=4, cols=512, ld=512, n=512, bits=4, alpha=0.0, ot=-1.0,
        codes=FAKE, scales=FAKE, mask=FAKE, xh=None):
    return lib.quest_hadamard_quantize(x, dtype, rows, cols, ld, n, bits, alpha, ot, codes, scales,
                                       mask, xh, None)


def test_quantizer_rejects_bad_arguments(lib):
    assert _hq(lib, x=None) == 1 and _hq(lib, codes=None) == 1 and _hq(lib, scales=None) == 1
    assert _hq(lib, dtype=7) == 6
    for bits in (0, 5, 6, 7, 9, 16, -1):
        assert _hq(lib, bits=bits) == 3
    assert _hq(lib, cols=0) == 2 and _hq(lib, cols=508) == 2 and _hq(lib, cols=32768, ld=32768, n=8) == 2
    assert _hq(lib, rows=-1) == 2 and _hq(lib, ld=256) == 2
    assert _hq(lib, n=3) == 4 and _hq(lib, n=0) == 4 and _hq(lib, n=1024) == 4 and _hq(lib, cols=768, ld=768, n=512) == 4
    assert _hq(lib, x=ctypes.c_void_p(0x10008)) == 5 and _hq(lib, mask=ctypes.c_void_p(0x10001)) == 5
    assert _hq(lib, ld=516) == 5                      # bf16 row stride not a multiple of 16 bytes
    assert _hq(lib, alpha=float("nan")) == 8 and _hq(lib, ot=float("inf")) == 8
    assert _hq(lib, rows=0) == 0                      # empty input is a no-op, nothing is launched


def _pair(lib, x=FAKE, rows_x=4, ld_x=512, codes_x=FAKE, scales_x=FAKE, mask_x=FAKE, w=FAKE, rows_w=4, ld_w=512,
          codes_w=FAKE, scales_w=FAKE, mask_w=FAKE, dtype=1, cols=512, n=512, bits=4, alpha=0.0, ot=-1.0):
    return lib.quest_hadamard_quantize_pair(x, rows_x, ld_x, codes_x, scales_x, mask_x, w, rows_w, ld_w, codes_w,
                                            scales_w, mask_w, dtype, cols, n, bits, alpha, ot, None)


def test_pair_quantizer_rejects_bad_arguments(lib):
    """Either operand of the two-operand call is validated like the operand of the single call."""
    assert _pair(lib, x=None) == 1 and _pair(lib, w=None) == 1 and _pair(lib, codes_w=None) == 1
    assert _pair(lib, scales_x=None) == 1 and _pair(lib, scales_w=None) == 1
    assert _pair(lib, dtype=7) == 6 and _pair(lib, bits=5) == 3
    assert _pair(lib, rows_w=-1) == 2 and _pair(lib, ld_w=256) == 2 and _pair(lib, cols=508) == 2
    assert _pair(lib, n=3) == 4 and _pair(lib, cols=768, ld_x=768, ld_w=768, n=512) == 4
    assert _pair(lib, w=ctypes.c_void_p(0x10008)) == 5 and _pair(lib, mask_w=ctypes.c_void_p(0x10001)) == 5
    assert _pair(lib, ld_w=516) == 5
    assert _pair(lib, mask_x=None) == 8 and _pair(lib, mask_w=None) == 8     # both masks or neither
    assert _pair(lib, alpha=float("nan")) == 8
    assert _pair(lib, rows_x=0, rows_w=0) == 0 and _pair(lib, rows_x=0, rows_w=0, mask_x=None, mask_w=None) == 0


def test_fp4_pair_quantizer_and_backward_pair_reject_bad_arguments(lib):
    """The other two-operand calls validate either operand like their single calls do."""
    def fp4(x=FAKE, rows_x=4, ld_x=512, codes_x=FAKE, scales_x=FAKE, mask_x=FAKE, w=FAKE, rows_w=4, ld_w=512,
            codes_w=FAKE, scales_w=FAKE, mask_w=FAKE, dtype=1, cols=512, n=512, alpha=0.0):
        return lib.quest_hadamard_quantize_fp4_pair(x, rows_x, ld_x, codes_x, scales_x, mask_x, w, rows_w, ld_w,
                                                    codes_w, scales_w, mask_w, dtype, cols, n, alpha, None)
    assert fp4(x=None) == 1 and fp4(scales_w=None) == 1 and fp4(dtype=7) == 6
    assert fp4(rows_x=-1) == 2 and fp4(ld_x=256) == 2 and fp4(n=3) == 4
    assert fp4(codes_w=ctypes.c_void_p(0x10008)) == 5 and fp4(mask_w=None) == 8 and fp4(alpha=float("inf")) == 8
    assert fp4(rows_x=0, rows_w=0) == 0 and fp4(rows_x=0, rows_w=0, x=None, codes_x=None, scales_x=None) == 0

    def back(g_x=FAKE, mask_x=FAKE, rows_x=4, out_x=FAKE, g_w=FAKE, mask_w=FAKE, rows_w=4, out_w=FAKE, gd=1,
             cols=512, n=512, od=1):
        return lib.quest_trust_backward_pair(g_x, mask_x, rows_x, out_x, g_w, mask_w, rows_w, out_w, gd, cols, n,
                                             od, None)
    assert back(g_x=None) == 1 and back(out_w=None) == 1 and back(gd=3) == 6 and back(od=-1) == 6
    assert back(cols=20) == 2 and back(rows_w=-1) == 2 and back(n=48) == 4
    assert back(out_w=ctypes.c_void_p(0x10002)) == 5 and back(mask_x=ctypes.c_void_p(0x10001)) == 5
    assert back(mask_x=None) == 8 and back(mask_w=None) == 8                  # both masks or neither
    assert back(rows_x=0, rows_w=0) == 0 and back(rows_x=0, rows_w=0, g_w=None, out_w=None) == 0
    assert back(rows_x=0, rows_w=0, mask_x=None) == 0                         # an empty gradient's mask is not looked at


def test_gemm_backward_and_grad_gemm_reject_bad_arguments(lib):
    def gemm(a=FAKE, sa=FAKE, M=0, b=FAKE, sb=FAKE, N=0, K=512, bits=4, y=FAKE, ld=0, acc=None, ws=None, wsb=0):
        return lib.quest_lowbit_gemm(a, sa, M, b, sb, N, K, bits, y, ld, acc, ws, wsb, None)
    assert gemm() == 0
    assert gemm(a=None) == 1 and gemm(y=None) == 1 and gemm(y=None, acc=FAKE) == 0
    assert gemm(bits=8) == 3 and gemm(bits=0) == 3
    assert gemm(K=96) == 2 and gemm(K=0) == 2 and gemm(M=-1) == 2 and gemm(N=8, ld=4) == 2
    assert gemm(a=ctypes.c_void_p(0x10004)) == 5
    # per-lane operand offsets are 32-bit: max(M, N) * K / 2 must stay below 2^32 (a million tokens at K = 8192 do not)
    assert gemm(M=1 << 20, N=1 << 20, K=8192, ld=1 << 20) == 2 and gemm(M=(1 << 20) - 64, N=64, K=8192, ld=64, y=None) == 1
    assert q.quest_lowbit_gemm_workspace_bytes(1 << 20, 64, 8192, 4) == -1
    # scratch for the 1- and 2-bit fast path: both operands as nibbles; too small is an argument error
    assert q.quest_lowbit_gemm_workspace_bytes(512, 256, 1024, 2) == (512 + 256) * 512
    assert q.quest_lowbit_gemm_workspace_bytes(512, 256, 1024, 4) == 0
    assert q.quest_lowbit_gemm_workspace_bytes(64, 256, 1024, 1) == 0      # below the tile kernels' sizes
    assert q.quest_lowbit_gemm_workspace_bytes(512, 256, 1024, 8) == -1
    assert gemm(M=512, N=256, K=1024, bits=2, ld=256, ws=FAKE, wsb=(512 + 256) * 512 - 1) == 8
    assert gemm(M=512, N=256, K=1024, bits=2, ld=256, ws=ctypes.c_void_p(0x10008), wsb=1 << 20) == 5
    assert gemm(wsb=-1) == 8

    # the variant with the built-in scratch buffer: same checks, plus its size limit (32 MiB)
    def static(a=FAKE, sa=FAKE, M=0, b=FAKE, sb=FAKE, N=0, K=512, bits=4, y=FAKE, ld=0, acc=None):
        return lib.quest_lowbit_gemm_static(a, sa, M, b, sb, N, K, bits, y, ld, acc, None)
    assert static() == 0 and static(a=None) == 1 and static(bits=7) == 3 and static(K=100) == 2
    assert static(M=65536, N=8192, K=1024, bits=2, ld=8192) == 9          # (M + N) K / 2 = 36 MiB of scratch
    assert static(M=65536, N=8192, K=1024, bits=4, ld=8192, a=None) == 1  # 4-bit codes need none: not rejected for it
    assert "scratch" in q.status_string(9)

    def back(g=FAKE, gd=1, mask=FAKE, rows=0, cols=512, n=512, out=FAKE, od=1):
        return lib.quest_trust_backward(g, gd, mask, rows, cols, n, out, od, None)
    assert back() == 0 and back(mask=None) == 0
    assert back(g=None) == 1 and back(out=None) == 1 and back(gd=3) == 6 and back(od=-1) == 6
    assert back(cols=20) == 2 and back(n=48) == 4 and back(out=ctypes.c_void_p(0x10002)) == 5

    def grad(which=0, dy=FAKE, qc=FAKE, qs=FAKE, bits=4, M=0, N=0, K=0, out=FAKE, ws=None, wsb=0):
        return lib.quest_grad_gemm(which, dy, qc, qs, bits, M, N, K, out, ws, wsb, None)
    assert grad() == 0
    assert grad(which=2) == 8 and grad(dy=None) == 1 and grad(bits=8) == 3 and grad(M=32) == 2
    # scratch: the expanded operand (bf16), plus two 256 KiB partial-tile slots per compute unit when tiles are split
    assert q.quest_grad_gemm_workspace_bytes(0, 64, 64, 64) == 0            # small-shape kernel: none
    need = q.quest_grad_gemm_workspace_bytes(1, 8192, 768, 512)
    assert need >= 8192 * 512 * 2 and need % 256 == 0
    assert q.quest_grad_gemm_workspace_bytes(0, 512, 256, 512) == 256 * 512 * 2    # whole tiles only
    assert q.quest_grad_gemm_workspace_bytes(2, 512, 256, 512) == -1 and q.quest_grad_gemm_workspace_bytes(0, 32, 64, 64) == -1
    assert grad(which=1, M=8192, N=768, K=512) == 8                         # workspace missing
    assert grad(which=1, M=8192, N=768, K=512, ws=FAKE, wsb=need - 1) == 8  # too small
    assert grad(which=1, M=8192, N=768, K=512, ws=ctypes.c_void_p(0x10004), wsb=need) == 5


def test_variant_entry_points_reject_bad_arguments(lib):
    def absmax(x=FAKE, dtype=1, rows=0, cols=512, ld=512, n=512, bits=4, codes=FAKE, scales=FAKE, mask=None):
        return lib.quest_hadamard_quantize_absmax(x, dtype, rows, cols, ld, n, bits, codes, scales, mask, None, None)
    assert absmax() == 0 and absmax(n=1) == 0
    assert absmax(x=None) == 1 and absmax(bits=5) == 3 and absmax(n=48) == 4 and absmax(cols=20) == 2

    def fp4(x=FAKE, dtype=1, rows=0, cols=512, ld=512, n=512, alpha=0.0, codes=FAKE, scales=FAKE, mask=None):
        return lib.quest_hadamard_quantize_fp4(x, dtype, rows, cols, ld, n, alpha, codes, scales, mask, None, None)
    assert fp4() == 0 and fp4(alpha=3.0) == 0
    assert fp4(codes=None) == 1 and fp4(dtype=9) == 6 and fp4(alpha=float("nan")) == 8 and fp4(ld=100) == 2

    def gemm4(a=FAKE, sa=FAKE, M=0, b=FAKE, sb=FAKE, N=0, K=512, y=FAKE, ld=0, acc=None):
        return lib.quest_lowbit_gemm_fp4(a, sa, M, b, sb, N, K, y, ld, acc, None)
    assert gemm4() == 0 and gemm4(y=None, acc=FAKE) == 0
    assert gemm4(b=None) == 1 and gemm4(y=None) == 1
    assert gemm4(K=64) == 2 and gemm4(K=192) == 2 and gemm4(K=131072) == 2 and gemm4(N=8, ld=4) == 2
    assert gemm4(b=ctypes.c_void_p(0x10004)) == 5

    def grad4(which=0, dy=FAKE, qc=FAKE, qs=FAKE, M=0, N=0, K=0, out=FAKE, ws=None, wsb=0):
        return lib.quest_grad_gemm_fp4(which, dy, qc, qs, M, N, K, out, ws, wsb, None)
    assert grad4() == 0 and grad4(which=2) == 8 and grad4(qc=None) == 1
    assert grad4(M=64, N=256, K=256) == 2 and grad4(M=256, N=32, K=256) == 2 and grad4(M=256, N=256, K=64) == 2
    assert q.quest_grad_gemm_fp4_workspace_bytes(0, 64, 256, 256) == -1
    assert q.quest_grad_gemm_fp4_workspace_bytes(0, 512, 256, 512) == 256 * 512 * 2
    assert grad4(M=512, N=256, K=512) == 8 and grad4(M=512, N=256, K=512, ws=FAKE, wsb=100) == 8

    def wonly(x=FAKE, wc=FAKE, ws=FAKE, bits=4, M=0, N=0, K=0, y=FAKE, scratch=None, sb=0):
        return lib.quest_weight_only_gemm(x, wc, ws, bits, M, N, K, y, scratch, sb, None)
    assert q.quest_weight_only_gemm_workspace_bytes(256, 256, 64) == 256 * 64 * 2
    assert q.quest_weight_only_gemm_workspace_bytes(64, 256, 64) == -1
    assert wonly(M=256, N=256, K=64) == 8
    assert wonly() == 0
    assert wonly(x=None) == 1 and wonly(bits=8) == 3
    assert wonly(M=64, N=256, K=64) == 2 and wonly(M=256, N=256, K=32) == 2 and wonly(M=256, N=192 + 8, K=64) == 2
    assert wonly(y=ctypes.c_void_p(0x10002)) == 5


def test_probe_library_exports_what_its_header_declares(lib):
    """The benchmark's measurement aid (include/quest_probe.h) is a library of its own."""
    from paper_2502_05003_amd import build
    header = open(os.path.join(ROOT, "include", "quest_probe.h")).read()
    declared = set(re.findall(r"\b(quest_[a-z_0-9]+)\s*\(", header))
    assert declared == {"quest_probe_mfma_loop"}
    probe = ctypes.CDLL(build.PROBE_LIB)
    probe.quest_probe_mfma_loop.restype = ctypes.c_int32
    probe.quest_probe_mfma_loop.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                            ctypes.c_int32, ctypes.c_void_p]
    assert probe.quest_probe_mfma_loop(0, None, FAKE, 1, 1, None) == 1          # validation before any launch
    assert probe.quest_probe_mfma_loop(2, FAKE, FAKE, 1, 1, None) == 1 and probe.quest_probe_mfma_loop(0, FAKE, FAKE, 0, 1, None) == 1


def test_status_strings(lib):
    assert q.status_string(0) == "ok"
    assert len({q.status_string(s) for s in range(10)}) == 10
    assert "unknown" in q.status_string(99)
