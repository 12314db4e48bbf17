// The two 16-bit gradient matmuls of Algorithm 2 (arXiv 2502.05003, Sec. 3.3): the upstream
// gradient dy against a code-packed operand whose value is bf16(s * u), contracted on the bf16
// matrix cores with fp32 accumulation.
//   which = 0:  out[M, K] = dy[M, N]   * what_h[N, K]   (contraction over N)
//   which = 1:  out[N, K] = dy[M, N]^T * xhat_h[M, K]   (contraction over M)
#include <utility>

#include "quest_device.h"
#include "quest_internal.h"

namespace quest {
namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kTile = 64;      // output tile is 64 x 64, one 32 x 32 quadrant per wave
constexpr int kStep = 32;      // contraction elements per main-loop step
constexpr int kThreads = 256;
constexpr int kStride = 40;    // LDS row stride in bf16: 32 payload + 8 pad

/*
 * TRANSPOSED = false: left operand rows are dy rows (out row = m, contraction index = n).
 * TRANSPOSED = true:  left operand rows are dy columns (out row = n, contraction index = m).
 * q is [C, K*cb/8] packed codes with one scale per contraction row; C is the contraction length.
 */
template <bool TRANSPOSED>
__global__ __launch_bounds__(kThreads) void grad_gemm_kernel(
    const uint16_t *__restrict__ dy, int64_t ld_dy, const uint8_t *__restrict__ q_codes,
    const float *__restrict__ q_scales, int levels, int cb, int C, int K,
    uint16_t *__restrict__ out)
{
    __shared__ __attribute__((aligned(16))) uint16_t left[kTile * kStride];   // [out row][c]
    __shared__ __attribute__((aligned(16))) uint16_t right[kTile * kStride];  // [k][c]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int r0 = blockIdx.y * kTile, k0 = blockIdx.x * kTile;
    const int64_t q_row_bytes = (int64_t)K * cb / 8;

    v16f acc;
#pragma unroll
    for (int r = 0; r < 16; ++r)
        acc[r] = 0.0f;

    for (int c0 = 0; c0 < C; c0 += kStep) {
        __syncthreads();
        if constexpr (!TRANSPOSED) {
            // 64 rows x 32 contraction elements, 16 bytes per thread, already c-contiguous
            const int row = tid >> 2, chunk = tid & 3;
            const uint4 v = *reinterpret_cast<const uint4 *>(dy + (int64_t)(r0 + row) * ld_dy + c0 +
                                                             chunk * 8);
            *reinterpret_cast<uint4 *>(left + row * kStride + chunk * 8) = v;
        } else {
            // 32 contraction rows x 64 output rows; transpose through LDS
            const int crow = tid >> 3, chunk = tid & 7;
            const uint4 v = *reinterpret_cast<const uint4 *>(dy + (int64_t)(c0 + crow) * ld_dy + r0 +
                                                             chunk * 8);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                left[(chunk * 8 + e) * kStride + crow] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
        }
        {
            // 32 contraction rows x 64 k of codes: eight codes per thread, dequantized to bf16(s u)
            const int crow = tid >> 3, chunk = tid & 7;
            const uint8_t *src = q_codes + (int64_t)(c0 + crow) * q_row_bytes +
                                 (int64_t)(k0 + chunk * 8) * cb / 8;
            uint32_t bits = 0;
            for (int byte = 0; byte < cb; ++byte)
                bits |= (uint32_t)src[byte] << (8 * byte);
            const float s = q_scales[c0 + crow];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int c = (int)((bits >> (e * cb)) & ((1u << cb) - 1u));
                const float value = __fmul_rn(s, (float)(2 * c - (levels - 1)));
                right[(chunk * 8 + e) * kStride + crow] = (uint16_t)float_to_bf16_bits(value);
            }
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < kStep / 16; ++s) {
            const int off = s * 16 + (lane >> 5) * 8;
            const v8bf a = *reinterpret_cast<const v8bf *>(left + (wr * 32 + (lane & 31)) * kStride + off);
            const v8bf b = *reinterpret_cast<const v8bf *>(right + (wc * 32 + (lane & 31)) * kStride + off);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
        }
    }

    const int k = k0 + wc * 32 + (lane & 31);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = r0 + wr * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        out[(int64_t)row * K + k] = (uint16_t)float_to_bf16_bits(acc[r]);
    }
}


// ------------------------------------------------------------------------------------------
// Main kernel: 256 x 256 outputs per workgroup, four waves of 128 x 128 (sixteen 32 x 32 fp32
// accumulator tiles), 64 contraction elements per step, two LDS stages of 64 KiB, one workgroup
// per CU.  Both operands sit in LDS as [row][contraction] bf16, 128 bytes per row, so every MFMA
// fragment is one 128-bit LDS read.
//   left operand  (rows = output rows):   dy rows as they are (which = 0), or dy columns,
//                                          transposed 8 x 8 in registers on the way in (which = 1);
//   right operand (rows = output columns): the code-packed matrix, dequantized to bf16(s u) and
//                                          transposed on the way in (pairs of contraction rows are
//                                          converted together, which is the transpose).
// ------------------------------------------------------------------------------------------

constexpr int GT = 256;                        // tile edge
constexpr int GC = 64;                         // contraction elements per step
constexpr int kGemmThreads = 256;
constexpr int kGRowBytes = GC * 2;             // 128
constexpr int kGStage = 2 * GT * kGRowBytes;   // 64 KiB: left rows, then right rows
constexpr int kGLds = 2 * kGStage;             // 128 KiB, reused by the epilogue

// chunk c (0..7) of row `row` lives at chunk c ^ gswz(row): sixteen consecutive rows reading the
// same logical chunk hit sixteen different 16-byte slots modulo 256 bytes
__device__ __forceinline__ int gswz(int row)
{
    return (row >> 1) & 7;
}

__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi)
{
    typedef __bf16 v2bf16 __attribute__((ext_vector_type(2)));
    v2bf16 p;
    p[0] = (__bf16)lo;
    p[1] = (__bf16)hi;
    uint32_t u;
    __builtin_memcpy(&u, &p, 4);
    return u;
}

// compile-time loop: f(std::integral_constant<int, 0>) ... f(std::integral_constant<int, N - 1>)
template <int... Is, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F &&f)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

template <bool TRANSPOSED>
__global__ __launch_bounds__(kGemmThreads, 1) void grad_gemm_tile_kernel(
    const uint16_t *__restrict__ dy, int64_t ld_dy, const uint8_t *__restrict__ q_codes,
    const float *__restrict__ q_scales, int levels, int C, int K, int tiles_r, int tiles_k,
    uint16_t *__restrict__ out)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // workgroup -> tile: one contiguous run of tiles per XCD, four tile-rows deep
    const int total = tiles_r * tiles_k;
    const int per_xcd = (total + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total)
        return;
    const int band = logical / (4 * tiles_k);
    const int band_rows = min(4, tiles_r - band * 4);
    const int in_band = logical - band * 4 * tiles_k;
    const int r0 = (band * 4 + in_band % band_rows) * GT;
    const int k0 = (in_band / band_rows) * GT;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int lm = lane & 31, lh = lane >> 5;
    const int64_t q_row_bytes = (int64_t)K / 2;
    const float offset = -(float)(levels - 1);

    // staging roles
    //   direct left operand: chunk tid % 8 of rows tid / 8 + 32 i
    //   transposed operands: 8 x 8 sub-block, contraction group mg = tid % 8, column group cg = tid / 8
    const int mg = tid & 7, cg = tid >> 3;
    // every global address is a wave-uniform base plus a 32-bit per-thread byte offset that does not
    // change from step to step (one register per stream instead of one pointer per piece)
    // which = 0: the left pieces go from global memory straight into LDS (no registers): lane l of a
    // wave lands at LDS offset 16 l of the wave's 1 KiB (8 rows x 128 bytes), so it fetches the
    // logical chunk that belongs in that physical slot
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int dma_row = tid >> 3;                                   // + 32 jj
    const int dma_chunk = (tid & 7) ^ gswz(dma_row);                // gswz(row + 32 jj) = gswz(row)
    const uint32_t left_toff = TRANSPOSED ? (uint32_t)((8 * mg) * ld_dy + 8 * cg) * 2u
                                          : (uint32_t)(dma_row * ld_dy + 8 * dma_chunk) * 2u;
    const uint32_t code_toff = (uint32_t)((8 * mg) * q_row_bytes + 4 * cg);
    const uint32_t scale_toff = (uint32_t)(8 * mg) * 4u;
    const char *left_base = reinterpret_cast<const char *>(TRANSPOSED ? dy + r0 : dy + (int64_t)r0 * ld_dy);
    const char *code_base = reinterpret_cast<const char *>(q_codes + k0 / 2);
    const char *scale_base = reinterpret_cast<const char *>(q_scales);
    const int steps = C / GC;

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0.0f;

    // Staged pieces of one step (plain arrays indexed by compile-time constants only, so that they
    // live in registers): left operand, eight 16-byte pieces; right operand, eight codes of each of
    // eight contraction rows and the scales of those rows.
    uint4 gl[8];
    uint32_t gq[8];
    float gs[8];
    auto fetch_piece = [&](auto rc, int64_t c0) {
        constexpr int r = decltype(rc)::value;
        if (TRANSPOSED)
            gl[r] = *reinterpret_cast<const uint4 *>(left_base + (c0 + r) * ld_dy * 2 + left_toff);
        gq[r] = *reinterpret_cast<const uint32_t *>(code_base + (c0 + r) * q_row_bytes + code_toff);
        gs[r] = *reinterpret_cast<const float *>(scale_base + (c0 + r) * 4 + scale_toff);
    };
    // which = 0: rows 8 wave + 32 jj .. + 8 of the left tile, global -> LDS
    auto dma_left_piece = [&](auto jc, uint8_t *stage, int64_t c0) {
        constexpr int jj = decltype(jc)::value;
        const char *src = left_base + ((int64_t)(32 * jj) * ld_dy + c0) * 2 + left_toff;
        lds_dma16(src, lds_address(stage) + (8 * wave_u + 32 * jj) * kGRowBytes);
    };
    // which = 1: column jj of the 8 x 8 sub-block, built by one byte permute per pair of rows
    // (2a, 2a+1), becomes chunk mg of left row 8 cg + jj
    auto stash_left_piece = [&](auto jc, uint8_t *stage) {
        constexpr int jj = decltype(jc)::value;
        uint32_t d[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const uint4 lo = gl[2 * a], hi = gl[2 * a + 1];
            const uint32_t wl = (jj >> 1) == 0 ? lo.x : (jj >> 1) == 1 ? lo.y : (jj >> 1) == 2 ? lo.z : lo.w;
            const uint32_t wh = (jj >> 1) == 0 ? hi.x : (jj >> 1) == 1 ? hi.y : (jj >> 1) == 2 ? hi.z : hi.w;
            d[a] = __builtin_amdgcn_perm(wh, wl, (jj & 1) ? 0x07060302u : 0x05040100u);
        }
        const int row = 8 * cg + jj;
        *reinterpret_cast<uint4 *>(stage + row * kGRowBytes + ((mg ^ gswz(row)) << 4)) =
            make_uint4(d[0], d[1], d[2], d[3]);
    };
    // codes of contraction rows (2a, 2a+1), column e of the sub-block -> one bf16 pair, word a of
    // right chunk e.  value = bf16(fp32(s * u)), u = 2 c - (L - 1).
    uint32_t chunk[8][4];
    auto dequant_pair = [&](auto kc) {
        constexpr int a = decltype(kc)::value >> 3, e = decltype(kc)::value & 7;
        float v[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t q = gq[2 * a + h];
            const uint32_t nib = (e & 1) ? (q >> 4) : q;
            const float c = (float)((nib >> (8 * (e >> 1))) & 0xfu);
            v[h] = __fmul_rn(gs[2 * a + h], __fmaf_rn(c, 2.0f, offset));
        }
        chunk[e][a] = pack2_bf16(v[0], v[1]);
    };
    auto stash_right_piece = [&](auto jc, uint8_t *stage) {
        constexpr int jj = decltype(jc)::value;
        const int row = 8 * cg + jj;
        *reinterpret_cast<uint4 *>(stage + GT * kGRowBytes + row * kGRowBytes + ((mg ^ gswz(row)) << 4)) =
            make_uint4(chunk[jj][0], chunk[jj][1], chunk[jj][2], chunk[jj][3]);
    };

    static_for<8>([&](auto r) { fetch_piece(r, 0); });
    if constexpr (TRANSPOSED)
        static_for<8>([&](auto j) { stash_left_piece(j, smem); });
    else
        static_for<8>([&](auto j) { dma_left_piece(j, smem, 0); });
    static_for<32>([&](auto k) { dequant_pair(k); });
    static_for<8>([&](auto j) { stash_right_piece(j, smem); });
    static_for<8>([&](auto r) { fetch_piece(r, (int64_t)min(1, steps - 1) * GC); });
    wait_vmcnt<0>();
    __syncthreads();

    // fragments: chunk 2 s + lh of a row holds this lane's eight contraction elements of k-step s
    const int left_off = (wr * 128 + lm) * kGRowBytes;
    const int right_off = GT * kGRowBytes + (wc * 128 + lm) * kGRowBytes;
    const int x = gswz(lm);   // rows lm + 32 i share bits 1..3
    v8bf lf[2][4], rf[2][4];
    auto load_frag = [&](const uint8_t *stage, int ks, int which_frag) {
        const int off = ((2 * ks + lh) ^ x) << 4;
        const int i = which_frag & 3;
        if (which_frag < 4)
            lf[ks & 1][i] = *reinterpret_cast<const v8bf *>(stage + left_off + i * 32 * kGRowBytes + off);
        else
            rf[ks & 1][i] = *reinterpret_cast<const v8bf *>(stage + right_off + i * 32 * kGRowBytes + off);
    };
#pragma unroll
    for (int f = 0; f < 8; ++f)
        load_frag(smem, 0, f);

    // One wave per SIMD: nothing else hides the staging work, so it is cut into 64 slices and one
    // slice follows each of the 64 MFMAs of a step, pinned there by scheduling barriers:
    //    0..7   left pieces of step + 1: global -> LDS (which = 0) or permute and store (which = 1)
    //    0..31  dequantize two codes each (rows 2a, 2a+1 of column e) into a word of a right chunk
    //   32..39  store the eight right chunks (which = 0: and fetch the codes of step + 2)
    //   48..55  which = 1: fetch step + 2
    //   (the first eight MFMAs of a k-step also carry the fragment loads of the next one)
    for (int step = 0; step < steps; ++step) {
        uint8_t *cur = smem + (step & 1) * kGStage;
        uint8_t *nxt = smem + ((step + 1) & 1) * kGStage;
        // registers hold step + 1; which = 0 moves the left tile of step + 1 straight into the idle
        // stage and can refill its (small) code registers early; which = 1 refills late, after its
        // left pieces have been permuted out of their registers
        const int64_t c_one = (int64_t)min(step + 1, steps - 1) * GC;
        const int64_t c_two = (int64_t)min(step + 2, steps - 1) * GC;
        static_for<64>([&](auto kc) {
            constexpr int k = decltype(kc)::value;
            constexpr int ks = k >> 4, i = (k >> 2) & 3, j = k & 3;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rf[ks & 1][j], lf[ks & 1][i], acc[i][j], 0, 0, 0);
            if constexpr ((k & 15) < 8 && ks < 3)
                load_frag(cur, ks + 1, k & 15);
            if constexpr (k < 8 && TRANSPOSED)
                stash_left_piece(std::integral_constant<int, k & 7>{}, nxt);
            if constexpr (k < 32) {
                dequant_pair(std::integral_constant<int, k & 31>{});
                // after the slice's first use of the code registers: the wait for those (older)
                // loads must not also cover the transfer just issued
                if constexpr (k < 8 && !TRANSPOSED)
                    dma_left_piece(std::integral_constant<int, k & 7>{}, nxt, c_one);
            } else if constexpr (k < 40) {
                stash_right_piece(std::integral_constant<int, (k - 32) & 7>{}, nxt);
                if constexpr (!TRANSPOSED)
                    fetch_piece(std::integral_constant<int, (k - 32) & 7>{}, c_two);
            } else if constexpr (k >= 48 && k < 56) {
                if constexpr (TRANSPOSED)
                    fetch_piece(std::integral_constant<int, (k - 48) & 7>{}, c_two);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        if constexpr (!TRANSPOSED)
            wait_vmcnt<8>();   // the eight transfers (issued before this step's eight code fetches) landed
        __syncthreads();
#pragma unroll
        for (int f = 0; f < 8; ++f)
            load_frag(nxt, 0, f);
    }

    // Epilogue.  Each accumulator tile is a transposed output tile: lane l holds output row l % 32
    // and, in register r, output column 8 (r / 4) + 4 (l / 32) + r % 4.  Each wave parks its
    // 128 x 128 block as bf16 in its own 32 KiB of LDS (chunks swizzled by row) and writes it out as
    // 256-byte row segments.
    __syncthreads();
    uint8_t *park = smem + wave * 32768;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = i * 32 + lm;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = j * 32 + 8 * q + 4 * lh;
                const int chunk = (col >> 3) ^ (row & 15);
                *reinterpret_cast<uint2 *>(park + row * 256 + chunk * 16 + (col & 4) * 2) =
                    make_uint2(pack2_bf16(acc[i][j][4 * q + 0], acc[i][j][4 * q + 1]),
                               pack2_bf16(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]));
            }
        }
    }
    uint16_t *out_base = out + (int64_t)(r0 + wr * 128) * K + k0 + wc * 128;
#pragma unroll 4
    for (int pass = 0; pass < 32; ++pass) {
        const int row = pass * 4 + (lane >> 4);
        const int c = lane & 15;
        const uint4 v = *reinterpret_cast<const uint4 *>(park + row * 256 + ((c ^ (row & 15)) << 4));
        *reinterpret_cast<uint4 *>(out_base + (int64_t)row * K + c * 8) = v;
    }
}

}  // namespace

hipError_t launch_grad_gemm(const GradGemmArgs &a, hipStream_t stream)
{
    if (a.M == 0 || a.N == 0 || a.K == 0)
        return hipSuccess;
    const int levels = 1 << a.bits;
    const auto *dy = static_cast<const uint16_t *>(a.dy);
    auto *out = static_cast<uint16_t *>(a.out);
    const int64_t out_rows = a.which == 0 ? a.M : a.N, contraction = a.which == 0 ? a.N : a.M;
    if (a.cb == 4 && (out_rows % GT) == 0 && (a.K % GT) == 0 && (contraction % GC) == 0) {
        const int tiles_r = (int)(out_rows / GT), tiles_k = (int)(a.K / GT);
        const dim3 grid((unsigned)(((tiles_r * tiles_k + 7) / 8) * 8));
        static bool attr_set = false;
        if (!attr_set) {
            hipError_t err = hipFuncSetAttribute(
                reinterpret_cast<const void *>(grad_gemm_tile_kernel<false>),
                hipFuncAttributeMaxDynamicSharedMemorySize, kGLds);
            if (err == hipSuccess)
                err = hipFuncSetAttribute(reinterpret_cast<const void *>(grad_gemm_tile_kernel<true>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, kGLds);
            if (err != hipSuccess)
                return err;
            attr_set = true;
        }
        if (a.which == 0)
            hipLaunchKernelGGL(grad_gemm_tile_kernel<false>, grid, dim3(kGemmThreads), kGLds, stream, dy,
                               a.N, a.q_codes, a.q_scales, levels, (int)contraction, (int)a.K, tiles_r,
                               tiles_k, out);
        else
            hipLaunchKernelGGL(grad_gemm_tile_kernel<true>, grid, dim3(kGemmThreads), kGLds, stream, dy,
                               a.N, a.q_codes, a.q_scales, levels, (int)contraction, (int)a.K, tiles_r,
                               tiles_k, out);
        return hipGetLastError();
    }
    if (a.which == 0) {
        const dim3 grid((unsigned)(a.K / kTile), (unsigned)(a.M / kTile));
        hipLaunchKernelGGL(grad_gemm_kernel<false>, grid, dim3(kThreads), 0, stream, dy, a.N,
                           a.q_codes, a.q_scales, levels, a.cb, (int)a.N, (int)a.K, out);
    } else {
        const dim3 grid((unsigned)(a.K / kTile), (unsigned)(a.N / kTile));
        hipLaunchKernelGGL(grad_gemm_kernel<true>, grid, dim3(kThreads), 0, stream, dy, a.N,
                           a.q_codes, a.q_scales, levels, a.cb, (int)a.M, (int)a.K, out);
    }
    return hipGetLastError();
}

}  // namespace quest
