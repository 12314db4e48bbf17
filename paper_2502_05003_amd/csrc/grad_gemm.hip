// The two 16-bit gradient matmuls of Algorithm 2 (arXiv 2502.05003, Sec. 3.3): the upstream
// gradient dy against a code-packed operand whose value is bf16(s * u), contracted on the bf16
// matrix cores with fp32 accumulation.
//   which = 0:  out[M, K] = dy[M, N]   * what_h[N, K]   (contraction over N)
//   which = 1:  out[N, K] = dy[M, N]^T * xhat_h[M, K]   (contraction over M)
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

struct GradStaged {
    uint4 left[8];     // left operand: eight 16-byte pieces
    uint32_t code[8];  // right operand: eight codes of each of eight contraction rows
    float scale[8];    // and the scales of those rows
};

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
    const uint16_t *left_src = TRANSPOSED ? dy + (int64_t)(8 * mg) * ld_dy + r0 + 8 * cg
                                          : dy + (int64_t)(r0 + (tid >> 3)) * ld_dy + 8 * (tid & 7);
    const uint8_t *code_src = q_codes + (int64_t)(8 * mg) * q_row_bytes + (k0 + 8 * cg) / 2;
    const float *scale_src = q_scales + 8 * mg;
    const int steps = C / GC;

    auto fetch = [&](int step, GradStaged &g) {
        const int64_t c0 = (int64_t)min(step, steps - 1) * GC;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (TRANSPOSED)
                g.left[i] = *reinterpret_cast<const uint4 *>(left_src + (c0 + i) * ld_dy);
            else
                g.left[i] = *reinterpret_cast<const uint4 *>(left_src + (int64_t)(32 * i) * ld_dy + c0);
            g.code[i] = *reinterpret_cast<const uint32_t *>(code_src + (c0 + i) * q_row_bytes);
            g.scale[i] = scale_src[c0 + i];
        }
    };

    auto stash_left = [&](uint8_t *stage, const GradStaged &g) {
        if (TRANSPOSED) {
            // left[r] holds dy[c0 + 8 mg + r][r0 + 8 cg .. + 8]; column j of the sub-block becomes
            // chunk mg of left row 8 cg + j: halves of rows (2a, 2a+1) are paired by one byte permute
            const uint32_t w[8][4] = {
                {g.left[0].x, g.left[0].y, g.left[0].z, g.left[0].w}, {g.left[1].x, g.left[1].y, g.left[1].z, g.left[1].w},
                {g.left[2].x, g.left[2].y, g.left[2].z, g.left[2].w}, {g.left[3].x, g.left[3].y, g.left[3].z, g.left[3].w},
                {g.left[4].x, g.left[4].y, g.left[4].z, g.left[4].w}, {g.left[5].x, g.left[5].y, g.left[5].z, g.left[5].w},
                {g.left[6].x, g.left[6].y, g.left[6].z, g.left[6].w}, {g.left[7].x, g.left[7].y, g.left[7].z, g.left[7].w}};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint32_t d[4];
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    d[a] = __builtin_amdgcn_perm(w[2 * a + 1][j >> 1], w[2 * a][j >> 1],
                                                 (j & 1) ? 0x07060302u : 0x05040100u);
                const int row = 8 * cg + j;
                *reinterpret_cast<uint4 *>(stage + row * kGRowBytes + ((mg ^ gswz(row)) << 4)) =
                    make_uint4(d[0], d[1], d[2], d[3]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = (tid >> 3) + 32 * i;
                *reinterpret_cast<uint4 *>(stage + row * kGRowBytes + (((tid & 7) ^ gswz(row)) << 4)) =
                    g.left[i];
            }
        }
    };

    // codes of contraction rows (2a, 2a+1), columns 0..7 of the sub-block -> bf16 pairs, i.e. word a
    // of the eight right-operand chunks.  value = bf16(fp32(s * u)), u = 2 c - (L - 1).
    auto stash_right_pair = [&](uint8_t *stage, const GradStaged &g, int a, uint32_t (&word)[8]) {
        (void)stage;
        float v[2][8];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t q = g.code[2 * a + h];
            const uint32_t even = q & 0x0f0f0f0fu, odd = (q >> 4) & 0x0f0f0f0fu;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t bytes = (e & 1) ? odd : even;
                const float c = (float)((bytes >> (8 * (e >> 1))) & 0xffu);
                v[h][e] = __fmul_rn(g.scale[2 * a + h], __fmaf_rn(c, 2.0f, offset));
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e)
            word[e] = pack2_bf16(v[0][e], v[1][e]);
    };
    auto stash_right = [&](uint8_t *stage, const GradStaged &g) {
        uint32_t chunk[8][4];
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            uint32_t word[8];
            stash_right_pair(stage, g, a, word);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                chunk[e][a] = word[e];
        }
        uint8_t *right = stage + GT * kGRowBytes;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int row = 8 * cg + j;
            *reinterpret_cast<uint4 *>(right + row * kGRowBytes + ((mg ^ gswz(row)) << 4)) =
                make_uint4(chunk[j][0], chunk[j][1], chunk[j][2], chunk[j][3]);
        }
    };

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0.0f;

    GradStaged g;
    fetch(0, g);
    stash_left(smem, g);
    stash_right(smem, g);
    fetch(1, g);
    __syncthreads();

    // fragments: chunk 2 s + lh of a row holds this lane's eight contraction elements of k-step s
    const int left_off = (wr * 128 + lm) * kGRowBytes;
    const int right_off = GT * kGRowBytes + (wc * 128 + lm) * kGRowBytes;
    const int x = gswz(lm);   // rows lm + 32 i share bits 1..3
    auto load_frags = [&](const uint8_t *stage, int ks, v8bf (&lf)[4], v8bf (&rf)[4]) {
        const int off = ((2 * ks + lh) ^ x) << 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            lf[i] = *reinterpret_cast<const v8bf *>(stage + left_off + i * 32 * kGRowBytes + off);
            rf[i] = *reinterpret_cast<const v8bf *>(stage + right_off + i * 32 * kGRowBytes + off);
        }
    };
    auto multiply = [&](const v8bf (&lf)[4], const v8bf (&rf)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)   // right fragment as the row operand: transposed tiles
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rf[j], lf[i], acc[i][j], 0, 0, 0);
    };

    v8bf lf[2][4], rf[2][4];
    load_frags(smem, 0, lf[0], rf[0]);
    for (int step = 0; step < steps; ++step) {
        uint8_t *cur = smem + (step & 1) * kGStage;
        uint8_t *nxt = smem + ((step + 1) & 1) * kGStage;
        // g holds step + 1; it is written to the idle stage between the MFMAs and refilled with
        // step + 2 (past the end: the last step again, into a stage nobody reads)
        load_frags(cur, 1, lf[1], rf[1]);
        multiply(lf[0], rf[0]);
        stash_left(nxt, g);
        load_frags(cur, 2, lf[0], rf[0]);
        multiply(lf[1], rf[1]);
        stash_right(nxt, g);
        load_frags(cur, 3, lf[1], rf[1]);
        multiply(lf[0], rf[0]);
        fetch(step + 2, g);
        multiply(lf[1], rf[1]);
        __syncthreads();
        load_frags(nxt, 0, lf[0], rf[0]);
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
