// Low-bit integer GEMM with a dequantizing bf16 epilogue: y = xhat_h what_h^T computed on the
// packed codes (Algorithm 1, last step; Sec. 5 "Kernel Overview" stage 3 of arXiv 2502.05003).
// The codes are widened to the signed odd integers u = 2c - (L - 1) on their way into LDS and
// contracted on the INT8 matrix cores; acc = sum_k u_a u_b is exact in int32.
#include "quest_device.h"
#include "quest_internal.h"

namespace quest {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 128;          // block tile rows (activations)
constexpr int BN = 128;          // block tile columns (weights)
constexpr int BK = 64;           // contraction elements per main-loop step
constexpr int kThreads = 256;    // 4 waves in a 2 x 2 arrangement, 64 x 64 outputs per wave
constexpr int kRowStride = 80;   // LDS bytes per tile row: 64 payload + 16 pad (conflict-free b128 reads)

/*
 * Widen 32 consecutive codes (CB bits each, little-endian) to 32 signed bytes u = 2c - (L - 1),
 * four per dword.  The order of the 32 bytes is a fixed permutation of the element order; both
 * GEMM operands go through this same function, so products still pair element k with element k.
 */
template <int CB>
__device__ __forceinline__ void widen32(const uint32_t *packed, uint32_t bias, uint32_t (&out)[8])
{
    uint32_t c[8];
    if constexpr (CB == 4) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            c[2 * i] = packed[i] & 0x0f0f0f0fu;
            c[2 * i + 1] = (packed[i] >> 4) & 0x0f0f0f0fu;
        }
    } else if constexpr (CB == 2) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int d = 0; d < 4; ++d)
                c[4 * i + d] = (packed[i] >> (2 * d)) & 0x03030303u;
    } else {
#pragma unroll
        for (int d = 0; d < 8; ++d)
            c[d] = (packed[0] >> d) & 0x01010101u;
    }
    // per byte: (2c + 128) - (L - 1), then flip the top bit -> two's complement 2c - (L - 1);
    // every byte stays >= 128 - 15 before the subtraction, so no borrow crosses bytes
#pragma unroll
    for (int i = 0; i < 8; ++i)
        out[i] = (((c[i] << 1) | 0x80808080u) - bias) ^ 0x80808080u;
}

template <int CB>
__global__ __launch_bounds__(kThreads) void lowbit_gemm_kernel(
    const uint8_t *__restrict__ a_codes, const float *__restrict__ a_scales,
    const uint8_t *__restrict__ b_codes, const float *__restrict__ b_scales, int M, int N, int K,
    int levels, uint16_t *__restrict__ y, int64_t ld_y, int32_t *__restrict__ acc_out)
{
    __shared__ __attribute__((aligned(16))) uint8_t a_tile[BM * kRowStride];
    __shared__ __attribute__((aligned(16))) uint8_t b_tile[BN * kRowStride];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

    // staging role: thread -> (tile row, which half of the 64-element step)
    const int ld_row = tid >> 1, ld_half = tid & 1;
    constexpr int kChunkBytes = 32 * CB / 8;             // packed bytes of 32 elements
    constexpr int kChunkWords = kChunkBytes / 4 > 0 ? kChunkBytes / 4 : 1;
    const int64_t row_bytes = (int64_t)K * CB / 8;
    const int a_row = min(m0 + ld_row, M - 1), b_row = min(n0 + ld_row, N - 1);
    const uint8_t *a_src = a_codes + a_row * row_bytes + ld_half * kChunkBytes;
    const uint8_t *b_src = b_codes + b_row * row_bytes + ld_half * kChunkBytes;
    const uint32_t bias = (uint32_t)(levels - 1) * 0x01010101u;

    v16i acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0;

    auto fetch = [&](const uint8_t *src, uint32_t (&w)[kChunkWords]) {
        if constexpr (CB == 4) {
            const uint4 v = *reinterpret_cast<const uint4 *>(src);
            w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
        } else if constexpr (CB == 2) {
            const uint2 v = *reinterpret_cast<const uint2 *>(src);
            w[0] = v.x; w[1] = v.y;
        } else {
            w[0] = *reinterpret_cast<const uint32_t *>(src);
        }
    };

    uint32_t a_next[kChunkWords], b_next[kChunkWords];
    fetch(a_src, a_next);
    fetch(b_src, b_next);

    for (int k0 = 0; k0 < K; k0 += BK) {
        uint32_t a_wide[8], b_wide[8];
        widen32<CB>(a_next, bias, a_wide);
        widen32<CB>(b_next, bias, b_wide);
        __syncthreads();  // previous step's MFMA reads are done
        uint4 *a_dst = reinterpret_cast<uint4 *>(a_tile + ld_row * kRowStride + ld_half * 32);
        uint4 *b_dst = reinterpret_cast<uint4 *>(b_tile + ld_row * kRowStride + ld_half * 32);
        a_dst[0] = make_uint4(a_wide[0], a_wide[1], a_wide[2], a_wide[3]);
        a_dst[1] = make_uint4(a_wide[4], a_wide[5], a_wide[6], a_wide[7]);
        b_dst[0] = make_uint4(b_wide[0], b_wide[1], b_wide[2], b_wide[3]);
        b_dst[1] = make_uint4(b_wide[4], b_wide[5], b_wide[6], b_wide[7]);
        if (k0 + BK < K) {  // prefetch the next step while this one is multiplied
            fetch(a_src + (int64_t)(k0 + BK) * CB / 8, a_next);
            fetch(b_src + (int64_t)(k0 + BK) * CB / 8, b_next);
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            v4i a_frag[2], b_frag[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = wm * 64 + i * 32 + (lane & 31);
                a_frag[i] = *reinterpret_cast<const v4i *>(a_tile + row * kRowStride + s * 32 +
                                                           (lane >> 5) * 16);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int row = wn * 64 + j * 32 + (lane & 31);
                b_frag[j] = *reinterpret_cast<const v4i *>(b_tile + row * kRowStride + s * 32 +
                                                           (lane >> 5) * 16);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a_frag[i], b_frag[j],
                                                                      acc[i][j], 0, 0, 0);
        }
    }

    // Epilogue.  In the 32 x 32 accumulator tile, lane l holds column l % 32 and, in register r,
    // row 8 (r / 4) + 4 (l / 32) + r % 4.
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn * 64 + j * 32 + (lane & 31);
        if (n >= N)
            continue;
        const float sb = b_scales[n];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (m >= M)
                    continue;
                const int a = acc[i][j][r];
                if (acc_out)
                    acc_out[(int64_t)m * N + n] = a;
                if (y)
                    y[(int64_t)m * ld_y + n] =
                        (uint16_t)float_to_bf16_bits(__fmul_rn(__fmul_rn((float)a, a_scales[m]), sb));
            }
        }
    }
}

}  // namespace

hipError_t launch_lowbit_gemm(const GemmArgs &a, hipStream_t stream)
{
    if (a.M == 0 || a.N == 0)
        return hipSuccess;
    const dim3 grid((unsigned)((a.N + BN - 1) / BN), (unsigned)((a.M + BM - 1) / BM));
    const dim3 block(kThreads);
    const int levels = 1 << a.bits;
    auto *y = static_cast<uint16_t *>(a.y);
    switch (a.cb) {
    case 4:
        hipLaunchKernelGGL(lowbit_gemm_kernel<4>, grid, block, 0, stream, a.a_codes, a.a_scales,
                           a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, levels, y, a.ld_y,
                           a.acc_out);
        break;
    case 2:
        hipLaunchKernelGGL(lowbit_gemm_kernel<2>, grid, block, 0, stream, a.a_codes, a.a_scales,
                           a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, levels, y, a.ld_y,
                           a.acc_out);
        break;
    default:
        hipLaunchKernelGGL(lowbit_gemm_kernel<1>, grid, block, 0, stream, a.a_codes, a.a_scales,
                           a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, levels, y, a.ld_y,
                           a.acc_out);
        break;
    }
    return hipGetLastError();
}

}  // namespace quest
