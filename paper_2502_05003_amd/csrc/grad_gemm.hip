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

}  // namespace

hipError_t launch_grad_gemm(const GradGemmArgs &a, hipStream_t stream)
{
    if (a.M == 0 || a.N == 0 || a.K == 0)
        return hipSuccess;
    const int levels = 1 << a.bits;
    const auto *dy = static_cast<const uint16_t *>(a.dy);
    auto *out = static_cast<uint16_t *>(a.out);
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
