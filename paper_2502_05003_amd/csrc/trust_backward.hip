// Trust-masked inverse Hadamard transform, out = IHT(M (.) g) (Algorithm 2; Sec. 3.2 of
// arXiv 2502.05003).  The normalised Sylvester transform is symmetric and orthogonal, so the
// inverse is the same block transform as the forward one.
#include "quest_device.h"
#include "quest_internal.h"

namespace quest {
namespace {

constexpr int kGenericThreads = 256;

/*
 * Generic kernel: one workgroup per row at a time, row in LDS as fp32.  The mask byte of each
 * group of eight elements zeroes the untrusted ones as they are loaded; index bits 0..2 are
 * transformed in registers, the rest in LDS passes; the 1/sqrt(n) factor and the output rounding
 * are applied on the way out.
 */
template <typename In, typename Out>
__global__ __launch_bounds__(kGenericThreads) void tb_generic_kernel(
    const In *__restrict__ g, const uint8_t *__restrict__ mask, int64_t rows, int cols, int log2n,
    Out *__restrict__ out)
{
    extern __shared__ float lds[];
    float *row = lds;
    const int groups = cols >> 3;
    const float inv_sqrt_n = (log2n & 1) ? 0.70710678118654752440f / (float)(1 << (log2n >> 1))
                                         : 1.0f / (float)(1 << (log2n >> 1));

    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const In *src = g + r * (int64_t)cols;
        for (int grp = threadIdx.x; grp < groups; grp += blockDim.x) {
            float v[8];
            load8(src + 8 * grp, v);
            const uint32_t m = mask ? mask[r * (int64_t)groups + grp] : 0xffu;
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v[i] = ((m >> i) & 1u) ? v[i] : 0.0f;
            butterflies8(v, log2n < 3 ? log2n : 3);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                row[lds_pad(8 * grp + i)] = v[i];
        }
        lds_butterfly_passes(row, cols, log2n);
        Out *dst = out + r * (int64_t)cols;
        for (int grp = threadIdx.x; grp < groups; grp += blockDim.x) {
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v[i] = __fmul_rn(row[lds_pad(8 * grp + i)], inv_sqrt_n);
            store8(dst + 8 * grp, v);
        }
        __syncthreads();
    }
}

template <typename In, typename Out>
hipError_t launch_generic(const BackwardArgs &a, hipStream_t stream)
{
    const int cols = (int)a.cols;
    const size_t lds_bytes = (size_t)(cols + (cols >> 5) + 1) * sizeof(float);
    const int64_t max_blocks = 256 * 8;
    const dim3 grid((unsigned)(a.rows < max_blocks ? a.rows : max_blocks));
    auto kernel = tb_generic_kernel<In, Out>;
    if (lds_bytes > 48 * 1024) {
        hipError_t err = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), (int)lds_bytes);
        if (err != hipSuccess)
            return err;
    }
    hipLaunchKernelGGL(kernel, grid, dim3(kGenericThreads), lds_bytes, stream,
                       static_cast<const In *>(a.g), a.mask, a.rows, cols, a.log2n,
                       static_cast<Out *>(a.out));
    return hipGetLastError();
}

}  // namespace

hipError_t prepare_trust_backward_kernels()
{
    constexpr int kMaxLds = (QUEST_MAX_COLS + (QUEST_MAX_COLS >> 5) + 1) * (int)sizeof(float);
    hipError_t err = allow_dynamic_lds(reinterpret_cast<const void *>(tb_generic_kernel<uint16_t, uint16_t>), kMaxLds);
    if (err == hipSuccess)
        err = allow_dynamic_lds(reinterpret_cast<const void *>(tb_generic_kernel<uint16_t, float>), kMaxLds);
    if (err == hipSuccess)
        err = allow_dynamic_lds(reinterpret_cast<const void *>(tb_generic_kernel<float, uint16_t>), kMaxLds);
    if (err == hipSuccess)
        err = allow_dynamic_lds(reinterpret_cast<const void *>(tb_generic_kernel<float, float>), kMaxLds);
    return err;
}

hipError_t launch_trust_backward(const BackwardArgs &a, hipStream_t stream)
{
    if (a.rows2 != 0) {
        // two gradients: one launch where the matrix-core kernel covers the shape, else one after the other
        if (a.rows != 0 && launch_trust_backward_mfma(a, stream))
            return hipGetLastError();
        BackwardArgs first = a, second = a;
        first.g2 = nullptr;
        first.rows2 = 0;
        second.g = a.g2;
        second.mask = a.mask2;
        second.rows = a.rows2;
        second.out = a.out2;
        second.g2 = nullptr;
        second.rows2 = 0;
        const hipError_t err = launch_trust_backward(first, stream);
        return err != hipSuccess ? err : launch_trust_backward(second, stream);
    }
    if (a.rows == 0)
        return hipSuccess;
    if (launch_trust_backward_mfma(a, stream))
        return hipGetLastError();
    if (a.g_dtype == QUEST_BF16)
        return a.out_dtype == QUEST_BF16 ? launch_generic<uint16_t, uint16_t>(a, stream)
                                         : launch_generic<uint16_t, float>(a, stream);
    return a.out_dtype == QUEST_BF16 ? launch_generic<float, uint16_t>(a, stream)
                                     : launch_generic<float, float>(a, stream);
}

}  // namespace quest
