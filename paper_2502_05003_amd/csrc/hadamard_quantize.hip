// Fused block-Hadamard transform + RMS + clip/round + pack + trust mask (Algorithm 1, one operand;
// Sec. 3.1 and 3.2 of arXiv 2502.05003).  One pass over the operand: each row is read once from
// HBM, transformed on chip, and only the packed codes, the per-row scale and the mask bitmap are
// written back.
#include "quest_device.h"
#include "quest_internal.h"

namespace quest {
namespace {

constexpr int kGenericThreads = 256;

// Per-row constants of the projection, all in fp32 (the precision the codes are decided in), every
// operation correctly rounded (sqrtf and the _rn division are; the _rn square-root intrinsic is the
// hardware's approximation), so that an fp32 evaluation elsewhere reproduces them bit for bit.
struct RowQuant {
    float inv_step;   // (L - 1) / (2 alpha rms): x_h * inv_step is the position in grid cells
    float trust_abs;  // trust_edge * rms
    float scale;      // alpha rms / (L - 1)
    bool zero;        // rms == 0: every element maps to k = 0, trusted
};

__device__ __forceinline__ RowQuant row_quant(float sumsq, int cols, int levels, float alpha,
                                              float trust_edge)
{
    RowQuant q;
    const float rms = sqrtf(__fdiv_rn(sumsq, (float)cols));
    const float clip = __fmul_rn(alpha, rms);
    q.zero = !(rms > 0.0f);
    q.inv_step = q.zero ? 0.0f : __fdiv_rn((float)(levels - 1), __fmul_rn(2.0f, clip));
    q.trust_abs = __fmul_rn(trust_edge, rms);
    q.scale = __fdiv_rn(clip, (float)(levels - 1));
    return q;
}

// AbsMax variant (the comparison quantizer of Sec. 4.1): the clip is the row's largest magnitude,
// nothing is clipped and every element is trusted.
__device__ __forceinline__ RowQuant row_quant_absmax(float amax, int levels)
{
    RowQuant q;
    q.zero = !(amax > 0.0f);
    q.inv_step = q.zero ? 0.0f : __fdiv_rn((float)(levels - 1), __fmul_rn(2.0f, amax));
    q.trust_abs = amax;
    q.scale = __fdiv_rn(amax, (float)(levels - 1));
    return q;
}

// FP4 variant (Sec. 4.4): the grid is the E2M1 value set {0, .5, 1, 1.5, 2, 3, 4, 6} scaled so that 6
// sits on the clip; inv_step = 6 / (alpha rms) maps x_h to E2M1 units, scale = alpha rms / 6.
__device__ __forceinline__ RowQuant row_quant_fp4(float sumsq, int cols, float alpha, float trust_edge)
{
    RowQuant q;
    const float rms = sqrtf(__fdiv_rn(sumsq, (float)cols));
    const float clip = __fmul_rn(alpha, rms);
    q.zero = !(rms > 0.0f);
    q.inv_step = q.zero ? 0.0f : __fdiv_rn(6.0f, clip);
    q.trust_abs = __fmul_rn(trust_edge, rms);
    q.scale = __fdiv_rn(clip, 6.0f);
    return q;
}

// E2M1 code of one element: nearest magnitude (a tie goes to the even code), sign in bit 3.
__device__ __forceinline__ uint32_t quantize_fp4(float xh, const RowQuant &q)
{
    const float t = fminf(__fmul_rn(fabsf(xh), q.inv_step), 6.0f);
    const uint32_t index = (t > 0.25f) + (t >= 0.75f) + (t > 1.25f) + (t >= 1.75f) + (t > 2.5f) +
                           (t >= 3.5f) + (t > 5.0f);
    return index | (xh < 0.0f ? 8u : 0u);
}

// Code c = clamp(floor(x_h * inv_step), -L/2, L/2 - 1) + L/2 for one element.
__device__ __forceinline__ uint32_t quantize_one(float xh, const RowQuant &q, int levels)
{
    const float half = (float)(levels >> 1);
    float cell = floorf(__fmul_rn(xh, q.inv_step));
    cell = fminf(fmaxf(cell, -half), half - 1.0f);
    return (uint32_t)((int)cell + (levels >> 1));
}

/*
 * Generic kernel: any cols (multiple of 8, <= QUEST_MAX_COLS), any power-of-two block, any
 * supported bit width.  One workgroup per row at a time; the row lives in LDS as fp32.
 * Index bits 0..2 are transformed in registers straight from the 128-bit loads, the remaining
 * bits in LDS passes of three bits each.
 */
template <typename In>
__global__ __launch_bounds__(kGenericThreads) void hq_generic_kernel(
    const In *__restrict__ x, int64_t rows, int cols, int64_t ld, int log2n, int bits, int cb,
    float alpha, float trust_edge, int mode, uint8_t *__restrict__ codes,
    float *__restrict__ scales, uint8_t *__restrict__ mask, float *__restrict__ xh_out)
{
    extern __shared__ float lds[];
    float *row = lds;
    __shared__ float partial[kGenericThreads / kWave];
    __shared__ float partial_max[kGenericThreads / kWave];

    const int levels = 1 << bits;
    const int groups = cols >> 3;
    // 1/sqrt(n), correctly rounded: a power of two, or 1/sqrt(2) times one
    const float inv_sqrt_n = (log2n & 1) ? 0.70710678118654752440f / (float)(1 << (log2n >> 1))
                                         : 1.0f / (float)(1 << (log2n >> 1));

    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        const In *src = x + r * ld;
        for (int g = threadIdx.x; g < groups; g += blockDim.x) {
            float v[8];
            load8(src + 8 * g, v);
            butterflies8(v, log2n < 3 ? log2n : 3);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                row[lds_pad(8 * g + i)] = v[i];
        }
        lds_butterfly_passes(row, cols, log2n);

        // x_h = raw / sqrt(n); row sum of squares and largest magnitude
        float sumsq = 0.0f, amax = 0.0f;
        for (int g = threadIdx.x; g < groups; g += blockDim.x) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float xh = __fmul_rn(row[lds_pad(8 * g + i)], inv_sqrt_n);
                row[lds_pad(8 * g + i)] = xh;
                sumsq = __fmaf_rn(xh, xh, sumsq);
                amax = fmaxf(amax, fabsf(xh));
            }
        }
        sumsq = wave_sum(sumsq);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1)
            amax = fmaxf(amax, __shfl_xor(amax, off, kWave));
        if ((threadIdx.x & (kWave - 1)) == 0) {
            partial[threadIdx.x / kWave] = sumsq;
            partial_max[threadIdx.x / kWave] = amax;
        }
        __syncthreads();
        float total = 0.0f, total_max = 0.0f;
#pragma unroll
        for (int w = 0; w < kGenericThreads / kWave; ++w) {
            total += partial[w];
            total_max = fmaxf(total_max, partial_max[w]);
        }
        const RowQuant q = mode == kQuantAbsMax ? row_quant_absmax(total_max, levels)
                           : mode == kQuantFp4  ? row_quant_fp4(total, cols, alpha, trust_edge)
                                                : row_quant(total, cols, levels, alpha, trust_edge);
        if (threadIdx.x == 0)
            scales[r] = q.scale;

        uint8_t *code_row = codes + r * ((int64_t)cols * cb / 8);
        for (int g = threadIdx.x; g < groups; g += blockDim.x) {
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v[i] = row[lds_pad(8 * g + i)];
            uint64_t packed = 0;
            uint32_t trusted = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t c = mode == kQuantFp4 ? (q.zero ? 0u : quantize_fp4(v[i], q))
                                   : q.zero         ? (uint32_t)(levels >> 1)
                                                    : quantize_one(v[i], q, levels);
                packed |= (uint64_t)c << (i * cb);
                trusted |= ((q.zero || fabsf(v[i]) <= q.trust_abs) ? 1u : 0u) << i;
            }
            switch (cb) {
            case 1: code_row[g] = (uint8_t)packed; break;
            case 2: reinterpret_cast<uint16_t *>(code_row)[g] = (uint16_t)packed; break;
            case 4: reinterpret_cast<uint32_t *>(code_row)[g] = (uint32_t)packed; break;
            default: reinterpret_cast<uint64_t *>(code_row)[g] = packed; break;
            }
            if (mask)
                mask[r * (int64_t)(cols >> 3) + g] = (uint8_t)trusted;
            if (xh_out)
                store8(xh_out + r * (int64_t)cols + 8 * g, v);
        }
        __syncthreads();  // the row buffer and `partial` are reused by the next row
    }
}



}  // namespace

// the longest row the entry points accept, as padded fp32
constexpr int kGenericMaxLds = (QUEST_MAX_COLS + (QUEST_MAX_COLS >> 5) + 1) * (int)sizeof(float);

hipError_t prepare_quantize_kernels()
{
    hipError_t err = allow_dynamic_lds(reinterpret_cast<const void *>(hq_generic_kernel<uint16_t>), kGenericMaxLds);
    if (err == hipSuccess)
        err = allow_dynamic_lds(reinterpret_cast<const void *>(hq_generic_kernel<float>), kGenericMaxLds);
    return err;
}

hipError_t launch_hadamard_quantize(const QuantizeArgs &a, hipStream_t stream)
{
    if (a.rows2 != 0) {
        // two operands: one launch where the matrix-core kernel covers the shape, else one after the other
        if (a.rows != 0 && launch_hadamard_quantize_mfma(a, stream))
            return hipGetLastError();
        QuantizeArgs first = a, second = a;
        first.x2 = nullptr;
        first.rows2 = 0;
        second.x = a.x2;
        second.rows = a.rows2;
        second.ld = a.ld2;
        second.codes = a.codes2;
        second.scales = a.scales2;
        second.mask = a.mask2;
        second.xh_out = nullptr;
        second.x2 = nullptr;
        second.rows2 = 0;
        const hipError_t err = launch_hadamard_quantize(first, stream);
        return err != hipSuccess ? err : launch_hadamard_quantize(second, stream);
    }
    if (a.rows == 0)
        return hipSuccess;
    if (launch_hadamard_quantize_mfma(a, stream))
        return hipGetLastError();
    const int cols = (int)a.cols;
    const size_t lds_bytes = (size_t)(cols + (cols >> 5) + 1) * sizeof(float);
    const int64_t max_blocks = 256 * 8;
    const dim3 grid((unsigned)(a.rows < max_blocks ? a.rows : max_blocks));
    const dim3 block(kGenericThreads);
    hipError_t err = hipSuccess;
    if (a.dtype == QUEST_BF16) {
        auto kernel = hq_generic_kernel<uint16_t>;
        if (lds_bytes > 48 * 1024)
            err = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), (int)lds_bytes);
        if (err != hipSuccess)
            return err;
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream,
                           static_cast<const uint16_t *>(a.x), a.rows, cols, a.ld, a.log2n, a.bits,
                           a.cb, a.alpha, a.trust_edge, a.mode, a.codes, a.scales, a.mask, a.xh_out);
    } else {
        auto kernel = hq_generic_kernel<float>;
        if (lds_bytes > 48 * 1024)
            err = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), (int)lds_bytes);
        if (err != hipSuccess)
            return err;
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream,
                           static_cast<const float *>(a.x), a.rows, cols, a.ld, a.log2n, a.bits,
                           a.cb, a.alpha, a.trust_edge, a.mode, a.codes, a.scales, a.mask, a.xh_out);
    }
    return hipGetLastError();
}

}  // namespace quest
