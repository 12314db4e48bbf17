// Fused block-Hadamard transform + RMS + clip/round + pack + trust mask (Algorithm 1, one operand;
// Sec. 3.1 and 3.2 of arXiv 2502.05003).  One pass over the operand: each row is read once from
// HBM, transformed on chip, and only the packed codes, the per-row scale and the mask bitmap are
// written back.
#include "quest_device.h"
#include "quest_internal.h"

namespace quest {
namespace {

constexpr int kGenericThreads = 256;

// Per-row constants of the projection, all in fp32 (the precision the codes are decided in).
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
    const float rms = __fsqrt_rn(__fdiv_rn(sumsq, (float)cols));
    const float clip = __fmul_rn(alpha, rms);
    q.zero = !(rms > 0.0f);
    q.inv_step = q.zero ? 0.0f : __fdiv_rn((float)(levels - 1), __fmul_rn(2.0f, clip));
    q.trust_abs = __fmul_rn(trust_edge, rms);
    q.scale = __fdiv_rn(clip, (float)(levels - 1));
    return q;
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
    float alpha, float trust_edge, uint8_t *__restrict__ codes, float *__restrict__ scales,
    uint8_t *__restrict__ mask, float *__restrict__ xh_out)
{
    extern __shared__ float lds[];
    float *row = lds;
    __shared__ float partial[kGenericThreads / kWave];

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

        // x_h = raw / sqrt(n); row sum of squares
        float sumsq = 0.0f;
        for (int g = threadIdx.x; g < groups; g += blockDim.x) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float xh = __fmul_rn(row[lds_pad(8 * g + i)], inv_sqrt_n);
                row[lds_pad(8 * g + i)] = xh;
                sumsq = __fmaf_rn(xh, xh, sumsq);
            }
        }
        sumsq = wave_sum(sumsq);
        if ((threadIdx.x & (kWave - 1)) == 0)
            partial[threadIdx.x / kWave] = sumsq;
        __syncthreads();
        float total = 0.0f;
#pragma unroll
        for (int w = 0; w < kGenericThreads / kWave; ++w)
            total += partial[w];
        const RowQuant q = row_quant(total, cols, levels, alpha, trust_edge);
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
                const uint32_t c = q.zero ? (uint32_t)(levels >> 1) : quantize_one(v[i], q, levels);
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


// ------------------------------------------------------------------------------------------
// Matrix-core assisted kernel for bf16 rows of 512 * HT elements (HT <= 11), 4-bit containers.
//
// One wavefront owns one row at a time.  The row is cut into tiles of 1024 elements seen as
// 32 x 32 matrices X[p][q] (element 32 p + q).  Index bits 0..4 (q) are transformed by one
// 32x32x32 bf16 MFMA product X . H_32 per tile: the inputs are bf16 and the matrix is +-1, so
// every product is exact and the fp32 accumulation is the only rounding, as in a butterfly.
// This takes five of the eleven stages off the vector ALU, which would otherwise bound the
// kernel (about 18 fp32 ops per element against 2.6 bytes per element).  The remaining
// stages run on the fp32 accumulators in registers:
//   after the MFMA lane (l & 31) holds q' (bits 0..4), l >> 5 = h holds bit 7 and register r
//   holds p = 8 (r >> 2) + 4 h + (r & 3), i.e. bits 5, 6 in r & 3 and bits 8, 9 in r >> 2;
//   bit 7 is brought into registers by one half-wave swap (h then holds bit 5);
//   bits >= 10 pair whole tiles.
// Codes and mask bits are produced in that register order, packed per lane, transposed across
// lanes (8 x 8 nibbles, 32 x 32 bits) through the LDS crossbar, and stored as coalesced dwords
// in natural element order.
// ------------------------------------------------------------------------------------------

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kMfmaThreads = 256;

// in-lane element index iota = b6 + 2 b7 + 4 b8 + 8 b9 + 16 tile  ->  accumulator register in
// its tile (after the half-wave swap: b7 = r & 1, b6 = (r >> 1) & 1, b8 = (r >> 2) & 1, b9 = r >> 3)
__host__ __device__ constexpr int reg_of_iota(int iota)
{
    return ((iota >> 1) & 1) | ((iota & 1) << 1) | (((iota >> 2) & 1) << 2) | (((iota >> 3) & 1) << 3);
}

__device__ __forceinline__ void bfly(float &a, float &b)
{
    const float t = a;
    a = t + b;
    b = t - b;
}

__device__ __forceinline__ uint32_t swizzle_xor(uint32_t v, int lane_xor)
{
    switch (lane_xor) {
    case 1: return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, (1 << 10) | 0x1f);
    case 2: return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, (2 << 10) | 0x1f);
    case 4: return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, (4 << 10) | 0x1f);
    case 8: return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, (8 << 10) | 0x1f);
    default: return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, (16 << 10) | 0x1f);
    }
}

// Transpose a STAGES-bit lane index against a STAGES-bit field index inside each dword:
// fields are (32 >> STAGES... ) no: fields are FIELD bits wide; after the call, field i of
// lane a holds what field a of lane i held (lanes taken modulo 2^STAGES within their group).
template <int STAGES, int FIELD>
__device__ __forceinline__ uint32_t lane_field_transpose(uint32_t d, int lane)
{
#pragma unroll
    for (int s = 0; s < STAGES; ++s) {
        const int sh = FIELD << s;
        // positions whose field-index bit s is 0
        uint32_t lo = 0;
#pragma unroll
        for (int f = 0; f < (1 << STAGES); ++f)
            if (((f >> s) & 1) == 0)
                lo |= ((FIELD == 32 ? 0xffffffffu : ((1u << FIELD) - 1u)) << (f * FIELD));
        const bool up = (lane >> s) & 1;
        const uint32_t keep = up ? ~lo : lo;
        const uint32_t partner = swizzle_xor(d, 1 << s);
        const uint32_t rotated = __builtin_amdgcn_alignbit(partner, partner, up ? sh : 32 - sh);
        d = (keep & d) | (~keep & rotated);
    }
    return d;
}

template <int HT>
__global__ __launch_bounds__(kMfmaThreads) void hq_mfma_kernel(
    const uint16_t *__restrict__ x, int64_t rows, int64_t ld, int log2n, int bits, float alpha,
    float trust_edge, uint8_t *__restrict__ codes, float *__restrict__ scales,
    uint8_t *__restrict__ mask, float *__restrict__ xh_out)
{
    constexpr int T = (HT + 1) / 2;        // tiles of 1024 elements; the last one may be half
    constexpr int NI = 8 * HT;             // elements per lane
    constexpr int cols = 512 * HT;
    constexpr bool kHalfTail = (HT & 1) != 0;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, h = lane >> 5;
    const int levels = 1 << bits;

    // B operand: rows q = 16 h + 8 s + e of I (x) H_min(n,32), column q' = m, as bf16 +-1 / 0
    v8bf bmat[2];
    {
        const int nb = log2n < 5 ? log2n : 5;
        const int low = (1 << nb) - 1;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int q = 16 * h + 8 * s + e;
                uint32_t v = 0;
                if ((q >> nb) == (m >> nb))
                    v = (__builtin_popcount(q & m & low) & 1) ? 0xBF80u : 0x3F80u;
                if (e & 1)
                    w[e >> 1] |= v << 16;
                else
                    w[e >> 1] = v;
            }
            __builtin_memcpy(&bmat[s], w, 16);
        }
    }
    const float inv_sqrt_n = (log2n & 1) ? 0.70710678118654752440f / (float)(1 << (log2n >> 1))
                                         : 1.0f / (float)(1 << (log2n >> 1));
    const float sqrt_n = (log2n & 1) ? 1.41421356237309504880f * (float)(1 << (log2n >> 1))
                                     : (float)(1 << (log2n >> 1));

    for (int64_t row = (int64_t)blockIdx.x * (kMfmaThreads / 64) + wave; row < rows;
         row += (int64_t)gridDim.x * (kMfmaThreads / 64)) {
        const uint16_t *src = x + row * ld + 32 * m + 16 * h;
        float acc[T][16];
        float sumsq = 0.0f;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            uint4 a0 = make_uint4(0, 0, 0, 0), a1 = make_uint4(0, 0, 0, 0);
            if (!(kHalfTail && t == T - 1) || m < 16) {
                a0 = *reinterpret_cast<const uint4 *>(src + 1024 * t);
                a1 = *reinterpret_cast<const uint4 *>(src + 1024 * t + 8);
            }
            const uint32_t w[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                v2bf pair;
                __builtin_memcpy(&pair, &w[i], 4);
                sumsq = __builtin_amdgcn_fdot2_f32_bf16(pair, pair, sumsq, false);
            }
            v8bf f0, f1;
            __builtin_memcpy(&f0, &a0, 16);
            __builtin_memcpy(&f1, &a1, 16);
            v16f z;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                z[r] = 0.0f;
            z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0, bmat[0], z, 0, 0, 0);
            z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1, bmat[1], z, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[t][r] = z[r];
        }
        // The block transform is orthonormal, so the row sum of squares of x_h equals that of x.
        sumsq = wave_sum(sumsq);

        // stages on bits 5 and 6 (register bits 0 and 1)
        if (log2n > 5) {
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int r = 0; r < 16; r += 2)
                    bfly(acc[t][r], acc[t][r + 1]);
        }
        if (log2n > 6) {
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (!(r & 2))
                        bfly(acc[t][r], acc[t][r + 2]);
        }
        // bit 7 lives in the half-wave index: swap it with register bit 0, then it is in registers
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[t][r]),
                                                                 __float_as_uint(acc[t][r + 1]),
                                                                 false, false);
                acc[t][r] = __uint_as_float(sw[0]);
                acc[t][r + 1] = __uint_as_float(sw[1]);
            }
        if (log2n > 7) {
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int r = 0; r < 16; r += 2)
                    bfly(acc[t][r], acc[t][r + 1]);
        }
        if (log2n > 8) {
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (!(r & 4))
                        bfly(acc[t][r], acc[t][r + 4]);
        }
        if (log2n > 9) {
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int r = 0; r < 8; ++r)
                    bfly(acc[t][r], acc[t][r + 8]);
        }
#pragma unroll
        for (int k = 0; (1 << k) < T; ++k) {
            if (log2n > 10 + k) {
#pragma unroll
                for (int t = 0; t < T; ++t)
                    if (!(t & (1 << k)) && (t | (1 << k)) < T) {
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            bfly(acc[t][r], acc[t | (1 << k)][r]);
                    }
            }
        }

        // per-row constants, in the un-normalised ("raw") domain: x_h = raw / sqrt(n)
        const RowQuant q = row_quant(sumsq, cols, levels, alpha, trust_edge);
        const float raw_to_cell = __fmul_rn(q.inv_step, inv_sqrt_n);
        const float trust_raw = __fmul_rn(q.trust_abs, sqrt_n);
        if (lane == 0)
            scales[row] = q.scale;

        if (xh_out) {
            float *dst = xh_out + row * cols + lane;   // element = lane + 64 iota
#pragma unroll
            for (int i = 0; i < NI; ++i)
                dst[64 * i] = __fmul_rn(acc[i >> 4][reg_of_iota(i & 15)], inv_sqrt_n);
        }

        // codes: eight per dword in iota order, then an 8 x 8 nibble transpose across lanes
        uint32_t *code_row = reinterpret_cast<uint32_t *>(codes + row * (cols / 2));
        const int code_word = ((lane >> 3) & 3) + 4 * h + 8 * (lane & 7);
#pragma unroll
        for (int d = 0; d < HT; ++d) {
            uint32_t packed;
            if (bits == 4) {
                // byte = sat_u8(rne(16 cell + 128 - 1/2)): its high nibble is clamp(floor(cell) + 8, 0, 15)
                const float s16 = __fmul_rn(raw_to_cell, 16.0f);
                uint32_t even = 0, odd = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float v = acc[(8 * d + i) >> 4][reg_of_iota((8 * d + i) & 15)];
                    const float t = __fmaf_rn(v, s16, 127.5f);
                    if (i & 1)
                        odd = __builtin_amdgcn_cvt_pk_u8_f32(t, i >> 1, odd);
                    else
                        even = __builtin_amdgcn_cvt_pk_u8_f32(t, i >> 1, even);
                }
                packed = ((even >> 4) & 0x0f0f0f0fu) | (odd & 0xf0f0f0f0u);
            } else {
                const float half = (float)(levels >> 1);
                packed = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float v = acc[(8 * d + i) >> 4][reg_of_iota((8 * d + i) & 15)];
                    const float t = fmaxf(__fmaf_rn(v, raw_to_cell, half), 0.0f);
                    const uint32_t c = min((uint32_t)t, (uint32_t)(levels - 1));
                    packed |= c << (4 * i);
                }
            }
            packed = lane_field_transpose<3, 4>(packed, lane);
            code_row[code_word + 64 * d] = packed;
        }

        // trust mask: one bit per element in iota order, then a 32 x 32 bit transpose across lanes
        if (mask) {
            uint32_t *mask_row = reinterpret_cast<uint32_t *>(mask + row * (cols / 8));
#pragma unroll
            for (int c = 0; c * 32 < NI; ++c) {
                const int count = (NI - 32 * c) < 32 ? (NI - 32 * c) : 32;
                uint32_t untrusted = 0;
#pragma unroll
                for (int i = count - 1; i >= 0; --i) {
                    const float v = acc[(32 * c + i) >> 4][reg_of_iota((32 * c + i) & 15)];
                    const float slack = trust_raw - fabsf(v);          // negative <=> untrusted
                    untrusted = __builtin_amdgcn_alignbit(untrusted, __float_as_uint(slack), 31);
                }
                uint32_t trusted = ~untrusted;
                if (count < 32)
                    trusted &= (1u << count) - 1u;
                trusted = lane_field_transpose<5, 1>(trusted, lane);
                if (m < count)
                    mask_row[h + 2 * (m + 32 * c)] = trusted;
            }
        }
    }
}

template <int HT>
void launch_mfma(const QuantizeArgs &a, hipStream_t stream)
{
    const int64_t blocks_needed = (a.rows + 3) / 4;
    const int64_t max_blocks = 256 * 8;
    const dim3 grid((unsigned)(blocks_needed < max_blocks ? blocks_needed : max_blocks));
    hipLaunchKernelGGL(hq_mfma_kernel<HT>, grid, dim3(kMfmaThreads), 0, stream,
                       static_cast<const uint16_t *>(a.x), a.rows, a.ld, a.log2n, a.bits, a.alpha,
                       a.trust_edge, a.codes, a.scales, a.mask, a.xh_out);
}

// true if the matrix-core kernel covers this call
bool mfma_path_applies(const QuantizeArgs &a)
{
    if (a.dtype != QUEST_BF16 || a.cb != 4 || (a.cols % 512) != 0)
        return false;
    const int ht = (int)(a.cols / 512);
    if (!(ht == 1 || ht == 2 || ht == 4 || ht == 8 || ht == 11))
        return false;
    // blocks above 1024 pair whole tiles, so they must cover a power-of-two number of them
    return (int64_t(1) << a.log2n) <= a.cols;
}

}  // namespace

hipError_t launch_hadamard_quantize(const QuantizeArgs &a, hipStream_t stream)
{
    if (a.rows == 0)
        return hipSuccess;
    if (mfma_path_applies(a)) {
        switch ((int)(a.cols / 512)) {
        case 1: launch_mfma<1>(a, stream); break;
        case 2: launch_mfma<2>(a, stream); break;
        case 4: launch_mfma<4>(a, stream); break;
        case 8: launch_mfma<8>(a, stream); break;
        default: launch_mfma<11>(a, stream); break;
        }
        return hipGetLastError();
    }
    const int cols = (int)a.cols;
    const size_t lds_bytes = (size_t)(cols + (cols >> 5) + 1) * sizeof(float);
    const int64_t max_blocks = 256 * 8;
    const dim3 grid((unsigned)(a.rows < max_blocks ? a.rows : max_blocks));
    const dim3 block(kGenericThreads);
    hipError_t err = hipSuccess;
    if (a.dtype == QUEST_BF16) {
        auto kernel = hq_generic_kernel<uint16_t>;
        if (lds_bytes > 48 * 1024)
            err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (err != hipSuccess)
            return err;
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream,
                           static_cast<const uint16_t *>(a.x), a.rows, cols, a.ld, a.log2n, a.bits,
                           a.cb, a.alpha, a.trust_edge, a.codes, a.scales, a.mask, a.xh_out);
    } else {
        auto kernel = hq_generic_kernel<float>;
        if (lds_bytes > 48 * 1024)
            err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (err != hipSuccess)
            return err;
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream,
                           static_cast<const float *>(a.x), a.rows, cols, a.ld, a.log2n, a.bits,
                           a.cb, a.alpha, a.trust_edge, a.codes, a.scales, a.mask, a.xh_out);
    }
    return hipGetLastError();
}

}  // namespace quest
