// Pieces shared by the tile matmul kernels on packed codes (INT8 and FP4 matrix instructions).
#pragma once

#include <type_traits>
#include <utility>

#include "quest_device.h"

namespace quest {

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

// two floats -> packed bf16 pair (round to nearest even), low half = first
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    v2bf p;
    p[0] = (__bf16)lo;
    p[1] = (__bf16)hi;
    uint32_t u;
    __builtin_memcpy(&u, &p, 4);
    return u;
}

// Epilogue shared by the tile kernels.  Each 32 x 32 accumulator tile is the transpose of an output
// tile: lane l holds output row l % 32 and, in register r, output column 8 (r / 4) + 4 (l / 32) +
// r % 4, i.e. runs of four consecutive columns.  A wave owns a block of 32 AF rows by 64 columns at
// (row0, col0): it writes the raw accumulators if asked to, converts the block to bf16
// (float(acc) * s_a, then * s_b), parks it in its own LDS (128-byte rows, 16-byte chunks swizzled
// by row) and writes it out as 128-byte row segments.  Integer accumulators carry a factor 2^CARRY
// (sa_reg already holds s_a / 2^CARRY); fp32 accumulators (the FP4 kernel) have CARRY = 0.  Every
// wave of the workgroup must be done with the LDS that `park` points into.
template <int AF, int CARRY, typename Vec, typename Raw>
__device__ __forceinline__ void store_wave_block(const Vec (&acc)[AF][2], const float (&sa_reg)[AF],
                                                 const float *scale_lds_wave, uint8_t *park, int row0, int col0,
                                                 int M, int N, uint16_t *__restrict__ y, int64_t ld_y,
                                                 Raw *__restrict__ acc_out, int lane)
{
    constexpr bool kInteger = std::is_integral<Raw>::value;
    const int lm = lane & 31, lh = lane >> 5;
    if (acc_out) {
#pragma unroll
        for (int i = 0; i < AF; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = row0 + i * 32 + lm;
                    const int n = col0 + j * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                    if (m < M && n < N) {
                        if constexpr (kInteger)
                            acc_out[(int64_t)m * N + n] = acc[i][j][r] >> CARRY;   // exact: a multiple of 2^CARRY
                        else
                            acc_out[(int64_t)m * N + n] = acc[i][j][r];
                    }
                }
    }
    if (!y)
        return;
    // the weight scales of this lane's columns, read once (the park writes below would otherwise keep
    // the compiler from re-using them across the row blocks)
    float4 sb_reg[2][4];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            sb_reg[j][q] = *reinterpret_cast<const float4 *>(scale_lds_wave + j * 32 + 8 * q + 4 * lh);
#pragma unroll
    for (int i = 0; i < AF; ++i) {
        const int row = i * 32 + lm;   // row within the wave's block
        const float sa = sa_reg[i];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = j * 32 + 8 * q + 4 * lh;   // first of four consecutive columns
                const float4 sb = sb_reg[j][q];
                const float v0 = __fmul_rn(__fmul_rn((float)acc[i][j][4 * q + 0], sa), sb.x);
                const float v1 = __fmul_rn(__fmul_rn((float)acc[i][j][4 * q + 1], sa), sb.y);
                const float v2 = __fmul_rn(__fmul_rn((float)acc[i][j][4 * q + 2], sa), sb.z);
                const float v3 = __fmul_rn(__fmul_rn((float)acc[i][j][4 * q + 3], sa), sb.w);
                const int chunk = (col >> 3) ^ (row & 7);
                *reinterpret_cast<uint2 *>(park + row * 128 + chunk * 16 + (col & 4) * 2) =
                    make_uint2(pack_bf16(v0, v1), pack_bf16(v2, v3));
            }
        }
    }
    // each pass: 8 rows of 128 bytes, lane l takes 16-byte chunk l % 8 of row l / 8
    uint16_t *y_base = y + (int64_t)row0 * ld_y + col0;
    const bool vector_ok = ((ld_y & 7) == 0) && ((reinterpret_cast<uintptr_t>(y) & 15) == 0) && (col0 + 64 <= N);
#pragma unroll 4
    for (int pass = 0; pass < 4 * AF; ++pass) {
        const int row = pass * 8 + (lane >> 3);
        const int c = lane & 7;
        const uint4 v = *reinterpret_cast<const uint4 *>(park + row * 128 + ((c ^ (row & 7)) << 4));
        if (row0 + row >= M)
            continue;
        uint16_t *dst = y_base + (int64_t)row * ld_y + c * 8;
        if (vector_ok) {
            *reinterpret_cast<uint4 *>(dst) = v;
        } else {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (col0 + c * 8 + e < N)
                    dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
        }
    }
}

}  // namespace quest
