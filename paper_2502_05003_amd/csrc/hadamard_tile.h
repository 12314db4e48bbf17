// Pieces shared by the two matrix-core Hadamard kernels (the fused quantizer and the trust-masked
// inverse transform): a row is cut into tiles of 1024 elements seen as 32 x 32 matrices X[p][q]
// (element 32 p + q).  Index bits 0..4 (q) go through one exact +-1 MFMA product per tile, after
// which lane (m = l & 31, h = l >> 5) holds column q' = m and register r holds
// p = 8 (r >> 2) + 4 h + (r & 3); the other stages run on those registers.
#pragma once

#include "quest_device.h"

namespace quest {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// In-lane element index iota = b6 + 2 b7 + 4 b8 + 8 b9 + 16 tile (bN = index bit N of the
// element) -> accumulator register within its tile, after the half-wave swap:
// b7 = r & 1, b6 = (r >> 1) & 1, b8 = (r >> 2) & 1, b9 = r >> 3.
__host__ __device__ constexpr int reg_of_iota(int iota)
{
    return ((iota >> 1) & 1) | ((iota & 1) << 1) | (((iota >> 2) & 1) << 2) |
           (((iota >> 3) & 1) << 3);
}

__device__ __forceinline__ void bfly(float &a, float &b)
{
    const float t = a;
    a = t + b;
    b = t - b;
}

// B operand of the tile product D = X . (I (x) H_min(n,32)): rows q = 16 h + 8 s + e (s = which of
// the two 32 x 32 x 16 instructions, e = element) of that matrix, column q' = m, as bf16 +-1 / 0.
// FULL: the block is at least 32 wide, every entry is +-1: the signs of eight consecutive rows are
// parity(base & m) ^ parity(e & m), the second factor one of eight byte patterns.
template <bool FULL>
__device__ __forceinline__ void hadamard_operand(int log2n, int m, int h, v8bf (&bmat)[2])
{
    if constexpr (FULL) {
        const uint32_t pattern = ((m & 1) ? 0xAAu : 0u) ^ ((m & 2) ? 0xCCu : 0u) ^ ((m & 4) ? 0xF0u : 0u);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int base = 16 * h + 8 * s;
            const uint32_t minus = (__builtin_popcount(base & m) & 1) ? pattern ^ 0xFFu : pattern;   // bit e: entry is -1
            uint32_t w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                w[k] = 0x3F803F80u | ((minus << (15 - 2 * k)) & 0x8000u) | ((minus << (30 - 2 * k)) & 0x80000000u);
            __builtin_memcpy(&bmat[s], w, 16);
        }
        return;
    }
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

// 1 / sqrt(n) and sqrt(n), correctly rounded: powers of two, times sqrt(2) for odd log2(n).
__device__ __forceinline__ float inv_sqrt_pow2(int log2n)
{
    return (log2n & 1) ? 0.70710678118654752440f / (float)(1 << (log2n >> 1)) : 1.0f / (float)(1 << (log2n >> 1));
}

__device__ __forceinline__ float sqrt_pow2(int log2n)
{
    return (log2n & 1) ? 1.41421356237309504880f * (float)(1 << (log2n >> 1)) : (float)(1 << (log2n >> 1));
}

// The stages on index bits 5 .. LOG2N - 1 of G tiles held as MFMA accumulators: bits 5, 6, 8, 9 are
// register-to-register, bit 7 is the half-wave index and is swapped with register bit 0 first
// (after which h holds bit 5; the swap is made for every block size so that the element order of
// the registers does not depend on it), bits >= 10 pair whole tiles.  PAIRED: the stage on bit 10
// (tile 2 j with tile 2 j + 1) has already been applied by the caller.
template <int LOG2N, int G, bool PAIRED = false>
__device__ __forceinline__ void tile_stages(float (&acc)[G][16])
{
    if (LOG2N > 5) {  // bit 5 = register bit 0
#pragma unroll
        for (int u = 0; u < G; ++u)
#pragma unroll
            for (int r = 0; r < 16; r += 2)
                bfly(acc[u][r], acc[u][r + 1]);
    }
    if (LOG2N > 6) {  // bit 6 = register bit 1
#pragma unroll
        for (int u = 0; u < G; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (!(r & 2))
                    bfly(acc[u][r], acc[u][r + 2]);
    }
#pragma unroll
    for (int u = 0; u < G; ++u)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[u][r]),
                                                             __float_as_uint(acc[u][r + 1]), false, false);
            acc[u][r] = __uint_as_float(sw[0]);
            acc[u][r + 1] = __uint_as_float(sw[1]);
        }
    if (LOG2N > 7) {
#pragma unroll
        for (int u = 0; u < G; ++u)
#pragma unroll
            for (int r = 0; r < 16; r += 2)
                bfly(acc[u][r], acc[u][r + 1]);
    }
    if (LOG2N > 8) {  // bit 8 = register bit 2
#pragma unroll
        for (int u = 0; u < G; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (!(r & 4))
                    bfly(acc[u][r], acc[u][r + 4]);
    }
    if (LOG2N > 9) {  // bit 9 = register bit 3
#pragma unroll
        for (int u = 0; u < G; ++u)
#pragma unroll
            for (int r = 0; r < 8; ++r)
                bfly(acc[u][r], acc[u][r + 8]);
    }
#pragma unroll
    for (int k = PAIRED ? 1 : 0; (1 << k) < G; ++k) {  // bits >= 10 pair whole tiles
        if (LOG2N > 10 + k) {
#pragma unroll
            for (int u = 0; u < G; ++u)
                if (!(u & (1 << k)) && (u | (1 << k)) < G) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        bfly(acc[u][r], acc[u | (1 << k)][r]);
                }
        }
    }
}

}  // namespace quest
