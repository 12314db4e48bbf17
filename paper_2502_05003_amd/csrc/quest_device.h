// Device-side helpers shared by the QuEST HIP kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace quest {

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16)
{
    return __uint_as_float(bits16 << 16);
}

// Round-to-nearest-even float -> bf16 bits (NaN kept quiet).
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Eight consecutive row elements widened to fp32.  The pointer must be 16-byte aligned.
__device__ __forceinline__ void load8(const float *p, float (&v)[8])
{
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

__device__ __forceinline__ void load8(const uint16_t *p, float (&v)[8])
{
    const uint4 w = *reinterpret_cast<const uint4 *>(p);
    v[0] = __uint_as_float(w.x << 16); v[1] = __uint_as_float(w.x & 0xffff0000u);
    v[2] = __uint_as_float(w.y << 16); v[3] = __uint_as_float(w.y & 0xffff0000u);
    v[4] = __uint_as_float(w.z << 16); v[5] = __uint_as_float(w.z & 0xffff0000u);
    v[6] = __uint_as_float(w.w << 16); v[7] = __uint_as_float(w.w & 0xffff0000u);
}

__device__ __forceinline__ void store8(float *p, const float (&v)[8])
{
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}

__device__ __forceinline__ void store8(uint16_t *p, const float (&v)[8])
{
    uint4 w;
    w.x = float_to_bf16_bits(v[0]) | (float_to_bf16_bits(v[1]) << 16);
    w.y = float_to_bf16_bits(v[2]) | (float_to_bf16_bits(v[3]) << 16);
    w.z = float_to_bf16_bits(v[4]) | (float_to_bf16_bits(v[5]) << 16);
    w.w = float_to_bf16_bits(v[6]) | (float_to_bf16_bits(v[7]) << 16);
    *reinterpret_cast<uint4 *>(p) = w;
}

// Un-normalised Sylvester butterflies over the low `STAGES` index bits of a 2^STAGES register
// array: after the call v[i] = sum_j (-1)^popcount(i & j) v_in[j].
template <int STAGES>
__device__ __forceinline__ void butterflies(float (&v)[1 << STAGES])
{
#pragma unroll
    for (int s = 0; s < STAGES; ++s) {
        const int h = 1 << s;
#pragma unroll
        for (int i = 0; i < (1 << STAGES); ++i) {
            if ((i & h) == 0) {
                const float a = v[i], b = v[i + h];
                v[i] = a + b;
                v[i + h] = a - b;
            }
        }
    }
}

// Same, for a runtime stage count 0..3 on an 8-element array (stages beyond `stages` skipped).
__device__ __forceinline__ void butterflies8(float (&v)[8], int stages)
{
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        if (s < stages) {
            const int h = 1 << s;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if ((i & h) == 0) {
                    const float a = v[i], b = v[i + h];
                    v[i] = a + b;
                    v[i + h] = a - b;
                }
            }
        }
    }
}

// LDS index with one pad word per 32 so that power-of-two strides spread over the banks.
__device__ __forceinline__ int lds_pad(int i)
{
    return i + (i >> 5);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        v += __shfl_xor(v, off, kWave);
    return v;
}

// Same sum through the data-parallel-primitive lane patterns (no LDS crossbar, no address
// arithmetic): within quads, within rows of sixteen lanes by the two mirror patterns, then across the
// four rows by the two row broadcasts, after which lane 63 holds the total.  The result is
// wave-uniform.  The order of the additions differs from wave_sum's.
__device__ __forceinline__ float wave_sum_dpp(float v)
{
    auto moved = [](float x, auto ctrl, auto row_mask) {
        constexpr int kCtrl = decltype(ctrl)::value, kRows = decltype(row_mask)::value;
        return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(x), kCtrl, kRows, 0xF, false));
    };
    using std::integral_constant;
    v += moved(v, integral_constant<int, 0xB1>{}, integral_constant<int, 0xF>{});    // quad_perm [1, 0, 3, 2]
    v += moved(v, integral_constant<int, 0x4E>{}, integral_constant<int, 0xF>{});    // quad_perm [2, 3, 0, 1]
    v += moved(v, integral_constant<int, 0x141>{}, integral_constant<int, 0xF>{});   // row_half_mirror
    v += moved(v, integral_constant<int, 0x140>{}, integral_constant<int, 0xF>{});   // row_mirror
    v += moved(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{});   // row_bcast:15 into rows 1, 3
    v += moved(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{});   // row_bcast:31 into rows 2, 3
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(v), 63));
}

/*
 * Remaining butterfly stages (index bits 3 .. log2n-1) of one row held in LDS as padded fp32,
 * three bits per pass.  Bits 0..2 must already have been applied.  Every thread of the block
 * must call this; the row is consistent in LDS after the trailing barrier.
 */
__device__ __forceinline__ void lds_butterfly_passes(float *row, int cols, int log2n)
{
    for (int s = 3; s < log2n; s += 3) {
        const int r = (log2n - s) < 3 ? (log2n - s) : 3;
        const int groups = cols >> r;
        __syncthreads();
        for (int g = threadIdx.x; g < groups; g += blockDim.x) {
            const int base = ((g >> s) << (s + r)) | (g & ((1 << s) - 1));
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v[i] = (i < (1 << r)) ? row[lds_pad(base + (i << s))] : 0.0f;
            butterflies8(v, r);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (i < (1 << r))
                    row[lds_pad(base + (i << s))] = v[i];
        }
    }
    __syncthreads();
}

/*
 * 16 bytes per lane from global memory straight into LDS: lane l of the wave lands at
 * lds_base + 16 l.  lds_base is the wave-uniform LDS byte address.  Written as inline assembly so
 * that the compiler does not serialise the transfer against later LDS reads of other stages; the
 * caller orders it explicitly: wait_vmcnt<N>() (transfers complete in issue order) and a barrier
 * before any wave reads the destination.
 */
__device__ __forceinline__ void lds_dma16(const void *global_src, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(global_src), "s"(lds_base)
                 : "memory");
}

// Same, the source given as a wave-uniform base plus a per-lane unsigned 32-bit byte offset.
__device__ __forceinline__ void lds_dma16(const void *uniform_base, uint32_t lane_offset, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_offset), "s"(uniform_base), "s"(lds_base)
                 : "memory");
}

// Same, the LDS destination given as a wave-uniform base plus a compile-time byte offset: one
// scalar instruction writes M0 (the addition sets SCC, which is declared clobbered).
template <int LDS_IMM>
__device__ __forceinline__ void lds_dma16_at(const void *uniform_base, uint32_t lane_offset, uint32_t lds_base)
{
    static_assert(LDS_IMM >= 0, "byte offset into LDS");
    asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_offset), "s"(uniform_base), "s"(lds_base), "n"(LDS_IMM)
                 : "memory", "scc");
}

// LDS byte address of a pointer into shared memory
__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

// wait until at most N vector-memory operations of this wave are outstanding (N <= 63; the
// count's low four bits sit in bits 3:0 of the immediate, its high two in bits 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a six-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// ---- rows staged through LDS by the memory system (fused quantizer, trust backward) ----
// A wave requests its next row with global -> LDS transfers, which hold no registers while in flight,
// and goes on with the current row; when it comes back for the row, the vector-memory operations it
// has issued since (its stores) may still be outstanding, the transfers, issued before them, may not
// (a wave's vector-memory operations complete in issue order).  So the stores are issued by hand,
// counted, and the wait is for "all but that many".

// one streaming dword store per lane, as an instruction the compiler neither merges nor moves
__device__ __forceinline__ void store_word_counted(uint32_t *p, uint32_t v)
{
    asm volatile("global_store_dword %0, %1, off nt" : : "v"(p), "v"(v) : "memory");
}

// 16 bytes per lane from global memory straight into LDS (lane l lands at lds_base + 16 l), streaming
// (the input is read once).  Source = wave-uniform base + per-lane byte offset.
__device__ __forceinline__ void lds_dma16_stream(const void *uniform_base, uint32_t lane_offset, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :
                 : "v"(lane_offset), "s"(uniform_base), "s"(lds_base)
                 : "memory");
}

// wait until at most n (0 .. 24; larger values wait as for 24) vector-memory operations are outstanding
__device__ __forceinline__ void wait_vmcnt_upto(int n)
{
    switch (n) {
#define QUEST_WAIT_CASE(N) case N: wait_vmcnt<N>(); break;
    QUEST_WAIT_CASE(0) QUEST_WAIT_CASE(1) QUEST_WAIT_CASE(2) QUEST_WAIT_CASE(3) QUEST_WAIT_CASE(4)
    QUEST_WAIT_CASE(5) QUEST_WAIT_CASE(6) QUEST_WAIT_CASE(7) QUEST_WAIT_CASE(8) QUEST_WAIT_CASE(9)
    QUEST_WAIT_CASE(10) QUEST_WAIT_CASE(11) QUEST_WAIT_CASE(12) QUEST_WAIT_CASE(13) QUEST_WAIT_CASE(14)
    QUEST_WAIT_CASE(15) QUEST_WAIT_CASE(16) QUEST_WAIT_CASE(17) QUEST_WAIT_CASE(18) QUEST_WAIT_CASE(19)
    QUEST_WAIT_CASE(20) QUEST_WAIT_CASE(21) QUEST_WAIT_CASE(22) QUEST_WAIT_CASE(23)
#undef QUEST_WAIT_CASE
    default: wait_vmcnt<24>(); break;
    }
    asm volatile("" ::: "memory");   // the compiler keeps later LDS reads behind the wait
}

// 4 bytes per lane (lane l lands at lds_base + 4 l), streaming
__device__ __forceinline__ void lds_dma4_stream(const void *uniform_base, uint32_t lane_offset, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1 nt"
                 :
                 : "v"(lane_offset), "s"(uniform_base), "s"(lds_base)
                 : "memory");
}

}  // namespace quest
