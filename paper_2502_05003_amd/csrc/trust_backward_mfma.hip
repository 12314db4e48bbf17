// Matrix-core assisted trust-masked inverse Hadamard transform, bf16 in, bf16 or fp32 out (Algorithm 2,
// out = IHT(M (.) g); Sec. 3.2 of arXiv 2502.05003).  Same data flow as the fused quantizer
// (hadamard_quantize_mfma.hip), which see for the index bookkeeping:
//   * one wavefront per row of 128 * U elements, tiles of 1024 elements seen as 32 x 32 matrices;
//     lane (m = l & 31, h = l >> 5) loads the 32 contiguous bytes of tile row m holding columns
//     16 h .. 16 h + 15 together with their 16 mask bits, and zeroes the untrusted bf16 values;
//   * index bits 0..4 are transformed by one exact +-1 bf16 MFMA product per tile, the other stages
//     run on the fp32 accumulators in registers (bit 7 through one half-wave swap);
//   * afterwards lane l & 31 holds index bits 0..4, l >> 5 bit 5, and the in-lane index iota the
//     bits from 6 up; values are scaled by 1 / sqrt(n), rounded to bf16 in pairs (iota, iota + 1),
//     and one exchange with the neighbouring lane turns those into pairs of adjacent elements, so
//     that a wave stores 256 contiguous bytes per instruction;
//   * fp32 outputs are stored as they are, 64 consecutive floats per wave instruction;
//   * rows made of whole 1 KiB pieces, up to 4096 elements, come in through LDS one row ahead, with
//     their mask bytes behind them (see the quantizer): the next row's memory latency runs under
//     this row's arithmetic and stores.
#include "hadamard_tile.h"
#include "quest_internal.h"

namespace quest {
namespace {

typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int kMaxBlocks = 1024;   // four workgroups of four waves per compute unit, each wave walking over its rows
constexpr int kThreads = 256;
constexpr int kRowsPerBlock = kThreads / 64;

__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi)
{
    v2bf p;
    p[0] = (__bf16)lo;
    p[1] = (__bf16)hi;
    uint32_t u;
    __builtin_memcpy(&u, &p, 4);
    return u;
}

// zero the halves of `pair` whose mask bits (bit 0: low half, bit 1: high half) are clear
__device__ __forceinline__ uint32_t keep_trusted(uint32_t pair, uint32_t mask_bits, int first_bit)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_sbfe((int)mask_bits, first_bit, 1);      // 0 or ~0
    const uint32_t hi = (uint32_t)__builtin_amdgcn_sbfe((int)mask_bits, first_bit + 1, 1);
    return pair & __builtin_amdgcn_perm(hi, lo, 0x07060100u);   // low half from lo, high half from hi
}

// Rows of whole 1 KiB pieces, at most 4096 elements (four workgroups' buffers fit a CU's LDS), and few
// enough stores per row and lane for the wait on the vector-memory counter to tell them from the
// transfers (the counter has six bits).
constexpr bool tb_rows_through_lds(int u, bool f32_out)
{
    return (u % 8) == 0 && u <= 32 && (f32_out ? 4 * u : 2 * u) / 2 <= 48;
}
// LDS per wave: the row, then its mask bytes rounded up to whole 256-byte transfers
constexpr int tb_wave_buffer_bytes(int u)
{
    return 256 * u + 256 * ((16 * u + 255) / 256);
}

template <int U, int LOG2N, bool WITH_MASK, typename Out = uint16_t>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4)))
void tb_mfma_kernel(const uint16_t *__restrict__ g_a, const uint8_t *__restrict__ mask_a, int64_t rows_a,
                    int log2n, Out *__restrict__ out_a, const uint16_t *__restrict__ g_b,
                    const uint8_t *__restrict__ mask_b, int64_t rows_b, Out *__restrict__ out_b)
{
    // One launch serves up to two gradients of the same row length (rows_b = 0: one): rows
    // [0, rows_a) of the launch are the first one's, the rest the second one's.
    const int64_t rows = rows_a + rows_b;
    constexpr bool kF32Out = sizeof(Out) == 4;
    constexpr int T = (U + 7) / 8;         // tiles of 1024 elements; the last one may be partial
    constexpr int NI = 2 * U;              // elements per lane
    constexpr int cols = 128 * U;
    constexpr int kTailRows = (U % 8) ? 4 * (U % 8) : 32;   // rows of the last tile that exist
    // tiles transformed together: those one Hadamard block spans
    constexpr int kSpan = LOG2N > 10 ? (1 << (LOG2N - 10)) : 1;
    constexpr int G = kSpan < T ? kSpan : T;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, h = lane >> 5;

    // Row staging through LDS, as in the fused quantizer: each wave owns a buffer of one gradient row
    // (pieces of 16 tile rows of 64 bytes, chunk c of tile row r in slot c ^ ((r >> 2) & 3)) followed
    // by the row's mask bytes, both filled by global -> LDS transfers that are requested one row ahead.
    constexpr int kStoresPerRow = kF32Out ? NI : NI / 2;
    constexpr bool kLdsRow = tb_rows_through_lds(U, kF32Out);
    constexpr int kPieces = U / 4;
    constexpr int kMaskBytes = 16 * U, kMaskPieces = (kMaskBytes + 255) / 256;
    constexpr int kWaveBuffer = tb_wave_buffer_bytes(U);
    extern __shared__ __attribute__((aligned(16))) uint8_t row_buffers[];
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint8_t *my_buffer = row_buffers + wave_u * kWaveBuffer;
    const uint32_t my_buffer_addr = lds_address(row_buffers) + (uint32_t)(wave_u * kWaveBuffer);
    const uint32_t piece_offset = (uint32_t)(64 * (lane >> 2) + 16 * ((lane & 3) ^ ((lane >> 4) & 3)));
    auto request_row = [&](int64_t row_of_launch) {
        const bool from_b = row_of_launch >= rows_a;
        const int64_t row = from_b ? row_of_launch - rows_a : row_of_launch;
        const uint16_t *g = from_b ? g_b : g_a;
        const uint8_t *mask = from_b ? mask_b : mask_a;
        const char *base = reinterpret_cast<const char *>(g + row * cols);
#pragma unroll
        for (int i = 0; i < kPieces; ++i)
            lds_dma16_stream(base + 1024 * i, piece_offset, my_buffer_addr + 1024 * i);
        if constexpr (WITH_MASK) {
            // lanes past the end of the row's mask fetch its last dword again (in bounds, never read)
            const char *mask_base = reinterpret_cast<const char *>(mask + row * (cols / 8));
#pragma unroll
            for (int i = 0; i < kMaskPieces; ++i)
                lds_dma4_stream(mask_base, (uint32_t)min(256 * i + 4 * lane, kMaskBytes - 4),
                                my_buffer_addr + 256 * U + 256 * i);
        }
    };
    const int64_t row_stride = (int64_t)gridDim.x * kRowsPerBlock;
    int64_t row_of_launch = (int64_t)blockIdx.x * kRowsPerBlock + wave_u;
    if constexpr (kLdsRow) {
        if (row_of_launch < rows)
            request_row(row_of_launch);   // before anything else is set up
    }

    // B operand: rows q = 16 h + 8 s + e of I (x) H_min(n,32), column q' = m, as bf16 +-1 / 0
    v8bf bmat[2];
    hadamard_operand<(LOG2N > 5)>(log2n, m, h, bmat);
    // rows of two tiles under one block of 2048: the stage that pairs the tiles is taken into the
    // matrix instructions' accumulation
    constexpr bool kFold = T == 2 && LOG2N == 11;
    v8bf bneg[2];
    if constexpr (kFold) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            uint32_t words[4];
            __builtin_memcpy(words, &bmat[s], 16);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                words[i] ^= 0x80008000u;   // every entry is +-1 here: flip the signs
            __builtin_memcpy(&bneg[s], words, 16);
        }
    }
    const float inv_sqrt_n = inv_sqrt_pow2(log2n);
    // exchange with lane ^ 1: even lanes keep the low halves, odd lanes the high halves
    const uint32_t pair_sel = (lane & 1) ? 0x03020706u : 0x05040100u;

    int stores_after_request = 0;   // stores issued since the transfers of the row about to be read
    for (; row_of_launch < rows; row_of_launch += row_stride) {
        const bool from_b = row_of_launch >= rows_a;
        const int64_t row = from_b ? row_of_launch - rows_a : row_of_launch;
        const uint16_t *g = from_b ? g_b : g_a;
        const uint8_t *mask = from_b ? mask_b : mask_a;
        Out *out = from_b ? out_b : out_a;
        const uint16_t *src = g + row * cols + 32 * m + 16 * h;
        const uint8_t *mask_src = mask + row * (cols / 8) + 4 * m + 2 * h;
        // the whole row's inputs, out of LDS, before the buffer is handed to the next row
        v4u staged[kLdsRow ? T : 1][2];
        uint32_t staged_bits[kLdsRow ? T : 1];
        if constexpr (kLdsRow) {
            wait_vmcnt_upto(stores_after_request);   // this row has landed
            const int slot0 = (2 * h) ^ ((m >> 2) & 3), slot1 = (2 * h + 1) ^ ((m >> 2) & 3);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                staged[t][0] = *reinterpret_cast<const v4u *>(my_buffer + 2048 * t + 64 * m + 16 * slot0);
                staged[t][1] = *reinterpret_cast<const v4u *>(my_buffer + 2048 * t + 64 * m + 16 * slot1);
                staged_bits[t] = WITH_MASK ? *reinterpret_cast<const uint16_t *>(my_buffer + 256 * U + 128 * t + 4 * m + 2 * h)
                                           : 0xffffu;
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0): the buffer has been read, it may be refilled
            if (row_of_launch + row_stride < rows)
                request_row(row_of_launch + row_stride);
            stores_after_request = kStoresPerRow;
        }
        // tiles that one Hadamard block couples are transformed together, the others one after another
#pragma unroll
        for (int g0 = 0; g0 < T; g0 += G) {
            float acc[G][16];
            v8bf frag[G][2];   // masked inputs of the group's tiles as matrix-instruction operands
#pragma unroll
            for (int u = 0; u < G; ++u) {
                const int t = g0 + u;
                v4u n0 = {0, 0, 0, 0}, n1 = {0, 0, 0, 0};
                uint32_t bits = 0xffffu;
                if constexpr (kLdsRow) {   // whole tiles only
                    n0 = staged[t][0];
                    n1 = staged[t][1];
                    bits = staged_bits[t];
                } else if (t < T && (t < T - 1 || m < kTailRows)) {
                    n0 = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(src + 1024 * t));
                    n1 = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(src + 1024 * t + 8));
                    if (WITH_MASK)
                        bits = *reinterpret_cast<const uint16_t *>(mask_src + 128 * t);
                }
                uint32_t w[8] = {n0.x, n0.y, n0.z, n0.w, n1.x, n1.y, n1.z, n1.w};
                if (WITH_MASK) {
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        w[i] = keep_trusted(w[i], bits, 2 * i);
                }
                __builtin_memcpy(&frag[u][0], &w[0], 16);
                __builtin_memcpy(&frag[u][1], &w[4], 16);
            }
#pragma unroll
            for (int u = 0; u < G; ++u) {
                v16f z;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    z[r] = 0.0f;
                if constexpr (kFold) {   // tile 0 +- tile 1 in the accumulation: the second tile meets -H for the difference
                    z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[0][0], bmat[0], z, 0, 0, 0);
                    z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[0][1], bmat[1], z, 0, 0, 0);
                    z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[1][0], u == 0 ? bmat[0] : bneg[0], z, 0, 0, 0);
                    z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[1][1], u == 0 ? bmat[1] : bneg[1], z, 0, 0, 0);
                } else {
                    z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[u][0], bmat[0], z, 0, 0, 0);
                    z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[u][1], bmat[1], z, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[u][r] = z[r];
            }

            tile_stages<LOG2N, G, kFold>(acc);

            // element = (lane & 31) + 32 h + 64 iota; this group holds iota = 16 g0 .. as far as the row goes
            constexpr int kGroupI = 16 * G;
            const int first = 16 * g0;
            const int count_i = (NI - first) < kGroupI ? (NI - first) : kGroupI;
            if constexpr (kF32Out) {
                float *dst = out + row * cols + lane + 64 * first;
#pragma unroll
                for (int i = 0; i < kGroupI; ++i)
                    if (i < count_i) {
                        const float v = __fmul_rn(acc[i >> 4][reg_of_iota(i & 15)], inv_sqrt_n);
                        if constexpr (kLdsRow)
                            store_word_counted(reinterpret_cast<uint32_t *>(dst + 64 * i), __float_as_uint(v));
                        else
                            __builtin_nontemporal_store(v, dst + 64 * i);
                    }
            } else {
                // Round (iota, iota + 1) to a bf16 pair, swap halves with lane ^ 1: an even lane then
                // holds elements (l, l + 1) of iota, an odd lane elements (l - 1, l) of iota + 1.  A wave
                // instruction stores 2 x 128 contiguous bytes.
                uint32_t *dst = reinterpret_cast<uint32_t *>(out + row * cols) + (m >> 1) + 16 * h +
                                32 * (lane & 1) + 32 * first;
#pragma unroll
                for (int i = 0; i < kGroupI; i += 2) {
                    if (i < count_i) {
                        const float v0 = __fmul_rn(acc[i >> 4][reg_of_iota(i & 15)], inv_sqrt_n);
                        const float v1 = __fmul_rn(acc[(i + 1) >> 4][reg_of_iota((i + 1) & 15)], inv_sqrt_n);
                        const uint32_t own = pack_bf16_pair(v0, v1);
                        const uint32_t other = (uint32_t)__builtin_amdgcn_ds_swizzle((int)own, (1 << 10) | 0x1f);
                        if constexpr (kLdsRow)
                            store_word_counted(dst + 32 * i, __builtin_amdgcn_perm(other, own, pair_sel));
                        else
                            __builtin_nontemporal_store(__builtin_amdgcn_perm(other, own, pair_sel), dst + 32 * i);
                    }
                }
            }
        }
    }
}

template <int U, int LOG2N, typename Out = uint16_t>
void launch(const BackwardArgs &a, hipStream_t stream)
{
    const int64_t blocks_needed = (a.rows + a.rows2 + kRowsPerBlock - 1) / kRowsPerBlock;
    const int64_t max_blocks = kMaxBlocks;
    const dim3 grid((unsigned)(blocks_needed < max_blocks ? blocks_needed : max_blocks));
    const auto *g = static_cast<const uint16_t *>(a.g);
    auto *out = static_cast<Out *>(a.out);
    const auto *g2 = static_cast<const uint16_t *>(a.g2);
    auto *out2 = static_cast<Out *>(a.out2);
    constexpr unsigned lds_bytes = tb_rows_through_lds(U, sizeof(Out) == 4) ? kRowsPerBlock * tb_wave_buffer_bytes(U) : 0;
    static_assert(lds_bytes <= 40960, "four workgroups per CU");
    if (a.mask)
        hipLaunchKernelGGL((tb_mfma_kernel<U, LOG2N, true, Out>), grid, dim3(kThreads), lds_bytes, stream, g,
                           a.mask, a.rows, a.log2n, out, g2, a.mask2, a.rows2, out2);
    else
        hipLaunchKernelGGL((tb_mfma_kernel<U, LOG2N, false, Out>), grid, dim3(kThreads), lds_bytes, stream, g,
                           a.mask, a.rows, a.log2n, out, g2, a.mask2, a.rows2, out2);
}

}  // namespace

// Makes the runtime load this file's code object now (a query of one kernel's attributes does), so
// that the first launch, which may be under graph capture, does not.
hipError_t prepare_trust_backward_mfma_kernels()
{
    hipFuncAttributes attr;
    return hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(tb_mfma_kernel<16, 11, true, uint16_t>));
}

// Launches the matrix-core kernel if it covers the call; returns false (nothing launched) otherwise.
// Covered (U = row length / 128): bf16 in; bf16 out for rows of 512, 1024, 2048, 4096, 5632 or 11008
// elements with a Hadamard block of at most 32, or 128, 256 (11008 only), 512, 1024, 2048, 4096 where
// it divides the row, and for the other widths of the paper's model family (640, 768, 1280, 1664,
// 1792, 2816, 3584, 4608) with a block of at most 32 or their widest one; fp32 out (a weight
// gradient for an fp32 optimizer) for all of these row lengths with their widest block.
bool launch_trust_backward_mfma(const BackwardArgs &a, hipStream_t stream)
{
    if (a.g_dtype != QUEST_BF16 || (a.cols % 128) != 0)
        return false;
    const int u = (int)(a.cols / 128);
    const int l = a.log2n <= 5 ? 5 : a.log2n;
    if (a.out_dtype != QUEST_BF16) {
#define QUEST_F32_OUT_CASE(U_, L_)                 \
    if (u == U_ && l == L_) {                      \
        launch<U_, L_, float>(a, stream);          \
        return true;                               \
    }
        QUEST_F32_OUT_CASE(4, 9) QUEST_F32_OUT_CASE(8, 10) QUEST_F32_OUT_CASE(16, 11) QUEST_F32_OUT_CASE(32, 12)
        QUEST_F32_OUT_CASE(44, 9) QUEST_F32_OUT_CASE(86, 8)
        QUEST_F32_OUT_CASE(5, 7) QUEST_F32_OUT_CASE(6, 8) QUEST_F32_OUT_CASE(10, 8) QUEST_F32_OUT_CASE(13, 7)
        QUEST_F32_OUT_CASE(14, 8) QUEST_F32_OUT_CASE(22, 8) QUEST_F32_OUT_CASE(28, 9) QUEST_F32_OUT_CASE(36, 9)
#undef QUEST_F32_OUT_CASE
        return false;
    }
#define QUEST_CASE(U_, L_)                        \
    if (u == U_ && l == L_) {                     \
        launch<U_, L_>(a, stream);                \
        return true;                              \
    }
    QUEST_CASE(4, 5) QUEST_CASE(4, 7) QUEST_CASE(4, 9)
    QUEST_CASE(8, 5) QUEST_CASE(8, 7) QUEST_CASE(8, 9) QUEST_CASE(8, 10)
    QUEST_CASE(16, 5) QUEST_CASE(16, 7) QUEST_CASE(16, 9) QUEST_CASE(16, 10) QUEST_CASE(16, 11)
    QUEST_CASE(32, 5) QUEST_CASE(32, 7) QUEST_CASE(32, 9) QUEST_CASE(32, 10) QUEST_CASE(32, 11) QUEST_CASE(32, 12)
    QUEST_CASE(44, 5) QUEST_CASE(44, 7) QUEST_CASE(44, 9)
    QUEST_CASE(86, 5) QUEST_CASE(86, 7) QUEST_CASE(86, 8)   // 11008 = 86 x 128: ends three quarters into a tile
    // the other widths of the paper's models (hidden 640 .. 1664, MLP 1792 .. 4608): no transform / widest block
    QUEST_CASE(5, 5) QUEST_CASE(5, 7) QUEST_CASE(6, 5) QUEST_CASE(6, 8) QUEST_CASE(10, 5) QUEST_CASE(10, 8)
    QUEST_CASE(13, 5) QUEST_CASE(13, 7) QUEST_CASE(14, 5) QUEST_CASE(14, 8) QUEST_CASE(22, 5) QUEST_CASE(22, 8)
    QUEST_CASE(28, 5) QUEST_CASE(28, 9) QUEST_CASE(36, 5) QUEST_CASE(36, 9)
#undef QUEST_CASE
    return false;
}

}  // namespace quest
