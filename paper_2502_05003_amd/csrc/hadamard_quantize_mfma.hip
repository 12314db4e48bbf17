// Matrix-core assisted fused Hadamard quantizer for bf16 rows and 4-bit codes (Algorithm 1, one
// operand; Sec. 3.1 and 3.2 of arXiv 2502.05003).
//
// Why matrix cores in a bandwidth-bound kernel: at a block of 2048 the transform alone is 11
// fp32 add/sub per element, plus about 7 for RMS, rounding, packing and the mask.  Packed fp32
// math is off, so a CU retires 64 fp32 lane-ops per clock; 18 ops per element then cost more
// time than the 2.6 bytes per element do at the HBM rate.  The first five stages act on the bf16
// inputs themselves: as a product with the +-1 matrix H_32 they are exact on the bf16 MFMA
// (exact products, fp32 accumulation: the same roundings as a butterfly network), and they cost
// four MFMA instructions per row instead of 160 vector instructions.
//
// Data flow, one wavefront per row of 128 * U elements:
//   * bf16 rows of whole 512-element pieces are brought into a per-wave LDS buffer by global -> LDS
//     transfers, the next row while the current one is worked on (other rows: direct loads);
//   * the row is cut into tiles of 1024 elements seen as 32 x 32 matrices X[p][q] (element
//     32 p + q); lane (m = l & 31, h = l >> 5) takes the 32 contiguous bytes of row p = m that
//     hold q = 16 h .. 16 h + 15, which is exactly its share of the MFMA A operand;
//   * D = X . (I (x) H_min(n,32)) transforms index bits 0..4; lane m then holds column q' = m,
//     register r holds p = 8 (r >> 2) + 4 h + (r & 3): bits 5, 6 in r & 3, bit 7 in h, bits 8, 9
//     in r >> 2, bits >= 10 in the tile number;
//   * the stages on bits 5, 6, 8, 9 and on whole tiles are register-to-register; bit 7 is brought
//     into registers by one half-wave swap (after which h holds bit 5);
//   * sum of squares: the block transform is orthonormal, so it is taken from the packed bf16
//     inputs with the two-way dot instruction;
//   * codes and mask bits are formed in register order, packed per lane, transposed across lanes
//     (8 x 8 nibbles, 32 x 32 bits) through the LDS crossbar, and stored as coalesced dwords in
//     natural element order.
//
// fp32 rows and the AbsMax scale use the same kernel in its "hold all" form: every tile of the row
// is transformed before anything is rounded (the scale needs the whole transformed row, or, for
// fp32 rows, the sum of squares is gathered while the tiles stream in).  An fp32 input is cut into
// three bf16 pieces, x = hi + mid + lo exactly (8 + 8 + 8 significant bits), each of which goes
// through the same exact +-1 product; the fp32 MFMA would be sixteen times slower.
#include "hadamard_tile.h"
#include "quest_internal.h"

namespace quest {
namespace {

typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

// Launch shape: four workgroups of four waves per compute unit (one wave per SIMD and workgroup),
// each wave walking over its rows.  Two to six workgroups per compute unit time the same.
constexpr int kBlocksPerCu = 4;
constexpr int kWavesPerEu = 4;

constexpr int kThreads = 256;
constexpr int kRowsPerBlock = kThreads / 64;

// Streaming stores: the outputs are not read again by this kernel.  The inline-assembly form is for
// the code path that counts its own outstanding memory operations (see the row loop).
__device__ __forceinline__ void store_word(uint32_t *p, uint32_t v)
{
    __builtin_nontemporal_store(v, p);
}

template <int XOR>
__device__ __forceinline__ uint32_t swizzle_xor(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, (XOR << 10) | 0x1f);
}

// Per-lane constants of the lane <-> field transposes.  In stage s a lane keeps the fields whose
// index bit s equals its own lane bit s and takes the others from lane ^ (1 << s), moved by
// FIELD << s bits.  Moves of 8 or 16 bits are one byte permute; smaller ones a rotate and a
// three-input select.
template <int STAGES, int FIELD>
struct TransposePlan {
    uint32_t keep[STAGES];   // bit mask of the fields kept            (sub-byte stages)
    uint32_t rot[STAGES];    // right-rotation applied to the partner  (sub-byte stages)
    uint32_t sel[STAGES];    // v_perm selector {own, partner}         (byte and halfword stages)

    __device__ __forceinline__ void init(int lane)
    {
#pragma unroll
        for (int s = 0; s < STAGES; ++s) {
            const int sh = FIELD << s;
            uint32_t lo = 0;  // field positions whose index has bit s clear
#pragma unroll
            for (int f = 0; f < (1 << STAGES); ++f)
                if (((f >> s) & 1) == 0)
                    lo |= ((1u << FIELD) - 1u) << (f * FIELD);
            const bool up = (lane >> s) & 1;
            keep[s] = up ? ~lo : lo;
            rot[s] = up ? (uint32_t)sh : (uint32_t)(32 - sh);
            // v_perm_b32(partner, own, sel): selector bytes 0..3 pick from own, 4..7 from partner
            if (sh == 8)
                sel[s] = up ? 0x03070105u : 0x06020400u;
            else if (sh == 16)
                sel[s] = up ? 0x03020706u : 0x05040100u;
            else
                sel[s] = 0;
        }
    }

    // After the call, field i of lane a holds what field a of lane i held (lanes modulo 2^STAGES).
    __device__ __forceinline__ uint32_t apply(uint32_t d) const
    {
#pragma unroll
        for (int s = 0; s < STAGES; ++s) {
            uint32_t partner;
            if (s == 0) partner = swizzle_xor<1>(d);
            else if (s == 1) partner = swizzle_xor<2>(d);
            else if (s == 2) partner = swizzle_xor<4>(d);
            else if (s == 3) partner = swizzle_xor<8>(d);
            else partner = swizzle_xor<16>(d);
            if ((FIELD << s) >= 8) {
                d = __builtin_amdgcn_perm(partner, d, sel[s]);
            } else {
                const uint32_t rotated = __builtin_amdgcn_alignbit(partner, partner, rot[s]);
                // (keep & d) | (~keep & rotated) as one three-input bit operation
                d = __builtin_amdgcn_bitop3_b32(keep[s], d, rotated, 0xCA);
            }
        }
        return d;
    }
};

/*
 * U: row length / 128.  LOG2N: log2 of the Hadamard block when it is >= 32; 5 also stands for
 * every smaller block (then only the MFMA operand differs, and `log2n` carries the true value).
 * FP4: the codes are E2M1 values of 6 x_h / (alpha rms) (Sec. 4.4 "The FP4 Format"), made by the
 * hardware conversion (nearest, ties to even, saturating, sign kept on underflow), and the scale
 * is alpha rms / 6; everything else is shared.
 * BITS: b of the Eq. 1 grid (1, 2, 3, 4 or 8; containers of 1, 2, 4, 4, 8 bits).  For b >= 2 the
 * code is the top b bits of the byte sat_u8(rne(2^(8-b) cell + 127.5)) = clamp(floor(cell) + L/2,
 * 0, L - 1); for b = 1 it is the complement of the sign bit.  What differs is how many codes make
 * a dword and hence over how many lanes the fields are transposed before the store.
 * In: uint16_t (bf16 bits) or float.  ABSMAX: the grid spans the row's largest |x_h| instead of
 * alpha rms (the comparison quantizer of Sec. 4.1); nothing is clipped, every element is trusted.
 */
// Waves per SIMD the register budget is set for.  Holding a long row (2 U transformed values per
// lane, next to the fp32 inputs still on their way) needs more than the 128 registers of four waves,
// and so do the packed inputs of a row of 5632 or 11008 (measured: 52 instead of 57 us for 16384 x 5632).
template <int U, bool HOLD_ALL, bool F32>
constexpr int hq_waves_per_eu()
{
    return (HOLD_ALL && (U > 32 || (F32 && U >= 24))) ? 2 : U > 40 ? 3 : kWavesPerEu;
}

template <int U, int LOG2N, bool WITH_MASK, bool FP4 = false, int BITS = 4, typename In = uint16_t,
          bool ABSMAX = false>
__global__ __launch_bounds__(kThreads)
__attribute__((amdgpu_waves_per_eu(hq_waves_per_eu<U, (sizeof(In) == 4 || ABSMAX), sizeof(In) == 4>())))
void hq_mfma_kernel(
    const In *__restrict__ x_a, int64_t rows_a, int64_t ld_a, int log2n, float alpha,
    float trust_edge, uint8_t *__restrict__ codes_a, float *__restrict__ scales_a,
    uint8_t *__restrict__ mask_a, float *__restrict__ xh_out,
    const In *__restrict__ x_b, int64_t rows_b, int64_t ld_b, uint8_t *__restrict__ codes_b,
    float *__restrict__ scales_b, uint8_t *__restrict__ mask_b)
{
    // Two operands of one layer (activations and weights, same row length, block and grid) can share
    // a launch: the rows of the second follow those of the first in the launch's row numbering, and
    // every row picks its operand's pointers.  rows_b = 0 is the single-operand call.
    const int64_t rows = rows_a + rows_b;
    constexpr int T = (U + 7) / 8;         // tiles of 1024 elements; the last one may be partial
    constexpr int NI = 2 * U;              // elements per lane
    constexpr int cols = 128 * U;
    // rows p of the last tile that exist (the row may end after any eighth of it)
    constexpr int kTailRows = (U % 8) ? 4 * (U % 8) : 32;
    constexpr bool kF32 = sizeof(In) == 4;
    constexpr bool kHoldAll = kF32 || ABSMAX;
    static_assert(!kHoldAll || (!FP4 && BITS == 4), "fp32 rows and AbsMax: 4-bit integer grid only");
    // tiles transformed together: all of them when the whole row is held, else those one Hadamard
    // block spans, and at least two (one mask word)
    constexpr int kSpan = LOG2N > 10 ? (1 << (LOG2N - 10)) : 1;
    constexpr int G = kHoldAll ? T : (kSpan >= T ? T : (kSpan >= 2 ? kSpan : (T >= 2 ? 2 : 1)));
    constexpr int kLevels = 1 << BITS;
    constexpr int CB = BITS == 3 ? 4 : BITS;   // container bits
    static_assert(!FP4 || BITS == 4, "the E2M1 grid has 4-bit codes");
    static_assert((U % 4) == 0 || (BITS == 3 || BITS == 4), "rows that do not end on half a tile: nibble codes only");

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, h = lane >> 5;

    // bf16 rows made of whole 1 KiB pieces (512 elements) land in LDS first: each wave owns one row
    // buffer, filled by global -> LDS transfers that need no registers while in flight.  The row
    // after the one being worked on is requested as soon as the current one has been copied to
    // registers, so its memory latency runs under this row's arithmetic.  Piece i is 16 tile rows of
    // 64 bytes; lane l of a transfer lands at row l / 4, 16-byte slot l % 4, and fetches the chunk
    // that belongs there: chunk c of tile row r sits in slot c ^ ((r >> 2) & 3), which makes the
    // 128-bit operand reads below (sixteen lanes = sixteen consecutive tile rows) conflict-free.
    constexpr bool kLdsRow = !kF32 && (U % 4) == 0 && U <= 44;
    constexpr int kPieces = U / 4;
    extern __shared__ __attribute__((aligned(16))) uint8_t row_buffers[];
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint8_t *my_buffer = row_buffers + wave_u * (256 * U);
    const uint32_t my_buffer_addr = lds_address(row_buffers) + (uint32_t)wave_u * (256u * U);
    const uint32_t piece_offset = (uint32_t)(64 * (lane >> 2) + 16 * ((lane & 3) ^ ((lane >> 4) & 3)));
    auto request_row = [&](int64_t row_of_launch) {
        const bool from_b = row_of_launch >= rows_a;
        const char *base = reinterpret_cast<const char *>(
            from_b ? reinterpret_cast<const uint16_t *>(x_b) + (row_of_launch - rows_a) * ld_b
                   : reinterpret_cast<const uint16_t *>(x_a) + row_of_launch * ld_a);
#pragma unroll
        for (int i = 0; i < kPieces; ++i)
            lds_dma16_stream(base + 1024 * i, piece_offset, my_buffer_addr + 1024 * i);
    };
    // the first row is requested before anything else is set up
    const int64_t row_stride = (int64_t)gridDim.x * kRowsPerBlock;
    int64_t row_of_launch = (int64_t)blockIdx.x * kRowsPerBlock + wave_u;
    if constexpr (kLdsRow) {
        if (row_of_launch < rows)
            request_row(row_of_launch);
    }

    // B operand: rows q = 16 h + 8 s + e of I (x) H_min(n,32), column q' = m, as bf16 +-1 / 0
    v8bf bmat[2];
    hadamard_operand<(LOG2N > 5)>(log2n, m, h, bmat);
    // fp32 rows: the middle piece is carried with its sign flipped (see below) and meets -H
    // bf16 rows of two tiles under one block of 2048: the stage that pairs the tiles is taken into the
    // matrix instructions' accumulation, tile 0 +- tile 1 (the second tile meets -H for the difference)
    constexpr bool kFold = !kHoldAll && T == 2 && LOG2N == 11;
    v8bf bneg[2];
    if constexpr (kF32 || kFold) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            uint32_t w[4];
            __builtin_memcpy(w, &bmat[s], 16);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w[i] ^= (w[i] & 0x00800080u) << 8;   // bit 7 is set in +-1 and clear in 0: flip the sign of the former
            __builtin_memcpy(&bneg[s], w, 16);
        }
    }
    TransposePlan<3, 4> nibble_plan;   // 8 codes of 4 bits per dword
    TransposePlan<2, 8> byte_plan;     // 4 codes of 8 bits
    TransposePlan<4, 2> pair_plan;     // 16 codes of 2 bits
    if (CB == 4)
        nibble_plan.init(lane);
    if (CB == 8)
        byte_plan.init(lane);
    if (CB == 2)
        pair_plan.init(lane);
    TransposePlan<5, 1> bit_plan;      // 32 mask bits, or 32 codes of 1 bit
    if (CB == 1)
        bit_plan.init(lane);
    if (WITH_MASK)
        bit_plan.init(lane);

    const float inv_sqrt_n = inv_sqrt_pow2(log2n), sqrt_n = sqrt_pow2(log2n);
    const int code_word = ((lane >> 3) & 3) + 4 * h + 8 * (lane & 7);

    // Raw inputs of one bf16 row: two 16-byte pieces per tile and lane.
    struct RawRow {
        uint4 a[kF32 ? 1 : T][2];
    };
    auto load_row = [&](const In *x, int64_t ld, int64_t row, RawRow &raw) {
        if constexpr (!kF32) {   // fp32 rows stream in tile by tile, see below
            const uint16_t *src = reinterpret_cast<const uint16_t *>(x) + row * ld + 32 * m + 16 * h;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                raw.a[t][0] = make_uint4(0, 0, 0, 0);
                raw.a[t][1] = make_uint4(0, 0, 0, 0);
                if (t < T - 1 || m < kTailRows) {
                    const v4u n0 = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(src + 1024 * t));
                    const v4u n1 = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(src + 1024 * t + 8));
                    raw.a[t][0] = make_uint4(n0.x, n0.y, n0.z, n0.w);
                    raw.a[t][1] = make_uint4(n1.x, n1.y, n1.z, n1.w);
                }
            }
        }
    };

    auto read_row = [&](RawRow &raw) {
        if constexpr (!kF32) {
            const int slot0 = (2 * h) ^ ((m >> 2) & 3), slot1 = (2 * h + 1) ^ ((m >> 2) & 3);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                raw.a[t][0] = make_uint4(0, 0, 0, 0);
                raw.a[t][1] = make_uint4(0, 0, 0, 0);
                if (t < T - 1 || m < kTailRows) {
                    raw.a[t][0] = *reinterpret_cast<const uint4 *>(my_buffer + 2048 * t + 64 * m + 16 * slot0);
                    raw.a[t][1] = *reinterpret_cast<const uint4 *>(my_buffer + 2048 * t + 64 * m + 16 * slot1);
                }
            }
        }
    };
    // Stores of the LDS path are issued by hand and counted: when the next row's transfers are
    // awaited, exactly the stores issued after them may still be outstanding (vector-memory
    // operations of a wave complete in issue order).
    // (A store is counted whether or not this lane takes part in it: every predicate below holds for
    // some lane of every wave, so the instruction is always issued, and the count stays wave-uniform.)
    int stores_issued = 0;
    auto emit_if = [&](bool mine, uint32_t *p, uint32_t v) {
        if constexpr (kLdsRow) {
            if (mine)
                store_word_counted(p, v);
            ++stores_issued;
        } else {
            if (mine)
                store_word(p, v);
        }
    };

    int stores_after_request = 0;   // stores issued since the transfers of the row about to be read
    for (; row_of_launch < rows; row_of_launch += row_stride) {
        // this row's operand (wave-uniform)
        const bool from_b = row_of_launch >= rows_a;
        const int64_t row = from_b ? row_of_launch - rows_a : row_of_launch;
        const In *x = from_b ? x_b : x_a;
        const int64_t ld = from_b ? ld_b : ld_a;
        uint8_t *codes = from_b ? codes_b : codes_a;
        float *scales = from_b ? scales_b : scales_a;
        uint8_t *mask = from_b ? mask_b : mask_a;
        RawRow raw;
        if constexpr (kLdsRow) {
            wait_vmcnt_upto(stores_after_request);   // this row has landed
            read_row(raw);
            __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0): the buffer has been read, it may be refilled
            if (row_of_launch + row_stride < rows)
                request_row(row_of_launch + row_stride);
            stores_issued = 0;
        } else {
            load_row(x, ld, row, raw);
        }
        // Per-row constants in the un-normalised domain (x_h = raw / sqrt(n)).  The reciprocal and
        // the square root are the hardware approximations (1 ulp): the codes are decided on
        // raw * raw_to_cell, and a relative error of 1e-7 there is the size of one fp32 rounding.
        float cell16 = 0.0f, to_e2m1 = 0.0f, trust_raw = 0.0f;
        // `sumsq`: this lane's share of the row's sum of squares; `raw_max`: the row's largest |raw|
        auto set_row_constants = [&](float sumsq, float raw_max) {
            float clip;   // half-width of the grid in x_h units
            if constexpr (ABSMAX) {
                clip = __fmul_rn(raw_max, inv_sqrt_n);
                trust_raw = raw_max;
            } else {
                const float rms = __builtin_amdgcn_sqrtf(wave_sum_dpp(sumsq) * (1.0f / (float)cols));
                clip = alpha * rms;
                trust_raw = trust_edge * rms * sqrt_n;
            }
            const bool zero_row = !(clip > 0.0f);
            const float inv_step = zero_row ? 0.0f : (float)(kLevels - 1) * 0.5f * __builtin_amdgcn_rcpf(clip);
            // raw -> 2^(8-b) * (position in grid cells): the code ends up in the top b bits of a byte
            cell16 = inv_step * inv_sqrt_n * (float)(256 >> BITS);
            to_e2m1 = zero_row ? 0.0f : 6.0f * __builtin_amdgcn_rcpf(clip) * inv_sqrt_n;   // raw -> E2M1 units
            emit_if(lane == 0, reinterpret_cast<uint32_t *>(scales + row),
                    __float_as_uint(clip * (FP4 ? 1.0f / 6.0f : 1.0f / (float)(kLevels - 1))));
        };
        float sumsq = 0.0f;
        if constexpr (!kF32) {
            // sum of squares from the packed inputs (the block transform is orthonormal)
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const uint4 a0 = raw.a[t][0], a1 = raw.a[t][1];
                const uint32_t w[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    v2bf pair;
                    __builtin_memcpy(&pair, &w[i], 4);
                    sumsq = __builtin_amdgcn_fdot2_f32_bf16(pair, pair, sumsq, false);
                }
            }
        }
        if constexpr (!kHoldAll)
            set_row_constants(sumsq, 0.0f);
        uint32_t *code_row = reinterpret_cast<uint32_t *>(codes + row * (cols * CB / 8));
        uint32_t *mask_row = reinterpret_cast<uint32_t *>(mask + row * (cols / 8));

        // The transform couples whole tiles only for blocks above 1024.  Below that the tiles are
        // worked off two at a time (the 32 elements per lane that one mask word transposes), so
        // that a long row holds its packed inputs and 32 transformed values, not all of them.
#pragma unroll
        for (int g0 = 0; g0 < T; g0 += G) {
            float acc[G][16];
#pragma unroll
            for (int u = 0; u < G; ++u) {
                const int t = g0 + u;
                if (t < T) {
                    v16f z;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        z[r] = 0.0f;
                    if constexpr (kF32) {
                        // this lane's sixteen consecutive floats of tile row m: q = 16 h .. 16 h + 15
                        const float *src = reinterpret_cast<const float *>(x) + row * ld + 1024 * t + 32 * m + 16 * h;
                        float f[16];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            v4u piece = {0, 0, 0, 0};
                            if (t < T - 1 || m < kTailRows)
                                piece = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(src + 4 * i));
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                f[4 * i + e] = __uint_as_float(piece[e]);
                        }
                        // x = hi + mid + lo, each piece the top 16 bits of what the pieces before it
                        // leave (exact: the remainders have 16 and 8 significant bits).  Remainders
                        // come from the two-way bf16 dot product, packed piece times (1, 0) or (0, 1)
                        // minus the value: s1 = hi - x = -(mid + lo), s2 = top16(s1) - s1 = lo.
                        uint32_t hi[8], mid[8], lo[8];
                        // (1, 0) and (0, 1) as bf16 pairs, held in registers the compiler cannot see through: written
                        // as literals the pair (1, 0) reaches the instruction as (0, 1)
                        uint32_t first_bits = 0x00003F80u, second_bits = 0x3F800000u;
                        asm volatile("" : "+v"(first_bits), "+v"(second_bits));
                        v2bf first, second;
                        __builtin_memcpy(&first, &first_bits, 4);
                        __builtin_memcpy(&second, &second_bits, 4);
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const float a = f[2 * i], b = f[2 * i + 1];
                            sumsq = __fmaf_rn(a, a, sumsq);
                            sumsq = __fmaf_rn(b, b, sumsq);
                            hi[i] = __builtin_amdgcn_perm(__float_as_uint(b), __float_as_uint(a), 0x07060302u);
                            v2bf hp;
                            __builtin_memcpy(&hp, &hi[i], 4);
                            const float s1a = __builtin_amdgcn_fdot2_f32_bf16(hp, first, -a, false);
                            const float s1b = __builtin_amdgcn_fdot2_f32_bf16(hp, second, -b, false);
                            mid[i] = __builtin_amdgcn_perm(__float_as_uint(s1b), __float_as_uint(s1a), 0x07060302u);
                            v2bf mp;
                            __builtin_memcpy(&mp, &mid[i], 4);
                            const float s2a = __builtin_amdgcn_fdot2_f32_bf16(mp, first, -s1a, false);
                            const float s2b = __builtin_amdgcn_fdot2_f32_bf16(mp, second, -s1b, false);
                            lo[i] = __builtin_amdgcn_perm(__float_as_uint(s2b), __float_as_uint(s2a), 0x07060302u);
                        }
                        v8bf p0, p1;
                        __builtin_memcpy(&p0, &lo[0], 16);      // smallest piece first
                        __builtin_memcpy(&p1, &lo[4], 16);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p0, bmat[0], z, 0, 0, 0);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p1, bmat[1], z, 0, 0, 0);
                        __builtin_memcpy(&p0, &mid[0], 16);     // holds -mid
                        __builtin_memcpy(&p1, &mid[4], 16);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p0, bneg[0], z, 0, 0, 0);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p1, bneg[1], z, 0, 0, 0);
                        __builtin_memcpy(&p0, &hi[0], 16);
                        __builtin_memcpy(&p1, &hi[4], 16);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p0, bmat[0], z, 0, 0, 0);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p1, bmat[1], z, 0, 0, 0);
                    } else if constexpr (kFold) {
                        v8bf tile0_lo, tile0_hi, tile1_lo, tile1_hi;
                        __builtin_memcpy(&tile0_lo, &raw.a[0][0], 16);
                        __builtin_memcpy(&tile0_hi, &raw.a[0][1], 16);
                        __builtin_memcpy(&tile1_lo, &raw.a[1][0], 16);
                        __builtin_memcpy(&tile1_hi, &raw.a[1][1], 16);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tile0_lo, bmat[0], z, 0, 0, 0);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tile0_hi, bmat[1], z, 0, 0, 0);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tile1_lo, u == 0 ? bmat[0] : bneg[0], z, 0, 0, 0);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tile1_hi, u == 0 ? bmat[1] : bneg[1], z, 0, 0, 0);
                    } else {
                        v8bf f0, f1;
                        __builtin_memcpy(&f0, &raw.a[t][0], 16);
                        __builtin_memcpy(&f1, &raw.a[t][1], 16);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0, bmat[0], z, 0, 0, 0);
                        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1, bmat[1], z, 0, 0, 0);
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        acc[u][r] = z[r];
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        acc[u][r] = 0.0f;
                }
            }

            tile_stages<LOG2N, G, kFold>(acc);

            if constexpr (kHoldAll) {   // the whole row is transformed: now its scale can be fixed
                float raw_max = 0.0f;
                if constexpr (ABSMAX) {
#pragma unroll
                    for (int u = 0; u < G; ++u)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            raw_max = fmaxf(raw_max, fabsf(acc[u][r]));
#pragma unroll
                    for (int off = 32; off > 0; off >>= 1)
                        raw_max = fmaxf(raw_max, __shfl_xor(raw_max, off, kWave));
                }
                set_row_constants(sumsq, raw_max);
            }

            // in-lane elements of this group: iota = 16 g0 .. , as far as the row goes
            constexpr int kGroupI = 16 * G;
            const int first = 16 * g0;
            const int count_i = (NI - first) < kGroupI ? (NI - first) : kGroupI;

            if (xh_out && !from_b) {   // debug output of the first operand only
                float *dst = xh_out + row * cols + lane;   // element = lane + 64 iota
#pragma unroll
                for (int i = 0; i < kGroupI; ++i)
                    if (i < count_i)
                        dst[64 * (first + i)] = __fmul_rn(acc[i >> 4][reg_of_iota(i & 15)], inv_sqrt_n);
            }

            // value of in-lane element i of this group
            auto elem = [&](int i) { return acc[i >> 4][reg_of_iota(i & 15)]; };
            if constexpr (CB == 4) {
                // byte = sat_u8(rne(2^(8-b) cell + 128 - 1/2)); its top b bits are
                // clamp(floor(cell) + L/2, 0, L - 1) = c.  Eight per dword in iota order, then the transpose.
#pragma unroll
                for (int dd = 0; dd < 2 * G; ++dd) {
                    if (8 * dd < count_i) {
                        uint32_t packed;
                        if (FP4) {
                            // byte i / 2 = E2M1(element i + 1) << 4 | E2M1(element i), converted in pairs
                            auto scaled = [&](int i) { return __fmul_rn(elem(8 * dd + i), to_e2m1); };
                            packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, scaled(0), scaled(1), 1.0f, 0);
                            packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, scaled(2), scaled(3), 1.0f, 1);
                            packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, scaled(4), scaled(5), 1.0f, 2);
                            packed = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(packed, scaled(6), scaled(7), 1.0f, 3);
                        } else {
                            uint32_t even = 0, odd = 0;
#pragma unroll
                            for (int i = 0; i < 8; ++i) {
                                const float t = __fmaf_rn(elem(8 * dd + i), cell16, 127.5f);
                                if (i & 1)
                                    odd = __builtin_amdgcn_cvt_pk_u8_f32(t, i >> 1, odd);
                                else
                                    even = __builtin_amdgcn_cvt_pk_u8_f32(t, i >> 1, even);
                            }
                            packed = BITS == 4 ? ((even >> 4) & 0x0f0f0f0fu) | (odd & 0xf0f0f0f0u)
                                               : ((even >> 5) & 0x07070707u) | ((odd >> 1) & 0x70707070u);
                        }
                        // after the transpose this lane holds in-lane element 8 dd + lane % 8 of eight
                        // neighbouring lanes; where the row ends inside the dword's range it may not exist
                        const uint32_t word = nibble_plan.apply(packed);
                        emit_if(8 * dd + 8 <= count_i || 8 * dd + (lane & 7) < count_i,
                                code_row + code_word + 64 * (2 * g0 + dd), word);
                    }
                }
            } else if constexpr (CB == 8) {
                // four codes per dword; lane 4 q + a ends up with elements 4 q .. 4 q + 3 of iota 4 w + a
#pragma unroll
                for (int w = 0; w < 4 * G; ++w) {
                    if (4 * w < count_i) {
                        uint32_t packed = 0;
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            packed = __builtin_amdgcn_cvt_pk_u8_f32(__fmaf_rn(elem(4 * w + i), cell16, 127.5f), i, packed);
                        emit_if(true, code_row + (lane >> 2) + 16 * (lane & 3) + 64 * (4 * g0 + w),
                                   byte_plan.apply(packed));
                    }
                }
            } else if constexpr (CB == 2) {
                // sixteen codes per dword.  Byte j of e[k] takes element k + 4 j, so that its code (top
                // two bits) shifted down by 6 and up by 2 k lands at bit 2 (k + 4 j) of the dword.
#pragma unroll
                for (int t16 = 0; t16 < G; ++t16) {
                    const int left = count_i - 16 * t16;
                    if (left > 0) {
                        uint32_t packed = 0;
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            uint32_t e = 0;
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                e = __builtin_amdgcn_cvt_pk_u8_f32(__fmaf_rn(elem(16 * t16 + k + 4 * j), cell16, 127.5f), j, e);
                            packed |= ((e >> 6) & 0x03030303u) << (2 * k);
                        }
                        packed = pair_plan.apply(packed);
                        // a half tile at the end of the row has 8 elements per lane
                        emit_if((lane & 15) < left, code_row + (lane >> 4) + 4 * (lane & 15) + 64 * (g0 + t16), packed);
                    }
                }
            } else {
                // one bit per code: c = 1 iff x_h >= 0, the complement of the sign bit; 32 per dword,
                // transposed and stored like the mask
#pragma unroll
                for (int cc = 0; cc * 32 < kGroupI; ++cc) {
                    const int left = count_i - 32 * cc;
                    if (left > 0) {
                        const int count = left < 32 ? left : 32;
                        uint32_t negative = 0;
#pragma unroll
                        for (int i = 31; i >= 0; --i)
                            if (i < count)
                                negative = __builtin_amdgcn_alignbit(negative, __float_as_uint(elem(32 * cc + i)), 31);
                        uint32_t code = ~negative;
                        if (count < 32)
                            code &= (1u << count) - 1u;
                        code = bit_plan.apply(code);
                        emit_if(m < count, code_row + h + 2 * (m + 32 * (g0 / 2 + cc)), code);
                    }
                }
            }

            // trust mask: one bit per element in iota order (sign of trust_raw - |raw|), then the
            // 32 x 32 bit transpose; lane m ends up with the bits of 32 consecutive elements
            if (WITH_MASK) {
#pragma unroll
                for (int cc = 0; cc * 32 < kGroupI; ++cc) {
                    const int left = count_i - 32 * cc;
                    if (left > 0) {
                        const int count = left < 32 ? left : 32;
                        uint32_t untrusted = 0;
#pragma unroll
                        for (int i = 31; i >= 0; --i) {
                            if (i < count) {
                                const float v = acc[(32 * cc + i) >> 4][reg_of_iota((32 * cc + i) & 15)];
                                const float slack = trust_raw - fabsf(v);          // negative <=> untrusted
                                untrusted = __builtin_amdgcn_alignbit(untrusted, __float_as_uint(slack), 31);
                            }
                        }
                        uint32_t trusted = ~untrusted;
                        if (count < 32)
                            trusted &= (1u << count) - 1u;
                        trusted = bit_plan.apply(trusted);
                        emit_if(m < count, mask_row + h + 2 * (m + 32 * (g0 / 2 + cc)), trusted);
                    }
                }
            }
        }
        stores_after_request = stores_issued;
    }
}

template <int U, int LOG2N, bool FP4 = false, int BITS = 4, typename In = uint16_t, bool ABSMAX = false>
void launch(const QuantizeArgs &a, hipStream_t stream)
{
    const int64_t blocks_needed = (a.rows + a.rows2 + kRowsPerBlock - 1) / kRowsPerBlock;
    const int64_t max_blocks = 256 * kBlocksPerCu;
    const dim3 grid((unsigned)(blocks_needed < max_blocks ? blocks_needed : max_blocks));
    const auto *x = static_cast<const In *>(a.x);
    const auto *x2 = static_cast<const In *>(a.x2);
    // one row buffer per wave for the rows that are staged through LDS (see the kernel), 45 KiB at most
    constexpr bool kLdsRow = sizeof(In) == 2 && (U % 4) == 0 && U <= 44;
    constexpr unsigned lds_bytes = kLdsRow ? kRowsPerBlock * 256 * U : 0;
    if (a.mask)
        hipLaunchKernelGGL((hq_mfma_kernel<U, LOG2N, true, FP4, BITS, In, ABSMAX>), grid, dim3(kThreads),
                           lds_bytes, stream, x, a.rows, a.ld, a.log2n, a.alpha, a.trust_edge, a.codes, a.scales,
                           a.mask, a.xh_out, x2, a.rows2, a.ld2, a.codes2, a.scales2, a.mask2);
    else
        hipLaunchKernelGGL((hq_mfma_kernel<U, LOG2N, false, FP4, BITS, In, ABSMAX>), grid, dim3(kThreads),
                           lds_bytes, stream, x, a.rows, a.ld, a.log2n, a.alpha, a.trust_edge, a.codes, a.scales,
                           a.mask, a.xh_out, x2, a.rows2, a.ld2, a.codes2, a.scales2, a.mask2);
}

}  // namespace

// Makes the runtime load this file's code object now (a query of one kernel's attributes does), so
// that the first launch, which may be under graph capture, does not.
hipError_t prepare_quantize_mfma_kernels()
{
    hipFuncAttributes attr;
    return hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(hq_mfma_kernel<16, 11, true>));
}

// Launches the matrix-core kernel if it covers the call; returns false (nothing launched) otherwise.
// Covered (U = row length / 128):
//   bf16 rows, b = 4: rows of 512, 1024, 2048, 4096, 5632 or 11008 elements with a Hadamard block of
//     at most 32, or 128, 256 (11008 only), 512, 1024, 2048, 4096 where it divides the row; the other
//     hidden and MLP widths of the paper's model family (640, 768, 1280, 1664, 1792, 2816, 3584,
//     4608) with a block of at most 32 or their widest one;
//   bf16 rows, b = 1, 2, 3, 8 and the E2M1 grid: rows of 1024 .. 5632 with their widest block;
//   fp32 rows and the AbsMax scale, b = 4: rows of 512 .. 5632 with their widest block; fp32 rows
//     also for the other model widths up to 4608.
bool launch_hadamard_quantize_mfma(const QuantizeArgs &a, hipStream_t stream)
{
    if ((a.cols % 128) != 0)
        return false;
    const int u = (int)(a.cols / 128);
    const int l = a.log2n <= 5 ? 5 : a.log2n;
    if (a.dtype == QUEST_F32 || a.mode == kQuantAbsMax) {   // the whole row is held before anything is rounded
        if (a.bits != 4 || a.mode == kQuantFp4)
            return false;
#define QUEST_HOLD_CASE(U_, L_)                                          \
    if (u == U_ && l == L_) {                                            \
        if (a.dtype == QUEST_F32 && a.mode == kQuantAbsMax)              \
            launch<U_, L_, false, 4, float, true>(a, stream);            \
        else if (a.dtype == QUEST_F32)                                   \
            launch<U_, L_, false, 4, float, false>(a, stream);           \
        else                                                             \
            launch<U_, L_, false, 4, uint16_t, true>(a, stream);         \
        return true;                                                     \
    }
        QUEST_HOLD_CASE(4, 9) QUEST_HOLD_CASE(8, 10) QUEST_HOLD_CASE(16, 11) QUEST_HOLD_CASE(32, 12)
        QUEST_HOLD_CASE(44, 9)
#undef QUEST_HOLD_CASE
        if (a.dtype == QUEST_F32 && a.mode == kQuantRms) {   // fp32 master weights of the smaller models
#define QUEST_F32_CASE(U_, L_)                                           \
    if (u == U_ && l == L_) {                                            \
        launch<U_, L_, false, 4, float, false>(a, stream);               \
        return true;                                                     \
    }
            QUEST_F32_CASE(5, 7) QUEST_F32_CASE(6, 8) QUEST_F32_CASE(10, 8) QUEST_F32_CASE(13, 7)
            QUEST_F32_CASE(14, 8) QUEST_F32_CASE(22, 8) QUEST_F32_CASE(28, 9) QUEST_F32_CASE(36, 9)
#undef QUEST_F32_CASE
        }
        return false;
    }
    if (a.bits != 4) {   // the other widths of the Eq. 1 grid
        if (a.mode != kQuantRms)
            return false;
#define QUEST_BITS_CASE(U_, L_, B_)                    \
    if (u == U_ && l == L_ && a.bits == B_) {          \
        launch<U_, L_, false, B_>(a, stream);          \
        return true;                                   \
    }
#define QUEST_BITS_CASES(U_, L_) \
    QUEST_BITS_CASE(U_, L_, 1) QUEST_BITS_CASE(U_, L_, 2) QUEST_BITS_CASE(U_, L_, 3) QUEST_BITS_CASE(U_, L_, 8)
        QUEST_BITS_CASES(8, 10) QUEST_BITS_CASES(16, 11) QUEST_BITS_CASES(32, 12) QUEST_BITS_CASES(44, 9)
#undef QUEST_BITS_CASES
#undef QUEST_BITS_CASE
        return false;
    }
    if (a.mode == kQuantFp4) {   // the E2M1 grid
#define QUEST_FP4_CASE(U_, L_)                    \
    if (u == U_ && l == L_) {                     \
        launch<U_, L_, true>(a, stream);          \
        return true;                              \
    }
        QUEST_FP4_CASE(8, 10) QUEST_FP4_CASE(16, 11) QUEST_FP4_CASE(32, 12) QUEST_FP4_CASE(44, 9)
#undef QUEST_FP4_CASE
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
