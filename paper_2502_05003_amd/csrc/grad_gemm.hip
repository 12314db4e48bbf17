// The two 16-bit gradient matmuls of Algorithm 2 (arXiv 2502.05003, Sec. 3.3): the upstream
// gradient dy against a code-packed operand whose value is bf16(s * u), contracted on the bf16
// matrix cores with fp32 accumulation.
//   which = 0:  out[M, K] = dy[M, N]   * what_h[N, K]   (contraction over N)
//   which = 1:  out[N, K] = dy[M, N]^T * xhat_h[M, K]   (contraction over M)
// and, with the same machinery, the weight-only forward product (Sec. 4.4):
//   which = 2:  out[M, N] = x[M, K]    * what_h[N, K]^T (contraction over K)
#include <algorithm>
#include <numeric>
#include <utility>

#include "gemm_tile.h"
#include "quest_internal.h"

namespace quest {
namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

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


// ------------------------------------------------------------------------------------------
// Main path.  The code-packed operand is first expanded once to bf16(s u), [C, K] row-major, in
// the caller's workspace (every 256 x 256 output tile would otherwise repeat that work for the
// whole contraction); the matmul itself is then a plain bf16 x bf16 contraction whose main loop
// holds nothing but matrix instructions, LDS reads and global -> LDS transfers.
//
// 256 x 256 outputs per workgroup, four waves of 128 x 128 (sixteen 32 x 32 fp32 accumulator
// tiles, one wave per SIMD), 32 contraction elements per step, a ring of LDS stages of 32 KiB that
// the transfers fill several steps ahead of the step being multiplied.  An operand whose rows are
// contraction rows in memory ([c][k]: the expanded operand, and dy for which = 1) is staged as it
// is and read with the transposing LDS load, which hands each lane four contraction elements of
// one column; an operand whose rows are output rows (dy for which = 0) is read with 128-bit loads.
// ------------------------------------------------------------------------------------------

constexpr int GT = 256;                        // tile edge
constexpr int GC = 32;                         // contraction elements per step
constexpr int kGemmThreads = 256;
constexpr int kOperandBytes = GT * GC * 2;     // 16 KiB per operand and step
constexpr int kGStage = 2 * kOperandBytes;     // left operand, then right operand
constexpr int kParkBytes = 4 * 32768;          // epilogue: 32 KiB per wave

typedef __bf16 v4bf __attribute__((ext_vector_type(4)));

// One LDS read of the main loop: operand, fragment, and which half of the fragment's eight
// contraction elements a transposing read fetches (-1: a 128-bit read of the row form, both halves).
struct ReadOp {
    bool left;
    int idx, half;
};
// right fragment j feeds matrix instructions j, 4 + j, ..., left fragment i instructions 4 i .. 4 i + 3
constexpr ReadOp kReadsTransposed[16] = {{false, 0, 0}, {false, 0, 1}, {true, 0, 0},  {true, 0, 1},
                                         {false, 1, 0}, {false, 1, 1}, {false, 2, 0}, {false, 2, 1},
                                         {false, 3, 0}, {false, 3, 1}, {true, 1, 0},  {true, 1, 1},
                                         {true, 2, 0},  {true, 2, 1},  {true, 3, 0},  {true, 3, 1}};
constexpr ReadOp kReadsRows[8] = {{false, 0, -1}, {true, 0, -1}, {false, 1, -1}, {false, 2, -1},
                                  {false, 3, -1}, {true, 1, -1},  {true, 2, -1},  {true, 3, -1}};
constexpr ReadOp kReadsPlain[12] = {{false, 0, 0}, {false, 0, 1}, {true, 0, -1}, {false, 1, 0},
                                    {false, 1, 1}, {false, 2, 0}, {false, 2, 1}, {false, 3, 0},
                                    {false, 3, 1}, {true, 1, -1}, {true, 2, -1}, {true, 3, -1}};

// Expands packed codes to bf16(fp32(s * u)), u = 2 c - (L - 1): eight elements per thread.
// levels = 0 stands for E2M1 codes (Sec. 4.4): u is then the signed E2M1 value of the code.
__global__ __launch_bounds__(256) void expand_codes_kernel(const uint8_t *__restrict__ codes,
                                                           const float *__restrict__ scales, int levels,
                                                           int cb, int K, int64_t groups,
                                                           uint16_t *__restrict__ qhat)
{
    // a workgroup takes 1024 consecutive groups of eight elements, a thread four of them, 256 apart:
    // every load instruction of a wave reads 256 contiguous bytes of codes (at 4 bits), every store
    // writes 1 KiB, and a thread has four independent chains in flight
    const int per_row = K / 8;
    const float offset = -(float)(levels - 1);
    const uint32_t field = (1u << cb) - 1u;
#pragma unroll
    for (int part = 0; part < 4; ++part) {
    const int64_t g = (int64_t)blockIdx.x * 1024 + part * 256 + threadIdx.x;   // group of eight elements
    if (g >= groups)
        continue;
    const int64_t row = g / per_row;
    const uint8_t *src = codes + g * cb;
    uint32_t bits = 0;
    if (cb == 4) {
        bits = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(src));
    } else {
        for (int byte = 0; byte < cb; ++byte)
            bits |= (uint32_t)src[byte] << (8 * byte);
    }
    const float s = scales[row];
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t c = (bits >> (e * cb)) & field;
        if (levels == 0) {
            // magnitudes 0 .5 1 1.5 | 2 3 4 6: index < 4 is index / 2, else (2 + (index & 1)) * 2^((index >> 1) - 2)
            const uint32_t i = c & 7u;
            const float mag = i < 4u ? 0.5f * (float)i : (float)((2u + (i & 1u)) << ((i >> 1) - 2u));
            v[e] = __fmul_rn(s, (c & 8u) ? -mag : mag);
        } else {
            v[e] = __fmul_rn(s, __fmaf_rn((float)c, 2.0f, offset));
        }
    }
    *reinterpret_cast<uint4 *>(qhat + g * 8) = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]),
                                                          pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
    }
}

// Work is counted in (tile, step) units: tile t owns the units [t * steps, (t + 1) * steps) and
// workgroup b (in XCD-major order) the units [b * per_block, (b + 1) * per_block).  With
// per_block = steps every workgroup computes one whole tile.  When the tiles do not fill the CUs
// evenly the launcher hands every CU the same number of units instead; a workgroup then computes
// one segment per tile its range touches, and a segment that is not a whole tile leaves its fp32
// accumulators in partial-tile slot 2 b (segment continues a tile) or 2 b + 1 (segment starts one)
// of the workspace for grad_gemm_fixup_kernel to add up.  A slot is [wave][accumulator quad 0..63][lane] float4.
//
// Workgroups that are phase_period apart in that order walk through their tiles at the same
// contraction position all the time, and with the tiles numbered along the longer side of the tile
// grid (a run of neighbours shares one operand panel, and the longer the run, the more often two
// such workgroups fall into the same one) they tend to work on tiles of one tile-row or
// tile-column, that is on the same operand rows at the same moment.  Such
// workgroups are placed on one XCD (hardware deals workgroup ids out to the eight XCDs in turn) so
// that they share the fetch through that XCD's L2.  phase_period = 0: whole tiles, all in phase.
constexpr int kSlotQuads = 4 * 64 * 64;   // float4 per partial tile (256 KiB)

__device__ __forceinline__ void tile_origin(int tile, int tiles_r, int tiles_k, int phase_period, int &r0,
                                            int &k0)
{
    if (phase_period != 0) {   // split tiles: plain order along the longer side of the tile grid
        if (tiles_k > tiles_r) {
            r0 = (tile / tiles_k) * GT;
            k0 = (tile % tiles_k) * GT;
        } else {
            r0 = (tile % tiles_r) * GT;
            k0 = (tile / tiles_r) * GT;
        }
        return;
    }
    // four tile-rows deep, column by column: neighbours in the order share operand rows in L2
    const int band = tile / (4 * tiles_k);
    const int band_rows = min(4, tiles_r - band * 4);
    const int in_band = tile - band * 4 * tiles_k;
    r0 = (band * 4 + in_band % band_rows) * GT;
    k0 = (in_band / band_rows) * GT;
}

/*
 * LDS layouts of one operand of one step (16 KiB), both free of bank conflicts for the reads below.
 *   row form  [256 rows][4 chunks of 8 contraction elements]: chunk c of row r sits at chunk
 *             c ^ ((r >> 2) & 3).  Lane l of a 128-bit fragment read takes row l % 32 and chunk
 *             2 ks + l / 32 of k-step ks.
 *   column form [32 contraction rows][32 chunks of 8 columns]: chunk c of contraction row q sits at
 *             chunk c ^ ((q & 3) << 2).  A transposing 64-bit read works on 16 lanes: lanes 4 a ..
 *             4 a + 3 point at contraction row a of a block of four, sixteen columns wide, and lane
 *             i receives column i of it (four contraction elements).  Two such reads give a lane
 *             its eight contraction elements of one matrix-instruction operand.
 * A transfer instruction moves 1 KiB (lane l to offset 16 l): sixteen rows of the row form, two
 * contraction rows of the column form; each lane fetches the chunk that belongs in its slot.
 */
/*
 * MODE 0: out[M, K] = dy[M, N] what[N, K]        left = dy rows (row form),     right = expanded [c][k]
 * MODE 1: out[N, K] = dy[M, N]^T xhat[M, K]      left = dy columns (column form), right = expanded [c][k]
 * MODE 2: out[M, N] = x[M, K] what[N, K]^T       left = x rows (row form),       right = expanded rows
 *         (row form: the weight-only forward product, contraction over the expanded matrix's columns)
 * `left` has row pitch ld_left elements, the expanded operand ld_right, `out` is [R, K] (K columns).
 * R and K need not be whole tiles: the transfers of an edge tile fetch the last rows or columns
 * that exist in place of those that do not (results of those positions are never stored).
 */
constexpr int kSpreadModes = 5;   // bit m: MODE m spreads its transfers over the whole step (measured, see below)

template <int MODE, int STAGES>
__global__ __launch_bounds__(kGemmThreads, 1) void grad_gemm_tile_kernel(
    const uint16_t *__restrict__ dy, int64_t ld_dy, const uint16_t *__restrict__ qhat, int64_t ld_right,
    int C, int R, int K, int tiles_r, int tiles_k, int per_block, int phase_period, uint16_t *__restrict__ out,
    float4 *__restrict__ partial)
{
    constexpr bool TRANSPOSED = MODE == 1;   // left operand in column form
    constexpr bool RIGHT_ROWS = MODE == 2;   // right operand in row form
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    static_assert(STAGES * kGStage >= kParkBytes, "the epilogue reuses the stages");

    const int steps = C / GC;
    const int64_t total_units = (int64_t)tiles_r * tiles_k * steps;
    int block;
    if (phase_period != 0) {
        // XCD x holds the phase classes x c .. x c + c - 1 (c = phase_period / 8) of every period
        const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3, classes = phase_period >> 3;
        block = (idx / classes) * phase_period + xcd * classes + idx % classes;
    } else {
        block = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);   // one contiguous run per XCD
    }
    const int64_t unit_begin = (int64_t)block * per_block;
    const int64_t unit_end = min(unit_begin + per_block, total_units);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int wr = wave >> 1, wc = wave & 1;
    const int lm = lane & 31, lh = lane >> 5;
    const int l16 = lane & 15, lg = lane >> 4;
    const uint32_t smem_addr = lds_address(smem);

    // byte advance per step
    const int64_t left_step = TRANSPOSED ? (int64_t)GC * ld_dy * 2 : (int64_t)GC * 2;
    const int64_t right_step = RIGHT_ROWS ? (int64_t)GC * 2 : (int64_t)GC * ld_right * 2;

    // Fragment reads, byte offsets from the operand's place in a stage.
    //   row form, fragment i, k-step ks:      row_off[ks] + 2048 i
    //   column form, fragment j, k-step ks, half t:  col_off[j] + 512 (16 ks + 4 t)
    // (column form: lane group g = l / 16 covers columns 16 (g % 2) .. + 16 and contraction rows
    //  8 (g / 2) .. of the k-step; lane i of the group points at row i / 4, columns 4 (i % 4) ..)
    auto column_offsets = [&](int w, uint32_t (&off)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int crow = 8 * (lg >> 1) + (l16 >> 2);
            const int chunk = ((4 * w + (j ^ (l16 >> 2))) << 2) + 2 * (lg & 1) + ((l16 >> 1) & 1);
            off[j] = (uint32_t)(crow * 512 + chunk * 16 + 8 * (l16 & 1));
        }
    };
    auto row_offsets = [&](int w, uint32_t (&off)[4]) {
        const int x = (lm >> 2) & 3;
        off[0] = (uint32_t)((w * 128 + lm) * 64 + ((lh ^ x) << 4));
        off[1] = (uint32_t)((w * 128 + lm) * 64 + (((2 + lh) ^ x) << 4));
        off[2] = off[3] = 0;
    };
    uint32_t left_off[4], right_off[4];
    if (RIGHT_ROWS)
        row_offsets(wc, right_off);
    else
        column_offsets(wc, right_off);
    if (TRANSPOSED)
        column_offsets(wr, left_off);
    else
        row_offsets(wr, left_off);

    for (int64_t unit = unit_begin; unit < unit_end;) {
    const int tile = (int)(unit / steps);
    const int s_begin = (int)(unit - (int64_t)tile * steps);
    const int s_end = (int)min((int64_t)steps, unit_end - (int64_t)tile * steps);
    unit += s_end - s_begin;
    int r0, k0;
    tile_origin(tile, tiles_r, tiles_k, phase_period, r0, k0);
    // Transfers: piece q (0..3) of an operand is the 1 KiB at offset (4 q + wave) KiB.  Per-lane
    // byte offsets from the operand's position of the step:
    //   row form:    row 16 (4 q + wave) + l / 4, chunk (l % 4) ^ ((l / 16) & 3)
    //   column form: contraction row 2 (4 q + wave) + l / 32, chunk (l % 32) ^ ((2 wave + l / 32) & 3) << 2
    // with rows and columns beyond the output's edge replaced by the last ones inside it.
    uint32_t left_voff[4], right_voff[4];
    {
        const int rows_left = R - r0, cols_left = K - k0;   // what exists of this tile: >= 64, multiples of 8
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int piece = 4 * q + wave;
            const int crow = 2 * piece + lh;
            const int column = ((lane & 31) ^ ((crow & 3) << 2)) * 8;    // first of the chunk's eight columns
            const int row_form_row = 16 * piece + (lane >> 2);
            const uint32_t row_form_chunk = (uint32_t)(((lane & 3) ^ ((lane >> 4) & 3)) << 4);
            right_voff[q] = RIGHT_ROWS ? (uint32_t)min(row_form_row, cols_left - 1) * (uint32_t)ld_right * 2u + row_form_chunk
                                       : (uint32_t)crow * (uint32_t)ld_right * 2u + (uint32_t)min(column, cols_left - 8) * 2u;
            left_voff[q] = TRANSPOSED ? (uint32_t)crow * (uint32_t)ld_dy * 2u + (uint32_t)min(column, rows_left - 8) * 2u
                                      : (uint32_t)min(row_form_row, rows_left - 1) * (uint32_t)ld_dy * 2u + row_form_chunk;
        }
    }
    // operand positions of contraction step 0 (wave-uniform)
    const char *left_base = reinterpret_cast<const char *>(TRANSPOSED ? dy + r0 : dy + (int64_t)r0 * ld_dy);
    const char *right_base = reinterpret_cast<const char *>(RIGHT_ROWS ? qhat + (int64_t)k0 * ld_right : qhat + k0);

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0.0f;

    // eight transfers per wave fill the stage at LDS byte address `stage` with contraction step `step`
    auto transfer = [&](auto pc, uint32_t stage, int step) {
        constexpr int p = decltype(pc)::value;
        const int at = min(step, s_end - 1);   // past the end: a valid step again, never used
        if constexpr (p < 4)
            lds_dma16(left_base + at * left_step, left_voff[p], stage + (4 * p + wave_u) * 1024);
        else
            lds_dma16(right_base + at * right_step, right_voff[p - 4],
                      stage + kOperandBytes + (4 * (p - 4) + wave_u) * 1024);
    };

    // the same from operand positions that the caller keeps up to date
    // (`wave_stage`: LDS byte address of the stage plus 1024 * wave)
    auto transfer_from = [&](auto pc, uint32_t wave_stage, const char *left_at, const char *right_at) {
        constexpr int p = decltype(pc)::value;
        if constexpr (p < 4)
            lds_dma16_at<4096 * p>(left_at, left_voff[p], wave_stage);
        else
            lds_dma16_at<kOperandBytes + 4096 * (p - 4)>(right_at, right_voff[p - 4], wave_stage);
    };

    // fragments as halves of four contraction elements: [k-step][fragment][half]
    v4bf lf[2][4][2], rf[2][4][2];
    // read number n of k-step ks out of `stage`, in the order the matrix instructions want them
    auto load_frag = [&](auto nc, const uint8_t *stage, auto ksc) {
        constexpr int ks = decltype(ksc)::value;
        constexpr ReadOp op = (MODE == 1 ? kReadsTransposed : MODE == 0 ? kReadsPlain : kReadsRows)[decltype(nc)::value];
        if constexpr (op.half < 0) {
            const uint32_t off = (op.left ? left_off[ks] : kOperandBytes + right_off[ks]) + 2048 * op.idx;
            const v8bf v = *reinterpret_cast<const v8bf *>(stage + off);
            if constexpr (op.left) {
                lf[ks][op.idx][0] = __builtin_shufflevector(v, v, 0, 1, 2, 3);
                lf[ks][op.idx][1] = __builtin_shufflevector(v, v, 4, 5, 6, 7);
            } else {
                rf[ks][op.idx][0] = __builtin_shufflevector(v, v, 0, 1, 2, 3);
                rf[ks][op.idx][1] = __builtin_shufflevector(v, v, 4, 5, 6, 7);
            }
        } else {
            const uint32_t off = (op.left ? left_off[op.idx] : kOperandBytes + right_off[op.idx]) +
                                 512 * (16 * ks + 4 * op.half);
            const v4bf v = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                (__attribute__((address_space(3))) v4bf *)(stage + off));
            if constexpr (op.left)
                lf[ks][op.idx][op.half] = v;
            else
                rf[ks][op.idx][op.half] = v;
        }
    };
    constexpr int kReads = MODE == 1 ? 16 : MODE == 0 ? 12 : 8;

    // Ring of STAGES stages: while step s is multiplied out of stage s % STAGES, the transfers of the
    // next steps are in flight or done.  Two ways to refill:
    //   late   the transfers of step s + STAGES - 1 go into the stage that step s - 1 has left, which is
    //          free once every wave has passed this step's barrier: second half of the step only;
    //   spread the transfers of step s + STAGES - 2 go into the stage that step s - 2 has left, free
    //          since the previous step's barrier: one transfer every fourth matrix instruction, all
    //          through the step, at the price of one step less of look-ahead.
    // Spreading is 1-3 % faster when the left operand is in row form (G_x: 320 instead of 328 us on
    // one box, 334 instead of 338 on another) and 0-1 % slower when both operands are in column form.
    constexpr bool kSpread = kSpreadModes & (1 << MODE);
    constexpr int kAhead = kSpread ? STAGES - 2 : STAGES - 1;   // steps in flight beyond the current one
    static_for<kAhead>([&](auto sc) {
        static_for<8>([&](auto pc) {
            transfer(pc, smem_addr + decltype(sc)::value * kGStage, s_begin + decltype(sc)::value);
        });
    });
    wait_vmcnt<8 * (kAhead - 1)>();
    __builtin_amdgcn_s_barrier();
    static_for<kReads>([&](auto nc) { load_frag(nc, smem, std::integral_constant<int, 0>{}); });

    // Scalar bookkeeping of a step is kept to additions and selects (one wave per SIMD: a chain of
    // dependent scalar instructions between two matrix instructions is time the matrix pipe idles):
    // byte offsets of the current stage and of the stage being refilled, and the operands' positions
    // at the step being fetched, min(step + kAhead, s_end - 1).
    constexpr int kRing = STAGES * kGStage;
    int cur_off = 0;
    int refill_off = (kSpread ? kAhead : STAGES - 1) * kGStage;
    const char *left_fetch = left_base + (int64_t)min(s_begin + kAhead, s_end - 1) * left_step;
    const char *right_fetch = right_base + (int64_t)min(s_begin + kAhead, s_end - 1) * right_step;
    for (int step = s_begin; step < s_end; ++step) {
        const uint8_t *cur_stage = smem + cur_off;
        const int nxt_off = cur_off + kGStage == kRing ? 0 : cur_off + kGStage;
        const uint8_t *nxt_stage = smem + nxt_off;
        const uint32_t refill = smem_addr + refill_off + wave_u * 1024;
        // 32 matrix instructions; each is followed by one slice of the other work, pinned in place:
        //    0..15  fragment reads of the step's second k-step
        //   15      transfers of step + 1 have landed (all but the newer groups), barrier
        //   16..31  fragment reads of the next step's first k-step
        //   16, 18, .. 30 (late) or 0, 4, .. 28 (spread)  transfers of a later step (never back to back:
        //           a wave issues in order, and a transfer that finds the memory pipeline's queue full
        //           holds up the MFMAs behind it)
        static_for<32>([&](auto kc) {
            constexpr int k = decltype(kc)::value;
            constexpr int ks = k >> 4, i = (k >> 2) & 3, j = k & 3;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_shufflevector(rf[ks][j][0], rf[ks][j][1], 0, 1, 2, 3, 4, 5, 6, 7),
                __builtin_shufflevector(lf[ks][i][0], lf[ks][i][1], 0, 1, 2, 3, 4, 5, 6, 7), acc[i][j], 0, 0, 0);
            if constexpr (kSpread && (k & 3) == 0)
                transfer_from(std::integral_constant<int, k / 4>{}, refill, left_fetch, right_fetch);
            if constexpr (k < 16) {
                if constexpr (k < kReads)
                    load_frag(std::integral_constant<int, k>{}, cur_stage, std::integral_constant<int, 1>{});
                if constexpr (k == 15) {
                    // all transfers of step + 1 have landed: what may still be in flight are the groups of
                    // the steps after it and, when spread, the four transfers this step has issued so far
                    wait_vmcnt<8 * (kAhead - 2) + (kSpread ? 4 : 0)>();
                    __builtin_amdgcn_s_barrier();
                }
            } else {
                if constexpr (k - 16 < kReads)
                    load_frag(std::integral_constant<int, k - 16>{}, nxt_stage, std::integral_constant<int, 0>{});
                if constexpr (!kSpread && (k & 1) == 0)
                    transfer_from(std::integral_constant<int, (k - 16) / 2>{}, refill, left_fetch, right_fetch);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        cur_off = nxt_off;
        refill_off = refill_off + kGStage == kRing ? 0 : refill_off + kGStage;
        if (step + 1 + kAhead < s_end) {
            left_fetch += left_step;
            right_fetch += right_step;
        }
    }
    wait_vmcnt<0>();   // the look-ahead transfers still write into the stages

    // Epilogue.  A segment that is not a whole tile leaves its accumulators as they are, in fp32.
    __syncthreads();
    if (s_begin != 0 || s_end != steps) {
        float4 *slot = partial + ((int64_t)(2 * block + (s_begin == 0 ? 1 : 0)) * 4 + wave) * (64 * 64) + lane;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    __builtin_nontemporal_store(
                        v4f{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]},
                        reinterpret_cast<v4f *>(slot + ((i * 4 + j) * 4 + q) * 64));
        continue;   // LDS untouched since the barrier
    }
    // Each accumulator tile is a transposed output tile: lane l holds output row l % 32
    // and, in register r, output column 8 (r / 4) + 4 (l / 32) + r % 4.  Each wave parks its
    // 128 x 128 block as bf16 in its own 32 KiB of LDS (chunks swizzled by row) and writes it out as
    // 256-byte row segments.
    uint8_t *park = smem + wave * 32768;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = i * 32 + lm;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = j * 32 + 8 * q + 4 * lh;
                const int chunk = (col >> 3) ^ (row & 15);
                *reinterpret_cast<uint2 *>(park + row * 256 + chunk * 16 + (col & 4) * 2) =
                    make_uint2(pack_bf16(acc[i][j][4 * q + 0], acc[i][j][4 * q + 1]),
                               pack_bf16(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]));
            }
        }
    }
    uint16_t *out_base = out + (int64_t)(r0 + wr * 128) * K + k0 + wc * 128;
#pragma unroll 4
    for (int pass = 0; pass < 32; ++pass) {
        const int row = pass * 4 + (lane >> 4);
        const int c = lane & 15;
        const uint4 v = *reinterpret_cast<const uint4 *>(park + row * 256 + ((c ^ (row & 15)) << 4));
        if (r0 + wr * 128 + row < R && k0 + wc * 128 + c * 8 < K)
            *reinterpret_cast<uint4 *>(out_base + (int64_t)row * K + c * 8) = v;
    }
    __syncthreads();   // the next segment's first stage overwrites the parked block
    }
}

/*
 * Adds up the partial tiles of every tile that more than one workgroup worked on (in workgroup
 * order, so the sum does not depend on timing) and writes the bf16 result.  One wave per 32 x 32
 * accumulator tile: quadrant = the 128 x 128 block of one wave of the main kernel, (i, j) = the
 * accumulator tile in it, j = the wave of a workgroup.  (Sixty-four waves per output tile, and
 * several partial tiles in flight per lane: a small output split over many CUs has few tiles and
 * many partial tiles each, and the sum is a chain of loads.)
 */
__global__ __launch_bounds__(256) void grad_gemm_fixup_kernel(const float4 *__restrict__ partial, int steps,
                                                             int per_block, int phase_period, int R, int K,
                                                             int tiles_r, int tiles_k,
                                                             uint16_t *__restrict__ out)
{
    __shared__ __attribute__((aligned(16))) uint8_t park_all[4 * 2048];
    const int tile = blockIdx.x >> 4, quadrant = (blockIdx.x >> 2) & 3, i = blockIdx.x & 3, j = threadIdx.x >> 6;
    uint8_t *park = park_all + j * 2048;
    const int64_t first_unit = (int64_t)tile * steps, last_unit = first_unit + steps - 1;
    const int b_first = (int)(first_unit / per_block), b_last = (int)(last_unit / per_block);
    if (b_first == b_last)
        return;   // computed whole by one workgroup, already written
    const int lane = threadIdx.x & 63;
    const int lm = lane & 31, lh = lane >> 5;
    float4 sum[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
        sum[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll 4
    for (int b = b_first; b <= b_last; ++b) {
        const bool continues = (int64_t)b * per_block > first_unit;
        const float4 *slot = partial + ((int64_t)(2 * b + (continues ? 0 : 1)) * 4 + quadrant) * (64 * 64) + lane;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 v = slot[((i * 4 + j) * 4 + q) * 64];
            sum[q].x += v.x; sum[q].y += v.y; sum[q].z += v.z; sum[q].w += v.w;
        }
    }
    // park the 32 x 32 tile as bf16 (row lm, 64 bytes), write 16-byte chunks: 4 per row, 2 passes
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int col = 8 * q + 4 * lh;
        *reinterpret_cast<uint2 *>(park + lm * 64 + col * 2) =
            make_uint2(pack_bf16(sum[q].x, sum[q].y), pack_bf16(sum[q].z, sum[q].w));
    }
    __syncthreads();
    int r0, k0;
    tile_origin(tile, tiles_r, tiles_k, phase_period, r0, k0);
    const int row0 = r0 + (quadrant >> 1) * 128 + i * 32, col0 = k0 + (quadrant & 1) * 128 + j * 32;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int prow = pass * 16 + (lane >> 2);
        const int c = lane & 3;
        const uint4 v = *reinterpret_cast<const uint4 *>(park + prow * 64 + c * 16);
        if (row0 + prow < R && col0 + c * 8 < K)
            *reinterpret_cast<uint4 *>(out + (int64_t)(row0 + prow) * K + col0 + c * 8) = v;
    }
}

}  // namespace

namespace {

constexpr int kStages = 5;
constexpr int kLds = kStages * kGStage;

// How a call is carried out: which kernels, how the tiles are dealt out, what scratch it needs.
struct GradGemmPlan {
    bool covered;      // some kernel handles the shape
    bool tile_path;    // the 256 x 256 tile kernels (else the small-shape kernel, no scratch)
    bool split;        // tiles split over the CUs, partial tiles summed by the fix-up kernel
    int tiles_r, tiles_k, steps, blocks, per_block, phase_period;
    int64_t out_rows, out_cols, contraction, q_rows, ld_left;
    size_t expanded_bytes, partial_bytes;
};

GradGemmPlan plan_grad_gemm(int which, bool fp4, int64_t M, int64_t N, int64_t K, int cus)
{
    GradGemmPlan p = {};
    // which = 0: out[M, K] = dy what;  1: out[N, K] = dy^T xhat;  2: out[M, N] = x what^T (weight-only)
    p.out_rows = which == 1 ? N : M;
    p.out_cols = which == 2 ? N : K;
    p.contraction = which == 0 ? N : which == 1 ? M : K;
    p.q_rows = which == 1 ? M : N;          // rows of the code-packed operand [q_rows, K]
    p.ld_left = which == 2 ? K : N;
    // the tile kernels: edge tiles may be partial (every size is a multiple of 64), offsets are 32-bit
    p.tile_path = p.out_rows >= GT / 2 && p.out_cols >= GT / 2 && (p.contraction % GC) == 0 &&
                  p.out_rows * p.out_cols < ((int64_t)1 << 31) &&
                  std::max(M, N) * std::max(K, N) < ((int64_t)1 << 30);
    p.covered = p.tile_path || !(which == 2 || fp4);   // only the tile kernels know these two forms
    if (!p.tile_path)
        return p;
    p.tiles_r = (int)((p.out_rows + GT - 1) / GT);
    p.tiles_k = (int)((p.out_cols + GT - 1) / GT);
    p.steps = (int)(p.contraction / GC);
    const int tiles = p.tiles_r * p.tiles_k;
    // One workgroup per CU at a time.  When rounds of whole tiles would leave CUs idle, every CU
    // can get the same share of (tile, step) units instead, the split tiles being summed by a
    // second, small kernel.  That pays when the steps saved outweigh the partial tiles written
    // and read back (two 256 KiB slots per workgroup at most, one per tile at least).
    const int rounds = cus > 0 ? (tiles + cus - 1) / cus : 0;
    const int64_t units = (int64_t)tiles * p.steps;
    // measured on this kernel: 0.6 us per step, 0.08 us per partial tile written and read, 10 us for the second launch
    const double whole_cost = 0.6 * rounds * p.steps;
    const double split_cost = cus > 0 ? 0.6 * (double)((units + cus - 1) / cus) + 0.08 * (cus + tiles) + 10.0 : 0.0;
    p.split = cus >= 8 && split_cost < whole_cost && units >= 4 * (int64_t)cus;
    p.blocks = (tiles + 7) / 8 * 8;
    p.per_block = p.steps;
    p.phase_period = 0;
    if (!p.split && cus >= 8 && tiles > cus) {
        // more whole tiles than compute units: one workgroup per unit walks over several tiles, so that
        // no tile after the first waits for a workgroup to be dispatched (7 us per tile here)
        p.blocks = cus;
        p.per_block = (tiles + cus - 1) / cus * p.steps;
    }
    if (p.split) {
        p.blocks = cus;
        p.per_block = (int)((units + p.blocks - 1) / p.blocks);
        // workgroups b and b + period are at the same contraction position at all times
        const int period = p.steps / std::gcd(p.per_block, p.steps);
        p.phase_period = (period % 8 == 0 && p.blocks % period == 0) ? period : 8;
        if (p.blocks % p.phase_period != 0)
            p.phase_period = p.blocks;
    }
    p.expanded_bytes = ((size_t)p.q_rows * K * 2 + 255) / 256 * 256;
    p.partial_bytes = p.split ? (size_t)2 * p.blocks * kSlotQuads * sizeof(float4) : 0;
    return p;
}

}  // namespace

int64_t grad_gemm_workspace_bytes(int which, bool fp4, int64_t M, int64_t N, int64_t K, int cus)
{
    if (M == 0 || N == 0 || K == 0)
        return 0;
    const GradGemmPlan p = plan_grad_gemm(which, fp4, M, N, K, cus);
    if (!p.covered)
        return -1;
    return p.tile_path ? (int64_t)(p.expanded_bytes + p.partial_bytes) : 0;
}

hipError_t prepare_grad_gemm_kernels()
{
    hipError_t err = allow_dynamic_lds(reinterpret_cast<const void *>(grad_gemm_tile_kernel<0, kStages>), kLds);
    if (err == hipSuccess)
        err = allow_dynamic_lds(reinterpret_cast<const void *>(grad_gemm_tile_kernel<1, kStages>), kLds);
    if (err == hipSuccess)
        err = allow_dynamic_lds(reinterpret_cast<const void *>(grad_gemm_tile_kernel<2, kStages>), kLds);
    return err;
}

hipError_t launch_grad_gemm(const GradGemmArgs &a, hipStream_t stream)
{
    if (a.M == 0 || a.N == 0 || a.K == 0)
        return hipSuccess;
    const int levels = a.fp4 ? 0 : 1 << a.bits;
    const auto *dy = static_cast<const uint16_t *>(a.dy);
    auto *out = static_cast<uint16_t *>(a.out);
    const GradGemmPlan p = plan_grad_gemm(a.which, a.fp4, a.M, a.N, a.K, device_compute_units());
    if (!p.covered)
        return hipErrorInvalidValue;
    if (p.tile_path) {
        if (a.workspace == nullptr || (size_t)a.workspace_bytes < p.expanded_bytes + p.partial_bytes)
            return hipErrorInvalidValue;
        hipError_t err = prepare_grad_gemm_kernels();
        if (err != hipSuccess)
            return err;
        // the caller's scratch: the expanded operand, then the partial tiles
        char *memory = static_cast<char *>(a.workspace);
        auto *qhat = reinterpret_cast<uint16_t *>(memory);
        auto *partial = p.split ? reinterpret_cast<float4 *>(memory + p.expanded_bytes) : nullptr;
        const int tiles_r = p.tiles_r, tiles_k = p.tiles_k, per_block = p.per_block, phase_period = p.phase_period;
        const int64_t ld_left = p.ld_left, contraction = p.contraction, out_rows = p.out_rows, out_cols = p.out_cols;

        const int64_t groups = p.q_rows * a.K / 8;
        hipLaunchKernelGGL(expand_codes_kernel, dim3((unsigned)((groups + 1023) / 1024)), dim3(256), 0, stream,
                           a.q_codes, a.q_scales, levels, a.cb, (int)a.K, groups, qhat);
        err = hipGetLastError();
        if (err != hipSuccess)
            return err;
        const dim3 grid((unsigned)p.blocks), block(kGemmThreads);
        if (a.which == 0)
            hipLaunchKernelGGL((grad_gemm_tile_kernel<0, kStages>), grid, block, kLds, stream, dy, ld_left, qhat,
                               a.K, (int)contraction, (int)out_rows, (int)out_cols, tiles_r, tiles_k, per_block,
                               phase_period, out, partial);
        else if (a.which == 1)
            hipLaunchKernelGGL((grad_gemm_tile_kernel<1, kStages>), grid, block, kLds, stream, dy, ld_left, qhat,
                               a.K, (int)contraction, (int)out_rows, (int)out_cols, tiles_r, tiles_k, per_block,
                               phase_period, out, partial);
        else
            hipLaunchKernelGGL((grad_gemm_tile_kernel<2, kStages>), grid, block, kLds, stream, dy, ld_left, qhat,
                               a.K, (int)contraction, (int)out_rows, (int)out_cols, tiles_r, tiles_k, per_block,
                               phase_period, out, partial);
        err = hipGetLastError();
        if (err == hipSuccess && p.split) {
            hipLaunchKernelGGL(grad_gemm_fixup_kernel, dim3((unsigned)(tiles_r * tiles_k * 16)), dim3(256), 0, stream,
                               partial, p.steps, per_block, phase_period, (int)out_rows, (int)out_cols, tiles_r,
                               tiles_k, out);
            err = hipGetLastError();
        }
        return err;
    }
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
