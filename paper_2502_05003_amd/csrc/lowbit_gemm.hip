// Low-bit integer GEMM with a dequantizing bf16 epilogue: y = xhat_h what_h^T computed on the
// packed codes (Algorithm 1, last step; Sec. 5 "Kernel Overview" stage 3 of arXiv 2502.05003).
// The codes are widened to signed bytes proportional to the odd integers u = 2c - (L - 1) (on their
// way into LDS in the general kernel, at the consumer in the tile kernels) and contracted on the
// INT8 matrix cores; acc = sum_k u_a u_b is exact in int32.
#include "gemm_tile.h"
#include "quest_internal.h"

namespace quest {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 128;          // block tile rows (activations)
constexpr int BN = 128;          // block tile columns (weights)
constexpr int BK = 64;           // contraction elements per main-loop step
constexpr int kThreads = 256;    // 4 waves in a 2 x 2 arrangement, 64 x 64 outputs per wave
constexpr int kRowStride = 80;   // LDS bytes per tile row: 64 payload + 16 pad (conflict-free b128 reads)

/*
 * Widen 32 consecutive codes (CB bits each, little-endian) to 32 signed bytes u = 2c - (L - 1),
 * four per dword.  The order of the 32 bytes is a fixed permutation of the element order; both
 * GEMM operands go through this same function, so products still pair element k with element k.
 */
template <int CB>
__device__ __forceinline__ void widen32(const uint32_t *packed, uint32_t bias, uint32_t (&out)[8])
{
    uint32_t c[8];
    if constexpr (CB == 4) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            c[2 * i] = packed[i] & 0x0f0f0f0fu;
            c[2 * i + 1] = (packed[i] >> 4) & 0x0f0f0f0fu;
        }
    } else if constexpr (CB == 2) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int d = 0; d < 4; ++d)
                c[4 * i + d] = (packed[i] >> (2 * d)) & 0x03030303u;
    } else {
#pragma unroll
        for (int d = 0; d < 8; ++d)
            c[d] = (packed[0] >> d) & 0x01010101u;
    }
    // per byte: (2c + 128) - (L - 1), then flip the top bit -> two's complement 2c - (L - 1);
    // every byte stays >= 128 - 15 before the subtraction, so no borrow crosses bytes
#pragma unroll
    for (int i = 0; i < 8; ++i)
        out[i] = (((c[i] << 1) | 0x80808080u) - bias) ^ 0x80808080u;
}

template <int CB>
__global__ __launch_bounds__(kThreads) void lowbit_gemm_kernel(
    const uint8_t *__restrict__ a_codes, const float *__restrict__ a_scales,
    const uint8_t *__restrict__ b_codes, const float *__restrict__ b_scales, int M, int N, int K,
    int levels, uint16_t *__restrict__ y, int64_t ld_y, int32_t *__restrict__ acc_out)
{
    __shared__ __attribute__((aligned(16))) uint8_t a_tile[BM * kRowStride];
    __shared__ __attribute__((aligned(16))) uint8_t b_tile[BN * kRowStride];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

    // staging role: thread -> (tile row, which half of the 64-element step)
    const int ld_row = tid >> 1, ld_half = tid & 1;
    constexpr int kChunkBytes = 32 * CB / 8;             // packed bytes of 32 elements
    constexpr int kChunkWords = kChunkBytes / 4 > 0 ? kChunkBytes / 4 : 1;
    const int64_t row_bytes = (int64_t)K * CB / 8;
    const int a_row = min(m0 + ld_row, M - 1), b_row = min(n0 + ld_row, N - 1);
    const uint8_t *a_src = a_codes + a_row * row_bytes + ld_half * kChunkBytes;
    const uint8_t *b_src = b_codes + b_row * row_bytes + ld_half * kChunkBytes;
    const uint32_t bias = (uint32_t)(levels - 1) * 0x01010101u;

    v16i acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0;

    auto fetch = [&](const uint8_t *src, uint32_t (&w)[kChunkWords]) {
        if constexpr (CB == 4) {
            const uint4 v = *reinterpret_cast<const uint4 *>(src);
            w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
        } else if constexpr (CB == 2) {
            const uint2 v = *reinterpret_cast<const uint2 *>(src);
            w[0] = v.x; w[1] = v.y;
        } else {
            w[0] = *reinterpret_cast<const uint32_t *>(src);
        }
    };

    uint32_t a_next[kChunkWords], b_next[kChunkWords];
    fetch(a_src, a_next);
    fetch(b_src, b_next);

    for (int k0 = 0; k0 < K; k0 += BK) {
        uint32_t a_wide[8], b_wide[8];
        widen32<CB>(a_next, bias, a_wide);
        widen32<CB>(b_next, bias, b_wide);
        __syncthreads();  // previous step's MFMA reads are done
        uint4 *a_dst = reinterpret_cast<uint4 *>(a_tile + ld_row * kRowStride + ld_half * 32);
        uint4 *b_dst = reinterpret_cast<uint4 *>(b_tile + ld_row * kRowStride + ld_half * 32);
        a_dst[0] = make_uint4(a_wide[0], a_wide[1], a_wide[2], a_wide[3]);
        a_dst[1] = make_uint4(a_wide[4], a_wide[5], a_wide[6], a_wide[7]);
        b_dst[0] = make_uint4(b_wide[0], b_wide[1], b_wide[2], b_wide[3]);
        b_dst[1] = make_uint4(b_wide[4], b_wide[5], b_wide[6], b_wide[7]);
        if (k0 + BK < K) {  // prefetch the next step while this one is multiplied
            fetch(a_src + (int64_t)(k0 + BK) * CB / 8, a_next);
            fetch(b_src + (int64_t)(k0 + BK) * CB / 8, b_next);
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            v4i a_frag[2], b_frag[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = wm * 64 + i * 32 + (lane & 31);
                a_frag[i] = *reinterpret_cast<const v4i *>(a_tile + row * kRowStride + s * 32 +
                                                           (lane >> 5) * 16);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int row = wn * 64 + j * 32 + (lane & 31);
                b_frag[j] = *reinterpret_cast<const v4i *>(b_tile + row * kRowStride + s * 32 +
                                                           (lane >> 5) * 16);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a_frag[i], b_frag[j],
                                                                      acc[i][j], 0, 0, 0);
        }
    }

    // Epilogue.  In the 32 x 32 accumulator tile, lane l holds column l % 32 and, in register r,
    // row 8 (r / 4) + 4 (l / 32) + r % 4.
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn * 64 + j * 32 + (lane & 31);
        if (n >= N)
            continue;
        const float sb = b_scales[n];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (m >= M)
                    continue;
                const int a = acc[i][j][r];
                if (acc_out)
                    acc_out[(int64_t)m * N + n] = a;
                if (y)
                    y[(int64_t)m * ld_y + n] =
                        (uint16_t)float_to_bf16_bits(__fmul_rn(__fmul_rn((float)a, a_scales[m]), sb));
            }
        }
    }
}


// ------------------------------------------------------------------------------------------
// Main kernel for b = 4 and b = 3 (nibble containers).  Workgroup tile 256 (M) x 128 (N), four waves of 128 x 64 (eight 32 x 32
// accumulator tiles each), 128 contraction elements per step, three LDS stages, two workgroups per
// CU so that one group's staging, barriers and epilogue hide behind the other's MFMAs.
//
// LDS holds the codes still packed (64 bytes per row and step): the LDS pipe moves 128 bytes per
// clock and CU, and widened bytes would need three quarters of that.  A nibble c moved to the top
// of a byte, with its top bit flipped (c - 8 in two's complement) and bit 3 set below it, is the
// signed byte 16 (c - 8) + 8 = 8 (2c - 15) = 8 u, so widening costs three vector ops per eight
// codes at the consumer.  Both operands carry the factor 8: the MFMAs accumulate
// 64 * sum u_a u_b (below 2^31 for K <= 65536), and the epilogue takes the 64 out exactly.
// ------------------------------------------------------------------------------------------

constexpr int TM = 256, TN = 128, TK = 128;
constexpr int kTileThreads = 256;
constexpr int kRowBytes = TK / 2;                      // packed bytes per tile row and step
constexpr int kStageBytes = (TM + TN) * kRowBytes;     // 24 KiB
constexpr int kStages = 3;
constexpr int kParkBytes = 4 * 128 * 64 * 2;           // epilogue: four waves x 128 x 64 bf16 (reuses the stages)
static_assert(kParkBytes <= kStages * kStageBytes, "the epilogue parks in the stages");
constexpr int kTileLds = kStages * kStageBytes + TN * 4;   // 72 KiB + the tile's weight scales

// 16-byte chunk c (0..3) of tile row `row` lives at chunk c ^ swz(row).  The LDS serves 128-bit
// accesses sixteen lanes at a time over 64 banks (256 bytes): sixteen consecutive rows reading
// the same logical chunk must hit sixteen different 16-byte slots modulo 256 bytes (measured).
__device__ __forceinline__ int swz(int row)
{
    return (row >> 2) & 3;
}

// Eight offset-binary codes c (one packed dword) -> the signed bytes 8 u = 16 (c - 8) + 8 of the
// odd and of the even elements.  With the nibble in the top half of its byte this is one
// three-input bit function of (word, 0xf0f0f0f0, 0x88888888): keep bits 4..6, invert bit 7 (the
// offset-binary -> two's-complement flip), force bit 3, clear bits 0..2.
// For b = 3 (codes 0..7 in the same nibbles, u = 2c - 7) one more shift puts the three bits at the
// top of the byte: (c << 5) with bit 7 inverted and bit 4 forced is 32 (c - 4) + 16 = 16 u; the
// function is the same with (0xe0e0e0e0, 0x90909090), and the products carry 256 instead of 64.
template <int BITS>
__device__ __forceinline__ void widen8(uint32_t w, uint32_t field_mask, int &even, int &odd)
{
    static_assert(BITS == 3 || BITS == 4, "nibble containers only");
    constexpr uint32_t forced = BITS == 4 ? 0x88888888u : 0x90909090u;
    odd = (int)__builtin_amdgcn_bitop3_b32(w << (4 - BITS), field_mask, forced, 0x6A);
    even = (int)__builtin_amdgcn_bitop3_b32(w << (8 - BITS), field_mask, forced, 0x6A);
}

template <int BITS>
__global__ __launch_bounds__(kTileThreads, 2) void lowbit_gemm_tile_kernel(
    const uint8_t *__restrict__ a_codes, const float *__restrict__ a_scales,
    const uint8_t *__restrict__ b_codes, const float *__restrict__ b_scales, int M, int N, int K,
    int tiles_m, int tiles_n, uint16_t *__restrict__ y, int64_t ld_y,
    int32_t *__restrict__ acc_out)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // Workgroup -> tile.  Consecutive workgroup ids go to different XCDs (8 of them, each with
    // its own L2), so give each XCD one contiguous run of tiles, ordered four tile-rows deep:
    // the tiles an XCD works on at a time share a few row panels of A and column panels of B.
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total)
        return;
    const int band = logical / (4 * tiles_n);
    const int band_rows = min(4, tiles_m - band * 4);
    const int in_band = logical - band * 4 * tiles_n;
    const int tile_m = band * 4 + in_band % band_rows;
    const int tile_n = in_band / band_rows;
    const int m0 = tile_m * TM, n0 = tile_n * TN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lm = lane & 31, lh = lane >> 5;

    // Staging: codes go from global memory straight into LDS, 16 bytes per lane.  A wave's 64 lanes
    // fill 1 KiB = 16 tile rows x 64 bytes; lane l lands at offset 16 l, i.e. row l / 4, physical
    // chunk l % 4, so it fetches the logical chunk that belongs there.  Six such pieces per step and
    // wave: rows 64 i + 16 wave .. + 16 of A (i < 4) and of B (i = 4, 5).
    const int st_row = 16 * wave + (lane >> 2);                       // + 64 i
    const int st_chunk = (lane & 3) ^ swz(st_row);                    // swz(row + 64 i) = swz(row)
    const int64_t row_bytes = (int64_t)K / 2;
    uint32_t src_off[6];   // per-thread byte offsets from a_codes / b_codes (rows clamped at the edge)
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        const int row = st_row + 64 * (i < 4 ? i : i - 4);
        const int64_t grow = i < 4 ? min(m0 + row, M - 1) : min(n0 + row, N - 1);
        src_off[i] = (uint32_t)(grow * row_bytes + st_chunk * 16);
    }

    v16i acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0;

    // kept in a vector register (opaque to constant folding) so that widen8 is one instruction
    constexpr int kCarry = BITS == 4 ? 6 : 8;   // log2 of the factor the products carry (8 u or 16 u per operand)
    uint32_t nibble_mask = BITS == 4 ? 0xf0f0f0f0u : 0xe0e0e0e0u;
    asm volatile("" : "+v"(nibble_mask));

    const int steps = K / TK;
    // piece I of contraction step STEP -> stage at LDS byte address STAGE (wave-uniform)
    const uint32_t smem_addr = lds_address(smem);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    // (WAVE_STAGE: LDS byte address of the stage plus this wave's 16 rows)
#define QUEST_DMA(WAVE_STAGE, I, STEP)                                                             \
    lds_dma16_at<((I) < 4 ? 0 : TM * kRowBytes) + 64 * ((I) < 4 ? (I) : (I)-4) * kRowBytes>(         \
        ((I) < 4 ? a_codes : b_codes) + (int64_t)min((STEP), steps - 1) * kRowBytes, src_off[I], (WAVE_STAGE))

    const uint32_t wave_smem = smem_addr + 16 * wave_u * kRowBytes;
    static_for<6>([&](auto i) { QUEST_DMA(wave_smem, decltype(i)::value, 0); });
    static_for<6>([&](auto i) { QUEST_DMA(wave_smem + kStageBytes, decltype(i)::value, 1); });
    // the epilogue's scales, fetched while the first stages are on their way: the weight scales of
    // the tile's columns into their own corner of LDS, this lane's four activation scales into
    // registers (float(64 acc) * (s_a / 64) rounds exactly like float(acc) * s_a)
    float *scale_lds = reinterpret_cast<float *>(smem + kStages * kStageBytes);
    if (tid < TN)
        scale_lds[tid] = b_scales[min(n0 + tid, N - 1)];
    float sa_reg[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        sa_reg[i] = a_scales[min(m0 + wm * 128 + i * 32 + lm, M - 1)] * (1.0f / (float)(1 << kCarry));
    wait_vmcnt<0>();
    __syncthreads();

    // fragment addresses: rows lm + 32 i share bits 2..3, hence one swizzle value per lane;
    // chunk 2 p + lh of a row feeds this lane's share of sub-steps 2 p and 2 p + 1
    const int x = swz(lm);
    const int a_off = (wm * 128 + lm) * kRowBytes;
    const int b_off = TM * kRowBytes + (wn * 64 + lm) * kRowBytes;
    uint4 af[2][4], bf[2][2];   // packed fragments of the two sub-step pairs
    auto load_frag = [&](const uint8_t *stage, int p, int f) {
        const int off = ((2 * p + lh) ^ x) << 4;
        if (f < 4)
            af[p][f] = *reinterpret_cast<const uint4 *>(stage + a_off + f * 32 * kRowBytes + off);
        else
            bf[p][f - 4] = *reinterpret_cast<const uint4 *>(stage + b_off + (f - 4) * 32 * kRowBytes + off);
    };
    static_for<6>([&](auto f) { load_frag(smem, 0, decltype(f)::value); });

    // Widened operands.  A fragment i sits in wa[i % 2] while its two instructions run; the B
    // fragments of sub-step g sit in wb[g % 2][j].  Sub-step g = 2 p + e takes words (x, y) (e = 0)
    // or (z, w) (e = 1) of the packed fragments of pair p.
    v4i wa[2], wb[2][2];
    auto widen_a = [&](auto gc, auto ic) {
        constexpr int g = decltype(gc)::value & 3, i = decltype(ic)::value;
        constexpr int p = g >> 1, e = g & 1;
        int w0, w1, w2, w3;
        widen8<BITS>(e ? af[p][i].z : af[p][i].x, nibble_mask, w0, w1);
        widen8<BITS>(e ? af[p][i].w : af[p][i].y, nibble_mask, w2, w3);
        wa[i & 1] = v4i{w0, w1, w2, w3};
    };
    auto widen_b = [&](auto gc, auto jc) {
        constexpr int g = decltype(gc)::value & 3, j = decltype(jc)::value;
        constexpr int p = g >> 1, e = g & 1;
        int w0, w1, w2, w3;
        widen8<BITS>(e ? bf[p][j].z : bf[p][j].x, nibble_mask, w0, w1);
        widen8<BITS>(e ? bf[p][j].w : bf[p][j].y, nibble_mask, w2, w3);
        wb[g & 1][j] = v4i{w0, w1, w2, w3};
    };
    widen_a(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    widen_b(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    widen_b(std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{});

    // Main loop: 32 MFMAs per step and wave, everything else pinned between them, at most one
    // widening (six vector ops) per MFMA so that the vector unit never has a burst to work off, and
    // every widening at least one MFMA ahead of the first instruction that reads its result (a
    // matrix instruction directly behind the vector op that writes its operand waits).
    //   MFMA k: sub-step g = k / 8, within it s = k % 8 multiplies A fragment s / 2 with B fragment s % 2
    //   after s = 0, 2, 4: widen A1, A2, A3    after s = 5, 6, 7: widen B0, A0, B1 of the next sub-step
    //   k = 0, 3, .. 15  start the transfers of step + 2 into the stage that was read in step - 1
    //               (spread out: a transfer that finds the memory queue full holds up the MFMAs)
    //   k = 2..7    load the packed fragments of pair 1 (first needed after k = 13)
    //   k = 16      wait for this wave's transfers of step + 1 (issued one step ago: all but the six
    //               newest), then the workgroup barrier: step + 1 is complete in LDS
    //   k = 17..22  load the packed fragments of pair 0 of step + 1 in the order of their first use
    //               (B0, A0, B1 are widened after k = 29, 30, 31)
    // Three stages: a transfer has almost two steps to land, and no wave waits on the barrier with
    // an empty MFMA queue.
    int stage_cur = 0;   // byte offsets of the stages holding step, step + 1, step + 2
    int stage_one = kStageBytes, stage_two = 2 * kStageBytes;
    for (int step = 0; step < steps; ++step) {
        const uint8_t *cur = smem + stage_cur;
        const uint8_t *one = smem + stage_one;
        static_for<32>([&](auto kc) {
            constexpr int k = decltype(kc)::value;
            constexpr int g = k >> 3, s = k & 7, i = s >> 1, j = s & 1;
            // weight fragment as the row operand: transposed accumulator tiles
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wb[g & 1][j], wa[i & 1], acc[i][j], 0, 0, 0);
            if constexpr (s == 0 || s == 2 || s == 4)
                widen_a(std::integral_constant<int, g>{}, std::integral_constant<int, s / 2 + 1>{});
            if constexpr (s == 5)
                widen_b(std::integral_constant<int, g + 1>{}, std::integral_constant<int, 0>{});
            if constexpr (s == 6)
                widen_a(std::integral_constant<int, g + 1>{}, std::integral_constant<int, 0>{});
            if constexpr (s == 7)
                widen_b(std::integral_constant<int, g + 1>{}, std::integral_constant<int, 1>{});
            if constexpr (k < 18 && k % 3 == 0)
                QUEST_DMA(wave_smem + stage_two, k / 3, step + 2);
            if constexpr (k >= 2 && k < 8)
                load_frag(cur, 1, k - 2);
            if constexpr (k == 16) {
                wait_vmcnt<6>();
                __builtin_amdgcn_s_barrier();
            }
            if constexpr (k >= 17 && k < 23) {
                constexpr int order[6] = {4, 0, 5, 1, 2, 3};   // B0, A0, B1, A1, A2, A3
                load_frag(one, 0, order[k - 17]);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        const int t = stage_cur;
        stage_cur = stage_one;
        stage_one = stage_two;
        stage_two = t;
    }
    wait_vmcnt<0>();   // all transfers landed before the stages are reused
#undef QUEST_DMA

    // Epilogue: each wave's 128 x 64 block (see store_wave_block), parked in the stages.
    __syncthreads();   // every wave is done with the stages
    store_wave_block<4, kCarry>(acc, sa_reg, scale_lds + wn * 64, smem + wave * (128 * 128), m0 + wm * 128,
                                n0 + wn * 64, M, N, y, ld_y, acc_out, lane);
}

// ------------------------------------------------------------------------------------------
// Small-tile kernel for launches that would leave the kernel above with fewer workgroups than the
// chip has slots (a prefill of a few thousand tokens): workgroup tile 128 x 128, four waves of
// 64 x 64 (four 32 x 32 accumulator tiles each), 128 contraction elements per step, three LDS
// stages of 16 KiB, three workgroups per CU.  Same layouts, transfers, widening and transposed
// accumulator tiles as above; a 64 x 64 wave tile needs one widening per matrix instruction, so
// the operands of a sub-step are widened during the sub-step before it, into the other of two
// register sets.
// ------------------------------------------------------------------------------------------

constexpr int STM = 128, STN = 128;
constexpr int kSmallStageBytes = (STM + STN) * kRowBytes;     // 16 KiB
constexpr int kSmallParkBytes = 4 * 64 * 64 * 2;             // epilogue: four waves x 64 x 64 bf16
static_assert(kSmallParkBytes <= kStages * kSmallStageBytes, "the epilogue parks in the stages");
constexpr int kSmallLds = kStages * kSmallStageBytes + STN * 4;

template <int BITS>
__global__ __launch_bounds__(kTileThreads, 3) void lowbit_gemm_small_kernel(
    const uint8_t *__restrict__ a_codes, const float *__restrict__ a_scales,
    const uint8_t *__restrict__ b_codes, const float *__restrict__ b_scales, int M, int N, int K,
    int tiles_m, int tiles_n, uint16_t *__restrict__ y, int64_t ld_y,
    int32_t *__restrict__ acc_out)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // workgroup -> tile: one contiguous run of tiles per XCD, eight tile-rows deep
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total)
        return;
    const int band = logical / (8 * tiles_n);
    const int band_rows = min(8, tiles_m - band * 8);
    const int in_band = logical - band * 8 * tiles_n;
    const int tile_m = band * 8 + in_band % band_rows;
    const int tile_n = in_band / band_rows;
    const int m0 = tile_m * STM, n0 = tile_n * STN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lm = lane & 31, lh = lane >> 5;

    // Staging as above: a wave's 64 lanes fill 16 tile rows x 64 bytes per transfer.  Four pieces per
    // step and wave: rows 64 i + 16 wave .. + 16 of A (i < 2) and of B (i = 2, 3).
    const int st_row = 16 * wave + (lane >> 2);
    const int st_chunk = (lane & 3) ^ swz(st_row);
    const int64_t row_bytes = (int64_t)K / 2;
    uint32_t src_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = st_row + 64 * (i & 1);
        const int64_t grow = i < 2 ? min(m0 + row, M - 1) : min(n0 + row, N - 1);
        src_off[i] = (uint32_t)(grow * row_bytes + st_chunk * 16);
    }

    v16i acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0;

    constexpr int kCarry = BITS == 4 ? 6 : 8;
    uint32_t nibble_mask = BITS == 4 ? 0xf0f0f0f0u : 0xe0e0e0e0u;
    asm volatile("" : "+v"(nibble_mask));

    const int steps = K / TK;
    const uint32_t smem_addr = lds_address(smem);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#define QUEST_SMALL_DMA(STAGE, I, STEP)                                                                 \
    lds_dma16(((I) < 2 ? a_codes : b_codes) + src_off[I] + (int64_t)min((STEP), steps - 1) * kRowBytes, \
              (STAGE) + ((I) < 2 ? 0 : STM * kRowBytes) + (64 * ((I)&1) + 16 * wave_u) * kRowBytes)

    static_for<4>([&](auto i) { QUEST_SMALL_DMA(smem_addr, decltype(i)::value, 0); });
    static_for<4>([&](auto i) { QUEST_SMALL_DMA(smem_addr + kSmallStageBytes, decltype(i)::value, 1); });
    float *scale_lds = reinterpret_cast<float *>(smem + kStages * kSmallStageBytes);
    if (tid < STN)
        scale_lds[tid] = b_scales[min(n0 + tid, N - 1)];
    float sa_reg[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
        sa_reg[i] = a_scales[min(m0 + wm * 64 + i * 32 + lm, M - 1)] * (1.0f / (float)(1 << kCarry));
    wait_vmcnt<0>();
    __syncthreads();

    const int x = swz(lm);
    const int a_off = (wm * 64 + lm) * kRowBytes;
    const int b_off = STM * kRowBytes + (wn * 64 + lm) * kRowBytes;
    uint4 af[2][2], bf[2][2];   // packed fragments of the two sub-step pairs
    auto load_frag = [&](const uint8_t *stage, int p, int f) {
        const int off = ((2 * p + lh) ^ x) << 4;
        if (f < 2)
            af[p][f] = *reinterpret_cast<const uint4 *>(stage + a_off + f * 32 * kRowBytes + off);
        else
            bf[p][f - 2] = *reinterpret_cast<const uint4 *>(stage + b_off + (f - 2) * 32 * kRowBytes + off);
    };
    static_for<4>([&](auto f) { load_frag(smem, 0, decltype(f)::value); });

    // widened operands of sub-step g in set g % 2
    v4i wa[2][2], wb[2][2];
    auto widen_a = [&](auto gc, auto ic) {
        constexpr int g = decltype(gc)::value & 3, i = decltype(ic)::value;
        constexpr int p = g >> 1, e = g & 1;
        int w0, w1, w2, w3;
        widen8<BITS>(e ? af[p][i].z : af[p][i].x, nibble_mask, w0, w1);
        widen8<BITS>(e ? af[p][i].w : af[p][i].y, nibble_mask, w2, w3);
        wa[g & 1][i] = v4i{w0, w1, w2, w3};
    };
    auto widen_b = [&](auto gc, auto jc) {
        constexpr int g = decltype(gc)::value & 3, j = decltype(jc)::value;
        constexpr int p = g >> 1, e = g & 1;
        int w0, w1, w2, w3;
        widen8<BITS>(e ? bf[p][j].z : bf[p][j].x, nibble_mask, w0, w1);
        widen8<BITS>(e ? bf[p][j].w : bf[p][j].y, nibble_mask, w2, w3);
        wb[g & 1][j] = v4i{w0, w1, w2, w3};
    };
    static_for<2>([&](auto f) {
        widen_a(std::integral_constant<int, 0>{}, f);
        widen_b(std::integral_constant<int, 0>{}, f);
    });

    // Main loop: 16 MFMAs per step and wave.
    //   MFMA k: sub-step g = k / 4, A fragment (k % 4) / 2, B fragment k % 2; after it one operand of
    //           sub-step g + 1 is widened (B0, A0, B1, A1)
    //   k = 0, 2, 4, 6   start the transfers of step + 2 into the stage that was read in step - 1
    //   k = 0..3         load the packed fragments of pair 1 (first widened after k = 4)
    //   k = 7            wait for this wave's transfers of step + 1 (all but the four newest), barrier
    //   k = 8..11        load the packed fragments of pair 0 of step + 1 (first widened after k = 12)
    int stage_cur = 0, stage_one = kSmallStageBytes, stage_two = 2 * kSmallStageBytes;
    for (int step = 0; step < steps; ++step) {
        const uint8_t *cur = smem + stage_cur;
        const uint8_t *one = smem + stage_one;
        static_for<16>([&](auto kc) {
            constexpr int k = decltype(kc)::value;
            constexpr int g = k >> 2, s = k & 3, i = s >> 1, j = s & 1;
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wb[g & 1][j], wa[g & 1][i], acc[i][j], 0, 0, 0);
            if constexpr (s == 0)
                widen_b(std::integral_constant<int, g + 1>{}, std::integral_constant<int, 0>{});
            if constexpr (s == 1)
                widen_a(std::integral_constant<int, g + 1>{}, std::integral_constant<int, 0>{});
            if constexpr (s == 2)
                widen_b(std::integral_constant<int, g + 1>{}, std::integral_constant<int, 1>{});
            if constexpr (s == 3)
                widen_a(std::integral_constant<int, g + 1>{}, std::integral_constant<int, 1>{});
            if constexpr (k < 8 && (k & 1) == 0)
                QUEST_SMALL_DMA(smem_addr + stage_two, k / 2, step + 2);
            if constexpr (k < 4)
                load_frag(cur, 1, k);
            if constexpr (k == 7) {
                wait_vmcnt<4>();
                __builtin_amdgcn_s_barrier();
            }
            if constexpr (k >= 8 && k < 12)
                load_frag(one, 0, k - 8);
            __builtin_amdgcn_sched_barrier(0);
        });
        const int t = stage_cur;
        stage_cur = stage_one;
        stage_one = stage_two;
        stage_two = t;
    }
    wait_vmcnt<0>();
#undef QUEST_SMALL_DMA

    // Epilogue: each wave's 64 x 64 block (see store_wave_block), parked in the stages.
    __syncthreads();
    store_wave_block<2, kCarry>(acc, sa_reg, scale_lds + wn * 64, smem + wave * (64 * 128), m0 + wm * 64,
                                n0 + wn * 64, M, N, y, ld_y, acc_out, lane);
}

// ------------------------------------------------------------------------------------------
// Wide kernel for b = 4 and long contractions (K >= 4096).  Workgroup tile 256 x 256, eight waves of
// 128 x 64 (two per SIMD), 256 contraction elements per step, two LDS stages of 64 KiB, one
// workgroup per CU.  The codes of a tile step have to come through the CU's vector-memory path
// (64 bytes per clock): (TM + TN) * TK / 2 bytes for TM * TN * TK multiply-adds.  256 x 256 tiles move a
// third less per multiply-add than 256 x 128, and with 256 contraction elements a row contributes a
// whole 128-byte line per step instead of half of one.  The price is an epilogue that no second
// workgroup hides, which only pays off when the main loop is long.  Everything else (packed codes
// in LDS, widening at the consumer, direct global -> LDS transfers, pinned instruction slices,
// transposed accumulator tiles) is as in the kernel above.
// ------------------------------------------------------------------------------------------

constexpr int WTM = 256, WTN = 256, WTK = 256;
constexpr int kWideThreads = 512;
constexpr int kWideRowBytes = WTK / 2;                      // packed bytes per tile row and step: 128
constexpr int kWideStageBytes = (WTM + WTN) * kWideRowBytes;     // 64 KiB
constexpr int kWideParkBytes = 8 * 128 * 64 * 2;           // epilogue: eight waves x 128 x 64 bf16 (reuses the stages)
static_assert(kWideParkBytes <= 2 * kWideStageBytes, "the epilogue parks in the stages");
constexpr int kWideLds = 2 * kWideStageBytes + WTN * 4;     // 128 KiB + the tile's weight scales

// 16-byte chunk c (0..7) of tile row `row` lives at chunk c ^ wide_swz(row).  The LDS serves 128-bit
// accesses sixteen lanes at a time over 64 banks (256 bytes): sixteen consecutive rows reading
// the same logical chunk must hit sixteen different 16-byte slots modulo 256 bytes (measured).
// Rows are 128 bytes, so even and odd rows already differ; (row >> 1) & 7 separates the rest.
__device__ __forceinline__ int wide_swz(int row)
{
    return (row >> 1) & 7;
}

template <int BITS>
__global__ __launch_bounds__(kWideThreads, 1) void lowbit_gemm_wide_kernel(
    const uint8_t *__restrict__ a_codes, const float *__restrict__ a_scales,
    const uint8_t *__restrict__ b_codes, const float *__restrict__ b_scales, int M, int N, int K,
    int tiles_m, int tiles_n, uint16_t *__restrict__ y, int64_t ld_y,
    int32_t *__restrict__ acc_out)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // Workgroup -> tile.  Consecutive workgroup ids go to different XCDs (8 of them, each with
    // its own L2), so give each XCD one contiguous run of tiles, ordered four tile-rows deep:
    // the tiles an XCD works on at a time share a few row panels of A and column panels of B.
    const int total = tiles_m * tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total)
        return;
    const int band = logical / (4 * tiles_n);
    const int band_rows = min(4, tiles_m - band * 4);
    const int in_band = logical - band * 4 * tiles_n;
    const int tile_m = band * 4 + in_band % band_rows;
    const int tile_n = in_band / band_rows;
    const int m0 = tile_m * WTM, n0 = tile_n * WTN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int lm = lane & 31, lh = lane >> 5;

    // Staging: codes go from global memory straight into LDS, 16 bytes per lane.  A wave's 64 lanes
    // fill 1 KiB = 8 tile rows x 128 bytes; lane l lands at offset 16 l, i.e. row l / 8, physical
    // chunk l % 8, so it fetches the logical chunk that belongs there.  Eight such pieces per step
    // and wave: rows 64 i + 8 wave .. + 8 of A (i < 4) and of B (i >= 4).
    const int st_row = 8 * wave + (lane >> 3);                        // + 64 i
    const int st_chunk = (lane & 7) ^ wide_swz(st_row);                    // wide_swz(row + 64 i) = wide_swz(row)
    const int64_t row_bytes = (int64_t)K / 2;
    uint32_t src_off[8];   // per-thread byte offsets from a_codes / b_codes (rows clamped at the edge)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = st_row + 64 * (i & 3);
        const int64_t grow = i < 4 ? min(m0 + row, M - 1) : min(n0 + row, N - 1);
        src_off[i] = (uint32_t)(grow * row_bytes + st_chunk * 16);
    }

    v16i acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0;

    // kept in a vector register (opaque to constant folding) so that widen8 is one instruction
    constexpr int kCarry = BITS == 4 ? 6 : 8;   // log2 of the factor the products carry (8 u or 16 u per operand)
    uint32_t nibble_mask = BITS == 4 ? 0xf0f0f0f0u : 0xe0e0e0e0u;
    asm volatile("" : "+v"(nibble_mask));

    const int steps = K / WTK;
    // piece I of contraction step STEP -> stage at LDS byte address STAGE (wave-uniform)
    const uint32_t smem_addr = lds_address(smem);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    // (WAVE_STAGE: LDS byte address of the stage plus this wave's 8 rows)
#define QUEST_WIDE_DMA(WAVE_STAGE, I, STEP)                                                            \
    lds_dma16_at<((I) < 4 ? 0 : WTM * kWideRowBytes) + 64 * ((I)&3) * kWideRowBytes>(                   \
        ((I) < 4 ? a_codes : b_codes) + (int64_t)min((STEP), steps - 1) * kWideRowBytes, src_off[I], (WAVE_STAGE))

    const uint32_t wave_smem = smem_addr + 8 * wave_u * kWideRowBytes;
    static_for<8>([&](auto i) { QUEST_WIDE_DMA(wave_smem, decltype(i)::value, 0); });
    // the epilogue's scales, fetched while the first stage is on its way (see the kernel above)
    float *scale_lds = reinterpret_cast<float *>(smem + 2 * kWideStageBytes);
    if (tid < WTN)
        scale_lds[tid] = b_scales[min(n0 + tid, N - 1)];
    float sa_reg[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        sa_reg[i] = a_scales[min(m0 + wm * 128 + i * 32 + lm, M - 1)] * (1.0f / (float)(1 << kCarry));
    wait_vmcnt<0>();
    __syncthreads();

    // fragment addresses: rows lm + 32 i share bits 1..3, hence one swizzle value per lane;
    // chunk 2 p + lh of a row feeds this lane's share of sub-steps 2 p and 2 p + 1
    const int x = wide_swz(lm);
    const int a_off = (wm * 128 + lm) * kWideRowBytes;
    const int b_off = WTM * kWideRowBytes + (wn * 64 + lm) * kWideRowBytes;
    uint4 af[2][4], bf[2][2];   // packed fragments of two consecutive sub-step pairs
    auto load_frag = [&](const uint8_t *stage, int p, int f) {
        const int off = ((2 * p + lh) ^ x) << 4;
        if (f < 4)
            af[p & 1][f] = *reinterpret_cast<const uint4 *>(stage + a_off + f * 32 * kWideRowBytes + off);
        else
            bf[p & 1][f - 4] = *reinterpret_cast<const uint4 *>(stage + b_off + (f - 4) * 32 * kWideRowBytes + off);
    };
    static_for<6>([&](auto f) { load_frag(smem, 0, decltype(f)::value); });

    // Widened operands, as in the 256 x 128 kernel: A fragment i in wa[i % 2], the B fragments of
    // sub-step g in wb[g % 2][j]; sub-step g (eight per step) takes words (x, y) (g even) or (z, w)
    // (g odd) of the packed fragments of pair g / 2, which sit in af / bf [(g / 2) % 2].
    v4i wa[2], wb[2][2];
    auto widen_a = [&](auto gc, auto ic) {
        constexpr int g = decltype(gc)::value & 7, i = decltype(ic)::value;
        constexpr int q = (g >> 1) & 1, e = g & 1;
        int w0, w1, w2, w3;
        widen8<BITS>(e ? af[q][i].z : af[q][i].x, nibble_mask, w0, w1);
        widen8<BITS>(e ? af[q][i].w : af[q][i].y, nibble_mask, w2, w3);
        wa[i & 1] = v4i{w0, w1, w2, w3};
    };
    auto widen_b = [&](auto gc, auto jc) {
        constexpr int g = decltype(gc)::value & 7, j = decltype(jc)::value;
        constexpr int q = (g >> 1) & 1, e = g & 1;
        int w0, w1, w2, w3;
        widen8<BITS>(e ? bf[q][j].z : bf[q][j].x, nibble_mask, w0, w1);
        widen8<BITS>(e ? bf[q][j].w : bf[q][j].y, nibble_mask, w2, w3);
        wb[g & 1][j] = v4i{w0, w1, w2, w3};
    };
    widen_a(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    widen_b(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    widen_b(std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{});

    // Main loop: 64 MFMAs per step and wave, everything else pinned between them, every widening
    // at least one MFMA ahead of the first instruction that reads its result.
    //   MFMA k: sub-step g = k / 8, within it s = k % 8 multiplies A fragment s / 2 with B fragment s % 2
    //   after s = 0, 2, 4: widen A1, A2, A3    after s = 5, 6, 7: widen B0, A0, B1 of the next sub-step
    //   k = 0..7         start the transfer of step + 1 into the other stage (last read in step - 1)
    //   k = 16 p + 0..5  load the fragments of pair p + 1 (p < 3; first needed after k = 16 p + 13)
    //   k = 47           wait for this wave's transfers, then the workgroup barrier: step + 1 is in LDS
    //   k = 48..53       load the fragments of pair 0 of step + 1 in the order of their first use
    // The barrier sits before the last pair, so no wave waits on it with an empty MFMA queue.
    for (int step = 0; step < steps; ++step) {
        const uint8_t *cur = smem + (step & 1) * kWideStageBytes;
        const uint8_t *nxt = smem + ((step + 1) & 1) * kWideStageBytes;
        const uint32_t nxt_addr = wave_smem + ((step + 1) & 1) * kWideStageBytes;
        static_for<64>([&](auto kc) {
            constexpr int k = decltype(kc)::value;
            constexpr int g = k >> 3, s = k & 7, i = s >> 1, j = s & 1;
            // weight fragment as the row operand: transposed accumulator tiles
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wb[g & 1][j], wa[i & 1], acc[i][j], 0, 0, 0);
            if constexpr (s == 0 || s == 2 || s == 4)
                widen_a(std::integral_constant<int, g>{}, std::integral_constant<int, s / 2 + 1>{});
            if constexpr (s == 5)
                widen_b(std::integral_constant<int, g + 1>{}, std::integral_constant<int, 0>{});
            if constexpr (s == 6)
                widen_a(std::integral_constant<int, g + 1>{}, std::integral_constant<int, 0>{});
            if constexpr (s == 7)
                widen_b(std::integral_constant<int, g + 1>{}, std::integral_constant<int, 1>{});
            if constexpr (k < 8)
                QUEST_WIDE_DMA(nxt_addr, k, step + 1);
            if constexpr (k < 48 && (k & 15) < 6)
                load_frag(cur, (k >> 4) + 1, k & 15);
            if constexpr (k == 47) {
                wait_vmcnt<0>();
                __builtin_amdgcn_s_barrier();
            }
            if constexpr (k >= 48 && k < 54) {
                constexpr int order[6] = {4, 0, 5, 1, 2, 3};   // B0, A0, B1, A1, A2, A3
                load_frag(nxt, 0, order[k - 48]);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    }
#undef QUEST_WIDE_DMA

    // Epilogue: each wave's 128 x 64 block (see store_wave_block), parked in the stages.
    __syncthreads();   // every wave is done with the stages
    store_wave_block<4, kCarry>(acc, sa_reg, scale_lds + wn * 64, smem + wave * (128 * 128), m0 + wm * 128,
                                n0 + wn * 64, M, N, y, ld_y, acc_out, lane);
}

// ------------------------------------------------------------------------------------------
// b = 1 and b = 2 on the tile kernels: the codes are first re-coded into nibbles that stand for the
// same odd integers on the 4-bit grid (u = 2c - (L - 1) = 2(c + (16 - L) / 2) - 15), sixteen codes
// per thread, into scratch memory the caller provides; the accumulators are unchanged.
// ------------------------------------------------------------------------------------------
template <int CB>
__global__ __launch_bounds__(256) void recode_to_nibbles_kernel(const uint8_t *__restrict__ in,
                                                                uint2 *__restrict__ out, int64_t groups)
{
    static_assert(CB == 1 || CB == 2, "containers narrower than a nibble");
    constexpr uint32_t kField = (1u << CB) - 1u, kOffset = (16u - (1u << CB)) / 2u;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups;
         g += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t w = CB == 2 ? reinterpret_cast<const uint32_t *>(in)[g]
                                   : (uint32_t) reinterpret_cast<const uint16_t *>(in)[g];
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            lo |= (((w >> (CB * j)) & kField) + kOffset) << (4 * j);
            hi |= (((w >> (CB * (j + 8))) & kField) + kOffset) << (4 * j);
        }
        out[g] = make_uint2(lo, hi);
    }
}

hipError_t launch_recode(const uint8_t *in, uint8_t *out, int64_t rows, int64_t K, int cb, hipStream_t stream)
{
    const int64_t groups = rows * K / 16;
    const int64_t blocks = (groups + 255) / 256;
    const dim3 grid((unsigned)(blocks < 8192 ? blocks : 8192));
    if (cb == 2)
        hipLaunchKernelGGL(recode_to_nibbles_kernel<2>, grid, dim3(256), 0, stream, in,
                           reinterpret_cast<uint2 *>(out), groups);
    else
        hipLaunchKernelGGL(recode_to_nibbles_kernel<1>, grid, dim3(256), 0, stream, in,
                           reinterpret_cast<uint2 *>(out), groups);
    return hipGetLastError();
}

}  // namespace

// the 1- and 2-bit product takes the re-coding path when the tile kernels cover the shape
static bool recode_path(int64_t M, int64_t N, int64_t K, int bits)
{
    return bits <= 2 && (K % TK) == 0 && M >= 128 && N >= 128;
}

int64_t lowbit_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int bits)
{
    return recode_path(M, N, K, bits) ? (M + N) * K / 2 : 0;
}

hipError_t prepare_lowbit_gemm_kernels()
{
    hipError_t err = allow_dynamic_lds(reinterpret_cast<const void *>(lowbit_gemm_wide_kernel<4>), kWideLds);
    if (err == hipSuccess)
        err = allow_dynamic_lds(reinterpret_cast<const void *>(lowbit_gemm_wide_kernel<3>), kWideLds);
    if (err == hipSuccess)
        err = allow_dynamic_lds(reinterpret_cast<const void *>(lowbit_gemm_small_kernel<4>), kSmallLds);
    if (err == hipSuccess)
        err = allow_dynamic_lds(reinterpret_cast<const void *>(lowbit_gemm_small_kernel<3>), kSmallLds);
    if (err == hipSuccess)
        err = allow_dynamic_lds(reinterpret_cast<const void *>(lowbit_gemm_tile_kernel<4>), kTileLds);
    if (err == hipSuccess)
        err = allow_dynamic_lds(reinterpret_cast<const void *>(lowbit_gemm_tile_kernel<3>), kTileLds);
    return err;
}

hipError_t launch_lowbit_gemm(const GemmArgs &args, hipStream_t stream)
{
    if (args.M == 0 || args.N == 0)
        return hipSuccess;
    GemmArgs a = args;
    // 1 and 2 bits with scratch from the caller: re-code, then the 4-bit tile kernels.  Without
    // scratch the general kernel below multiplies the narrow containers directly (slower).
    if (recode_path(a.M, a.N, a.K, a.bits) && a.workspace != nullptr) {
        if (a.workspace_bytes < lowbit_gemm_workspace_bytes(a.M, a.N, a.K, a.bits))
            return hipErrorInvalidValue;
        uint8_t *a_nibbles = static_cast<uint8_t *>(a.workspace);
        uint8_t *b_nibbles = a_nibbles + a.M * a.K / 2;
        hipError_t err = launch_recode(a.a_codes, a_nibbles, a.M, a.K, a.cb, stream);
        if (err == hipSuccess)
            err = launch_recode(a.b_codes, b_nibbles, a.N, a.K, a.cb, stream);
        if (err != hipSuccess)
            return err;
        a.a_codes = a_nibbles;
        a.b_codes = b_nibbles;
        a.bits = 4;
        a.cb = 4;
    }
    const int levels = 1 << a.bits;
    auto *y = static_cast<uint16_t *>(a.y);
    // the wide kernel runs one workgroup per CU: it needs about a round of 256 x 256 tiles to fill the chip
    const int64_t wide_tiles = ((a.M + WTM - 1) / WTM) * ((a.N + WTN - 1) / WTN);
    if ((a.bits == 4 || a.bits == 3) && (a.K % WTK) == 0 && a.K >= 4096 && a.M >= 512 && a.N >= 512 &&
        wide_tiles >= 192) {
        const int tiles_m = (int)((a.M + WTM - 1) / WTM), tiles_n = (int)((a.N + WTN - 1) / WTN);
        const int per_xcd = (tiles_m * tiles_n + 7) / 8;
        const hipError_t err = prepare_lowbit_gemm_kernels();
        if (err != hipSuccess)
            return err;
        const dim3 grid((unsigned)(per_xcd * 8)), block(kWideThreads);
        if (a.bits == 4)
            hipLaunchKernelGGL(lowbit_gemm_wide_kernel<4>, grid, block, kWideLds, stream, a.a_codes, a.a_scales,
                               a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, tiles_m, tiles_n, y, a.ld_y,
                               a.acc_out);
        else
            hipLaunchKernelGGL(lowbit_gemm_wide_kernel<3>, grid, block, kWideLds, stream, a.a_codes, a.a_scales,
                               a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, tiles_m, tiles_n, y, a.ld_y,
                               a.acc_out);
        return hipGetLastError();
    }
    // fewer 256 x 128 tiles than three quarters of the chip's slots (two per CU): 128 x 128 tiles
    const int64_t big_tiles = ((a.M + TM - 1) / TM) * ((a.N + TN - 1) / TN);
    if ((a.bits == 4 || a.bits == 3) && (a.K % TK) == 0 && a.M >= 128 && a.N >= 128 && big_tiles < 384) {
        const int tiles_m = (int)((a.M + STM - 1) / STM), tiles_n = (int)((a.N + STN - 1) / STN);
        const int per_xcd = (tiles_m * tiles_n + 7) / 8;
        const hipError_t err = prepare_lowbit_gemm_kernels();
        if (err != hipSuccess)
            return err;
        const dim3 grid((unsigned)(per_xcd * 8)), block(kTileThreads);
        if (a.bits == 4)
            hipLaunchKernelGGL(lowbit_gemm_small_kernel<4>, grid, block, kSmallLds, stream, a.a_codes, a.a_scales,
                               a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, tiles_m, tiles_n, y, a.ld_y,
                               a.acc_out);
        else
            hipLaunchKernelGGL(lowbit_gemm_small_kernel<3>, grid, block, kSmallLds, stream, a.a_codes, a.a_scales,
                               a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, tiles_m, tiles_n, y, a.ld_y,
                               a.acc_out);
        return hipGetLastError();
    }
    if ((a.bits == 4 || a.bits == 3) && (a.K % TK) == 0 && a.M >= 512 && a.N >= 256) {
        const int tiles_m = (int)((a.M + TM - 1) / TM), tiles_n = (int)((a.N + TN - 1) / TN);
        const int per_xcd = (tiles_m * tiles_n + 7) / 8;
        const hipError_t err = prepare_lowbit_gemm_kernels();
        if (err != hipSuccess)
            return err;
        const dim3 grid((unsigned)(per_xcd * 8)), block(kTileThreads);
        if (a.bits == 4)
            hipLaunchKernelGGL(lowbit_gemm_tile_kernel<4>, grid, block, kTileLds, stream, a.a_codes, a.a_scales,
                               a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, tiles_m, tiles_n, y, a.ld_y,
                               a.acc_out);
        else
            hipLaunchKernelGGL(lowbit_gemm_tile_kernel<3>, grid, block, kTileLds, stream, a.a_codes, a.a_scales,
                               a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, tiles_m, tiles_n, y, a.ld_y,
                               a.acc_out);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)((a.N + BN - 1) / BN), (unsigned)((a.M + BM - 1) / BM));
    const dim3 block(kThreads);
    switch (a.cb) {
    case 4:
        hipLaunchKernelGGL(lowbit_gemm_kernel<4>, grid, block, 0, stream, a.a_codes, a.a_scales,
                           a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, levels, y, a.ld_y,
                           a.acc_out);
        break;
    case 2:
        hipLaunchKernelGGL(lowbit_gemm_kernel<2>, grid, block, 0, stream, a.a_codes, a.a_scales,
                           a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, levels, y, a.ld_y,
                           a.acc_out);
        break;
    default:
        hipLaunchKernelGGL(lowbit_gemm_kernel<1>, grid, block, 0, stream, a.a_codes, a.a_scales,
                           a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K, levels, y, a.ld_y,
                           a.acc_out);
        break;
    }
    return hipGetLastError();
}

}  // namespace quest
