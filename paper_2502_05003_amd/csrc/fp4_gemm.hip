// FP4 x FP4 GEMM with a dequantizing bf16 epilogue for the FP4 variant of the method (Sec. 4.4
// "The FP4 Format" of arXiv 2502.05003): y = xhat_h what_h^T on E2M1 codes, contracted on the FP4
// matrix instruction (v_mfma_scale_f32_32x32x64_f8f6f4 with unit block scales).  Products of
// E2M1 values are multiples of 1/4 below 36, so the fp32 accumulators hold sum_k v_a v_b exactly
// for K <= 65536.
//
// Same structure as the INT8 kernel for the integer grid (256 x 128 tile, four waves of 128 x 64,
// 128 contraction elements per step, three LDS stages filled by direct global -> LDS transfers, two
// workgroups per CU, transposed accumulator tiles, LDS-parked epilogue), minus the widening: the
// quantizer packs two codes per byte in element order, which is the instruction's operand layout
// (lane l: row l % 32, elements 32 (l / 32) .. + 32 of the 64-element sub-step), so a 16-byte LDS
// read is an operand.
#include <algorithm>

#include "gemm_tile.h"
#include "quest_internal.h"

namespace quest {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int TM = 256, TN = 128, TK = 128;
constexpr int kTileThreads = 256;
constexpr int kRowBytes = TK / 2;                      // packed bytes per tile row and step
constexpr int kStageBytes = (TM + TN) * kRowBytes;     // 24 KiB
constexpr int kStages = 3;
constexpr int kParkBytes = 4 * 128 * 64 * 2;           // epilogue: four waves x 128 x 64 bf16 (reuses the stages)
static_assert(kParkBytes <= kStages * kStageBytes, "the epilogue parks in the stages");
constexpr int kTileLds = kStages * kStageBytes + TN * 4;   // 72 KiB + the tile's weight scales

// 16-byte chunk c (0..3) of tile row `row` lives at chunk c ^ swz(row): sixteen consecutive rows
// reading the same logical chunk hit sixteen different 16-byte slots modulo 256 bytes.
__device__ __forceinline__ int swz(int row)
{
    return (row >> 2) & 3;
}

__global__ __launch_bounds__(kTileThreads, 2) void fp4_gemm_tile_kernel(
    const uint8_t *__restrict__ a_codes, const float *__restrict__ a_scales,
    const uint8_t *__restrict__ b_codes, const float *__restrict__ b_scales, int M, int N, int K,
    int tiles_m, int tiles_n, uint16_t *__restrict__ y, int64_t ld_y,
    float *__restrict__ acc_out)
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

    v16f acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][j][r] = 0.0f;

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
    // registers
    float *scale_lds = reinterpret_cast<float *>(smem + kStages * kStageBytes);
    if (tid < TN)
        scale_lds[tid] = b_scales[min(n0 + tid, N - 1)];
    float sa_reg[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        sa_reg[i] = a_scales[min(m0 + wm * 128 + i * 32 + lm, M - 1)];
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

    // Main loop: 16 matrix instructions per step and wave.  A packed fragment (16 bytes per lane:
    // the 32 codes of its half of a 64-element sub-step) is the instruction's operand as it is.
    //   MFMA s: pair p = s / 8, A fragment i = (s / 2) % 4, B fragment j = s % 2
    //   s = 0, 2, .. 10  start the transfers of step + 2 into the stage that was read in step - 1
    //   s = 1..6    load the fragments of pair 1 (first needed at s = 8)
    //   s = 10      wait for this wave's transfers of step + 1 (all but the six newest), barrier
    //   s = 11..15  load the fragments of pair 0 of step + 1
    const int one = 0x7f7f7f7f;   // block scales 2^0 (the codes carry no block scale)
    auto operand = [](const uint4 &f) { return v8i{(int)f.x, (int)f.y, (int)f.z, (int)f.w, 0, 0, 0, 0}; };
    int stage_cur = 0;   // byte offsets of the stages holding step, step + 1, step + 2
    int stage_one = kStageBytes, stage_two = 2 * kStageBytes;
    for (int step = 0; step < steps; ++step) {
        const uint8_t *cur = smem + stage_cur;
        const uint8_t *one_stage = smem + stage_one;
        static_for<16>([&](auto kc) {
            constexpr int s = decltype(kc)::value;
            constexpr int p = s >> 3, i = (s >> 1) & 3, j = s & 1;
            // weight fragment as the row operand: transposed accumulator tiles
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(operand(bf[p][j]), operand(af[p][i]),
                                                                        acc[i][j], 4, 4, 0, one, 0, one);
            if constexpr (s <= 10 && (s & 1) == 0)
                QUEST_DMA(wave_smem + stage_two, s / 2, step + 2);
            if constexpr (s >= 1 && s <= 6)
                load_frag(cur, 1, s - 1);
            if constexpr (s == 10) {
                wait_vmcnt<6>();
                __builtin_amdgcn_s_barrier();
            }
            if constexpr (s == 11) {
                load_frag(one_stage, 0, 0);
                load_frag(one_stage, 0, 4);
            }
            if constexpr (s == 12)
                load_frag(one_stage, 0, 5);
            if constexpr (s >= 13)
                load_frag(one_stage, 0, s - 12);
            __builtin_amdgcn_sched_barrier(0);
        });
        const int t = stage_cur;
        stage_cur = stage_one;
        stage_one = stage_two;
        stage_two = t;
    }
    wait_vmcnt<0>();   // all transfers landed before the stages are reused
#undef QUEST_DMA

    // Epilogue: each wave's 128 x 64 block (see store_wave_block), parked in the stages.  (Storing
    // 16-byte pieces straight from registers after a lane-pair exchange, without the detour through
    // LDS, measured 5 % slower here and 1 % slower in the INT8 kernels: whole 128-byte row segments
    // per store instruction matter more than the LDS round trip.)
    __syncthreads();   // every wave is done with the stages
    store_wave_block<4, 0>(acc, sa_reg, scale_lds + wn * 64, smem + wave * (128 * 128), m0 + wm * 128,
                           n0 + wn * 64, M, N, y, ld_y, acc_out, lane);
}

}  // namespace

hipError_t prepare_fp4_gemm_kernels()
{
    return allow_dynamic_lds(reinterpret_cast<const void *>(fp4_gemm_tile_kernel), kTileLds);
}

hipError_t launch_fp4_gemm(const Fp4GemmArgs &a, hipStream_t stream)
{
    if (a.M == 0 || a.N == 0)
        return hipSuccess;
    const hipError_t attr_err = prepare_fp4_gemm_kernels();
    if (attr_err != hipSuccess)
        return attr_err;
    const int tiles_m = (int)((a.M + TM - 1) / TM), tiles_n = (int)((a.N + TN - 1) / TN);
    const int per_xcd = (tiles_m * tiles_n + 7) / 8;
    hipLaunchKernelGGL(fp4_gemm_tile_kernel, dim3((unsigned)(per_xcd * 8)), dim3(kTileThreads), kTileLds,
                       stream, a.a_codes, a.a_scales, a.b_codes, a.b_scales, (int)a.M, (int)a.N, (int)a.K,
                       tiles_m, tiles_n, static_cast<uint16_t *>(a.y), a.ld_y, a.acc_out);
    return hipGetLastError();
}

}  // namespace quest
