// C-ABI entry points of the QuEST hot path: argument validation and kernel dispatch only.
// See include/quest.h for the contract of every function.
#include <math.h>

#include <map>
#include <mutex>
#include <tuple>

#include "quest_internal.h"

namespace {

// Gaussian-MSE-optimal clip in RMS units for the 2^b-level zero-free symmetric grid
// (Sec. 3.1 "Gaussian Fitting" defines alpha*; the paper prints no values).  Obtained by
// minimising, over alpha, sum over cells of the integral of (xi - q_k)^2 phi(xi); b = 1 has the
// closed form sqrt(2 / pi).
constexpr double kAlphaStar1 = 0.7978845608028654;
constexpr double kAlphaStar2 = 1.4935300066;
constexpr double kAlphaStar3 = 2.0510680577;
constexpr double kAlphaStar4 = 2.5140046071;
constexpr double kAlphaStar8 = 3.9221998115;
// Same definition with the rounding to the E2M1 grid scaled to [-1, 1] (Sec. 4.4 "The FP4 Format"):
// ternary search on a piecewise Simpson integral of the error; the minimum is flat to 1e-7.
constexpr double kAlphaStarFp4 = 2.9224752;

double alpha_star(int bits)
{
    switch (bits) {
    case 1: return kAlphaStar1;
    case 2: return kAlphaStar2;
    case 3: return kAlphaStar3;
    case 4: return kAlphaStar4;
    case 8: return kAlphaStar8;
    default: return 0.0;
    }
}

int container_bits(int bits)
{
    switch (bits) {
    case 1: return 1;
    case 2: return 2;
    case 3: return 4;
    case 4: return 4;
    case 8: return 8;
    default: return 0;
    }
}

bool aligned16(const void *p)
{
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

// log2 of a power of two, -1 otherwise
int exact_log2(int64_t v)
{
    if (v <= 0 || (v & (v - 1)))
        return -1;
    int l = 0;
    while ((int64_t(1) << l) < v)
        ++l;
    return l;
}

quest_status shape_checks(int64_t rows, int64_t cols, int32_t had_block, int *log2n)
{
    if (rows < 0 || cols < 8 || cols > QUEST_MAX_COLS || (cols & 7))
        return QUEST_ERR_SHAPE;
    const int l = exact_log2(had_block);
    if (l < 0 || had_block > QUEST_MAX_HAD_BLOCK || cols % had_block)
        return QUEST_ERR_BLOCK;
    *log2n = l;
    return QUEST_OK;
}

}  // namespace

namespace quest {

hipError_t allow_dynamic_lds(const void *kernel, int bytes)
{
    static std::mutex guard;
    static std::map<std::tuple<const void *, int>, int> allowed;   // (kernel, device) -> bytes granted
    int device = 0;
    hipError_t err = hipGetDevice(&device);
    if (err != hipSuccess)
        return err;
    std::lock_guard<std::mutex> lock(guard);
    int &granted = allowed[std::make_tuple(kernel, device)];
    if (granted >= bytes)
        return hipSuccess;
    err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (err == hipSuccess)
        granted = bytes;
    return err;
}

/*
 * Device memory the library owns (the expanded operand and the partial tiles of the gradient
 * matmuls, re-coded operands of the 1- and 2-bit matmul): one buffer per device, grown on demand
 * and kept until the process ends.  All launches that use it on a device share it, so they must
 * not overlap (they do not when issued to one stream).  Growing frees the old buffer after a
 * device synchronisation.
 */
hipError_t library_memory(int device, size_t bytes, char **out_ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex guard;
    static void *buffer[kMaxDevices] = {};
    static size_t capacity[kMaxDevices] = {};
    if (device < 0 || device >= kMaxDevices)
        return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(guard);
    if (capacity[device] < bytes) {
        if (buffer[device] != nullptr) {
            hipError_t err = hipDeviceSynchronize();
            if (err == hipSuccess)
                err = hipFree(buffer[device]);
            if (err != hipSuccess)
                return err;
            buffer[device] = nullptr;
            capacity[device] = 0;
        }
        hipError_t err = hipMalloc(&buffer[device], bytes);
        if (err != hipSuccess)
            return err;
        capacity[device] = bytes;
    }
    *out_ptr = static_cast<char *>(buffer[device]);
    return hipSuccess;
}

}  // namespace quest

extern "C" {

float quest_alpha_star(int32_t bits)
{
    return (float)alpha_star(bits);
}

int32_t quest_container_bits(int32_t bits)
{
    return container_bits(bits);
}

const char *quest_status_string(quest_status status)
{
    switch (status) {
    case QUEST_OK: return "ok";
    case QUEST_ERR_NULL: return "a required pointer is NULL";
    case QUEST_ERR_SHAPE: return "shape out of the supported range";
    case QUEST_ERR_BITS: return "unsupported bit width";
    case QUEST_ERR_BLOCK: return "Hadamard block must be a power of two that divides cols";
    case QUEST_ERR_ALIGN: return "pointer or leading dimension not 16-byte aligned";
    case QUEST_ERR_DTYPE: return "unknown dtype";
    case QUEST_ERR_LAUNCH: return "the HIP runtime refused the launch";
    case QUEST_ERR_ARG: return "invalid argument";
    default: return "unknown status";
    }
}

namespace {

// Shared by the two quantizer entry points; absmax ignores alpha and outer_trust.
quest_status quantize_entry(const void *x, quest_dtype dtype, int64_t rows, int64_t cols, int64_t ld,
                            int32_t had_block, int32_t bits, float alpha, float outer_trust, int mode,
                            uint8_t *codes, float *scales, uint8_t *mask, float *xh_out, void *stream)
{
    if (!x || !codes || !scales)
        return QUEST_ERR_NULL;
    if (dtype != QUEST_F32 && dtype != QUEST_BF16)
        return QUEST_ERR_DTYPE;
    const int cb = container_bits(bits);
    if (cb == 0)
        return QUEST_ERR_BITS;
    int log2n = 0;
    const quest_status shape = shape_checks(rows, cols, had_block, &log2n);
    if (shape != QUEST_OK)
        return shape;
    if (ld < cols)
        return QUEST_ERR_SHAPE;
    const int64_t elem = dtype == QUEST_BF16 ? 2 : 4;
    if (!aligned16(x) || !aligned16(codes) || (mask && !aligned16(mask)) ||
        (xh_out && !aligned16(xh_out)) || ((ld * elem) & 15) ||
        (reinterpret_cast<uintptr_t>(scales) & 3u))
        return QUEST_ERR_ALIGN;
    if (isnan(alpha) || isinf(alpha) || isnan(outer_trust) || isinf(outer_trust))
        return QUEST_ERR_ARG;

    const int levels = 1 << bits;
    const double a = alpha > 0.0f ? (double)alpha : mode == quest::kQuantFp4 ? kAlphaStarFp4 : alpha_star(bits);
    const double ot = outer_trust < 0.0f ? 1.0 : (double)outer_trust;
    // trusted iff |x_h| <= edge * rms: the clip plus one trust width T (times outer_trust);
    // T = alpha / (L - 1) on the Eq. 1 grid, alpha / 6 (largest half-interval) on the FP4 grid
    const double width = mode == quest::kQuantFp4 ? 1.0 / 6.0 : 1.0 / (double)(levels - 1);

    quest::QuantizeArgs args;
    args.x = x;
    args.dtype = dtype;
    args.rows = rows;
    args.cols = cols;
    args.ld = ld;
    args.log2n = log2n;
    args.bits = bits;
    args.cb = cb;
    args.alpha = (float)a;
    args.trust_edge = (float)(a * (1.0 + ot * width));
    args.codes = codes;
    args.scales = scales;
    args.mask = mask;
    args.xh_out = xh_out;
    args.mode = mode;
    return quest::launch_hadamard_quantize(args, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUEST_OK
               : QUEST_ERR_LAUNCH;
}

}  // namespace

quest_status quest_hadamard_quantize(const void *x, quest_dtype dtype, int64_t rows, int64_t cols,
                                     int64_t ld, int32_t had_block, int32_t bits, float alpha,
                                     float outer_trust, uint8_t *codes, float *scales,
                                     uint8_t *mask, float *xh_out, void *stream)
{
    return quantize_entry(x, dtype, rows, cols, ld, had_block, bits, alpha, outer_trust, quest::kQuantRms, codes,
                          scales, mask, xh_out, stream);
}

quest_status quest_hadamard_quantize_absmax(const void *x, quest_dtype dtype, int64_t rows,
                                            int64_t cols, int64_t ld, int32_t had_block, int32_t bits,
                                            uint8_t *codes, float *scales, uint8_t *mask,
                                            float *xh_out, void *stream)
{
    return quantize_entry(x, dtype, rows, cols, ld, had_block, bits, 0.0f, -1.0f, quest::kQuantAbsMax, codes,
                          scales, mask, xh_out, stream);
}

quest_status quest_hadamard_quantize_fp4(const void *x, quest_dtype dtype, int64_t rows, int64_t cols,
                                         int64_t ld, int32_t had_block, float alpha, uint8_t *codes,
                                         float *scales, uint8_t *mask, float *xh_out, void *stream)
{
    return quantize_entry(x, dtype, rows, cols, ld, had_block, 4, alpha, -1.0f, quest::kQuantFp4, codes,
                          scales, mask, xh_out, stream);
}

float quest_alpha_star_fp4(void)
{
    return (float)kAlphaStarFp4;
}

quest_status quest_lowbit_gemm(const uint8_t *a_codes, const float *a_scales, int64_t M,
                               const uint8_t *b_codes, const float *b_scales, int64_t N, int64_t K,
                               int32_t bits, void *y, int64_t ld_y, int32_t *acc_out,
                               void *stream)
{
    if (!a_codes || !a_scales || !b_codes || !b_scales || (!y && !acc_out))
        return QUEST_ERR_NULL;
    if (bits < 1 || bits > 4)
        return QUEST_ERR_BITS;
    if (M < 0 || N < 0 || M > (int64_t(1) << 22) || N > (int64_t(1) << 22) || K < 64 ||
        K > 65536 || (K & 63))
        return QUEST_ERR_SHAPE;
    if (y && ld_y < N)
        return QUEST_ERR_SHAPE;
    if (!aligned16(a_codes) || !aligned16(b_codes) || (y && !aligned16(y)) ||
        (acc_out && !aligned16(acc_out)))
        return QUEST_ERR_ALIGN;

    quest::GemmArgs args;
    args.a_codes = a_codes;
    args.a_scales = a_scales;
    args.b_codes = b_codes;
    args.b_scales = b_scales;
    args.M = M;
    args.N = N;
    args.K = K;
    args.bits = bits;
    args.cb = container_bits(bits);
    args.y = y;
    args.ld_y = ld_y;
    args.acc_out = acc_out;
    return quest::launch_lowbit_gemm(args, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUEST_OK
               : QUEST_ERR_LAUNCH;
}

quest_status quest_lowbit_gemm_fp4(const uint8_t *a_codes, const float *a_scales, int64_t M,
                                   const uint8_t *b_codes, const float *b_scales, int64_t N, int64_t K,
                                   void *y, int64_t ld_y, float *acc_out, void *stream)
{
    if (!a_codes || !a_scales || !b_codes || !b_scales || (!y && !acc_out))
        return QUEST_ERR_NULL;
    if (M < 0 || N < 0 || M > (int64_t(1) << 22) || N > (int64_t(1) << 22) || K < 128 || K > 65536 ||
        (K & 127) || (M > N ? M : N) * (K / 2) >= (int64_t(1) << 32))
        return QUEST_ERR_SHAPE;
    if (y && ld_y < N)
        return QUEST_ERR_SHAPE;
    if (!aligned16(a_codes) || !aligned16(b_codes) || (reinterpret_cast<uintptr_t>(y) & 1u) ||
        (reinterpret_cast<uintptr_t>(acc_out) & 3u))
        return QUEST_ERR_ALIGN;
    quest::Fp4GemmArgs args;
    args.a_codes = a_codes;
    args.a_scales = a_scales;
    args.b_codes = b_codes;
    args.b_scales = b_scales;
    args.M = M;
    args.N = N;
    args.K = K;
    args.y = y;
    args.ld_y = ld_y;
    args.acc_out = acc_out;
    return quest::launch_fp4_gemm(args, static_cast<hipStream_t>(stream)) == hipSuccess ? QUEST_OK
                                                                                       : QUEST_ERR_LAUNCH;
}

quest_status quest_trust_backward(const void *g, quest_dtype g_dtype, const uint8_t *mask,
                                  int64_t rows, int64_t cols, int32_t had_block, void *out,
                                  quest_dtype out_dtype, void *stream)
{
    if (!g || !out)
        return QUEST_ERR_NULL;
    if ((g_dtype != QUEST_F32 && g_dtype != QUEST_BF16) ||
        (out_dtype != QUEST_F32 && out_dtype != QUEST_BF16))
        return QUEST_ERR_DTYPE;
    int log2n = 0;
    const quest_status shape = shape_checks(rows, cols, had_block, &log2n);
    if (shape != QUEST_OK)
        return shape;
    if (!aligned16(g) || !aligned16(out) || (mask && !aligned16(mask)))
        return QUEST_ERR_ALIGN;

    quest::BackwardArgs args;
    args.g = g;
    args.g_dtype = g_dtype;
    args.mask = mask;
    args.rows = rows;
    args.cols = cols;
    args.log2n = log2n;
    args.out = out;
    args.out_dtype = out_dtype;
    return quest::launch_trust_backward(args, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUEST_OK
               : QUEST_ERR_LAUNCH;
}

quest_status quest_grad_gemm(int32_t which, const void *dy, const uint8_t *q_codes,
                             const float *q_scales, int32_t bits, int64_t M, int64_t N, int64_t K,
                             void *out, void *stream)
{
    if (!dy || !q_codes || !q_scales || !out)
        return QUEST_ERR_NULL;
    if (which != 0 && which != 1)
        return QUEST_ERR_ARG;
    if (bits < 1 || bits > 4)
        return QUEST_ERR_BITS;
    if (M < 0 || N < 0 || K < 0 || (M & 63) || (N & 63) || (K & 63) || M > (int64_t(1) << 22) ||
        N > (int64_t(1) << 22) || K > (int64_t(1) << 22))
        return QUEST_ERR_SHAPE;
    if (!aligned16(dy) || !aligned16(q_codes) || !aligned16(out))
        return QUEST_ERR_ALIGN;

    quest::GradGemmArgs args;
    args.which = which;
    args.fp4 = false;
    args.dy = dy;
    args.q_codes = q_codes;
    args.q_scales = q_scales;
    args.bits = bits;
    args.cb = container_bits(bits);
    args.M = M;
    args.N = N;
    args.K = K;
    args.out = out;
    return quest::launch_grad_gemm(args, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUEST_OK
               : QUEST_ERR_LAUNCH;
}

quest_status quest_grad_gemm_fp4(int32_t which, const void *dy, const uint8_t *q_codes,
                                 const float *q_scales, int64_t M, int64_t N, int64_t K, void *out,
                                 void *stream)
{
    if (!dy || !q_codes || !q_scales || !out)
        return QUEST_ERR_NULL;
    if (which != 0 && which != 1)
        return QUEST_ERR_ARG;
    const int64_t out_rows = which == 0 ? M : N, contraction = which == 0 ? N : M;
    const bool empty = M == 0 || N == 0 || K == 0;
    if (M < 0 || N < 0 || K < 0 || (out_rows & 63) || (K & 63) || (contraction & 63) ||
        (!empty && (out_rows < 128 || K < 128)) || M > (int64_t(1) << 22) || N > (int64_t(1) << 22) || K > (int64_t(1) << 22) ||
        out_rows * K >= (int64_t(1) << 31) || (M > N ? M : N) * (K > N ? K : N) >= (int64_t(1) << 30))
        return QUEST_ERR_SHAPE;
    if (!aligned16(dy) || !aligned16(q_codes) || !aligned16(out))
        return QUEST_ERR_ALIGN;
    quest::GradGemmArgs args;
    args.which = which;
    args.fp4 = true;
    args.dy = dy;
    args.q_codes = q_codes;
    args.q_scales = q_scales;
    args.bits = 4;
    args.cb = 4;
    args.M = M;
    args.N = N;
    args.K = K;
    args.out = out;
    return quest::launch_grad_gemm(args, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUEST_OK
               : QUEST_ERR_LAUNCH;
}

quest_status quest_weight_only_gemm(const void *x, const uint8_t *w_codes, const float *w_scales,
                                    int32_t bits, int64_t M, int64_t N, int64_t K, void *y,
                                    void *stream)
{
    if (!x || !w_codes || !w_scales || !y)
        return QUEST_ERR_NULL;
    if (bits < 1 || bits > 4)
        return QUEST_ERR_BITS;
    const bool empty = M == 0 || N == 0 || K == 0;
    if (M < 0 || N < 0 || K < 0 || (M & 63) || (N & 63) || (K & 63) || (!empty && (M < 128 || N < 128)) ||
        M > (int64_t(1) << 22) ||
        N > (int64_t(1) << 22) || K > (int64_t(1) << 22) || M * N >= (int64_t(1) << 31) ||
        (M > N ? M : N) * (K > N ? K : N) >= (int64_t(1) << 30))
        return QUEST_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(w_codes) || !aligned16(y))
        return QUEST_ERR_ALIGN;

    quest::GradGemmArgs args;
    args.which = 2;
    args.fp4 = false;
    args.dy = x;
    args.q_codes = w_codes;
    args.q_scales = w_scales;
    args.bits = bits;
    args.cb = container_bits(bits);
    args.M = M;
    args.N = N;
    args.K = K;
    args.out = y;
    return quest::launch_grad_gemm(args, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUEST_OK
               : QUEST_ERR_LAUNCH;
}

}  // extern "C"
