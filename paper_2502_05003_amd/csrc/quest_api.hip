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

int device_compute_units()
{
    constexpr int kMaxDevices = 64;
    static std::mutex guard;
    static int known[kMaxDevices] = {};
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) {
        (void)hipGetLastError();   // host-only use: leave no sticky error behind
        return 256;
    }
    std::lock_guard<std::mutex> lock(guard);
    if (known[device] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus < 8) {
            (void)hipGetLastError();
            return 256;
        }
        known[device] = cus / 8 * 8;
    }
    return known[device];
}

}  // namespace quest

// Scratch of quest_lowbit_gemm_static: one copy per GPU the library runs on, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress; the device address it
// yields (per device) is what kernels, copies and fills are given.
static __device__ __align__(256) unsigned char scratch[QUEST_STATIC_SCRATCH_BYTES];

namespace {

// Device address of `scratch` on the current device, looked up once per device.
hipError_t static_scratch_address(void **out_ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex guard;
    static void *known[kMaxDevices] = {};
    int device = 0;
    hipError_t err = hipGetDevice(&device);
    if (err != hipSuccess)
        return err;
    if (device < 0 || device >= kMaxDevices)
        return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(guard);
    if (known[device] == nullptr) {
        void *ptr = nullptr;
        err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (err != hipSuccess)
            return err;
        if (ptr == nullptr)
            return hipErrorInvalidSymbol;
        known[device] = ptr;
    }
    *out_ptr = known[device];
    return hipSuccess;
}

}  // namespace

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
    case QUEST_ERR_SCRATCH: return "the call needs more scratch than the library's built-in buffer holds";
    default: return "unknown status";
    }
}

namespace {

// One operand of a quantizer call (rows of `cols` elements at stride ld, and its outputs).
struct QuantOperand {
    const void *x;
    int64_t rows, ld;
    uint8_t *codes;
    float *scales;
    uint8_t *mask;
};

// (`empty_may_be_null`: an operand of a pair call that has no rows needs no buffers)
quest_status check_quant_operand(const QuantOperand &o, quest_dtype dtype, int64_t cols, int32_t had_block,
                                 int *log2n, bool empty_may_be_null)
{
    if (!(empty_may_be_null && o.rows == 0) && (!o.x || !o.codes || !o.scales))
        return QUEST_ERR_NULL;
    const quest_status shape = shape_checks(o.rows, cols, had_block, log2n);
    if (shape != QUEST_OK)
        return shape;
    if (o.ld < cols)
        return QUEST_ERR_SHAPE;
    const int64_t elem = dtype == QUEST_BF16 ? 2 : 4;
    if (!aligned16(o.x) || !aligned16(o.codes) || (o.mask && !aligned16(o.mask)) || ((o.ld * elem) & 15) ||
        (reinterpret_cast<uintptr_t>(o.scales) & 3u))
        return QUEST_ERR_ALIGN;
    return QUEST_OK;
}

// Shared by the quantizer entry points; absmax ignores alpha and outer_trust.  `second` is the other
// operand of a pair call (same dtype, row length, block, grid and clip), or null.
quest_status quantize_entry(const QuantOperand &first, const QuantOperand *second, quest_dtype dtype, int64_t cols,
                            int32_t had_block, int32_t bits, float alpha, float outer_trust, int mode,
                            float *xh_out, void *stream)
{
    if (dtype != QUEST_F32 && dtype != QUEST_BF16)
        return (second && first.rows == 0) || (first.x && first.codes && first.scales) ? QUEST_ERR_DTYPE
                                                                                      : QUEST_ERR_NULL;
    const int cb = container_bits(bits);
    int log2n = 0;
    quest_status status = check_quant_operand(first, dtype, cols, had_block, &log2n, second != nullptr);
    if (status == QUEST_OK && second)
        status = check_quant_operand(*second, dtype, cols, had_block, &log2n, true);
    if (status == QUEST_ERR_NULL)
        return status;
    if (cb == 0)
        return QUEST_ERR_BITS;
    if (status != QUEST_OK)
        return status;
    if (xh_out && !aligned16(xh_out))
        return QUEST_ERR_ALIGN;
    if (second && first.rows != 0 && second->rows != 0 && ((first.mask == nullptr) != (second->mask == nullptr)))
        return QUEST_ERR_ARG;   // both masks or neither
    if (isnan(alpha) || isinf(alpha) || isnan(outer_trust) || isinf(outer_trust))
        return QUEST_ERR_ARG;

    const int levels = 1 << bits;
    const double a = alpha > 0.0f ? (double)alpha : mode == quest::kQuantFp4 ? kAlphaStarFp4 : alpha_star(bits);
    const double ot = outer_trust < 0.0f ? 1.0 : (double)outer_trust;
    // trusted iff |x_h| <= edge * rms: the clip plus one trust width T (times outer_trust);
    // T = alpha / (L - 1) on the Eq. 1 grid, alpha / 6 (largest half-interval) on the FP4 grid
    const double width = mode == quest::kQuantFp4 ? 1.0 / 6.0 : 1.0 / (double)(levels - 1);

    quest::QuantizeArgs args;
    args.x = first.x;
    args.dtype = dtype;
    args.rows = first.rows;
    args.cols = cols;
    args.ld = first.ld;
    args.log2n = log2n;
    args.bits = bits;
    args.cb = cb;
    args.alpha = (float)a;
    args.trust_edge = (float)(a * (1.0 + ot * width));
    args.codes = first.codes;
    args.scales = first.scales;
    args.mask = first.mask;
    args.xh_out = xh_out;
    args.mode = mode;
    if (second) {
        args.x2 = second->x;
        args.rows2 = second->rows;
        args.ld2 = second->ld;
        args.codes2 = second->codes;
        args.scales2 = second->scales;
        args.mask2 = second->mask;
    }
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
    return quantize_entry({x, rows, ld, codes, scales, mask}, nullptr, dtype, cols, had_block, bits, alpha,
                          outer_trust, quest::kQuantRms, xh_out, stream);
}

quest_status quest_hadamard_quantize_pair(const void *x, int64_t rows_x, int64_t ld_x, uint8_t *codes_x,
                                          float *scales_x, uint8_t *mask_x, const void *w, int64_t rows_w,
                                          int64_t ld_w, uint8_t *codes_w, float *scales_w, uint8_t *mask_w,
                                          quest_dtype dtype, int64_t cols, int32_t had_block, int32_t bits,
                                          float alpha, float outer_trust, void *stream)
{
    const QuantOperand second = {w, rows_w, ld_w, codes_w, scales_w, mask_w};
    return quantize_entry({x, rows_x, ld_x, codes_x, scales_x, mask_x}, &second, dtype, cols, had_block, bits,
                          alpha, outer_trust, quest::kQuantRms, nullptr, stream);
}

quest_status quest_hadamard_quantize_absmax(const void *x, quest_dtype dtype, int64_t rows,
                                            int64_t cols, int64_t ld, int32_t had_block, int32_t bits,
                                            uint8_t *codes, float *scales, uint8_t *mask,
                                            float *xh_out, void *stream)
{
    return quantize_entry({x, rows, ld, codes, scales, mask}, nullptr, dtype, cols, had_block, bits, 0.0f, -1.0f,
                          quest::kQuantAbsMax, xh_out, stream);
}

quest_status quest_hadamard_quantize_fp4(const void *x, quest_dtype dtype, int64_t rows, int64_t cols,
                                         int64_t ld, int32_t had_block, float alpha, uint8_t *codes,
                                         float *scales, uint8_t *mask, float *xh_out, void *stream)
{
    return quantize_entry({x, rows, ld, codes, scales, mask}, nullptr, dtype, cols, had_block, 4, alpha, -1.0f,
                          quest::kQuantFp4, xh_out, stream);
}

quest_status quest_hadamard_quantize_fp4_pair(const void *x, int64_t rows_x, int64_t ld_x, uint8_t *codes_x,
                                              float *scales_x, uint8_t *mask_x, const void *w,
                                              int64_t rows_w, int64_t ld_w, uint8_t *codes_w,
                                              float *scales_w, uint8_t *mask_w, quest_dtype dtype,
                                              int64_t cols, int32_t had_block, float alpha, void *stream)
{
    const QuantOperand second = {w, rows_w, ld_w, codes_w, scales_w, mask_w};
    return quantize_entry({x, rows_x, ld_x, codes_x, scales_x, mask_x}, &second, dtype, cols, had_block, 4,
                          alpha, -1.0f, quest::kQuantFp4, nullptr, stream);
}

float quest_alpha_star_fp4(void)
{
    return (float)kAlphaStarFp4;
}

namespace {

quest_status lowbit_gemm_entry(const uint8_t *a_codes, const float *a_scales, int64_t M,
                               const uint8_t *b_codes, const float *b_scales, int64_t N, int64_t K,
                               int32_t bits, void *y, int64_t ld_y, int32_t *acc_out, void *workspace,
                               int64_t workspace_bytes, void *stream)
{
    if (!a_codes || !a_scales || !b_codes || !b_scales || (!y && !acc_out))
        return QUEST_ERR_NULL;
    if (bits < 1 || bits > 4)
        return QUEST_ERR_BITS;
    // the tile kernels keep per-lane byte offsets into an operand (rows of K/2 bytes as nibbles) in 32 bits
    if (M < 0 || N < 0 || M > (int64_t(1) << 22) || N > (int64_t(1) << 22) || K < 64 ||
        K > 65536 || (K & 63) || (M > N ? M : N) * (K / 2) >= (int64_t(1) << 32))
        return QUEST_ERR_SHAPE;
    if (y && ld_y < N)
        return QUEST_ERR_SHAPE;
    if (!aligned16(a_codes) || !aligned16(b_codes) || (y && !aligned16(y)) ||
        (acc_out && !aligned16(acc_out)) || (workspace && !aligned16(workspace)))
        return QUEST_ERR_ALIGN;
    if (workspace_bytes < 0 ||
        (workspace && workspace_bytes < quest::lowbit_gemm_workspace_bytes(M, N, K, bits)))
        return QUEST_ERR_ARG;

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
    args.workspace = workspace;
    args.workspace_bytes = workspace_bytes;
    return quest::launch_lowbit_gemm(args, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUEST_OK
               : QUEST_ERR_LAUNCH;
}

}  // namespace

int64_t quest_lowbit_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int32_t bits)
{
    if (bits < 1 || bits > 4 || M < 0 || N < 0 || M > (int64_t(1) << 22) || N > (int64_t(1) << 22) || K < 64 ||
        K > 65536 || (K & 63) || (M > N ? M : N) * (K / 2) >= (int64_t(1) << 32))
        return -1;
    return quest::lowbit_gemm_workspace_bytes(M, N, K, bits);
}

quest_status quest_lowbit_gemm(const uint8_t *a_codes, const float *a_scales, int64_t M,
                               const uint8_t *b_codes, const float *b_scales, int64_t N, int64_t K,
                               int32_t bits, void *y, int64_t ld_y, int32_t *acc_out, void *workspace,
                               int64_t workspace_bytes, void *stream)
{
    return lowbit_gemm_entry(a_codes, a_scales, M, b_codes, b_scales, N, K, bits, y, ld_y, acc_out, workspace,
                             workspace_bytes, stream);
}

quest_status quest_lowbit_gemm_static(const uint8_t *a_codes, const float *a_scales, int64_t M,
                                      const uint8_t *b_codes, const float *b_scales, int64_t N, int64_t K,
                                      int32_t bits, void *y, int64_t ld_y, int32_t *acc_out, void *stream)
{
    // same validation as quest_lowbit_gemm, with no workspace; then the size against the built-in buffer
    const int64_t needed = quest_lowbit_gemm_workspace_bytes(M, N, K, bits);
    if (needed > QUEST_STATIC_SCRATCH_BYTES)
        return QUEST_ERR_SCRATCH;
    void *ptr = nullptr;
    int64_t bytes = 0;
    if (needed > 0 && a_codes && a_scales && b_codes && b_scales && (y || acc_out)) {
        if (static_scratch_address(&ptr) != hipSuccess)
            return QUEST_ERR_LAUNCH;
        bytes = QUEST_STATIC_SCRATCH_BYTES;
    }
    return lowbit_gemm_entry(a_codes, a_scales, M, b_codes, b_scales, N, K, bits, y, ld_y, acc_out, ptr, bytes,
                             stream);
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

namespace {

// One gradient of an inverse-transform call (rows of `cols` elements, its mask or null, its output).
struct BackwardOperand {
    const void *g;
    const uint8_t *mask;
    int64_t rows;
    void *out;
};

// `second` is the other gradient of a pair call (same dtypes, row length and block), or null; a
// gradient of a pair call that has no rows needs no buffers.
quest_status trust_backward_entry(const BackwardOperand &first, const BackwardOperand *second, quest_dtype g_dtype,
                                  int64_t cols, int32_t had_block, quest_dtype out_dtype, void *stream)
{
    const BackwardOperand *operands[2] = {&first, second};
    for (const BackwardOperand *o : operands)
        if (o && !(second && o->rows == 0) && (!o->g || !o->out))
            return QUEST_ERR_NULL;
    if ((g_dtype != QUEST_F32 && g_dtype != QUEST_BF16) ||
        (out_dtype != QUEST_F32 && out_dtype != QUEST_BF16))
        return QUEST_ERR_DTYPE;
    int log2n = 0;
    for (const BackwardOperand *o : operands) {
        if (!o)
            continue;
        const quest_status shape = shape_checks(o->rows, cols, had_block, &log2n);
        if (shape != QUEST_OK)
            return shape;
        if (!aligned16(o->g) || !aligned16(o->out) || (o->mask && !aligned16(o->mask)))
            return QUEST_ERR_ALIGN;
    }
    if (second && first.rows != 0 && second->rows != 0 && ((first.mask == nullptr) != (second->mask == nullptr)))
        return QUEST_ERR_ARG;   // both masks or neither

    quest::BackwardArgs args;
    args.g = first.g;
    args.g_dtype = g_dtype;
    args.mask = first.mask;
    args.rows = first.rows;
    args.cols = cols;
    args.log2n = log2n;
    args.out = first.out;
    args.out_dtype = out_dtype;
    if (second) {
        args.g2 = second->g;
        args.mask2 = second->mask;
        args.rows2 = second->rows;
        args.out2 = second->out;
    }
    return quest::launch_trust_backward(args, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUEST_OK
               : QUEST_ERR_LAUNCH;
}

}  // namespace

quest_status quest_trust_backward(const void *g, quest_dtype g_dtype, const uint8_t *mask,
                                  int64_t rows, int64_t cols, int32_t had_block, void *out,
                                  quest_dtype out_dtype, void *stream)
{
    return trust_backward_entry({g, mask, rows, out}, nullptr, g_dtype, cols, had_block, out_dtype, stream);
}

quest_status quest_trust_backward_pair(const void *g_x, const uint8_t *mask_x, int64_t rows_x, void *out_x,
                                       const void *g_w, const uint8_t *mask_w, int64_t rows_w, void *out_w,
                                       quest_dtype g_dtype, int64_t cols, int32_t had_block,
                                       quest_dtype out_dtype, void *stream)
{
    const BackwardOperand second = {g_w, mask_w, rows_w, out_w};
    return trust_backward_entry({g_x, mask_x, rows_x, out_x}, &second, g_dtype, cols, had_block, out_dtype,
                                stream);
}

namespace {

// Shape rules shared by the three entry points on the bf16 tile kernels and by their size queries.
// form: 0 / 1 = the gradient matmuls of Algorithm 2, 2 = the weight-only forward product.
bool grad_family_shape_ok(int form, bool fp4, int64_t M, int64_t N, int64_t K)
{
    const int64_t limit = int64_t(1) << 22;
    if (M < 0 || N < 0 || K < 0 || (M & 63) || (N & 63) || (K & 63) || M > limit || N > limit || K > limit)
        return false;
    if (M == 0 || N == 0 || K == 0)
        return true;
    return quest::grad_gemm_workspace_bytes(form, fp4, M, N, K, quest::device_compute_units()) >= 0;
}

quest_status grad_family_entry(int form, bool fp4, const void *left, const uint8_t *q_codes, const float *q_scales,
                               int32_t bits, int64_t M, int64_t N, int64_t K, void *out, void *workspace,
                               int64_t workspace_bytes, void *stream)
{
    if (!left || !q_codes || !q_scales || !out)
        return QUEST_ERR_NULL;
    if (bits < 1 || bits > 4)
        return QUEST_ERR_BITS;
    if (!grad_family_shape_ok(form, fp4, M, N, K))
        return QUEST_ERR_SHAPE;
    if (!aligned16(left) || !aligned16(q_codes) || !aligned16(out) || (workspace && !aligned16(workspace)))
        return QUEST_ERR_ALIGN;
    const int64_t needed = (M == 0 || N == 0 || K == 0)
                               ? 0
                               : quest::grad_gemm_workspace_bytes(form, fp4, M, N, K, quest::device_compute_units());
    if (workspace_bytes < 0 || (needed > 0 && (!workspace || workspace_bytes < needed)))
        return QUEST_ERR_ARG;

    quest::GradGemmArgs args;
    args.which = form;
    args.fp4 = fp4;
    args.dy = left;
    args.q_codes = q_codes;
    args.q_scales = q_scales;
    args.bits = bits;
    args.cb = container_bits(bits);
    args.M = M;
    args.N = N;
    args.K = K;
    args.out = out;
    args.workspace = workspace;
    args.workspace_bytes = workspace_bytes;
    return quest::launch_grad_gemm(args, static_cast<hipStream_t>(stream)) == hipSuccess
               ? QUEST_OK
               : QUEST_ERR_LAUNCH;
}

}  // namespace

int64_t quest_grad_gemm_workspace_bytes(int32_t which, int64_t M, int64_t N, int64_t K)
{
    if ((which != 0 && which != 1) || !grad_family_shape_ok(which, false, M, N, K))
        return -1;
    if (M == 0 || N == 0 || K == 0)
        return 0;
    return quest::grad_gemm_workspace_bytes(which, false, M, N, K, quest::device_compute_units());
}

quest_status quest_grad_gemm(int32_t which, const void *dy, const uint8_t *q_codes,
                             const float *q_scales, int32_t bits, int64_t M, int64_t N, int64_t K,
                             void *out, void *workspace, int64_t workspace_bytes, void *stream)
{
    if (which != 0 && which != 1)
        return QUEST_ERR_ARG;
    return grad_family_entry(which, false, dy, q_codes, q_scales, bits, M, N, K, out, workspace, workspace_bytes,
                             stream);
}

int64_t quest_grad_gemm_fp4_workspace_bytes(int32_t which, int64_t M, int64_t N, int64_t K)
{
    if ((which != 0 && which != 1) || !grad_family_shape_ok(which, true, M, N, K))
        return -1;
    if (M == 0 || N == 0 || K == 0)
        return 0;
    return quest::grad_gemm_workspace_bytes(which, true, M, N, K, quest::device_compute_units());
}

quest_status quest_grad_gemm_fp4(int32_t which, const void *dy, const uint8_t *q_codes,
                                 const float *q_scales, int64_t M, int64_t N, int64_t K, void *out,
                                 void *workspace, int64_t workspace_bytes, void *stream)
{
    if (which != 0 && which != 1)
        return QUEST_ERR_ARG;
    return grad_family_entry(which, true, dy, q_codes, q_scales, 4, M, N, K, out, workspace, workspace_bytes,
                             stream);
}

int64_t quest_weight_only_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (!grad_family_shape_ok(2, false, M, N, K))
        return -1;
    if (M == 0 || N == 0 || K == 0)
        return 0;
    return quest::grad_gemm_workspace_bytes(2, false, M, N, K, quest::device_compute_units());
}

quest_status quest_weight_only_gemm(const void *x, const uint8_t *w_codes, const float *w_scales,
                                    int32_t bits, int64_t M, int64_t N, int64_t K, void *y,
                                    void *workspace, int64_t workspace_bytes, void *stream)
{
    return grad_family_entry(2, false, x, w_codes, w_scales, bits, M, N, K, y, workspace, workspace_bytes,
                             stream);
}

quest_status quest_init(void)
{
    hipError_t err = quest::prepare_quantize_kernels();
    if (err == hipSuccess)
        err = quest::prepare_quantize_mfma_kernels();
    if (err == hipSuccess)
        err = quest::prepare_trust_backward_mfma_kernels();
    if (err == hipSuccess)
        err = quest::prepare_lowbit_gemm_kernels();
    if (err == hipSuccess)
        err = quest::prepare_fp4_gemm_kernels();
    if (err == hipSuccess)
        err = quest::prepare_trust_backward_kernels();
    if (err == hipSuccess)
        err = quest::prepare_grad_gemm_kernels();
    void *ptr = nullptr;
    if (err == hipSuccess)
        err = static_scratch_address(&ptr);
    return err == hipSuccess ? QUEST_OK : QUEST_ERR_LAUNCH;
}

}  // extern "C"
