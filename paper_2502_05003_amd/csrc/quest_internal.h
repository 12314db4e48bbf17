// Host-side declarations shared by the QuEST translation units: one launcher per kernel family.
// Launchers assume validated arguments (the C-ABI entry points validate) and only enqueue work.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/quest.h"

namespace quest {

enum { kQuantRms = 0, kQuantAbsMax = 1, kQuantFp4 = 2 };

struct QuantizeArgs {
    const void *x;
    quest_dtype dtype;
    int64_t rows, cols, ld;
    int log2n;         // log2(had_block)
    int bits;          // b
    int cb;            // container bits
    float alpha;       // clip in RMS units
    float trust_edge;  // alpha * (1 + outer_trust / (L - 1)): trusted iff |x_h| <= trust_edge * rms
    uint8_t *codes;
    float *scales;
    uint8_t *mask;     // may be null
    float *xh_out;     // may be null
    int mode;          // kQuantRms: Eq. 1 grid, clip alpha * rms;  kQuantAbsMax: Eq. 1 grid, clip = largest
                       // |x_h| of the row (alpha, trust_edge unused);  kQuantFp4: E2M1 grid, clip alpha * rms
    // a second operand with the same dtype, cols, block, grid and clip, quantized by the same launch
    // (rows2 = 0: none); its mask is given exactly when `mask` is; it has no xh_out
    const void *x2 = nullptr;
    int64_t rows2 = 0, ld2 = 0;
    uint8_t *codes2 = nullptr;
    float *scales2 = nullptr;
    uint8_t *mask2 = nullptr;
};

hipError_t launch_hadamard_quantize(const QuantizeArgs &a, hipStream_t stream);
// Matrix-core kernel for the common bf16 / 4-bit shapes; false means "not covered, nothing launched".
bool launch_hadamard_quantize_mfma(const QuantizeArgs &a, hipStream_t stream);

struct GemmArgs {
    const uint8_t *a_codes;
    const float *a_scales;
    const uint8_t *b_codes;
    const float *b_scales;
    int64_t M, N, K;
    int bits, cb;
    void *y;          // bf16, may be null
    int64_t ld_y;
    int32_t *acc_out; // may be null
    void *workspace;  // caller's scratch for the re-coded operands of 1- and 2-bit products; may be null
    int64_t workspace_bytes;
};

hipError_t launch_lowbit_gemm(const GemmArgs &a, hipStream_t stream);
// Scratch the fast path of a 1- or 2-bit product needs (both operands re-coded as nibbles); 0 when the
// shape or the bit width does not take that path.
int64_t lowbit_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int bits);

struct Fp4GemmArgs {
    const uint8_t *a_codes;
    const float *a_scales;
    const uint8_t *b_codes;
    const float *b_scales;
    int64_t M, N, K;
    void *y;          // bf16, may be null
    int64_t ld_y;
    float *acc_out;   // may be null
};

hipError_t launch_fp4_gemm(const Fp4GemmArgs &a, hipStream_t stream);

struct BackwardArgs {
    const void *g;
    quest_dtype g_dtype;
    const uint8_t *mask;  // may be null
    int64_t rows, cols;
    int log2n;
    void *out;
    quest_dtype out_dtype;
    // second gradient of the same row length, dtypes and block, served by the same launch where the
    // matrix-core kernel covers the shape (rows2 = 0: none)
    const void *g2 = nullptr;
    const uint8_t *mask2 = nullptr;
    int64_t rows2 = 0;
    void *out2 = nullptr;
};

hipError_t launch_trust_backward(const BackwardArgs &a, hipStream_t stream);
// Matrix-core kernel for bf16 in / bf16 out and the common shapes; false means "not covered".
bool launch_trust_backward_mfma(const BackwardArgs &a, hipStream_t stream);

struct GradGemmArgs {
    int which;
    const void *dy;
    const uint8_t *q_codes;
    const float *q_scales;
    int bits, cb;
    bool fp4;          // the codes are E2M1 codes (bits = cb = 4)
    int64_t M, N, K;
    void *out;
    void *workspace;   // caller's scratch: the expanded operand, then the partial tiles
    int64_t workspace_bytes;
};

// hipErrorInvalidValue: the shape is not one the kernels cover, or the workspace is too small
// (the entry points check both beforehand with grad_gemm_workspace_bytes).
hipError_t launch_grad_gemm(const GradGemmArgs &a, hipStream_t stream);
// Scratch bytes a call with these arguments needs on a device with `cus` compute units (0 for the
// small-shape kernel, which dequantizes in place); -1 when no kernel covers the shape.
int64_t grad_gemm_workspace_bytes(int which, bool fp4, int64_t M, int64_t N, int64_t K, int cus);

// Compute units of the current device, rounded down to a multiple of eight (one per XCD); 256, the
// MI355X's count, when no device can be asked (host-only use of the size queries).
int device_compute_units();

// Each family's kernels get their dynamic LDS limits on the current device, and the code objects of
// the files without such kernels are loaded (what quest_init does, so that no enqueue call has to
// change a kernel attribute or load code later).
hipError_t prepare_quantize_kernels();
hipError_t prepare_quantize_mfma_kernels();
hipError_t prepare_trust_backward_mfma_kernels();
hipError_t prepare_lowbit_gemm_kernels();
hipError_t prepare_fp4_gemm_kernels();
hipError_t prepare_trust_backward_kernels();
hipError_t prepare_grad_gemm_kernels();

// Raise the dynamic LDS limit of `kernel` to `bytes` on the current device.  The attribute is set
// once per (kernel, device, size) and remembered; safe to call from several host threads.
hipError_t allow_dynamic_lds(const void *kernel, int bytes);

}  // namespace quest
