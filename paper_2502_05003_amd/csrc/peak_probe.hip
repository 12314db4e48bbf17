// Register-only matrix-instruction loop: the rate the matrix pipes sustain on given operand data with
// no LDS or memory traffic (see include/quest_probe.h).  Measurement aid for bench.py.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/quest_probe.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Eight independent accumulator tiles per wave; operands rotate through four register copies so that
// consecutive instructions do not read the same registers.
template <int KIND>
__global__ __launch_bounds__(256) void mfma_loop_kernel(const uint4 *__restrict__ operands, int32_t *__restrict__ sink,
                                                        int iterations)
{
    const uint4 *mine = operands + (size_t)(blockIdx.x * 256 + threadIdx.x) * 2;
    uint4 a[4], b[4];
    a[0] = mine[0];
    b[0] = mine[1];
#pragma unroll
    for (int i = 1; i < 4; ++i) {   // lane-rotated copies: other values, same distribution
        a[i] = make_uint4(a[i - 1].y, a[i - 1].z, a[i - 1].w, a[i - 1].x);
        b[i] = make_uint4(b[i - 1].w, b[i - 1].x, b[i - 1].y, b[i - 1].z);
    }
    if constexpr (KIND == 0) {
        v16i acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][r] = 0;
        for (int it = 0; it < iterations; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint4 x = a[i & 3], y = b[(i + it) & 3];
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(v4i{(int)x.x, (int)x.y, (int)x.z, (int)x.w},
                                                               v4i{(int)y.x, (int)y.y, (int)y.z, (int)y.w}, acc[i], 0, 0, 0);
            }
        }
        int s = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                s += acc[i][r];
        sink[blockIdx.x * 256 + threadIdx.x] = s;
    } else {
        v16f acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[i][r] = 0.0f;
        for (int it = 0; it < iterations; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                v8bf x, y;
                __builtin_memcpy(&x, &a[i & 3], 16);
                __builtin_memcpy(&y, &b[(i + it) & 3], 16);
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc[i], 0, 0, 0);
            }
        }
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                s += acc[i][r];
        sink[blockIdx.x * 256 + threadIdx.x] = (int32_t)__float_as_uint(s);
    }
}

}  // namespace

extern "C" int32_t quest_probe_mfma_loop(int32_t kind, const void *operands, void *sink, int32_t workgroups,
                                         int32_t iterations, void *stream)
{
    if (!operands || !sink || workgroups <= 0 || iterations <= 0 || (kind != 0 && kind != 1))
        return 1;
    const dim3 grid((unsigned)workgroups), block(256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (kind == 0)
        hipLaunchKernelGGL(mfma_loop_kernel<0>, grid, block, 0, s, static_cast<const uint4 *>(operands),
                           static_cast<int32_t *>(sink), iterations);
    else
        hipLaunchKernelGGL(mfma_loop_kernel<1>, grid, block, 0, s, static_cast<const uint4 *>(operands),
                           static_cast<int32_t *>(sink), iterations);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
