// Measurement aid: the sustained rate of the matrix cores on caller-chosen operand values.
//
// The published dense bf16 peak assumes the nominal shader clock.  Under a long run of matrix
// instructions the clock is set by the power management, and the power drawn depends on how
// many operand bits toggle: zero or constant operands run near the nominal clock, normally
// distributed ones (what attention feeds the matrix cores) well below it.  This kernel issues
// nothing but independent v_mfma_f32_32x32x16_bf16 from registers, one wave per SIMD on every
// CU, so its rate is the ceiling any matrix-core-bound kernel can reach on the same data.
#include "ta_internal.h"

namespace ta {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kProbeBlocks = 256;    // one per CU
constexpr int kProbeThreads = 256;   // one wave per SIMD

__global__ __launch_bounds__(kProbeThreads) void matrix_core_probe_kernel(const u32x4* __restrict__ operands,
                                                                          int32_t iters, float* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = __builtin_bit_cast(bf16x8, operands[(2 * i) * 64 + lane]);
        b[i] = __builtin_bit_cast(bf16x8, operands[(2 * i + 1) * 64 + lane]);
    }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + u) & 3], b[i], acc[i], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    sink[blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

}  // namespace

int launch_matrix_core_probe(const void* operands, int32_t iters, void* sink, hipStream_t stream) {
    hipLaunchKernelGGL(matrix_core_probe_kernel, dim3(kProbeBlocks), dim3(kProbeThreads), 0, stream,
                       static_cast<const u32x4*>(operands), iters, static_cast<float*>(sink));
    TA_HIP_TRY(hipGetLastError());
    return TA_OK;
}

}  // namespace ta
