// Measurement aid: the sustained rate of the matrix cores on caller-chosen operand values.
//
// The published dense bf16 peak assumes the nominal shader clock.  Under a long run of matrix
// instructions the clock is set by the power management, and the power drawn depends on how
// many operand bits toggle: zero or constant operands run near the nominal clock, normally
// distributed ones (what attention feeds the matrix cores) well below it.  This kernel issues
// nothing but independent v_mfma_f32_32x32x16_bf16 from registers, one wave per SIMD on every
// CU, so its rate is the ceiling any matrix-core-bound kernel can reach on the same data.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ta_probe.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kProbeBlocks = 256;    // one per CU
constexpr int kProbeThreads = 256;   // one wave per SIMD
constexpr int kStreamBlocks = 8192;  // grid-stride; 32 workgroups per CU

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

// Streaming read: every byte of the buffer once, 16 bytes per lane, non-temporal, the access
// pattern of the decode kernel without its arithmetic.  Its rate is the read bandwidth the
// memory system delivers to a kernel of that shape.
__global__ __launch_bounds__(256) void stream_read_probe_kernel(const u32x4* __restrict__ src, size_t n_vec,
                                                                uint32_t* __restrict__ sink) {
    u32x4 acc = {0u, 0u, 0u, 0u};
    const size_t stride = size_t(gridDim.x) * blockDim.x * 4;
    size_t i = size_t(blockIdx.x) * blockDim.x * 4 + threadIdx.x;
    for (; i + 3 * 256 < n_vec; i += stride) {      // four independent loads in flight per lane
        const u32x4 a = __builtin_nontemporal_load(src + i);
        const u32x4 b = __builtin_nontemporal_load(src + i + 256);
        const u32x4 c = __builtin_nontemporal_load(src + i + 512);
        const u32x4 d = __builtin_nontemporal_load(src + i + 768);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n_vec; i += 256) acc ^= __builtin_nontemporal_load(src + i);   // ragged tail of the last block
    sink[blockIdx.x * blockDim.x + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

// Two waves per SIMD (512 threads on every CU); per iteration each wave issues NM independent
// matrix instructions and NV independent fp32 FMAs, interleaved.  Timing the three cases (matrix
// only, vector only, both) shows how much of a matrix instruction's time the vector issue port
// is unavailable to the other wave.
template <int NM, int NV>
__global__ __launch_bounds__(512) void issue_port_probe_kernel(float* __restrict__ sink, int32_t iters, float seed) {
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = static_cast<__bf16>(seed + i);
        b[i] = static_cast<__bf16>(seed * 0.5f + (threadIdx.x & 7));
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = seed + i + threadIdx.x;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (u < NM) acc[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[u & 3], 0, 0, 0);
#pragma unroll
            for (int w = 0; w < NV / 8; ++w) v[(u + w) & 7] = __builtin_fmaf(v[(u + w) & 7], 1.0001f, 0.5f);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
#pragma unroll
    for (int i = 0; i < 8; ++i) s += v[i];
    sink[blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace

extern "C" {

int ta_issue_port_probe(int32_t matrix_per_iter, int32_t vector_per_iter, int32_t iters, void* sink, void* hip_stream) {
    if (sink == nullptr || iters < 1 || (reinterpret_cast<uintptr_t>(sink) & 3) != 0) return -1;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    float* out = static_cast<float*>(sink);
    const dim3 grid(kProbeBlocks), block(512);
    if (matrix_per_iter == 8 && vector_per_iter == 0) hipLaunchKernelGGL((issue_port_probe_kernel<8, 0>), grid, block, 0, st, out, iters, 1.0f);
    else if (matrix_per_iter == 0 && vector_per_iter == 40) hipLaunchKernelGGL((issue_port_probe_kernel<0, 40>), grid, block, 0, st, out, iters, 1.0f);
    else if (matrix_per_iter == 0 && vector_per_iter == 80) hipLaunchKernelGGL((issue_port_probe_kernel<0, 80>), grid, block, 0, st, out, iters, 1.0f);
    else if (matrix_per_iter == 8 && vector_per_iter == 40) hipLaunchKernelGGL((issue_port_probe_kernel<8, 40>), grid, block, 0, st, out, iters, 1.0f);
    else if (matrix_per_iter == 8 && vector_per_iter == 80) hipLaunchKernelGGL((issue_port_probe_kernel<8, 80>), grid, block, 0, st, out, iters, 1.0f);
    else return -1;
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

int ta_stream_read_probe(const void* src, size_t bytes, void* sink, void* hip_stream) {
    if (src == nullptr || sink == nullptr || bytes == 0 || (bytes & 15) != 0) return -1;
    if ((reinterpret_cast<uintptr_t>(src) & 15) != 0 || (reinterpret_cast<uintptr_t>(sink) & 3) != 0) return -1;
    hipLaunchKernelGGL(stream_read_probe_kernel, dim3(kStreamBlocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const u32x4*>(src), bytes / 16, static_cast<uint32_t*>(sink));
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

int ta_matrix_core_probe(const void* operands, int32_t iters, void* sink, void* hip_stream) {
    if (operands == nullptr || sink == nullptr || iters < 1) return -1;
    if ((reinterpret_cast<uintptr_t>(operands) & 15) != 0 || (reinterpret_cast<uintptr_t>(sink) & 3) != 0) return -1;
    hipLaunchKernelGGL(matrix_core_probe_kernel, dim3(kProbeBlocks), dim3(kProbeThreads), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const u32x4*>(operands), iters,
                       static_cast<float*>(sink));
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

}  // extern "C"
