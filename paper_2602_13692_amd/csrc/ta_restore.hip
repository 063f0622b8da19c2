// KV page restore for gfx950: pages that a paused program left in pinned host
// memory are written back into free slots of the device page pool (ThunderAgent
// Sec. 4.3, Restore after Pause; host offloading in App. A.2 and A.4).  Bytes
// only: k_pool[dst[i]] = host_k[i], v_pool[dst[i]] = host_v[i].
//
// Two routes, chosen by how much staging the caller provides:
//   staged     large host-to-device copies into staging, then a scatter kernel
//              (device to device, HBM-bound, a small fraction of the link time);
//   zero-copy  the scatter kernel reads the pinned host pages over the link.
// The slot list always goes through the head of the staging buffer.
#include "ta_internal.h"

namespace ta {
namespace {

constexpr int kScatterThreads = 256;

// One workgroup per (page, K-or-V): copies page_bytes with 16-byte lanes.
__global__ __launch_bounds__(kScatterThreads) void scatter_pages_kernel(
    char* __restrict__ k_pool, char* __restrict__ v_pool, const char* __restrict__ src_k,
    const char* __restrict__ src_v, const int32_t* __restrict__ slots, int32_t first_page,
    int32_t n_pages, int64_t page_bytes) {
    const int i = blockIdx.x >> 1;
    if (i >= n_pages) return;
    const bool is_v = (blockIdx.x & 1) != 0;
    const int64_t slot = slots[first_page + i];
    const uint4* src = reinterpret_cast<const uint4*>((is_v ? src_v : src_k) + int64_t(i) * page_bytes);
    uint4* dst = reinterpret_cast<uint4*>((is_v ? v_pool : k_pool) + slot * page_bytes);
    const int64_t n16 = page_bytes / 16;
    int64_t t = threadIdx.x;
    // four independent 16-byte loads in flight per lane
    for (; t + 3 * kScatterThreads < n16; t += 4 * kScatterThreads) {
        const uint4 a = src[t];
        const uint4 b = src[t + kScatterThreads];
        const uint4 c = src[t + 2 * kScatterThreads];
        const uint4 d = src[t + 3 * kScatterThreads];
        dst[t] = a;
        dst[t + kScatterThreads] = b;
        dst[t + 2 * kScatterThreads] = c;
        dst[t + 3 * kScatterThreads] = d;
    }
    for (; t < n16; t += kScatterThreads) dst[t] = src[t];
}

}  // namespace

int launch_restore(void* k_pool, void* v_pool, size_t page_bytes, const void* host_k,
                   const void* host_v, const int32_t* dst_slots, int32_t n_pages, void* staging,
                   size_t staging_bytes, hipStream_t stream) {
    const size_t slot_bytes = ta_restore_staging_min_bytes(n_pages);
    int32_t* slots_dev = static_cast<int32_t*>(staging);
    TA_HIP_TRY(hipMemcpyAsync(slots_dev, dst_slots, sizeof(int32_t) * size_t(n_pages),
                              hipMemcpyHostToDevice, stream));
    char* kp = static_cast<char*>(k_pool);
    char* vp = static_cast<char*>(v_pool);
    const char* hk = static_cast<const char*>(host_k);
    const char* hv = static_cast<const char*>(host_v);

    const size_t room = staging_bytes - slot_bytes;
    const size_t half = (room / 2) & ~size_t(255);
    const int64_t per_round = static_cast<int64_t>(half / page_bytes);
    if (per_round < 1) {
        // zero-copy: pinned host memory is mapped into the device address space
        hipLaunchKernelGGL(scatter_pages_kernel, dim3(2u * unsigned(n_pages)), dim3(kScatterThreads), 0,
                           stream, kp, vp, hk, hv, slots_dev, 0, n_pages, int64_t(page_bytes));
        TA_HIP_TRY(hipGetLastError());
        return TA_OK;
    }
    char* stage_k = static_cast<char*>(staging) + slot_bytes;
    char* stage_v = stage_k + half;
    for (int64_t first = 0; first < n_pages; first += per_round) {
        const int64_t n = (n_pages - first) < per_round ? (n_pages - first) : per_round;
        const size_t bytes = size_t(n) * page_bytes;
        TA_HIP_TRY(hipMemcpyAsync(stage_k, hk + size_t(first) * page_bytes, bytes, hipMemcpyHostToDevice, stream));
        TA_HIP_TRY(hipMemcpyAsync(stage_v, hv + size_t(first) * page_bytes, bytes, hipMemcpyHostToDevice, stream));
        hipLaunchKernelGGL(scatter_pages_kernel, dim3(2u * unsigned(n)), dim3(kScatterThreads), 0, stream,
                           kp, vp, stage_k, stage_v, slots_dev, int32_t(first), int32_t(n),
                           int64_t(page_bytes));
        TA_HIP_TRY(hipGetLastError());
    }
    return TA_OK;
}

}  // namespace ta
