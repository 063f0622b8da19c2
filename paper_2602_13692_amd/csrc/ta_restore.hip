// KV page restore for gfx950: pages that a paused program left in pinned host
// memory are written back into free slots of the device page pool (ThunderAgent
// Sec. 4.3, Restore after Pause; host offloading in App. A.2 and A.4).  Bytes
// only: k_pool[dst[i]] = host_k[i], v_pool[dst[i]] = host_v[i].
//
// Two routes, chosen by how much staging the caller provides:
//   staged     large host-to-device copies into staging, then a scatter kernel
//              (device to device, HBM-bound, a small fraction of the link time);
//   zero-copy  the scatter kernel reads the pinned host pages over the link.
// The caller's slot list is host memory: it travels to the device inside the kernel
// arguments, a batch of slots per launch, so the call reads it completely before it
// returns, needs no copy from pageable memory and waits for nothing on the stream.
#include "ta_internal.h"

#include <mutex>

namespace ta {
namespace {

constexpr int kScatterThreads = 256;
constexpr int kTwoRoundPages = 256;    // shortest round worth a stream of its own (8 MiB of K at eight kv heads)
constexpr int kSlotsPerLaunch = 960;   // 3840 bytes of the 4 KiB a kernel's arguments may take

struct SlotBatch {
    int32_t slot[kSlotsPerLaunch];
};

// Fills a batch from the caller's host list; returns the number of slots taken.
int32_t fill_batch(SlotBatch& batch, const int32_t* slots, int64_t first, int64_t end) {
    const int64_t n = (end - first) < kSlotsPerLaunch ? (end - first) : kSlotsPerLaunch;
    for (int64_t i = 0; i < n; ++i) batch.slot[i] = slots[first + i];
    return static_cast<int32_t>(n);
}

// Moves (page, K-or-V) units between pool slots and a contiguous array (pinned host memory or device
// staging), 16 bytes per lane and access, two accesses in flight per lane; a workgroup takes units
// with the stride of the grid.  GATHER: pool -> array, else array -> pool.
//
// The kernel is written to run beside attention: a program is restored or paused while the other
// programs keep decoding (Sec. 4.3; the bench measures both at once).  The tile kernel's workgroup takes
// 496 of the 512 vector registers of every SIMD of its compute unit; a wave of this kernel takes the
// sixteen that are left, so a workgroup of four waves fits beside it, and neither waits for the
// other.  (At 26 registers, and with one workgroup per unit in flight all over the chip, decode
// ran 2.7 times slower while a zero-copy restore was on its way, and a staged restore took 1.46
// times as long beside decode steps, its scatter launches waiting for compute units; now 1.3 and
// 1.11.)
template <bool GATHER>
__global__ __launch_bounds__(kScatterThreads) __attribute__((amdgpu_num_vgpr(16))) void move_pages_kernel(
    char* __restrict__ k_pool, char* __restrict__ v_pool, char* __restrict__ lin_k, char* __restrict__ lin_v,
    const SlotBatch slots, int32_t n_pages, int64_t page_bytes) {
    for (int unit = blockIdx.x; unit < 2 * n_pages; unit += gridDim.x) {
        const int i = unit >> 1;
        const bool is_v = (unit & 1) != 0;
        char* pool = (is_v ? v_pool : k_pool) + int64_t(slots.slot[i]) * page_bytes;
        char* lin = (is_v ? lin_v : lin_k) + int64_t(i) * page_bytes;
        // both bases are the same for all lanes (scalar registers); a lane adds a 32-bit offset
        const char* src = GATHER ? pool : lin;
        char* dst = GATHER ? lin : pool;
        const uint32_t bytes = static_cast<uint32_t>(page_bytes);      // below 2 GiB: checked by the caller
        constexpr uint32_t kStep = kScatterThreads * 16;
        uint32_t at = threadIdx.x * 16;
        for (; at + kStep < bytes; at += 2 * kStep) {
            const uint4 a = *reinterpret_cast<const uint4*>(src + at);
            const uint4 b = *reinterpret_cast<const uint4*>(src + (at + kStep));
            *reinterpret_cast<uint4*>(dst + at) = a;
            *reinterpret_cast<uint4*>(dst + (at + kStep)) = b;
        }
        if (at < bytes) *reinterpret_cast<uint4*>(dst + at) = *reinterpret_cast<const uint4*>(src + at);
    }
}

// Workgroups of one launch.  Reading or writing pinned host memory directly, a few keep the host link
// full (55 GB/s x a few microseconds of latency is well under a megabyte in flight; measured: the
// same 65 ms for 3.7 GB read with 16 .. 256 workgroups, 79 ms with 8).  More of them do harm when
// attention runs beside the transfer: every access to host memory that is on its way seems to hold
// a place in queues that HBM traffic also passes through -- a decode step beside a restore ran 1.14 x
// its time alone with 8 workgroups, 1.31 x with 32, 1.61 x with 64, 3.6 x with 256 -- while the restore
// itself needs 32 to stay within a tenth of its time alone beside decode steps (16: 1.7 x).  Writes to
// host memory weigh more (decode 1.27 x with 16 workgroups, 1.72 x with 32) and an eviction is less
// pressed than a restore, for which a program waits: 16 there (1.29 x its time alone beside decode
// steps, 1.03 x when nothing else runs).  Between pool and device staging the kernel is bound by HBM
// and takes as many workgroups as it has units.
unsigned move_grid(int32_t n, bool over_the_link, bool to_host) {
    const unsigned units = 2u * unsigned(n);
    const unsigned cap = to_host ? 16u : 32u;
    return over_the_link && units > cap ? cap : units;
}

// The staged routes alternate between copies over the host link (DMA engines) and kernels between
// staging and pool.  On one stream each waits for the other: the link idles while a kernel runs, and
// beside attention, where a kernel launch waits for compute units behind a decode step, it idles
// for that wait too (a staged restore took 1.12 x its time alone there).  With staging for two
// rounds the kernels go to a stream of the library's own, one per GPU, at the default priority like
// the caller's, tied to the caller's stream by events in both directions:
//   restore   caller's: [wait until the scatter of round i - 2 has read buffer i % 2] copy round i
//             side: [wait for that copy] scatter round i;  at the end the caller's stream waits for both buffers
//   evict     side: [wait until the copy of round i - 2 has left buffer i % 2] gather round i
//             caller's: [wait for that gather] copy round i
// so whatever the caller enqueues after the call still comes after all of it, and the side stream
// starts only after what the caller enqueued before.  (The copies stay on the caller's stream on
// purpose: the runtime gives a stream's copies to a DMA engine only if it finds one free for that
// stream, else to a copy kernel, which reads host memory at half the link's rate; measured with
// the copies on the side stream after other streams had made copies: 120 ms instead of 66.)  A
// stream that is being captured into a graph keeps the single-stream order.
struct SideLane {
    hipStream_t stream = nullptr;
    hipEvent_t begin = nullptr, copied[2] = {nullptr, nullptr}, moved[2] = {nullptr, nullptr};
    bool tried = false, ok = false;
};
constexpr int kMaxDevices = 64;
SideLane g_lanes[kMaxDevices];
std::mutex g_lane_mutex;      // creation, and one staged call at a time enqueues on a GPU's lane

// The current device's lane, or nullptr if it cannot be had (the caller then stays on one stream).
SideLane* side_lane(hipStream_t caller) {
    // (a query that fails here only means "stay on one stream": its error must not be found later by
    // the checks after the kernel launches)
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(caller, &capturing) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    if (capturing != hipStreamCaptureStatusNone) return nullptr;
    SideLane& lane = g_lanes[dev];
    if (!lane.tried) {
        lane.tried = true;
        bool ok = hipStreamCreateWithFlags(&lane.stream, hipStreamNonBlocking) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&lane.begin, hipEventDisableTiming) == hipSuccess;
        for (int i = 0; i < 2 && ok; ++i)
            ok = hipEventCreateWithFlags(&lane.copied[i], hipEventDisableTiming) == hipSuccess &&
                 hipEventCreateWithFlags(&lane.moved[i], hipEventDisableTiming) == hipSuccess;
        lane.ok = ok;
        if (!ok) (void)hipGetLastError();
    }
    return lane.ok ? &lane : nullptr;
}

// KV append: one workgroup per new token copies its K row and its V row of every kv head
// (16-byte lanes) to the place the block table gives the token.
__global__ __launch_bounds__(256) void append_tokens_kernel(
    const char* __restrict__ new_k, const char* __restrict__ new_v, const int32_t* __restrict__ cu_new,
    char* __restrict__ k_pool, char* __restrict__ v_pool, const int32_t* __restrict__ block_table,
    int32_t block_table_stride, const int32_t* __restrict__ context_lens, int32_t batch, int32_t num_kv_heads,
    int64_t stride_page_bytes, int64_t stride_head_bytes) {
    const int row = blockIdx.x;                       // index into new_k / new_v
    if (row >= cu_new[batch]) return;
    // the program that owns the row: last b with cu_new[b] <= row
    int lo = 0, hi = batch - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (cu_new[mid] <= row) lo = mid; else hi = mid - 1;
    }
    const int b = lo;
    const int n = cu_new[b + 1] - cu_new[b];
    const int token = context_lens[b] - n + (row - cu_new[b]);
    const int64_t page = block_table[int64_t(b) * block_table_stride + token / kPageSize];
    const int64_t dst_row = page * stride_page_bytes + int64_t(token % kPageSize) * (kHeadDim * 2);
    const int64_t src_row = int64_t(row) * num_kv_heads * (kHeadDim * 2);
    // 16 lanes cover one 256-byte row
    for (int piece = threadIdx.x; piece < num_kv_heads * 16 * 2; piece += blockDim.x) {
        const int is_v = piece / (num_kv_heads * 16);
        const int rest = piece - is_v * num_kv_heads * 16;
        const int g = rest >> 4, c = rest & 15;
        const uint4 x = *reinterpret_cast<const uint4*>((is_v ? new_v : new_k) + src_row + g * (kHeadDim * 2) + c * 16);
        *reinterpret_cast<uint4*>((is_v ? v_pool : k_pool) + dst_row + g * stride_head_bytes + c * 16) = x;
    }
}

// The E4M3 code nearest to q: ties to the code with an even mantissa, saturation at +-448 (a cache
// never acquires a NaN the model did not produce), NaN stays NaN, the sign of zero is kept.
//   below 2^-6 the format is a fixed-point grid of 2^-9 steps: round(|q| * 512), 8 being the first normal code;
//   above, the fp32 pattern is rounded at its bit 20 (3 mantissa bits stay) and the exponent re-biased (127 -> 7).
// The sign is the element's own (the scale is positive; the sign a division gives a NaN is not defined).
__device__ __forceinline__ uint32_t quantise_e4m3(float q, uint32_t element_bits) {
    const uint32_t sign = (element_bits >> 24) & 0x80u;
    const uint32_t a = __builtin_bit_cast(uint32_t, q) & 0x7fffffffu;
    if (a > 0x7f800000u) return sign | 0x7fu;
    if (a >= 0x43e00000u) return sign | 0x7eu;                    // |q| >= 448
    if (a < 0x3c800000u)                                          // |q| < 2^-6
        return sign | static_cast<uint32_t>(__builtin_rintf(__builtin_bit_cast(float, a) * 512.0f));
    const uint32_t r = a + 0x7ffffu + ((a >> 20) & 1u);
    return sign | ((r >> 20) - (120u << 3));
}

// KV append into an FP8 cache: as append_tokens_kernel, the bf16 rows being quantised on the way
// (x / scale in fp32, correctly rounded).  A lane takes eight elements: 16 bytes in, 8 bytes out.
__global__ __launch_bounds__(256) void append_tokens_fp8_kernel(
    const char* __restrict__ new_k, const char* __restrict__ new_v, const int32_t* __restrict__ cu_new,
    char* __restrict__ k_pool, char* __restrict__ v_pool, const int32_t* __restrict__ block_table,
    int32_t block_table_stride, const int32_t* __restrict__ context_lens, int32_t batch, int32_t num_kv_heads,
    int64_t stride_page_bytes, int64_t stride_head_bytes, float k_scale, float v_scale) {
    const int row = blockIdx.x;
    if (row >= cu_new[batch]) return;
    int lo = 0, hi = batch - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (cu_new[mid] <= row) lo = mid; else hi = mid - 1;
    }
    const int b = lo;
    const int n = cu_new[b + 1] - cu_new[b];
    const int token = context_lens[b] - n + (row - cu_new[b]);
    const int64_t page = block_table[int64_t(b) * block_table_stride + token / kPageSize];
    const int64_t dst_row = page * stride_page_bytes + int64_t(token % kPageSize) * kHeadDim;
    const int64_t src_row = int64_t(row) * num_kv_heads * (kHeadDim * 2);
    for (int piece = threadIdx.x; piece < num_kv_heads * 16 * 2; piece += blockDim.x) {
        const int is_v = piece / (num_kv_heads * 16);
        const int rest = piece - is_v * num_kv_heads * 16;
        const int g = rest >> 4, c = rest & 15;
        const float scale = is_v ? v_scale : k_scale;
        const uint4 x = *reinterpret_cast<const uint4*>((is_v ? new_v : new_k) + src_row + g * (kHeadDim * 2) + c * 16);
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
        uint32_t codes[2] = {0u, 0u};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t lo_bits = w[i] << 16, hi_bits = w[i] & 0xffff0000u;   // elements 2 i and 2 i + 1 as fp32
            const uint32_t pair = quantise_e4m3(__builtin_bit_cast(float, lo_bits) / scale, lo_bits) |
                                  (quantise_e4m3(__builtin_bit_cast(float, hi_bits) / scale, hi_bits) << 8);
            codes[i >> 1] |= pair << (16 * (i & 1));
        }
        *reinterpret_cast<uint2*>((is_v ? v_pool : k_pool) + dst_row + g * stride_head_bytes + c * 8) =
            make_uint2(codes[0], codes[1]);
    }
}

}  // namespace

int launch_evict(const void* k_pool, const void* v_pool, size_t page_bytes, void* host_k, void* host_v,
                 const int32_t* src_slots, int32_t n_pages, void* staging, size_t staging_bytes,
                 hipStream_t stream) {
    const char* kp = static_cast<const char*>(k_pool);
    const char* vp = static_cast<const char*>(v_pool);
    char* hk = static_cast<char*>(host_k);
    char* hv = static_cast<char*>(host_v);
    const size_t half = staging != nullptr ? (staging_bytes / 2) & ~size_t(255) : 0;
    const int64_t per_round = static_cast<int64_t>(half / page_bytes);
    SlotBatch batch;
    if (per_round < 1) {
        // zero-copy: the kernel writes the pinned host pages itself
        for (int64_t first = 0; first < n_pages;) {
            const int32_t n = fill_batch(batch, src_slots, first, n_pages);
            hipLaunchKernelGGL(move_pages_kernel<true>, dim3(move_grid(n, true, true)), dim3(kScatterThreads), 0, stream,
                               const_cast<char*>(kp), const_cast<char*>(vp), hk + size_t(first) * page_bytes,
                               hv + size_t(first) * page_bytes, batch, n, int64_t(page_bytes));
            TA_HIP_TRY(hipGetLastError());
            first += n;
        }
        return TA_OK;
    }
    char* stage_k = static_cast<char*>(staging);
    char* stage_v = stage_k + half;
    // staging for two rounds of at least kTwoRoundPages pages each, and more than one round to go: gathers on the side stream
    const int64_t per_buffer = per_round / 2;
    std::unique_lock<std::mutex> hold(g_lane_mutex);
    SideLane* lane = (per_buffer >= kTwoRoundPages && n_pages > per_buffer) ? side_lane(stream) : nullptr;
    if (lane == nullptr) hold.unlock();
    const int64_t step = lane != nullptr ? per_buffer : per_round;
    hipStream_t kernel_stream = stream;
    if (lane != nullptr) {      // the gathers start after what the caller enqueued before this call
        kernel_stream = lane->stream;
        TA_HIP_TRY(hipEventRecord(lane->begin, stream));
        TA_HIP_TRY(hipStreamWaitEvent(kernel_stream, lane->begin, 0));
    }
    int64_t round = 0;
    for (int64_t first = 0; first < n_pages; first += step, ++round) {
        const int64_t end = (n_pages - first) < step ? n_pages : first + step;
        const int buf = lane != nullptr ? int(round & 1) : 0;
        char* sk = stage_k + size_t(buf) * size_t(per_buffer) * page_bytes;
        char* sv = stage_v + size_t(buf) * size_t(per_buffer) * page_bytes;
        if (lane != nullptr && round >= 2) TA_HIP_TRY(hipStreamWaitEvent(kernel_stream, lane->copied[buf], 0));
        for (int64_t at = first; at < end;) {
            const int32_t n = fill_batch(batch, src_slots, at, end);
            hipLaunchKernelGGL(move_pages_kernel<true>, dim3(move_grid(n, false, false)), dim3(kScatterThreads), 0,
                               kernel_stream, const_cast<char*>(kp), const_cast<char*>(vp),
                               sk + size_t(at - first) * page_bytes, sv + size_t(at - first) * page_bytes, batch, n,
                               int64_t(page_bytes));
            TA_HIP_TRY(hipGetLastError());
            at += n;
        }
        const size_t bytes = size_t(end - first) * page_bytes;
        if (lane != nullptr) {
            TA_HIP_TRY(hipEventRecord(lane->moved[buf], kernel_stream));
            TA_HIP_TRY(hipStreamWaitEvent(stream, lane->moved[buf], 0));
        }
        TA_HIP_TRY(hipMemcpyAsync(hk + size_t(first) * page_bytes, sk, bytes, hipMemcpyDeviceToHost, stream));
        TA_HIP_TRY(hipMemcpyAsync(hv + size_t(first) * page_bytes, sv, bytes, hipMemcpyDeviceToHost, stream));
        if (lane != nullptr) TA_HIP_TRY(hipEventRecord(lane->copied[buf], stream));
    }
    return TA_OK;
}

int launch_append(const Geometry& g, const void* new_k, const void* new_v, const int32_t* cu_new_lens,
                  void* k_pool, void* v_pool, const int32_t* block_table, int32_t block_table_stride,
                  const int32_t* context_lens, int32_t batch, int32_t total_new, hipStream_t stream) {
    if (g.kv_fp8) {
        hipLaunchKernelGGL(append_tokens_fp8_kernel, dim3(unsigned(total_new)), dim3(256), 0, stream,
                           static_cast<const char*>(new_k), static_cast<const char*>(new_v), cu_new_lens,
                           static_cast<char*>(k_pool), static_cast<char*>(v_pool), block_table,
                           block_table_stride, context_lens, batch, g.num_kv_heads, g.stride_page_bytes,
                           g.stride_head_bytes, g.k_scale, g.v_scale);
        TA_HIP_TRY(hipGetLastError());
        return TA_OK;
    }
    hipLaunchKernelGGL(append_tokens_kernel, dim3(unsigned(total_new)), dim3(256), 0, stream,
                       static_cast<const char*>(new_k), static_cast<const char*>(new_v), cu_new_lens,
                       static_cast<char*>(k_pool), static_cast<char*>(v_pool), block_table,
                       block_table_stride, context_lens, batch, g.num_kv_heads, g.stride_page_bytes,
                       g.stride_head_bytes);
    TA_HIP_TRY(hipGetLastError());
    return TA_OK;
}

int launch_restore(void* k_pool, void* v_pool, size_t page_bytes, const void* host_k,
                   const void* host_v, const int32_t* dst_slots, int32_t n_pages, void* staging,
                   size_t staging_bytes, hipStream_t stream) {
    char* kp = static_cast<char*>(k_pool);
    char* vp = static_cast<char*>(v_pool);
    const char* hk = static_cast<const char*>(host_k);
    const char* hv = static_cast<const char*>(host_v);
    const size_t half = staging != nullptr ? (staging_bytes / 2) & ~size_t(255) : 0;
    const int64_t per_round = static_cast<int64_t>(half / page_bytes);
    SlotBatch batch;
    if (per_round < 1) {
        // zero-copy: pinned host memory is mapped into the device address space
        for (int64_t first = 0; first < n_pages;) {
            const int32_t n = fill_batch(batch, dst_slots, first, n_pages);
            hipLaunchKernelGGL(move_pages_kernel<false>, dim3(move_grid(n, true, false)), dim3(kScatterThreads), 0, stream, kp, vp,
                               const_cast<char*>(hk) + size_t(first) * page_bytes,
                               const_cast<char*>(hv) + size_t(first) * page_bytes, batch, n, int64_t(page_bytes));
            TA_HIP_TRY(hipGetLastError());
            first += n;
        }
        return TA_OK;
    }
    char* stage_k = static_cast<char*>(staging);
    char* stage_v = stage_k + half;
    const int64_t per_buffer = per_round / 2;
    std::unique_lock<std::mutex> hold(g_lane_mutex);
    SideLane* lane = (per_buffer >= kTwoRoundPages && n_pages > per_buffer) ? side_lane(stream) : nullptr;
    if (lane == nullptr) hold.unlock();
    const int64_t step = lane != nullptr ? per_buffer : per_round;
    hipStream_t kernel_stream = lane != nullptr ? lane->stream : stream;
    int64_t round = 0;
    for (int64_t first = 0; first < n_pages; first += step, ++round) {
        const int64_t end = (n_pages - first) < step ? n_pages : first + step;
        const size_t bytes = size_t(end - first) * page_bytes;
        const int buf = lane != nullptr ? int(round & 1) : 0;
        char* sk = stage_k + size_t(buf) * size_t(per_buffer) * page_bytes;
        char* sv = stage_v + size_t(buf) * size_t(per_buffer) * page_bytes;
        if (lane != nullptr && round >= 2) TA_HIP_TRY(hipStreamWaitEvent(stream, lane->moved[buf], 0));
        TA_HIP_TRY(hipMemcpyAsync(sk, hk + size_t(first) * page_bytes, bytes, hipMemcpyHostToDevice, stream));
        TA_HIP_TRY(hipMemcpyAsync(sv, hv + size_t(first) * page_bytes, bytes, hipMemcpyHostToDevice, stream));
        if (lane != nullptr) {      // (the first scatter thereby also comes after what the caller enqueued before the call)
            TA_HIP_TRY(hipEventRecord(lane->copied[buf], stream));
            TA_HIP_TRY(hipStreamWaitEvent(kernel_stream, lane->copied[buf], 0));
        }
        for (int64_t at = first; at < end;) {
            const int32_t n = fill_batch(batch, dst_slots, at, end);
            hipLaunchKernelGGL(move_pages_kernel<false>, dim3(move_grid(n, false, false)), dim3(kScatterThreads), 0,
                               kernel_stream, kp, vp, sk + size_t(at - first) * page_bytes,
                               sv + size_t(at - first) * page_bytes, batch, n, int64_t(page_bytes));
            TA_HIP_TRY(hipGetLastError());
            at += n;
        }
        if (lane != nullptr) TA_HIP_TRY(hipEventRecord(lane->moved[buf], kernel_stream));
    }
    if (lane != nullptr) {      // the call is over, on the caller's stream, when the last scatters are
        TA_HIP_TRY(hipStreamWaitEvent(stream, lane->moved[0], 0));
        if (round >= 2) TA_HIP_TRY(hipStreamWaitEvent(stream, lane->moved[1], 0));
    }
    return TA_OK;
}

}  // namespace ta
