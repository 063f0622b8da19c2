// Host side of the C ABI: argument validation, workspace layout, error reporting.
// Every exported function validates what the host can see, then enqueues kernels
// on the caller's stream and returns without synchronising.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ta_internal.h"

namespace ta {

static thread_local int g_last_hip_error = 0;

int note_hip_error(hipError_t e) {
    g_last_hip_error = static_cast<int>(e);
    return TA_ERR_HIP;
}

static thread_local ProfileEvents g_profile_events = {nullptr, nullptr};

ProfileEvents profile_events() { return g_profile_events; }

static size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

int resolve_geometry(const ta_attn_desc* d, Geometry* g) {
    if (d == nullptr) return TA_ERR_INVALID_ARG;
    if (d->num_q_heads <= 0 || d->num_kv_heads <= 0) return TA_ERR_INVALID_ARG;
    if (d->num_q_heads % d->num_kv_heads != 0) return TA_ERR_INVALID_ARG;
    if (d->pool_pages < 0) return TA_ERR_INVALID_ARG;
    if (d->kv_format != TA_KV_BF16 && d->kv_format != TA_KV_FP8_E4M3) return TA_ERR_INVALID_ARG;
    const bool fp8 = d->kv_format == TA_KV_FP8_E4M3;
    if (fp8 && (!(d->k_scale > 0.0f) || !(d->v_scale > 0.0f) || std::isinf(d->k_scale) || std::isinf(d->v_scale)))
        return TA_ERR_INVALID_ARG;
    if (!(d->scale >= 0.0f) || std::isinf(d->scale)) return TA_ERR_INVALID_ARG;  // also rejects NaN
    if (d->pool_stride_page < 0 || d->pool_stride_head < 0 || d->pool_stride_token < 0)
        return TA_ERR_INVALID_ARG;
    if (d->head_dim != kHeadDim || d->page_size != kPageSize) return TA_ERR_UNSUPPORTED;
    const int group = d->num_q_heads / d->num_kv_heads;
    if (group != 1 && group != 2 && group != 4 && group != 8) return TA_ERR_UNSUPPORTED;
    const int64_t st = d->pool_stride_token ? d->pool_stride_token : kHeadDim;
    if (st != kHeadDim) return TA_ERR_UNSUPPORTED;
    const int64_t sh = d->pool_stride_head ? d->pool_stride_head : int64_t(kPageSize) * kHeadDim;
    const int64_t sp = d->pool_stride_page ? d->pool_stride_page : sh * d->num_kv_heads;
    // a (page, head) tile is read with 16-byte accesses
    const int64_t elem_bytes = fp8 ? 1 : 2;
    if ((sh * elem_bytes) % 16 != 0 || (sp * elem_bytes) % 16 != 0) return TA_ERR_UNSUPPORTED;
    if (sh < int64_t(kPageSize) * kHeadDim) return TA_ERR_INVALID_ARG;
    const int32_t cp = d->decode_chunk_pages;
    // with a bf16 cache chunks of 256 and 512 pages exist on the matrix-core tile kernel only: asking
    // for one also asks for that kernel
    if (cp != 0 && cp != 8 && cp != 16 && cp != 32 && cp != 64 && cp != 128 && cp != 256 && cp != 512)
        return TA_ERR_INVALID_ARG;
    if (d->prefill_key_chunks < 0 || d->prefill_key_chunks > 1024) return TA_ERR_INVALID_ARG;
    g->num_q_heads = d->num_q_heads;
    g->num_kv_heads = d->num_kv_heads;
    g->group = group;
    g->pool_pages = d->pool_pages;
    g->decode_chunk_pages = cp;
    g->prefill_key_chunks = d->prefill_key_chunks;
    g->scale = d->scale > 0.0f ? d->scale : 1.0f / std::sqrt(static_cast<float>(kHeadDim));
    g->scale_log2 = g->scale * kLog2e;
    g->stride_page_bytes = sp * elem_bytes;
    g->stride_head_bytes = sh * elem_bytes;
    g->kv_fp8 = fp8;
    g->k_scale = fp8 ? d->k_scale : 1.0f;
    g->v_scale = fp8 ? d->v_scale : 1.0f;
    return TA_OK;
}

// Split-K chunk length (pages per bulk chunk).  Every item costs a few microseconds of its
// workgroup's time (metadata, first loads in flight, the merge of its waves), so long chunks are
// cheaper; short ones are only chosen when a batch is too small to fill the chip otherwise.  The
// leftover of a program (less than one chunk) is cut finer and listed last, so that the launch
// ends on short items.
// Which kernel streams the private chunks of a bf16 cache.  The matrix-core tile kernel brings
// K/V in through global-to-LDS loads with three tiles in flight per CU and spends no vector
// instruction on them: with enough work to keep one eight-wave workgroup per CU on long items it
// streams faster than the vector-ALU kernel (measured with four query heads per kv head on 4 to
// 128 programs of 1k to 64k tokens: from about 5,000 to 10,000 pages in the batch).
// Below that the vector-ALU kernel's finer items fill the chip better.  With eight query heads
// per kv head the vector-ALU kernel does not exist (its per-head state would fill the register
// file).  The host knows only the batch and the bound on the context length: it takes their
// product, the most the batch can hold.
// Returns kRouteVector, kRouteTiles or kRouteOnDevice.  The last: the host's product says tiles, but
// the plan kernel, which sees the real lengths, has the last word -- under a bound far above them (a
// serving loop sizes it once) many short programs are better off on the vector-ALU kernel (1024
// programs of 256 to 1024 tokens: 0.75 of the HBM peak there, 0.65 on tiles; of 64 to 512 tokens:
// 0.71 against 0.45), whose launch then finds the list that the tile kernel's launch finds empty.
static int decode_route(const Geometry& g, int32_t batch, int32_t max_context_len) {
    if (g.kv_fp8) return kRouteVector;
    if (g.group == 8 || g.decode_chunk_pages >= 256) return kRouteTiles;
    if (g.decode_chunk_pages != 0) return kRouteVector;
    const int64_t pages = (int64_t(max_context_len) + kPageSize - 1) / kPageSize;
    // no context above one item of the vector-ALU kernel: nothing for the tile kernel's long items
    if (pages <= kMaxItemPages) return kRouteVector;
    return int64_t(batch) * pages >= 16000 ? kRouteOnDevice : kRouteVector;
}
static bool decode_on_tiles(const Geometry& g, int32_t batch, int32_t max_context_len) {
    return decode_route(g, batch, max_context_len) != kRouteVector;
}

static int32_t choose_chunk_pages(const Geometry& g, int32_t batch, int32_t max_context_len) {
    if (g.decode_chunk_pages != 0) return g.decode_chunk_pages;   // the caller's choice, validated with the descriptor
    const int64_t pages = (int64_t(max_context_len) + kPageSize - 1) / kPageSize;
    const bool on_tiles = decode_on_tiles(g, batch, max_context_len);
    if (on_tiles || g.kv_fp8) {
        // the tile kernel's per-item cost (filling the LDS ring anew, writing 32 to 128 rows of
        // partials) wants long items: up to 8192 tokens.  (Longer still would stream a little
        // faster, but the chunk is also the unit in which a shared prefix is recognised.)  The
        // kernel for FP8 caches likes them as long: the start of an item is a microsecond in which
        // its workgroup streams nothing.
        for (int32_t c : {512, 256, 128}) {
            const int64_t items = int64_t(batch) * g.num_kv_heads * ((pages + c - 1) / c);
            if (items >= 2048) return c;
        }
    }
    // The vector-ALU kernel's longest item; the plan shortens the chunk on the device, from the real
    // lengths, when a batch is too small to fill the chip with such items.
    if (!on_tiles) return 128;
    // (the tile route with a bound this small: the device-side choice does the rest)
    return 128;
}

constexpr int kPrefillRowsPerBlock = 256;  // score rows (tokens x heads of a group) per workgroup

WorkspaceLayout plan_workspace(const Geometry& g, int32_t batch, int32_t max_q_len,
                               int32_t max_context_len) {
    WorkspaceLayout w{};
    const int64_t pages = (int64_t(max_context_len) + kPageSize - 1) / kPageSize;
    size_t off = 0;
    if (max_q_len <= 1) {
        w.chunk_pages = choose_chunk_pages(g, batch, max_context_len);
        // the tile kernel takes a program's leftover as one item; the vector-ALU kernel gets it in quarters
        const bool all_on_tiles = decode_on_tiles(g, batch, max_context_len);
        w.private_on_tiles = decode_route(g, batch, max_context_len);
        w.rem_pages = all_on_tiles ? w.chunk_pages : (w.chunk_pages >= 32 ? w.chunk_pages / 4 : 8);
        w.slots_per_program = static_cast<int32_t>(pages / w.chunk_pages + w.chunk_pages / w.rem_pages);
        // (a route settled on the device: many short programs go to the vector-ALU kernel, whose items
        // are shorter than the tile kernel's; two slots a program let it cut a short context once)
        if (w.private_on_tiles == kRouteOnDevice && w.slots_per_program < 2) w.slots_per_program = 2;
        // (a chunk shortened on the device needs more slots than the host's chunk would: it is only
        // shortened while the batch has fewer than about 1200 / Hkv chunks, plus four pieces each)
        const int64_t slack = g.decode_chunk_pages == 0 ? 1200 / g.num_kv_heads + 1 : 0;
        w.max_chunks = static_cast<int32_t>(int64_t(batch) * w.slots_per_program + slack);
        w.direct = (!all_on_tiles && pages <= w.chunk_pages) ? 1 : 0;
        w.max_tiles = 0;
        w.off_chunk_start = off; off = align256(off + sizeof(int32_t) * (size_t(batch) + 1));
        w.off_items = off;       off = align256(off + sizeof(int32_t) * 4 * size_t(w.max_chunks));
        w.off_part_ml = off;     off = align256(off + sizeof(float) * 2 * size_t(w.max_chunks) * g.num_q_heads);
        w.off_part_o = off;      off = align256(off + sizeof(float) * kHeadDim * size_t(w.max_chunks) * g.num_q_heads);
        // a shared chunk serves at least two programs; when every chunk goes to the matrix-core
        // kernel, one item each at most
        // (a chunk chosen on the device may be shorter than the host's: room for the shortest one then)
        const int64_t finest = g.decode_chunk_pages == 0 ? kMinChunkPages : w.chunk_pages;
        const int64_t shared_off_tiles = (int64_t(batch) / 2) * (pages / finest);
        w.max_shared_items = static_cast<int32_t>(!all_on_tiles ? shared_off_tiles
                                                  : w.private_on_tiles == kRouteOnDevice && shared_off_tiles > w.max_chunks
                                                      ? shared_off_tiles
                                                      : w.max_chunks);
        w.off_counts = off;      off = align256(off + sizeof(int32_t) * 4);
        w.off_lcp = off;         off = align256(off + sizeof(int32_t) * size_t(batch));
        w.off_pred = off;        off = align256(off + sizeof(int32_t) * size_t(batch));
        w.off_order = off;       off = align256(off + sizeof(int32_t) * size_t(batch));
        w.off_shared_items = off; off = align256(off + sizeof(int32_t) * 4 * size_t(w.max_shared_items));
        w.off_tile_start = w.off_tiles = off;
    } else {
        w.chunk_pages = w.rem_pages = 0;
        w.max_chunks = 0;
        const int64_t tile_tokens = kPrefillRowsPerBlock / g.group;
        const int64_t per_prog = (int64_t(max_q_len) + tile_tokens - 1) / tile_tokens;
        w.max_tiles = static_cast<int32_t>(int64_t(batch) * per_prog);
        w.off_chunk_start = w.off_items = w.off_part_ml = w.off_part_o = off;
        w.off_tile_start = off; off = align256(off + sizeof(int32_t) * (size_t(batch) + 1));
        w.off_tiles = off;      off = align256(off + sizeof(int32_t) * 2 * size_t(w.max_tiles));
        // A workgroup walks all the keys of its query tile, and a compute unit holds one workgroup:
        // with few tiles (a tool result coming back for one or a few programs) most of the 256
        // compute units would stand idle for the whole walk.  Then the keys are cut into chunks of
        // even length and the chunks' partials merged afterwards.  The number of chunks is the one
        // with the least estimated time, in key tiles: rounds of 256 workgroups, each as long as a
        // chunk plus twelve tiles' worth of start, finish and merge (fitted to measured sweeps: what
        // matters is that the last round is nearly full).  (chunk, kv head) streams are dealt to
        // the eight XCDs in turn, so their number is kept a multiple of eight; cutting must win a
        // tenth to be worth the partials.
        w.prefill_split = 1;
        w.prefill_chunk_tiles = 0;
        {
            const int64_t wgs = int64_t(w.max_tiles) * g.num_kv_heads;
            const int64_t key_tiles = (int64_t(max_context_len) + 63) / 64;
            if (g.prefill_key_chunks > 1) {                   // the caller's choice
                int64_t split = g.prefill_key_chunks;
                while (split > 1 && key_tiles / split < 4) --split;
                if (split > 1) {
                    w.prefill_split = static_cast<int32_t>(split);
                    w.prefill_chunk_tiles = static_cast<int32_t>((key_tiles + split - 1) / split);
                }
            } else if (g.prefill_key_chunks == 0 && wgs <= 512 && key_tiles >= 32) {
                int64_t unit = 8;                                                  // 8 / gcd(8, kv heads)
                for (int64_t h = g.num_kv_heads; unit > 1 && h % 2 == 0; h /= 2) unit /= 2;
                auto estimate = [&](int64_t split) {
                    return (wgs * split + 255) / 256 * ((key_tiles + split - 1) / split + 12);
                };
                const int64_t uncut = estimate(1);
                int64_t best = uncut, best_split = 1;
                for (int64_t split = unit == 1 ? 2 : unit; wgs * split <= 1024 && key_tiles / split >= 8; split += unit) {
                    const int64_t e = estimate(split);
                    if (e < best) { best = e; best_split = split; }
                }
                if (best_split > 1 && best * 10 <= uncut * 9) {
                    w.prefill_split = static_cast<int32_t>(best_split);
                    w.prefill_chunk_tiles = static_cast<int32_t>((key_tiles + best_split - 1) / best_split);
                }
            }
            if (w.prefill_split > 1) {
                const size_t rows = size_t(batch) * size_t(max_q_len) * size_t(g.num_q_heads);
                w.off_part_ml = off; off = align256(off + sizeof(float) * 2 * rows * size_t(w.prefill_split));
                w.off_part_o = off;  off = align256(off + sizeof(float) * kHeadDim * rows * size_t(w.prefill_split));
            }
        }
        if (g.kv_fp8) {
            // the tile kernel reads a bf16 copy of the batch's pages: room for every program's bound
            w.wide_width = static_cast<int32_t>(pages);
            const size_t slots = size_t(batch) * size_t(pages);
            const size_t pool_bytes = slots * size_t(g.num_kv_heads) * kPageSize * kHeadDim * 2;
            w.off_wide_table = off; off = align256(off + sizeof(int32_t) * slots);
            w.off_wide_k = off;     off = align256(off + pool_bytes);
            w.off_wide_v = off;     off = align256(off + pool_bytes);
        }
    }
    w.total_bytes = off;
    return w;
}

}  // namespace ta

using namespace ta;

namespace ta {
namespace {

// Debug validation of the device-resident metadata: what a wrong entry would turn into a wild
// address inside the other kernels is caught here instead.  bit 0: a context length outside
// [0, max_context_len]; bit 1: a block-table entry below zero, or not below pool_pages when the
// descriptor states it, among the pages a program uses; bit 2: prefix sums not starting at zero,
// decreasing, or not ending at the stated total; bit 3: more new tokens than max_q_len or than
// the program's context holds.
//
// The flag word is a device variable of the library (one copy per GPU, found once per device
// through its symbol), so that the check needs no caller memory.
__device__ int32_t g_debug_flag;

__global__ void clear_flag_kernel(int32_t* flag) { *flag = 0; }

__global__ __launch_bounds__(256) void check_metadata_kernel(const int32_t* __restrict__ block_table,
                                                             int32_t block_table_stride,
                                                             const int32_t* __restrict__ context_lens,
                                                             const int32_t* __restrict__ cu_q_lens, int32_t batch,
                                                             int32_t max_context_len, int32_t total_q,
                                                             int32_t max_q_len, int32_t pool_pages,
                                                             int32_t* __restrict__ flag) {
    int bad = 0;
    for (int b = blockIdx.x * blockDim.x + threadIdx.x; b < batch; b += gridDim.x * blockDim.x) {
        const int L = context_lens[b];
        if (L < 0 || L > max_context_len) {
            bad |= 1;
            continue;
        }
        const int pages = (L + kPageSize - 1) / kPageSize;
        for (int i = 0; i < pages; ++i) {
            const int32_t e = block_table[int64_t(b) * block_table_stride + i];
            if (e < 0 || (pool_pages > 0 && e >= pool_pages)) bad |= 2;
        }
        if (cu_q_lens != nullptr) {
            const int n = cu_q_lens[b + 1] - cu_q_lens[b];
            if (n < 0 || (b == 0 && cu_q_lens[0] != 0) || (b == batch - 1 && cu_q_lens[batch] != total_q)) bad |= 4;
            if (n > max_q_len || n > L) bad |= 8;
        }
    }
    if (bad != 0) atomicOr(flag, bad);
}

// -1: not decided yet (the environment is consulted once), 0 / 1: off / on
std::atomic<int> g_debug_mode{-1};

bool debug_checks_enabled() {
    int mode = g_debug_mode.load(std::memory_order_acquire);
    if (mode < 0) {
        const char* env = std::getenv("TA_DEBUG");
        int expected = -1;
        g_debug_mode.compare_exchange_strong(expected, (env != nullptr && env[0] == '1') ? 1 : 0);
        mode = g_debug_mode.load(std::memory_order_acquire);
    }
    return mode == 1;
}

// Address of this device's copy of the flag word (looked up once per device).
int debug_flag_address(int32_t** out) {
    constexpr int kMaxDevices = 64;
    static std::atomic<int32_t*> cached[kMaxDevices];
    int device = 0;
    TA_HIP_TRY(hipGetDevice(&device));
    if (device < 0 || device >= kMaxDevices) return TA_ERR_UNSUPPORTED;
    int32_t* p = cached[device].load(std::memory_order_acquire);
    if (p == nullptr) {
        TA_HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(g_debug_flag)));
        cached[device].store(p, std::memory_order_release);
    }
    *out = p;
    return TA_OK;
}

// Synchronises the stream: debug mode only.
int check_metadata(const int32_t* block_table, int32_t block_table_stride, const int32_t* context_lens,
                   const int32_t* cu_q_lens, int32_t batch, int32_t max_context_len, int32_t total_q,
                   int32_t max_q_len, int32_t pool_pages, hipStream_t stream) {
    // The verdict has to reach the host, which a stream under graph capture cannot give: a call
    // that is being captured goes unchecked (check it once eagerly, before the capture).
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capture) == hipSuccess && capture != hipStreamCaptureStatusNone) return TA_OK;
    int32_t* flag = nullptr;
    const int rc = debug_flag_address(&flag);
    if (rc != TA_OK) return rc;
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, stream, flag);
    TA_HIP_TRY(hipGetLastError());
    const unsigned blocks = static_cast<unsigned>((batch + 255) / 256);
    hipLaunchKernelGGL(check_metadata_kernel, dim3(blocks < 1024 ? blocks : 1024), dim3(256), 0, stream, block_table,
                       block_table_stride, context_lens, cu_q_lens, batch, max_context_len, total_q, max_q_len,
                       pool_pages, flag);
    TA_HIP_TRY(hipGetLastError());
    int32_t host_flag = 0;
    TA_HIP_TRY(hipMemcpyAsync(&host_flag, flag, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
    TA_HIP_TRY(hipStreamSynchronize(stream));
    return host_flag == 0 ? TA_OK : TA_ERR_INVALID_ARG;
}


// The library's own scratch for ta_paged_decode_static: one array per GPU, held until the process
// ends.  In host code the array's name is only a handle; its device address comes from
// hipGetSymbolAddress, once per device, and that pointer is what kernels and copies are given.
__device__ __align__(256) unsigned char scratch[TA_STATIC_SCRATCH_BYTES];

int static_scratch_address(char** out) {
    constexpr int kMaxDevices = 64;
    static std::atomic<char*> cached[kMaxDevices];
    int device = 0;
    TA_HIP_TRY(hipGetDevice(&device));
    if (device < 0 || device >= kMaxDevices) return TA_ERR_UNSUPPORTED;
    char* p = cached[device].load(std::memory_order_acquire);
    if (p == nullptr) {
        TA_HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)));
        if (p == nullptr) return TA_ERR_HIP;
        cached[device].store(p, std::memory_order_release);
    }
    *out = p;
    return TA_OK;
}

// ta_paged_decode and ta_paged_decode_static: the same validation and the same kernels; the
// split-K workspace is the caller's buffer or this device's copy of the library's own array.
int decode_with_scratch(const ta_attn_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                        const int32_t* block_table, int32_t block_table_stride, const int32_t* context_lens,
                        int32_t batch, int32_t max_context_len, void* out, float* lse, void* workspace,
                        size_t workspace_bytes, bool own_scratch, void* hip_stream) {
    Geometry g;
    int rc = resolve_geometry(desc, &g);
    if (rc != TA_OK) return rc;
    if (batch < 0 || max_context_len < 0 || block_table_stride < 0) return TA_ERR_INVALID_ARG;
    if (batch == 0) return TA_OK;
    if (!q || !k_pool || !v_pool || !block_table || !context_lens || !out) return TA_ERR_INVALID_ARG;
    if (int64_t(block_table_stride) * kPageSize < int64_t(max_context_len)) return TA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_pool) |
         reinterpret_cast<uintptr_t>(v_pool) | reinterpret_cast<uintptr_t>(out)) & 15)
        return TA_ERR_INVALID_ARG;
    const WorkspaceLayout w = plan_workspace(g, batch, 1, max_context_len);
    if (own_scratch) {
        if (w.total_bytes > size_t(TA_STATIC_SCRATCH_BYTES)) return TA_ERR_TOO_LARGE;
        char* p = nullptr;
        rc = static_scratch_address(&p);
        if (rc != TA_OK) return rc;
        workspace = p;
    } else {
        if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255)) return TA_ERR_INVALID_ARG;
        if (workspace_bytes < w.total_bytes) return TA_ERR_INVALID_ARG;
    }
    if (debug_checks_enabled()) {
        rc = check_metadata(block_table, block_table_stride, context_lens, nullptr, batch, max_context_len, 0, 0,
                            g.pool_pages, static_cast<hipStream_t>(hip_stream));
        if (rc != TA_OK) return rc;
    }
    DecodeArgs a{};
    a.q = static_cast<const uint16_t*>(q);
    a.k_pool = static_cast<const uint16_t*>(k_pool);
    a.v_pool = static_cast<const uint16_t*>(v_pool);
    a.block_table = block_table;
    a.context_lens = context_lens;
    a.out = static_cast<uint16_t*>(out);
    a.lse = lse;
    a.block_table_stride = block_table_stride;
    a.batch = batch;
    a.max_context_len = max_context_len;
    return launch_decode(g, a, w, static_cast<char*>(workspace), static_cast<hipStream_t>(hip_stream));
}

}  // namespace
}  // namespace ta

extern "C" {

int32_t ta_version(void) { return 100; }

const char* ta_strerror(int status) {
    switch (status) {
        case TA_OK: return "ok";
        case TA_ERR_INVALID_ARG: return "invalid argument";
        case TA_ERR_UNSUPPORTED: return "unsupported configuration";
        case TA_ERR_HIP: return "HIP runtime error";
        case TA_ERR_TOO_LARGE: return "the call needs more scratch than the library's own array holds";
        default: return "unknown status";
    }
}

int ta_last_hip_error(void) { return g_last_hip_error; }

int ta_set_debug_checks(int on) {
    const bool before = ta::debug_checks_enabled();   // settles the environment's say first
    ta::g_debug_mode.store(on != 0 ? 1 : 0, std::memory_order_release);
    return before ? 1 : 0;
}

void ta_profile_events(void* start_event, void* stop_event) {
    const bool on = start_event != nullptr && stop_event != nullptr;
    g_profile_events.start = on ? static_cast<hipEvent_t>(start_event) : nullptr;
    g_profile_events.stop = on ? static_cast<hipEvent_t>(stop_event) : nullptr;
}

size_t ta_workspace_bytes(const ta_attn_desc* desc, int32_t batch, int32_t max_q_len,
                          int32_t max_context_len) {
    Geometry g;
    if (resolve_geometry(desc, &g) != TA_OK) return 0;
    if (batch < 0 || max_q_len < 0 || max_context_len < 0) return 0;
    if (batch == 0) return 256;
    const WorkspaceLayout w = plan_workspace(g, batch, max_q_len, max_context_len);
    return w.total_bytes < 256 ? 256 : w.total_bytes;
}

int ta_paged_decode(const ta_attn_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                    const int32_t* block_table, int32_t block_table_stride,
                    const int32_t* context_lens, int32_t batch, int32_t max_context_len, void* out,
                    float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return ta::decode_with_scratch(desc, q, k_pool, v_pool, block_table, block_table_stride, context_lens, batch,
                                   max_context_len, out, lse, workspace, workspace_bytes, /*own_scratch=*/false,
                                   hip_stream);
}

int ta_paged_decode_static(const ta_attn_desc* desc, const void* q, const void* k_pool, const void* v_pool,
                           const int32_t* block_table, int32_t block_table_stride,
                           const int32_t* context_lens, int32_t batch, int32_t max_context_len, void* out,
                           float* lse, void* hip_stream) {
    return ta::decode_with_scratch(desc, q, k_pool, v_pool, block_table, block_table_stride, context_lens, batch,
                                   max_context_len, out, lse, nullptr, 0, /*own_scratch=*/true, hip_stream);
}

int ta_append_prefill(const ta_attn_desc* desc, const void* q, const int32_t* cu_q_lens,
                      const void* k_pool, const void* v_pool, const int32_t* block_table,
                      int32_t block_table_stride, const int32_t* context_lens, int32_t batch,
                      int32_t total_q, int32_t max_q_len, int32_t max_context_len, void* out,
                      float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
    Geometry g;
    int rc = resolve_geometry(desc, &g);
    if (rc != TA_OK) return rc;
    if (batch < 0 || total_q < 0 || max_q_len < 0 || max_context_len < 0 || block_table_stride < 0)
        return TA_ERR_INVALID_ARG;
    if (batch == 0 || total_q == 0) return TA_OK;
    if (g.kv_fp8 && batch > 65535) return TA_ERR_UNSUPPORTED;   // the widening pass has one grid row per program
    if (!q || !cu_q_lens || !k_pool || !v_pool || !block_table || !context_lens || !out || !workspace)
        return TA_ERR_INVALID_ARG;
    if (max_q_len == 0 || max_q_len > max_context_len) return TA_ERR_INVALID_ARG;
    if (int64_t(max_q_len) * batch < int64_t(total_q)) return TA_ERR_INVALID_ARG;
    if (int64_t(block_table_stride) * kPageSize < int64_t(max_context_len)) return TA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_pool) |
         reinterpret_cast<uintptr_t>(v_pool) | reinterpret_cast<uintptr_t>(out)) & 15)
        return TA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return TA_ERR_INVALID_ARG;
    // the tile plan always uses the prefill layout, also when max_q_len == 1
    const WorkspaceLayout w = plan_workspace(g, batch, max_q_len < 2 ? 2 : max_q_len, max_context_len);
    if (workspace_bytes < w.total_bytes) return TA_ERR_INVALID_ARG;
    if (ta::debug_checks_enabled()) {
        rc = ta::check_metadata(block_table, block_table_stride, context_lens, cu_q_lens, batch, max_context_len,
                                total_q, max_q_len, g.pool_pages, static_cast<hipStream_t>(hip_stream));
        if (rc != TA_OK) return rc;
    }
    PrefillArgs a{};
    a.q = static_cast<const uint16_t*>(q);
    a.cu_q_lens = cu_q_lens;
    a.k_pool = static_cast<const uint16_t*>(k_pool);
    a.v_pool = static_cast<const uint16_t*>(v_pool);
    a.block_table = block_table;
    a.context_lens = context_lens;
    a.out = static_cast<uint16_t*>(out);
    a.lse = lse;
    a.block_table_stride = block_table_stride;
    a.batch = batch;
    a.total_q = total_q;
    a.max_q_len = max_q_len;
    a.max_context_len = max_context_len;
    return launch_prefill(g, a, w, static_cast<char*>(workspace), static_cast<hipStream_t>(hip_stream));
}

size_t ta_restore_staging_min_bytes(int32_t n_pages) {
    (void)n_pages;   // the slot list travels in the kernel arguments: no staging is required
    return 0;
}

size_t ta_restore_staging_full_bytes(int32_t n_pages, size_t page_bytes) {
    if (n_pages <= 0) return 0;
    // room for at least one K page and one V page per round
    return 2 * align256(page_bytes);
}

int ta_kv_page_restore(void* k_pool, void* v_pool, size_t page_bytes, const void* host_k,
                       const void* host_v, const int32_t* dst_slots, int32_t n_pages,
                       int32_t pool_pages, void* staging, size_t staging_bytes, void* hip_stream) {
    if (n_pages < 0 || pool_pages < 0) return TA_ERR_INVALID_ARG;
    if (n_pages == 0) return TA_OK;
    if (!k_pool || !v_pool || !host_k || !host_v || !dst_slots) return TA_ERR_INVALID_ARG;
    if (staging == nullptr && staging_bytes != 0) return TA_ERR_INVALID_ARG;
    if (page_bytes == 0 || page_bytes % 16 != 0) return TA_ERR_INVALID_ARG;
    if (page_bytes >= (size_t(1) << 31)) return TA_ERR_UNSUPPORTED;      // a lane's offset inside a page has 32 bits
    if (n_pages > pool_pages) return TA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(v_pool) |
         reinterpret_cast<uintptr_t>(host_k) | reinterpret_cast<uintptr_t>(host_v)) & 15)
        return TA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(staging) & 255) return TA_ERR_INVALID_ARG;
    // slots: in range and distinct (the list is host memory, so this is checked here)
    std::vector<uint8_t> seen(static_cast<size_t>(pool_pages), 0);
    for (int32_t i = 0; i < n_pages; ++i) {
        const int32_t s = dst_slots[i];
        if (s < 0 || s >= pool_pages || seen[static_cast<size_t>(s)]) return TA_ERR_INVALID_ARG;
        seen[static_cast<size_t>(s)] = 1;
    }
    return launch_restore(k_pool, v_pool, page_bytes, host_k, host_v, dst_slots, n_pages, staging,
                          staging_bytes, static_cast<hipStream_t>(hip_stream));
}

int ta_kv_page_evict(const void* k_pool, const void* v_pool, size_t page_bytes, void* host_k,
                     void* host_v, const int32_t* src_slots, int32_t n_pages, int32_t pool_pages,
                     void* staging, size_t staging_bytes, void* hip_stream) {
    if (n_pages < 0 || pool_pages < 0) return TA_ERR_INVALID_ARG;
    if (n_pages == 0) return TA_OK;
    if (!k_pool || !v_pool || !host_k || !host_v || !src_slots) return TA_ERR_INVALID_ARG;
    if (staging == nullptr && staging_bytes != 0) return TA_ERR_INVALID_ARG;
    if (page_bytes == 0 || page_bytes % 16 != 0) return TA_ERR_INVALID_ARG;
    if (page_bytes >= (size_t(1) << 31)) return TA_ERR_UNSUPPORTED;      // a lane's offset inside a page has 32 bits
    if ((reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(v_pool) |
         reinterpret_cast<uintptr_t>(host_k) | reinterpret_cast<uintptr_t>(host_v)) & 15)
        return TA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(staging) & 255) return TA_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n_pages; ++i)
        if (src_slots[i] < 0 || src_slots[i] >= pool_pages) return TA_ERR_INVALID_ARG;
    return launch_evict(k_pool, v_pool, page_bytes, host_k, host_v, src_slots, n_pages, staging,
                        staging_bytes, static_cast<hipStream_t>(hip_stream));
}

int ta_kv_append(const ta_attn_desc* desc, const void* new_k, const void* new_v,
                 const int32_t* cu_new_lens, void* k_pool, void* v_pool, const int32_t* block_table,
                 int32_t block_table_stride, const int32_t* context_lens, int32_t batch,
                 int32_t total_new, void* hip_stream) {
    Geometry g{};
    const int rc = resolve_geometry(desc, &g);
    if (rc != TA_OK) return rc;
    if (batch < 0 || total_new < 0 || block_table_stride < 0) return TA_ERR_INVALID_ARG;
    if (batch == 0 || total_new == 0) return TA_OK;
    if (!new_k || !new_v || !cu_new_lens || !k_pool || !v_pool || !block_table || !context_lens)
        return TA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(new_k) | reinterpret_cast<uintptr_t>(new_v) |
         reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(v_pool)) & 15)
        return TA_ERR_INVALID_ARG;
    if (ta::debug_checks_enabled()) {
        // a stale table entry or more new tokens than the context holds would overwrite other pages
        const int drc = ta::check_metadata(block_table, block_table_stride, context_lens, cu_new_lens, batch,
                                           static_cast<int32_t>(std::min<int64_t>(
                                               int64_t(block_table_stride) * kPageSize, 0x7fffffff)),
                                           total_new, total_new, g.pool_pages, static_cast<hipStream_t>(hip_stream));
        if (drc != TA_OK) return drc;
    }
    return launch_append(g, new_k, new_v, cu_new_lens, k_pool, v_pool, block_table, block_table_stride,
                         context_lens, batch, total_new, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
