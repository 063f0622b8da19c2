// Host side of the C ABI: argument validation, workspace layout, error reporting.
// Every exported function validates what the host can see, then enqueues kernels
// on the caller's stream and returns without synchronising.
#include <cmath>
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
    if (d->reserved != 0) return TA_ERR_INVALID_ARG;
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
    if (sh % 8 != 0 || sp % 8 != 0) return TA_ERR_UNSUPPORTED;
    if (sh < int64_t(kPageSize) * kHeadDim) return TA_ERR_INVALID_ARG;
    g->num_q_heads = d->num_q_heads;
    g->num_kv_heads = d->num_kv_heads;
    g->group = group;
    g->scale = d->scale > 0.0f ? d->scale : 1.0f / std::sqrt(static_cast<float>(kHeadDim));
    g->scale_log2 = g->scale * kLog2e;
    g->stride_page_bytes = sp * 2;
    g->stride_head_bytes = sh * 2;
    return TA_OK;
}

// Split-K chunk length.  Smaller chunks balance ragged batches better, larger
// ones write fewer partial results; 64 pages (1024 tokens) keeps the partials
// below one percent of the KV bytes, and batches too small to fill the chip
// with that get shorter chunks.
static int32_t choose_chunk_pages(const Geometry& g, int32_t batch, int32_t max_context_len) {
    const char* env = std::getenv("TA_DECODE_CHUNK_PAGES");
    if (env != nullptr) {
        const int v = std::atoi(env);
        if (v == 8 || v == 16 || v == 32 || v == 64) return v;
        if ((v == 128 || v == 256) && g.group == 8) return v;   // the tile kernel only
    }
    const int64_t pages = (int64_t(max_context_len) + kPageSize - 1) / kPageSize;
    if (g.group == 8) {
        // every chunk runs on the matrix-core tile kernel, whose per-item cost (filling the LDS
        // ring, writing 32 to 128 rows of partials) wants long items: up to 4096 tokens
        for (int32_t c : {256, 128}) {
            const int64_t items = int64_t(batch) * g.num_kv_heads * ((pages + c - 1) / c);
            if (items >= 2048) return c;
        }
    }
    for (int32_t c : {64, 32, 16}) {
        const int64_t items = int64_t(batch) * g.num_kv_heads * ((pages + c - 1) / c);
        if (items >= 4096) return c;
    }
    return 8;
}

constexpr int kPrefillRowsPerBlock = 256;  // score rows (tokens x heads of a group) per workgroup

WorkspaceLayout plan_workspace(const Geometry& g, int32_t batch, int32_t max_q_len,
                               int32_t max_context_len) {
    WorkspaceLayout w{};
    const int64_t pages = (int64_t(max_context_len) + kPageSize - 1) / kPageSize;
    size_t off = 0;
    if (max_q_len <= 1) {
        w.chunk_pages = choose_chunk_pages(g, batch, max_context_len);
        const int64_t per_prog = (pages + w.chunk_pages - 1) / w.chunk_pages;
        w.max_chunks = static_cast<int32_t>(int64_t(batch) * per_prog);
        w.max_tiles = 0;
        w.off_chunk_start = off; off = align256(off + sizeof(int32_t) * (size_t(batch) + 1));
        w.off_items = off;       off = align256(off + sizeof(int32_t) * 2 * size_t(w.max_chunks));
        w.off_part_ml = off;     off = align256(off + sizeof(float) * 2 * size_t(w.max_chunks) * g.num_q_heads);
        w.off_part_o = off;      off = align256(off + sizeof(float) * kHeadDim * size_t(w.max_chunks) * g.num_q_heads);
        // a shared chunk serves at least two programs; with eight heads per kv head every chunk
        // goes to the matrix-core kernel, one item each at most
        w.max_shared_items = g.group == 8 ? w.max_chunks
                                          : static_cast<int32_t>((int64_t(batch) / 2) * per_prog);
        w.off_counts = off;      off = align256(off + sizeof(int32_t) * 4);
        w.off_lcp = off;         off = align256(off + sizeof(int32_t) * size_t(batch));
        w.off_shared_items = off; off = align256(off + sizeof(int32_t) * 4 * size_t(w.max_shared_items));
        w.off_tile_start = w.off_tiles = off;
    } else {
        w.chunk_pages = 0;
        w.max_chunks = 0;
        const int64_t tile_tokens = kPrefillRowsPerBlock / g.group;
        const int64_t per_prog = (int64_t(max_q_len) + tile_tokens - 1) / tile_tokens;
        w.max_tiles = static_cast<int32_t>(int64_t(batch) * per_prog);
        w.off_chunk_start = w.off_items = w.off_part_ml = w.off_part_o = off;
        w.off_tile_start = off; off = align256(off + sizeof(int32_t) * (size_t(batch) + 1));
        w.off_tiles = off;      off = align256(off + sizeof(int32_t) * 2 * size_t(w.max_tiles));
    }
    w.total_bytes = off;
    return w;
}

}  // namespace ta

using namespace ta;

namespace ta {
namespace {

// Debug validation of the device-resident metadata (TA_DEBUG=1): what a wrong entry would turn
// into a wild address inside the attention kernels is caught here instead.  bit 0: a context
// length outside [0, max_context_len]; bit 1: a block-table entry below zero among the pages a
// program uses; bit 2: cu_q_lens not starting at zero, decreasing, or not ending at total_q;
// bit 3: more new tokens than max_q_len or than the program's context holds.
__global__ void clear_flag_kernel(int32_t* flag) { *flag = 0; }

__global__ __launch_bounds__(256) void check_metadata_kernel(const int32_t* __restrict__ block_table,
                                                             int32_t block_table_stride,
                                                             const int32_t* __restrict__ context_lens,
                                                             const int32_t* __restrict__ cu_q_lens, int32_t batch,
                                                             int32_t max_context_len, int32_t total_q,
                                                             int32_t max_q_len, int32_t* __restrict__ flag) {
    int bad = 0;
    for (int b = blockIdx.x * blockDim.x + threadIdx.x; b < batch; b += gridDim.x * blockDim.x) {
        const int L = context_lens[b];
        if (L < 0 || L > max_context_len) {
            bad |= 1;
            continue;
        }
        const int pages = (L + kPageSize - 1) / kPageSize;
        for (int i = 0; i < pages; ++i)
            if (block_table[int64_t(b) * block_table_stride + i] < 0) bad |= 2;
        if (cu_q_lens != nullptr) {
            const int n = cu_q_lens[b + 1] - cu_q_lens[b];
            if (n < 0 || (b == 0 && cu_q_lens[0] != 0) || (b == batch - 1 && cu_q_lens[batch] != total_q)) bad |= 4;
            if (n > max_q_len || n > L) bad |= 8;
        }
    }
    if (bad != 0) atomicOr(flag, bad);
}

bool debug_checks_enabled() {
    const char* env = std::getenv("TA_DEBUG");
    return env != nullptr && env[0] == '1';
}

// Synchronises the stream: debug mode only.  `flag` is the first word of the caller's workspace.
int check_metadata(const int32_t* block_table, int32_t block_table_stride, const int32_t* context_lens,
                   const int32_t* cu_q_lens, int32_t batch, int32_t max_context_len, int32_t total_q,
                   int32_t max_q_len, int32_t* flag, hipStream_t stream) {
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, stream, flag);
    TA_HIP_TRY(hipGetLastError());
    const unsigned blocks = static_cast<unsigned>((batch + 255) / 256);
    hipLaunchKernelGGL(check_metadata_kernel, dim3(blocks < 1024 ? blocks : 1024), dim3(256), 0, stream, block_table,
                       block_table_stride, context_lens, cu_q_lens, batch, max_context_len, total_q, max_q_len, flag);
    TA_HIP_TRY(hipGetLastError());
    int32_t host_flag = 0;
    TA_HIP_TRY(hipMemcpyAsync(&host_flag, flag, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
    TA_HIP_TRY(hipStreamSynchronize(stream));
    return host_flag == 0 ? TA_OK : TA_ERR_INVALID_ARG;
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
        default: return "unknown status";
    }
}

int ta_last_hip_error(void) { return g_last_hip_error; }

int ta_matrix_core_probe(const void* operands, int32_t iters, void* sink, void* hip_stream) {
    if (operands == nullptr || sink == nullptr || iters < 1) return TA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(operands) & 15) != 0 || (reinterpret_cast<uintptr_t>(sink) & 3) != 0)
        return TA_ERR_INVALID_ARG;
    return ta::launch_matrix_core_probe(operands, iters, sink, static_cast<hipStream_t>(hip_stream));
}

int ta_stream_read_probe(const void* src, size_t bytes, void* sink, void* hip_stream) {
    if (src == nullptr || sink == nullptr || bytes == 0 || (bytes & 15) != 0) return TA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) & 15) != 0 || (reinterpret_cast<uintptr_t>(sink) & 3) != 0)
        return TA_ERR_INVALID_ARG;
    return ta::launch_stream_read_probe(src, bytes, sink, static_cast<hipStream_t>(hip_stream));
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
    Geometry g;
    int rc = resolve_geometry(desc, &g);
    if (rc != TA_OK) return rc;
    if (batch < 0 || max_context_len < 0 || block_table_stride < 0) return TA_ERR_INVALID_ARG;
    if (batch == 0) return TA_OK;
    if (!q || !k_pool || !v_pool || !block_table || !context_lens || !out || !workspace)
        return TA_ERR_INVALID_ARG;
    if (int64_t(block_table_stride) * kPageSize < int64_t(max_context_len)) return TA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_pool) |
         reinterpret_cast<uintptr_t>(v_pool) | reinterpret_cast<uintptr_t>(out)) & 15)
        return TA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return TA_ERR_INVALID_ARG;
    const WorkspaceLayout w = plan_workspace(g, batch, 1, max_context_len);
    if (workspace_bytes < w.total_bytes) return TA_ERR_INVALID_ARG;
    if (ta::debug_checks_enabled()) {
        rc = ta::check_metadata(block_table, block_table_stride, context_lens, nullptr, batch, max_context_len, 0,
                                0, static_cast<int32_t*>(workspace), static_cast<hipStream_t>(hip_stream));
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
                                total_q, max_q_len, static_cast<int32_t*>(workspace),
                                static_cast<hipStream_t>(hip_stream));
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
    if (n_pages <= 0) return 0;
    return align256(sizeof(int32_t) * size_t(n_pages));
}

size_t ta_restore_staging_full_bytes(int32_t n_pages, size_t page_bytes) {
    if (n_pages <= 0) return 0;
    // slot list + room for at least one K page and one V page per round
    return ta_restore_staging_min_bytes(n_pages) + 2 * align256(page_bytes);
}

int ta_kv_page_restore(void* k_pool, void* v_pool, size_t page_bytes, const void* host_k,
                       const void* host_v, const int32_t* dst_slots, int32_t n_pages,
                       int32_t pool_pages, void* staging, size_t staging_bytes, void* hip_stream) {
    if (n_pages < 0 || pool_pages < 0) return TA_ERR_INVALID_ARG;
    if (n_pages == 0) return TA_OK;
    if (!k_pool || !v_pool || !host_k || !host_v || !dst_slots || !staging) return TA_ERR_INVALID_ARG;
    if (page_bytes == 0 || page_bytes % 16 != 0) return TA_ERR_INVALID_ARG;
    if (n_pages > pool_pages) return TA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(v_pool) |
         reinterpret_cast<uintptr_t>(host_k) | reinterpret_cast<uintptr_t>(host_v)) & 15)
        return TA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(staging) & 255) return TA_ERR_INVALID_ARG;
    if (staging_bytes < ta_restore_staging_min_bytes(n_pages)) return TA_ERR_INVALID_ARG;
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
    if (!k_pool || !v_pool || !host_k || !host_v || !src_slots || !staging) return TA_ERR_INVALID_ARG;
    if (page_bytes == 0 || page_bytes % 16 != 0) return TA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(v_pool) |
         reinterpret_cast<uintptr_t>(host_k) | reinterpret_cast<uintptr_t>(host_v)) & 15)
        return TA_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(staging) & 255) return TA_ERR_INVALID_ARG;
    if (staging_bytes < ta_restore_staging_min_bytes(n_pages)) return TA_ERR_INVALID_ARG;
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
    return launch_append(g, new_k, new_v, cu_new_lens, k_pool, v_pool, block_table, block_table_stride,
                         context_lens, batch, total_new, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
