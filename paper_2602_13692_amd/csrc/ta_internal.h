// Internal declarations shared by the HIP sources of the library (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ta.h"

namespace ta {

constexpr int kHeadDim = 128;
constexpr int kPageSize = 16;
constexpr int kWaveSize = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// Finite stand-in for "no key seen yet": keeps (m_old - m_new) free of inf - inf.
constexpr float kNegBig = -1.0e30f;
constexpr int kMinChunkPages = 8;    // the shortest split-K chunk (two 64-key tiles)
// which kernel streams the private chunks of a bf16 cache
constexpr int kRouteVector = 0, kRouteTiles = 1, kRouteOnDevice = 2;
constexpr int kMinAdaptedChunkPages = 32;   // the shortest chunk the library picks by itself

// Records a failed HIP call for ta_last_hip_error(); returns TA_ERR_HIP.
int note_hip_error(hipError_t e);

#define TA_HIP_TRY(expr)                                   \
    do {                                                   \
        hipError_t _e = (expr);                            \
        if (_e != hipSuccess) return ::ta::note_hip_error(_e); \
    } while (0)

// Benchmark instrumentation: events recorded around the dominant kernel (may be null).
struct ProfileEvents {
    hipEvent_t start;
    hipEvent_t stop;
};
ProfileEvents profile_events();

// Resolved geometry: strides in bytes, scale folded with log2(e).
struct Geometry {
    int32_t num_q_heads;
    int32_t num_kv_heads;
    int32_t group;            // Hq / Hkv
    int32_t pool_pages;       // pages per pool as stated by the caller (0 = not stated; debug checks only)
    int32_t decode_chunk_pages;  // the caller's split-K chunk length, 0 = chosen by the library
    int32_t prefill_key_chunks;  // the caller's number of key chunks per query tile of append-prefill, 0 = chosen by the library
    bool kv_fp8;              // pools hold E4M3 codes (one byte per element)
    float k_scale;            // fp8 only
    float v_scale;            // fp8 only
    float scale;              // multiplies q.k
    float scale_log2;         // scale * log2(e)
    int64_t stride_page_bytes;
    int64_t stride_head_bytes;
};

// Validates the descriptor; on TA_OK fills g.
int resolve_geometry(const ta_attn_desc* desc, Geometry* g);

// Layout of the caller's workspace for one call.  All offsets are multiples of 256 bytes.
//
// Decode cuts the pages of a program into bulk chunks of chunk_pages and cuts what is left
// (fewer than chunk_pages pages) into pieces of rem_pages; every chunk or piece has a slot for its
// partial result.  A program's slots are consecutive: bulk chunks first, then the pieces.
struct WorkspaceLayout {
    int32_t chunk_pages;        // pages per bulk chunk
    int32_t rem_pages;          // pages per piece of the remainder (divides chunk_pages)
    int32_t slots_per_program;  // upper bound on the slots of one program
    int32_t max_chunks;         // batch * slots_per_program: bound on slots and on vector-ALU items
    int32_t direct;             // 1: every context fits one item: no plan, no partials, no merge
    int32_t private_on_tiles;   // kRouteVector, kRouteTiles (every chunk runs on the matrix-core tile kernel, as groups
                                // of one program) or kRouteOnDevice (the plan kernel chooses between the two)
    int32_t max_tiles;          // upper bound on prefill query tiles (0 for decode)
    // append-prefill of few query tiles: every tile's keys are cut into prefill_split chunks of
    // prefill_chunk_tiles key tiles, one workgroup each, and their partials merged (1: no cutting)
    int32_t prefill_split;
    int32_t prefill_chunk_tiles;
    size_t off_chunk_start;     // int32 [batch + 1] first slot of each program
    size_t off_items;           // int4  [max_chunks] (program, first page, pages, slot)
    size_t off_part_ml;         // float [max_chunks][Hq][2]
    size_t off_part_o;          // float [max_chunks][Hq][128]
    int32_t max_shared_items;   // upper bound on the matrix-core kernel's items
    size_t off_counts;          // int32 [4]: vector-ALU items, matrix-core items, matrix-core work counter
    size_t off_lcp;             // int32 [batch] leading pages shared with the predecessor
    size_t off_pred;            // int32 [batch] predecessor: the nearest earlier program with the same first page
    size_t off_order;           // int32 [batch] programs listed group by group
    size_t off_shared_items;    // int4  [max_shared_items] (position in `order`, members, bulk chunk, first member)
    size_t off_tile_start;      // int32 [batch + 1]      (prefill)
    size_t off_tiles;           // int2  [max_tiles]      (prefill)
    // prefill over an FP8 cache: the batch's pages widened to bf16, program by program
    int32_t wide_width;         // pages per program in the widened pools (0: not used)
    size_t off_wide_table;      // int32 [batch][wide_width], entry (b, i) = b * wide_width + i
    size_t off_wide_k;          // bf16  [batch * wide_width][Hkv][16][128] code values of K
    size_t off_wide_v;          // the same for V
    size_t total_bytes;
};

WorkspaceLayout plan_workspace(const Geometry& g, int32_t batch, int32_t max_q_len,
                               int32_t max_context_len);

// ---- launchers (each validates nothing; callers have done that) ----

struct DecodeArgs {
    const uint16_t* q;
    const uint16_t* k_pool;
    const uint16_t* v_pool;
    const int32_t* block_table;
    const int32_t* context_lens;
    uint16_t* out;
    float* lse;
    int32_t block_table_stride;
    int32_t batch;
    int32_t max_context_len;
};

int launch_decode(const Geometry& g, const DecodeArgs& a, const WorkspaceLayout& w, char* workspace,
                  hipStream_t stream);

// Arguments of the kernels that work through the decode items (one workgroup per item and kv head).
struct ChunkParams {
    const uint16_t* q;
    const char* k_pool;
    const char* v_pool;
    const int32_t* block_table;
    const int32_t* context_lens;
    const int32_t* counts;       // counts[0] = number of items; shared form: counts[1] items, counts[3] chunk length in pages
    const int4* items;           // (program, first page, pages, slot)
    // shared form of the FP8 kernel only: chunks that a few programs share, as for the tile kernel
    const int4* shared_items;    // (position of the first member in `order`, members, bulk chunk, first member)
    const int32_t* order;        // programs listed group by group
    const int32_t* chunk_start;  // first partial slot of each program
    float* part_ml;
    float* part_o;
    uint16_t* out;               // direct mode only
    float* lse;                  // direct mode only, may be null
    int64_t stride_page_bytes;
    int64_t stride_head_bytes;
    int32_t block_table_stride;
    int32_t batch;
    int32_t num_q_heads;
    int32_t num_kv_heads;
    int32_t max_pages;           // direct mode only: pages the launch was sized for
    float scale_log2;            // fp8: the key scale is folded in
    float out_scale;             // fp8 direct mode: the value scale (1 otherwise)
};
constexpr int kMaxItemPages = 128;      // vector-ALU kernel: two page ids per lane
constexpr int kChunkGridCap = 16384;    // vector-ALU kernel: workgroups per launch at most (eight times what the chip holds at once)
constexpr int kMaxItemPagesFp8 = 512;   // FP8 kernel: the item's page ids sit in LDS

// The item kernel for pools of E4M3 codes (matrix cores, any group size up to 16).  Shared form:
// one workgroup per (shared chunk, kv head) computes the partials of up to 32 / group programs at
// once (their heads fill two sets of sixteen columns of the score tile).
int launch_fp8_items(const ChunkParams& p, int32_t group, bool direct, bool shared, unsigned blocks, hipStream_t stream);

// Widens the pages of a batch from E4M3 codes to bf16 code values (exact), program by program:
// logical page i of program b goes to slot b * width + i of the wide pools, and wide_table gets
// the identity map into them.  Pages beyond a program's context are left alone.
int launch_widen_pages(const Geometry& g, const void* k_codes, const void* v_codes, const int32_t* block_table,
                       int32_t block_table_stride, const int32_t* context_lens, int32_t batch, int32_t width,
                       void* wide_k, void* wide_v, int32_t* wide_table, hipStream_t stream);

struct PrefillArgs {
    const uint16_t* q;
    const int32_t* cu_q_lens;
    const uint16_t* k_pool;
    const uint16_t* v_pool;
    const int32_t* block_table;
    const int32_t* context_lens;
    uint16_t* out;
    float* lse;
    int32_t block_table_stride;
    int32_t batch;
    int32_t total_q;
    int32_t max_q_len;
    int32_t max_context_len;
};

int launch_prefill(const Geometry& g, const PrefillArgs& a, const WorkspaceLayout& w, char* workspace,
                   hipStream_t stream);

// Decode of the chunks that a group of programs shares (block tables with a common head):
// the matrix-core tile kernel computes the split-K partials of all members at once.
struct SharedPrefixArgs {
    const uint16_t* q;
    const uint16_t* k_pool;
    const uint16_t* v_pool;
    const int32_t* block_table;
    const int32_t* context_lens;
    const int32_t* shared_items;   // int4 per item: position of the first member in `order`, members, chunk, first member
    const int32_t* order;          // programs listed group by group
    int32_t* counts;               // counts[1] = number of items, counts[2] = work counter (starts at 0), counts[3] = chunk length in pages
    const int32_t* chunk_start;
    float* part_ml;
    float* part_o;
    int32_t block_table_stride;
    int32_t batch;
    int32_t max_items;
    int32_t private_on_tiles;      // 1: the batch's private chunks are in the list too
};

int launch_shared_prefix(const Geometry& g, const SharedPrefixArgs& a, hipStream_t stream);

int launch_restore(void* k_pool, void* v_pool, size_t page_bytes, const void* host_k,
                   const void* host_v, const int32_t* dst_slots, int32_t n_pages, void* staging,
                   size_t staging_bytes, hipStream_t stream);

int launch_evict(const void* k_pool, const void* v_pool, size_t page_bytes, void* host_k, void* host_v,
                 const int32_t* src_slots, int32_t n_pages, void* staging, size_t staging_bytes,
                 hipStream_t stream);

int launch_append(const Geometry& g, const void* new_k, const void* new_v, const int32_t* cu_new_lens,
                  void* k_pool, void* v_pool, const int32_t* block_table, int32_t block_table_stride,
                  const int32_t* context_lens, int32_t batch, int32_t total_new, hipStream_t stream);

}  // namespace ta
