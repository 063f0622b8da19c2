// Paged decode attention for gfx950: one query token per program attends to the
// program's whole cached context (ThunderAgent Sec. 2.1; the decode term of the
// cost decomposition, Sec. 4.2, Eq. 3).
//
// Kernels per call:
//   prefix  finds, for every program, the nearest earlier program whose block table starts
//           alike, and the leading pages the two have in common;
//   plan    cuts every program's pages into chunks of the key axis (bulk chunks, and finer
//           pieces of the leftover) and lists them flat, long items first, so ragged batches
//           keep all CUs busy and the launch ends on short items; chunks that a group of
//           programs shares go to the matrix-core tile kernel instead (one pass over the
//           shared pages for all members);
//   chunk   one workgroup per (item, kv head): streams the item's K and V pages from HBM once,
//           serves all Hq/Hkv query heads of the group from the same registers, keeps an
//           online softmax per 16-lane row, writes one partial (max, sum, unnormalised output)
//           per query head;
//   merge   combines the partials of a (program, query head) and writes bf16.
// When every context fits a single item (short contexts) the chunk kernel alone runs: it
// normalises and writes the output itself.
//
// The work is HBM-bound (4 flop per KV byte at group size 4), so the chunk kernel here runs on the
// vector ALUs: packed bf16 dot products for q.k, fp32 FMAs for p.v.  It serves small batches with
// up to four query heads per kv head.  With eight, its per-head state would fill the register file
// (one wave per SIMD, compute-bound); and a batch large enough to keep one eight-wave workgroup
// per CU on long items streams faster through the matrix-core tile kernel, whose K/V arrive by
// global-to-LDS loads: in both cases every chunk goes there (the host decides, once per call).
#include "ta_internal.h"

namespace ta {
namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kChunkThreads = 256;  // 4 waves
constexpr int kChunkWaves = 4;

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b),
                                           acc, false);
}

// Sum over the 16 lanes of a DPP row; every lane of the row ends with the total.
__device__ __forceinline__ float row16_sum(float x) {
    // quad_perm [1,0,3,2]
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
    // quad_perm [2,3,0,1]
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));
    // row_half_mirror: lane i <-> 7 - i, crosses the two quads of a half row
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));
    // row_mirror: lane i <-> 15 - i, crosses the two half rows
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));
    return x;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

__device__ __forceinline__ uint16_t to_bf16_rne(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

// ---------------------------------------------------------------------------
// shared-prefix detection, step 1 (one workgroup per program): forked agent branches list the
// same prefix pages at the head of their block tables, wherever they sit in the batch.  The
// predecessor of program b is the nearest earlier program whose table starts with the same page
// (both long enough to hold the shortest chunk there is); lcp[b] counts the leading pages the two
// have in common, as far as both fill them completely.  (The plan kernel, which chooses the chunk
// length, decides what of that is worth sharing.)  Programs linked this way form a chain whose
// first member leads the group; what all members share is the minimum along the chain.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void predecessor_prefix_kernel(const int32_t* __restrict__ block_table,
                                                                 int32_t block_table_stride,
                                                                 const int32_t* __restrict__ context_lens,
                                                                 int32_t* __restrict__ pred,
                                                                 int32_t* __restrict__ lcp) {
    __shared__ int best, first_diff;
    const int b = blockIdx.x;
    const int min_tokens = kMinChunkPages * kPageSize;
    const int lb = context_lens[b];
    if (b == 0 || lb < min_tokens) {           // nothing before it, or too short to share a chunk
        if (threadIdx.x == 0) { pred[b] = -1; lcp[b] = 0; }
        return;
    }
    if (threadIdx.x == 0) best = -1;
    __syncthreads();
    const int32_t first = block_table[int64_t(b) * block_table_stride];
    int cand = -1;
    for (int o = threadIdx.x; o < b; o += blockDim.x)    // ascending: the last hit is this thread's nearest
        if (block_table[int64_t(o) * block_table_stride] == first && context_lens[o] >= min_tokens) cand = o;
    if (cand >= 0) atomicMax(&best, cand);
    __syncthreads();
    const int a = best;
    if (a < 0) {                                          // the common case: nothing shared
        if (threadIdx.x == 0) { pred[b] = -1; lcp[b] = 0; }
        return;
    }
    const int la = context_lens[a];
    const int n = (la < lb ? la : lb) / kPageSize;        // pages both programs fill completely
    const int32_t* ta = block_table + int64_t(a) * block_table_stride;
    const int32_t* tb = block_table + int64_t(b) * block_table_stride;
    if (threadIdx.x == 0) first_diff = n;
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        if (ta[i] != tb[i]) {
            atomicMin(&first_diff, i);
            break;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) { pred[b] = a; lcp[b] = first_diff; }
}

// ---------------------------------------------------------------------------
// plan (one workgroup).  The host sized the workspace for chunks of chunk_pages_max pages, from
// the bound on the context length it was given; the real lengths may be far below that bound (a
// serving loop sizes it once), and chunks that long would then leave most of the chip without an
// item.  So the kernel first adds up the pages that exist and halves the chunk until the batch
// gives about as many items as the host's rule asks for (never more slots than the workspace
// holds).  A chunk length that the caller gave is kept as it is.  The length the kernel settles on
// is left in counts[3] for the tile kernel.
// A program's pages are cut into bulk chunks of chunk_pages and its
// leftover into pieces of rem_pages; every chunk or piece gets a slot for its partial result
// (chunk_start[b] + index, bulk chunks first).  Step 2 of the shared-prefix detection forms the
// groups (chains of predecessors), lists their members side by side in `order`, and hands the
// bulk chunks all members of a group share to the matrix-core kernel, one item per (group, chunk)
// for all members at once.  Everything else is listed flat for the vector-ALU kernel, bulk
// chunks first and the short pieces last, so that the launch ends on short items:
//   shared_items  (position of the first member in `order`, members, bulk chunk, first member)
//   items         (program, first page, pages, slot)
// counts[0] = number of items, counts[1] = number of shared items, counts[2] = 0 (the tile
// kernel's work counter), counts[3] = the chunk length in pages.
// With private_on_tiles (eight query heads per kv head, or a large batch) every remaining chunk
// is listed as a group of one program in shared_items instead, and `items` stays empty;
// rem_pages equals chunk_pages then, so a leftover is one item, and the leftovers are listed in
// four classes of length, long first.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void plan_decode_kernel(const int32_t* __restrict__ context_lens,
                                                           const int32_t* __restrict__ pred,
                                                           const int32_t* __restrict__ lcp,
                                                           int32_t batch, int32_t max_pages, int32_t chunk_pages_max,
                                                           int32_t adapt_chunk, int32_t num_kv_heads, int32_t max_chunks,
                                                           int32_t max_members,
                                                           int32_t max_shared_items, int32_t route,
                                                           int32_t* __restrict__ chunk_start,
                                                           int4* __restrict__ items,
                                                           int4* __restrict__ shared_items,
                                                           int32_t* __restrict__ order,
                                                           int32_t* __restrict__ counts) {
    __shared__ int32_t s_key[1024];      // (leader << 10 | program), sorted: groups side by side
    __shared__ int32_t s_lead[1024];     // leader of each program
    __shared__ int32_t s_lcp[1024];      // pages shared with the predecessor
    __shared__ int32_t s_shared[1024];   // leading bulk chunks of program b computed by its group
    __shared__ int32_t s_pos[1024];      // position of program b in `order`
    __shared__ int32_t s_count[1024];    // members of the group that program b leads
    __shared__ int32_t s_common[1024];   // per position: a sub-group's common prefix in pages, later in bulk chunks
    __shared__ int32_t wave_total[16];
    __shared__ unsigned long long wave_total64[16];
    __shared__ int32_t carry, n_shared;
    const int tid = threadIdx.x;
    const int nt = blockDim.x;           // a power of two, 64 .. 1024, at least the batch when the batch is at most 1024

    auto pages_of = [&](int b) {
        const int L = context_lens[b];
        const int n = L > 0 ? (L + kPageSize - 1) / kPageSize : 0;
        return n > max_pages ? max_pages : n;               // lengths above the host bound are clipped
    };
    // which kernel gets the private chunks: the host's word, or (kRouteOnDevice) settled in step 0
    bool private_on_tiles = route == kRouteTiles;
    int chunk_longest = chunk_pages_max;                                // of the route taken
    int chunk_pages = chunk_pages_max, rem_pages = chunk_pages_max;     // settled below
    auto pieces_of = [&](int pages) { return (pages % chunk_pages + rem_pages - 1) / rem_pages; };
    bool whole_leftovers = false;        // the vector-ALU kernel too, when slots are short
    auto set_chunk = [&](int c) {
        chunk_pages = c;
        // the tile kernel takes a program's leftover as one item; the vector-ALU kernel gets it in quarters
        rem_pages = (private_on_tiles || whole_leftovers) ? c : (c >= 32 ? c / 4 : kMinChunkPages);
    };
    // exclusive scan of `value` over one pass of the workgroup's threads (wave-level shuffles, then
    // the sixteen wave totals); returns this thread's offset including earlier passes
    auto block_scan = [&](int value) {
        const int lane = tid & 63, wv = tid >> 6;
        int x = value;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int y = __shfl_up(x, off);
            if (lane >= off) x += y;
        }
        if (lane == 63) wave_total[wv] = x;
        __syncthreads();
        int before = carry;
        for (int w = 0; w < wv; ++w) before += wave_total[w];
        __syncthreads();
        if (tid == nt - 1) carry = before + x;
        __syncthreads();
        return before + x - value;
    };

    // 0. the chunk: the longest one that still gives the item count the host's rule aims at
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < batch; base += nt) block_scan(base + tid < batch ? pages_of(base + tid) : 0);
    {
        const int64_t total_pages = carry;
        if (route == kRouteOnDevice) {
            // The tile kernel (one eight-wave workgroup per compute unit, a few microseconds to start
            // an item) wants long items and enough of them; measured on 4 to 4096 programs of 64 to
            // 64k tokens under a bound of 128k it wins from about 8,000 pages in the batch and 800
            // tokens a program on (1024 programs of 256-1024 tokens: the same on both; of 64-512
            // tokens: 258 us here against 334 us on tiles; 512 programs of 512-2048: 496 against 448).
            private_on_tiles = total_pages >= 8000 && total_pages >= int64_t(48) * batch;
            if (!private_on_tiles && chunk_longest > kMaxItemPages) chunk_longest = kMaxItemPages;
        }
        // (item, kv head) pairs to aim for, and the shortest chunk worth having: measured on 4 to 128
        // programs of 1k to 64k tokens, the best chunk is the longest one that still gives about 500
        // pairs on the vector-ALU kernel (whose leftovers come in quarters) and about 150 on the tile
        // kernel (whose items cost more and whose leftovers are one item each); below 32 pages an
        // item's fixed cost outweighs the balance it buys on either
        const int64_t target = private_on_tiles ? 150 : 500;
        const int shortest = kMinAdaptedChunkPages;
        int c = chunk_longest;
        while (adapt_chunk && c > shortest && total_pages * num_kv_heads / c < target) c >>= 1;
        set_chunk(c);
    }
    __syncthreads();

    // 1. partial slots (with the route's longest chunk if the shorter one would need more slots than
    //    there are; the host sized them for the tile kernel's items, so a batch whose route is settled
    //    here and came out for the vector-ALU kernel may have to leave its leftovers whole, or go to
    //    the tile kernel after all)
    for (int attempt = 0; attempt < 4; ++attempt) {
        if (tid == 0) carry = 0;
        __syncthreads();
        for (int base = 0; base < batch; base += nt) {
            const int b = base + tid;
            const int pages = b < batch ? pages_of(b) : 0;
            const int first = block_scan(b < batch ? pages / chunk_pages + pieces_of(pages) : 0);
            if (b < batch) chunk_start[b] = first;
        }
        const int total_slots = carry;
        __syncthreads();
        if (total_slots <= max_chunks) break;
        if (chunk_pages != chunk_longest) {
            set_chunk(chunk_longest);
        } else if (route == kRouteOnDevice && !private_on_tiles && !whole_leftovers) {
            whole_leftovers = true;
            set_chunk(chunk_longest);
        } else if (route == kRouteOnDevice && !private_on_tiles) {
            private_on_tiles = true;
            whole_leftovers = false;
            chunk_longest = chunk_pages_max;
            set_chunk(chunk_longest);
        } else {
            break;
        }
    }
    if (tid == 0) chunk_start[batch] = carry;

    // 2. groups of programs with common leading bulk chunks (batches of up to 1024 programs)
    const bool grouping = lcp != nullptr && batch <= 1024 && batch >= 2;
    s_shared[tid] = 0;
    s_pos[tid] = tid;
    s_count[tid] = 0;
    if (tid == 0) n_shared = 0;
    __syncthreads();
    __shared__ int32_t any_joins;
    if (tid == 0) any_joins = 0;
    __syncthreads();
    const bool joins = grouping && tid < batch && pred[tid] >= 0 && lcp[tid] >= chunk_pages;
    if (joins) any_joins = 1;
    __syncthreads();
    if (grouping && any_joins != 0) {      // the common case (no program has a predecessor) skips all of this
        s_lcp[tid] = joins ? lcp[tid] : 0;
        s_lead[tid] = joins ? pred[tid] : tid;
        __syncthreads();
        int log_n = 1;
        while ((2 << (log_n - 1)) < batch) ++log_n;
        for (int round = 0; round < log_n; ++round) {       // predecessors have smaller indices: 2^k hops suffice
            const int l = s_lead[s_lead[tid]];
            if (__syncthreads_or(l != s_lead[tid]) == 0) break;     // every chain has reached its leader
            s_lead[tid] = l;
            __syncthreads();
        }
        // Bitonic sort of the nt keys (the entries from `batch` on hold the largest key and stay
        // at the end), ascending; the keys are distinct.  Partners less than a wave apart trade
        // through a lane exchange, the others through LDS.
        int key = tid < batch ? ((s_lead[tid] << 10) | tid) : 0x7fffffff;
        for (int k = 2; k <= nt; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                int other;
                if (j >= kWaveSize) {
                    s_key[tid] = key;
                    __syncthreads();
                    other = s_key[tid ^ j];
                    __syncthreads();
                } else {
                    other = __shfl_xor(key, j);
                }
                const bool keep_low = ((tid & j) == 0) == ((tid & k) == 0);
                key = keep_low ? (key < other ? key : other) : (key > other ? key : other);
            }
        }
        s_key[tid] = key;
        // where each program went; members of each leader's group; nothing shared yet
        const int prog = key & 1023, lead = (key >> 10) & 1023;     // meaningless from position `batch` on
        if (tid < batch) {
            order[tid] = prog;
            s_pos[prog] = tid;
            atomicAdd(&s_count[lead], 1);
        }
        s_common[tid] = 0x7fffffff;
        __syncthreads();
        // a group sits side by side from its leader's position on (the leader has the smallest
        // key of its group); it is cut into tiles of max_members rows, each a sub-group whose
        // common prefix is the shortest prefix its members other than the leader share with theirs
        int head = 0, end = 0, sub_head = 0;
        if (tid < batch) {
            head = s_pos[lead];
            end = head + s_count[lead];
            sub_head = head + (tid - head) / max_members * max_members;
            if (prog != lead) atomicMin(&s_common[sub_head], s_lcp[prog]);
        }
        __syncthreads();
        int sc = 0, n_in_sub = 0;
        if (tid < batch && tid == sub_head) {
            n_in_sub = end - tid < max_members ? end - tid : max_members;
            if (n_in_sub >= 2) sc = s_common[tid] / chunk_pages;
        }
        __syncthreads();
        if (tid == 0) carry = 0;
        s_common[tid] = sc;                 // from here on: shared bulk chunks of the sub-group that starts here
        __syncthreads();
        const int first_item = block_scan(sc);
        if (tid == 0) n_shared = carry <= max_shared_items ? carry : 0;
        __syncthreads();
        if (n_shared > 0) {
            if (tid < batch) s_shared[prog] = s_common[sub_head];
            for (int c = 0; c < sc; ++c) shared_items[first_item + c] = make_int4(tid, n_in_sub, c, prog);
        }
    } else {
        for (int b = tid; b < batch; b += nt) order[b] = b;     // s_pos is the identity already
    }
    __syncthreads();

    // 3. the remaining bulk chunks, then the pieces, one item each
    const int tile_base = n_shared;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < batch; base += nt) {
        const int b = base + tid;
        const int bulk = b < batch ? pages_of(b) / chunk_pages : 0;
        const int sc = (b < batch && batch <= 1024) ? s_shared[b] : 0;
        const int first = block_scan(bulk - sc);
        if (b < batch) {
            const int slot0 = chunk_start[b];
            const int pos = batch <= 1024 ? s_pos[b] : b;
            for (int c = sc; c < bulk; ++c) {
                if (private_on_tiles) shared_items[tile_base + first + c - sc] = make_int4(pos, 1, c, b);
                else items[first + c - sc] = make_int4(b, c * chunk_pages, chunk_pages, slot0 + c);
            }
        }
    }
    __syncthreads();
    const int n_bulk = carry;
    __syncthreads();
    if (tid == 0) carry = 0;
    __syncthreads();
    // On the tile kernel a program's leftover is one item of up to chunk_pages pages, taken from a
    // work counter: listing the long leftovers first (four classes of length) lets the launch end
    // on short items.  The vector-ALU kernel's pieces are all short already: one pass.
    int n_rest = 0;
    if (private_on_tiles && batch <= nt) {
        // one pass: the four classes are counted side by side, 16 bits each (at most 1024 programs)
        const int b = tid;
        const int pages = b < batch ? pages_of(b) : 0;
        const int bulk = pages / chunk_pages;
        const int n = pieces_of(pages);                       // 0 or 1: a leftover is one item here
        const int cls = n > 0 ? 3 - ((pages - bulk * chunk_pages - 1) * 4) / chunk_pages : 0;   // 0 = the longest quarter
        const unsigned long long mine = n > 0 ? 1ull << (16 * cls) : 0ull;
        // exclusive scan of the packed counts (wave-level shuffles, then the wave totals)
        const int lane = tid & 63, wv = tid >> 6;
        unsigned long long x = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const unsigned long long y = __shfl_up(x, off);
            if (lane >= off) x += y;
        }
        if (lane == 63) wave_total64[wv] = x;
        __syncthreads();
        unsigned long long before = 0, total = 0;
        for (int w = 0; w < (nt >> 6); ++w) {
            if (w < wv) before += wave_total64[w];
            total += wave_total64[w];
        }
        const unsigned long long prefix = before + x - mine;
        int first = int((prefix >> (16 * cls)) & 0xffff);
        for (int k = 0; k < cls; ++k) first += int((total >> (16 * k)) & 0xffff);
        if (n > 0) shared_items[tile_base + n_bulk + first] = make_int4(s_pos[b], 1, bulk, b);
        n_rest = int(total & 0xffff) + int((total >> 16) & 0xffff) + int((total >> 32) & 0xffff) + int(total >> 48);
    } else {
    const int n_pass = private_on_tiles ? 4 : 1;
    for (int pass = 0; pass < n_pass; ++pass)
    for (int base = 0; base < batch; base += nt) {
        const int b = base + tid;
        const int pages = b < batch ? pages_of(b) : 0;
        const int bulk = pages / chunk_pages;
        int n = pieces_of(pages);
        if (n_pass > 1 && n > 0) {
            const int cls = 3 - ((pages - bulk * chunk_pages - 1) * 4) / chunk_pages;   // 0 = the longest quarter
            if (cls != pass) n = 0;
        }
        const int first = block_scan(n);
        if (b < batch) {
            const int slot0 = chunk_start[b];
            const int pos = batch <= 1024 ? s_pos[b] : b;
            for (int k = 0; k < n; ++k) {
                const int page0 = bulk * chunk_pages + k * rem_pages;
                const int left = pages - page0;
                if (private_on_tiles) shared_items[tile_base + n_bulk + first + k] = make_int4(pos, 1, bulk + k, b);
                else items[n_bulk + first + k] = make_int4(b, page0, left < rem_pages ? left : rem_pages, slot0 + bulk + k);
            }
        }
    }
    __syncthreads();
    n_rest = carry;
    }
    if (tid == 0) {
        counts[0] = private_on_tiles ? 0 : n_bulk + n_rest;
        counts[1] = private_on_tiles ? tile_base + n_bulk + n_rest : tile_base;
        counts[2] = 0;   // work counter of the tile kernel
        counts[3] = chunk_pages;
    }
}

// ---------------------------------------------------------------------------
// chunk kernel
// ---------------------------------------------------------------------------
struct PageRegs {
    u32x4 k[4];  // k[i]: token 4*i + (lane / 16), dims 8 * (lane % 16) .. + 7
    u32x4 v[4];
};

// The K/V stream is software-pipelined in source: the loads of the next page are
// written before the arithmetic on the current one, and a scheduling barrier
// right after them keeps the compiler from moving them back down next to their
// first use.  The waits themselves (s_waitcnt vmcnt) are the compiler's, so every
// register is known to have landed before it is read.
__device__ __forceinline__ void load_page(PageRegs& r, const char* k_tile, const char* v_tile, int lane) {
    const u32x4* kp = reinterpret_cast<const u32x4*>(k_tile) + lane;
    const u32x4* vp = reinterpret_cast<const u32x4*>(v_tile) + lane;
#pragma unroll
    for (int i = 0; i < 4; ++i) r.k[i] = __builtin_nontemporal_load(kp + i * 64);
#pragma unroll
    for (int i = 0; i < 4; ++i) r.v[i] = __builtin_nontemporal_load(vp + i * 64);
}

// One 16-token page against the G query heads of the group.
//   qreg[h][0..3]  this lane's 8 dims of query head h, packed bf16
//   m, l, o        online-softmax state of this lane's 16-lane row (raw-score max,
//                  sum of weights, unnormalised output for this lane's 8 dims)
//   valid          tokens of this page that exist (16 unless MASKED)
template <int G, bool MASKED>
__device__ __forceinline__ void process_page(const PageRegs& pg, const uint32_t (&qreg)[G][4],
                                             float (&m)[G], float (&l)[G], float (&o)[G][8],
                                             float scale_log2, int row, int valid) {
    float s[4][G];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t kw[4] = {pg.k[i].x, pg.k[i].y, pg.k[i].z, pg.k[i].w};
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float acc = 0.0f;
#pragma unroll
            for (int w = 0; w < 4; ++w) acc = dot2_bf16(kw[w], qreg[h][w], acc);
            s[i][h] = acc;
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int h = 0; h < G; ++h) s[i][h] = row16_sum(s[i][h]);

    if (MASKED) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool ok = (4 * i + row) < valid;
#pragma unroll
            for (int h = 0; h < G; ++h) s[i][h] = ok ? s[i][h] : -INFINITY;
        }
    }

    float p[4][G];
    float alpha[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float mx = fmaxf(fmaxf(s[0][h], s[1][h]), fmaxf(s[2][h], s[3][h]));
        const float m_new = fmaxf(m[h], mx);
        alpha[h] = fast_exp2((m[h] - m_new) * scale_log2);
        const float bias = -m_new * scale_log2;
        float psum = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p[i][h] = fast_exp2(fmaf(s[i][h], scale_log2, bias));
            psum += p[i][h];
        }
        m[h] = m_new;
        l[h] = fmaf(l[h], alpha[h], psum);
    }

    uint32_t vw[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        vw[i][0] = pg.v[i].x; vw[i][1] = pg.v[i].y; vw[i][2] = pg.v[i].z; vw[i][3] = pg.v[i].w;
    }
    if (MASKED) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool ok = (4 * i + row) < valid;
#pragma unroll
            for (int w = 0; w < 4; ++w) vw[i][w] = ok ? vw[i][w] : 0u;
        }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
#pragma unroll
        for (int c = 0; c < 8; ++c) o[h][c] *= alpha[h];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                o[h][2 * w] = fmaf(p[i][h], bf16_lo(vw[i][w]), o[h][2 * w]);
                o[h][2 * w + 1] = fmaf(p[i][h], bf16_hi(vw[i][w]), o[h][2 * w + 1]);
            }
        }
    }
}

// DIRECT: every program is one item (its whole context, at most kMaxItemPages pages); the
// workgroup normalises and writes the bf16 output itself: no plan, no partials, no merge.
// BEYOND_CAP: the host sizes the launch from the bound on the context length, which may be far above
// the real lengths, and half a million workgroups that find nothing to do cost 150 us.  So a launch
// has at most kChunkGridCap workgroups, one per (item, kv head) pair; pairs beyond that number (very
// large batches) belong to a second launch of as many workgroups, in this form, where a workgroup
// goes on to the pair one grid further until the list ends.  (Written as one loop for both forms;
// with the loop taken for real the compiler keeps more values in registers and the kernel loses a
// wave per SIMD, which is why the usual form is not the looping one.)
template <int G, bool DIRECT, bool BEYOND_CAP>
__device__ __forceinline__ void decode_chunk_body(const ChunkParams& p) {
    for (int pair = BEYOND_CAP ? kChunkGridCap + int(blockIdx.x) : int(blockIdx.x);; pair += gridDim.x) {
    const int item = pair / p.num_kv_heads;
    const int g = pair - item * p.num_kv_heads;
    int b, page0, n_here, slot = 0;
    if (DIRECT) {
        b = item;
        page0 = 0;
    } else {
        if (item >= p.counts[0]) return;
        const int4 it = p.items[item];
        b = it.x; page0 = it.y; n_here = it.z; slot = it.w;
    }
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row = lane >> 4;
    const int col = lane & 15;

    const int L = p.context_lens[b];
    int n_pages_b = L > 0 ? (L + kPageSize - 1) / kPageSize : 0;
    if (DIRECT) {
        n_pages_b = n_pages_b > p.max_pages ? p.max_pages : n_pages_b;
        n_here = n_pages_b;
    }
    const int tail_valid = L - (n_pages_b - 1) * kPageSize;           // 1..16 where the program's last page is reached
    const bool has_tail = n_here > 0 && (page0 + n_here == n_pages_b) && tail_valid < kPageSize;
    const int n_full = has_tail ? n_here - 1 : n_here;                // pages processed unmasked

    // page ids of this item, two per lane
    int my_id0 = 0, my_id1 = 0;
    {
        const int32_t* table = p.block_table + int64_t(b) * p.block_table_stride + page0;
        if (lane < n_here) my_id0 = table[lane];
        if (lane + 64 < n_here) my_id1 = table[lane + 64];
    }
    auto page_id = [&](int idx) -> int {                              // idx is wave-uniform
        const int lo = __builtin_amdgcn_readlane(my_id0, idx & 63);
        const int hi = __builtin_amdgcn_readlane(my_id1, idx & 63);
        return idx < 64 ? lo : hi;
    };

    // queries of the group: 8 dims per lane, the same in all four rows
    uint32_t qreg[G][4];
    {
        const uint16_t* qb = p.q + (int64_t(b) * p.num_q_heads + g * G) * kHeadDim + col * 8;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const uint4 t = *reinterpret_cast<const uint4*>(qb + h * kHeadDim);
            qreg[h][0] = t.x; qreg[h][1] = t.y; qreg[h][2] = t.z; qreg[h][3] = t.w;
        }
    }

    float m[G], l[G], o[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = kNegBig;
        l[h] = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) o[h][c] = 0.0f;
    }

    const char* k_head = p.k_pool + int64_t(g) * p.stride_head_bytes;
    const char* v_head = p.v_pool + int64_t(g) * p.stride_head_bytes;

    // this wave's full pages: chunk pages wave, wave + 4, ...
    const int n_mine = n_full > wave ? (n_full - wave + kChunkWaves - 1) / kChunkWaves : 0;
    if (n_mine > 0) {
        auto tile_of = [&](int j) -> int64_t { return int64_t(page_id(wave + kChunkWaves * j)) * p.stride_page_bytes; };
        PageRegs bufA, bufB;
        int64_t off = tile_of(0);
        load_page(bufA, k_head + off, v_head + off, lane);
        int j = 0;
        // two pages per trip, one basic block: each buffer is refilled right after its
        // page has been consumed and is consumed one page later.  The loop runs while a
        // third page exists, so no load is ever issued for a page that is not used.
        for (; j + 2 < n_mine; j += 2) {
            off = tile_of(j + 1);
            load_page(bufB, k_head + off, v_head + off, lane);
            __builtin_amdgcn_sched_barrier(0);
            process_page<G, false>(bufA, qreg, m, l, o, p.scale_log2, row, kPageSize);
            off = tile_of(j + 2);
            load_page(bufA, k_head + off, v_head + off, lane);
            __builtin_amdgcn_sched_barrier(0);
            process_page<G, false>(bufB, qreg, m, l, o, p.scale_log2, row, kPageSize);
        }
        // one or two pages are left; bufA holds page j
        if (j + 1 < n_mine) {
            off = tile_of(j + 1);
            load_page(bufB, k_head + off, v_head + off, lane);
            __builtin_amdgcn_sched_barrier(0);
            process_page<G, false>(bufA, qreg, m, l, o, p.scale_log2, row, kPageSize);
            process_page<G, false>(bufB, qreg, m, l, o, p.scale_log2, row, kPageSize);
        } else {
            process_page<G, false>(bufA, qreg, m, l, o, p.scale_log2, row, kPageSize);
        }
    }
    if (has_tail && ((n_here - 1) & (kChunkWaves - 1)) == wave) {
        PageRegs t;
        const int64_t off = int64_t(page_id(n_here - 1)) * p.stride_page_bytes;
        load_page(t, k_head + off, v_head + off, lane);
        process_page<G, true>(t, qreg, m, l, o, p.scale_log2, row, tail_valid);
    }

    // merge the four rows of the wave
    __shared__ float sm_o[kChunkWaves][G][kHeadDim];
    __shared__ float sm_m[kChunkWaves][G];
    __shared__ float sm_l[kChunkWaves][G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        float mt = fmaxf(m[h], __shfl_xor(m[h], 16));
        mt = fmaxf(mt, __shfl_xor(mt, 32));
        const float w = fast_exp2((m[h] - mt) * p.scale_log2);
        float lt = l[h] * w;
        lt += __shfl_xor(lt, 16);
        lt += __shfl_xor(lt, 32);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float x = o[h][c] * w;
            x += __shfl_xor(x, 16);
            x += __shfl_xor(x, 32);
            o[h][c] = x;
        }
        if (lane < 16) {
            float4* dst = reinterpret_cast<float4*>(&sm_o[wave][h][col * 8]);
            dst[0] = make_float4(o[h][0], o[h][1], o[h][2], o[h][3]);
            dst[1] = make_float4(o[h][4], o[h][5], o[h][6], o[h][7]);
        }
        if (lane == 0) {
            sm_m[wave][h] = mt;
            sm_l[wave][h] = lt;
        }
    }
    __syncthreads();

    // merge the four waves
    if (DIRECT) {
        // thread t owns two neighbouring dims of one head and writes them as bf16
        for (int idx = tid; idx < G * (kHeadDim / 2); idx += kChunkThreads) {
            const int h = idx / (kHeadDim / 2);
            const int c = 2 * (idx % (kHeadDim / 2));
            float mt = sm_m[0][h];
#pragma unroll
            for (int w = 1; w < kChunkWaves; ++w) mt = fmaxf(mt, sm_m[w][h]);
            float lt = 0.0f, a0 = 0.0f, a1 = 0.0f;
#pragma unroll
            for (int w = 0; w < kChunkWaves; ++w) {
                const float wt = fast_exp2((sm_m[w][h] - mt) * p.scale_log2);
                lt = fmaf(sm_l[w][h], wt, lt);
                a0 = fmaf(sm_o[w][h][c], wt, a0);
                a1 = fmaf(sm_o[w][h][c + 1], wt, a1);
            }
            const float inv = lt > 0.0f ? 1.0f / lt : 0.0f;
            const int64_t rid = int64_t(b) * p.num_q_heads + g * G + h;
            *reinterpret_cast<uint32_t*>(p.out + rid * kHeadDim + c) =
                uint32_t(to_bf16_rne(a0 * inv)) | (uint32_t(to_bf16_rne(a1 * inv)) << 16);
            if (p.lse != nullptr && c == 0)
                p.lse[rid] = lt > 0.0f ? (mt * p.scale_log2 + __builtin_amdgcn_logf(lt)) * kLn2 : -INFINITY;
        }
        return;
    }
    // thread t owns outputs t, t + 256, ...
    for (int idx = tid; idx < G * kHeadDim; idx += kChunkThreads) {
        const int h = idx / kHeadDim;
        const int c = idx % kHeadDim;
        float mt = sm_m[0][h];
#pragma unroll
        for (int w = 1; w < kChunkWaves; ++w) mt = fmaxf(mt, sm_m[w][h]);
        float lt = 0.0f, acc = 0.0f;
#pragma unroll
        for (int w = 0; w < kChunkWaves; ++w) {
            const float wt = fast_exp2((sm_m[w][h] - mt) * p.scale_log2);
            lt = fmaf(sm_l[w][h], wt, lt);
            acc = fmaf(sm_o[w][h][c], wt, acc);
        }
        const int64_t rowid = int64_t(slot) * p.num_q_heads + g * G + h;
        p.part_o[rowid * kHeadDim + c] = acc;
        if (c == 0) {
            p.part_ml[rowid * 2 + 0] = mt * p.scale_log2;  // max in the log2 domain
            p.part_ml[rowid * 2 + 1] = lt;
        }
    }
    if (!BEYOND_CAP) return;
    __syncthreads();      // the next pair reuses the merge buffers
    }
}

template <int G, bool DIRECT>
__global__ __launch_bounds__(kChunkThreads) void decode_chunk_kernel(ChunkParams p) {
    decode_chunk_body<G, DIRECT, false>(p);
}

template <int G>
__global__ __launch_bounds__(kChunkThreads) void decode_chunk_beyond_cap_kernel(ChunkParams p) {
    decode_chunk_body<G, false, true>(p);
}

// ---------------------------------------------------------------------------
// merge kernel: one wave per (program, query head)
// ---------------------------------------------------------------------------
struct MergeParams {
    const int32_t* chunk_start;
    const float* part_ml;
    const float* part_o;
    uint16_t* out;
    float* lse;
    int32_t batch;
    int32_t num_q_heads;
    float out_scale;     // 1, or the value scale of an fp8 cache
};

__global__ __launch_bounds__(256) void decode_merge_kernel(MergeParams p) {
    const int lane = threadIdx.x & 63;
    const int64_t rid = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (rid >= int64_t(p.batch) * p.num_q_heads) return;
    const int b = static_cast<int>(rid / p.num_q_heads);
    const int h = static_cast<int>(rid % p.num_q_heads);
    const int c0 = p.chunk_start[b];
    const int c1 = p.chunk_start[b + 1];

    float mt = kNegBig;
    for (int c = c0 + lane; c < c1; c += 64)
        mt = fmaxf(mt, p.part_ml[(int64_t(c) * p.num_q_heads + h) * 2]);
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) mt = fmaxf(mt, __shfl_xor(mt, s));

    float lt = 0.0f, o0 = 0.0f, o1 = 0.0f;
#pragma unroll 8
    for (int c = c0; c < c1; ++c) {
        const int64_t r = int64_t(c) * p.num_q_heads + h;
        const float wt = fast_exp2(p.part_ml[r * 2] - mt);
        lt = fmaf(p.part_ml[r * 2 + 1], wt, lt);
        const float2 v = *reinterpret_cast<const float2*>(p.part_o + r * kHeadDim + 2 * lane);
        o0 = fmaf(v.x, wt, o0);
        o1 = fmaf(v.y, wt, o1);
    }
    const float inv = lt > 0.0f ? p.out_scale / lt : 0.0f;
    const uint32_t packed = uint32_t(to_bf16_rne(o0 * inv)) | (uint32_t(to_bf16_rne(o1 * inv)) << 16);
    reinterpret_cast<uint32_t*>(p.out + rid * kHeadDim)[lane] = packed;
    if (p.lse != nullptr && lane == 0)
        p.lse[rid] = lt > 0.0f ? (mt + __builtin_amdgcn_logf(lt)) * kLn2 : -INFINITY;
}

}  // namespace

int launch_decode(const Geometry& g, const DecodeArgs& a, const WorkspaceLayout& w, char* workspace,
                  hipStream_t stream) {
    const ProfileEvents ev = profile_events();
    ChunkParams cp{};
    cp.q = a.q;
    cp.k_pool = reinterpret_cast<const char*>(a.k_pool);
    cp.v_pool = reinterpret_cast<const char*>(a.v_pool);
    cp.block_table = a.block_table;
    cp.context_lens = a.context_lens;
    cp.out = a.out;
    cp.lse = a.lse;
    cp.stride_page_bytes = g.stride_page_bytes;
    cp.stride_head_bytes = g.stride_head_bytes;
    cp.block_table_stride = a.block_table_stride;
    cp.batch = a.batch;
    cp.num_q_heads = g.num_q_heads;
    cp.num_kv_heads = g.num_kv_heads;
    cp.max_pages = (a.max_context_len + kPageSize - 1) / kPageSize;
    cp.scale_log2 = g.kv_fp8 ? g.scale_log2 * g.k_scale : g.scale_log2;
    cp.out_scale = g.kv_fp8 ? g.v_scale : 1.0f;

    if (w.direct) {
        // short contexts: one launch, one workgroup per (program, kv head), output written directly
        const int64_t blocks = int64_t(a.batch) * g.num_kv_heads;
        if (blocks > 0x7fffffff || cp.max_pages > (g.kv_fp8 ? kMaxItemPagesFp8 : kMaxItemPages)) return TA_ERR_INVALID_ARG;
        const dim3 grid(static_cast<unsigned>(blocks)), block(kChunkThreads);
        if (ev.start != nullptr) TA_HIP_TRY(hipEventRecord(ev.start, stream));
        if (g.kv_fp8) {
            const int rc = launch_fp8_items(cp, g.group, true, false, grid.x, stream);
            if (rc != TA_OK) return rc;
        } else {
            switch (g.group) {
                case 1: hipLaunchKernelGGL((decode_chunk_kernel<1, true>), grid, block, 0, stream, cp); break;
                case 2: hipLaunchKernelGGL((decode_chunk_kernel<2, true>), grid, block, 0, stream, cp); break;
                case 4: hipLaunchKernelGGL((decode_chunk_kernel<4, true>), grid, block, 0, stream, cp); break;
                default: return TA_ERR_UNSUPPORTED;
            }
            TA_HIP_TRY(hipGetLastError());
        }
        if (ev.stop != nullptr) TA_HIP_TRY(hipEventRecord(ev.stop, stream));
        return TA_OK;
    }

    int32_t* chunk_start = reinterpret_cast<int32_t*>(workspace + w.off_chunk_start);
    int4* items = reinterpret_cast<int4*>(workspace + w.off_items);
    float* part_ml = reinterpret_cast<float*>(workspace + w.off_part_ml);
    float* part_o = reinterpret_cast<float*>(workspace + w.off_part_o);
    int32_t* counts = reinterpret_cast<int32_t*>(workspace + w.off_counts);
    int32_t* lcp = reinterpret_cast<int32_t*>(workspace + w.off_lcp);
    int32_t* pred = reinterpret_cast<int32_t*>(workspace + w.off_pred);
    int32_t* order = reinterpret_cast<int32_t*>(workspace + w.off_order);
    int4* shared_items = reinterpret_cast<int4*>(workspace + w.off_shared_items);
    // sharing needs at least two programs with a bulk chunk each and a non-empty block table
    const bool look_for_sharing = a.batch >= 2 && a.batch <= 1024 && w.max_shared_items > 0 &&
                                  a.block_table_stride > 0 && cp.max_pages >= kMinChunkPages;
    // rows of one workgroup of the kernel that computes the shared chunks: 128 on the tile kernel,
    // two sets of sixteen columns of the score tile in the kernel for FP8 caches
    const int32_t max_members = (g.kv_fp8 ? 32 : 128) / g.group;
    // The workspace plan has decided which kernel streams the private chunks (and sized
    // shared_items for it): the matrix-core kernel takes them as groups of one program.
    const int route = w.private_on_tiles;                    // kRouteOnDevice: both kernels are launched, one finds its list empty
    const bool private_on_tiles = route != kRouteVector;     // the tile kernel may get private chunks

    if (look_for_sharing) {
        hipLaunchKernelGGL(predecessor_prefix_kernel, dim3(a.batch), dim3(256), 0, stream, a.block_table,
                           a.block_table_stride, a.context_lens, pred, lcp);
        TA_HIP_TRY(hipGetLastError());
    }
    // one workgroup, as small as the batch allows: its many barriers cost less with fewer waves
    unsigned plan_threads = 64;
    while (plan_threads < 1024 && plan_threads < static_cast<unsigned>(a.batch)) plan_threads <<= 1;
    hipLaunchKernelGGL(plan_decode_kernel, dim3(1), dim3(plan_threads), 0, stream, a.context_lens,
                       look_for_sharing ? pred : nullptr, look_for_sharing ? lcp : nullptr, a.batch, cp.max_pages,
                       w.chunk_pages, g.decode_chunk_pages == 0 ? 1 : 0, g.num_kv_heads, w.max_chunks, max_members,
                       w.max_shared_items,
                       route,
                       chunk_start, items, shared_items, order, counts);
    TA_HIP_TRY(hipGetLastError());

    cp.counts = counts;
    cp.items = items;
    cp.part_ml = part_ml;
    cp.part_o = part_o;
    if (look_for_sharing && g.kv_fp8) {
        // an FP8 cache: the shared chunks go through a form of the kernel that streams the private
        // ones, up to 32 / group member programs per workgroup
        cp.shared_items = shared_items;
        cp.order = order;
        cp.chunk_start = chunk_start;
        const int64_t walkers = w.max_shared_items < 256 ? w.max_shared_items : 256;     // each walks the list
        const int rc = launch_fp8_items(cp, g.group, false, true, static_cast<unsigned>(walkers * g.num_kv_heads), stream);
        if (rc != TA_OK) return rc;
    } else if (look_for_sharing || private_on_tiles) {
        SharedPrefixArgs sa{};
        sa.q = a.q;
        sa.k_pool = a.k_pool;
        sa.v_pool = a.v_pool;
        sa.block_table = a.block_table;
        sa.context_lens = a.context_lens;
        sa.shared_items = reinterpret_cast<const int32_t*>(shared_items);
        sa.order = order;
        sa.counts = counts;
        sa.chunk_start = chunk_start;
        sa.part_ml = part_ml;
        sa.part_o = part_o;
        sa.block_table_stride = a.block_table_stride;
        sa.batch = a.batch;
        sa.max_items = w.max_shared_items;
        sa.private_on_tiles = private_on_tiles ? 1 : 0;
        if (private_on_tiles && ev.start != nullptr) TA_HIP_TRY(hipEventRecord(ev.start, stream));
        const int rc = launch_shared_prefix(g, sa, stream);
        if (rc != TA_OK) return rc;
        if (private_on_tiles && ev.stop != nullptr) TA_HIP_TRY(hipEventRecord(ev.stop, stream));
    }

    if (w.max_chunks > 0 && route != kRouteTiles) {
        const int64_t blocks = int64_t(w.max_chunks) * g.num_kv_heads;
        // (a route settled on the device: the plan kernel keeps this kernel's items within its limit)
        if (blocks > 0x7fffffff ||
            (route == kRouteVector && w.chunk_pages > (g.kv_fp8 ? kMaxItemPagesFp8 : kMaxItemPages)))
            return TA_ERR_INVALID_ARG;
        const dim3 grid(static_cast<unsigned>(blocks < kChunkGridCap ? blocks : kChunkGridCap)), block(kChunkThreads);
        const bool timed = route == kRouteVector;     // else the events went around the tile kernel's launch
        if (timed && ev.start != nullptr) TA_HIP_TRY(hipEventRecord(ev.start, stream));
        if (g.kv_fp8) {
            const int rc = launch_fp8_items(cp, g.group, false, false, static_cast<unsigned>(blocks), stream);   // one workgroup per pair
            if (rc != TA_OK) return rc;
        } else {
            switch (g.group) {
                case 1: hipLaunchKernelGGL((decode_chunk_kernel<1, false>), grid, block, 0, stream, cp); break;
                case 2: hipLaunchKernelGGL((decode_chunk_kernel<2, false>), grid, block, 0, stream, cp); break;
                case 4: hipLaunchKernelGGL((decode_chunk_kernel<4, false>), grid, block, 0, stream, cp); break;
                default: return TA_ERR_UNSUPPORTED;
            }
            TA_HIP_TRY(hipGetLastError());
            if (blocks > kChunkGridCap) {        // the pairs beyond the first launch, if the batch has any
                switch (g.group) {
                    case 1: hipLaunchKernelGGL(decode_chunk_beyond_cap_kernel<1>, grid, block, 0, stream, cp); break;
                    case 2: hipLaunchKernelGGL(decode_chunk_beyond_cap_kernel<2>, grid, block, 0, stream, cp); break;
                    default: hipLaunchKernelGGL(decode_chunk_beyond_cap_kernel<4>, grid, block, 0, stream, cp); break;
                }
                TA_HIP_TRY(hipGetLastError());
            }
        }
        if (timed && ev.stop != nullptr) TA_HIP_TRY(hipEventRecord(ev.stop, stream));
    }

    MergeParams mp{};
    mp.chunk_start = chunk_start;
    mp.part_ml = part_ml;
    mp.part_o = part_o;
    mp.out = a.out;
    mp.lse = a.lse;
    mp.batch = a.batch;
    mp.num_q_heads = g.num_q_heads;
    mp.out_scale = g.kv_fp8 ? g.v_scale : 1.0f;
    const int64_t rows = int64_t(a.batch) * g.num_q_heads;
    hipLaunchKernelGGL(decode_merge_kernel, dim3(static_cast<unsigned>((rows + 3) / 4)), dim3(256), 0,
                       stream, mp);
    TA_HIP_TRY(hipGetLastError());
    return TA_OK;
}

}  // namespace ta
