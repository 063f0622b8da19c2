// Append-prefill attention for gfx950: the n new tokens of a program attend
// causally to the retained prefix plus themselves (ThunderAgent Sec. 4.2, the
// incremental-prefill term of Eq. 3; Sec. 2.1, c_{t+1} extends c_t).
//
// Here q.K^T and p.V are dense contractions, so both run on the matrix cores
// (v_mfma_f32_32x32x16_bf16).  One workgroup of eight waves (two per SIMD, so
// that one wave's vector work fills the issue slots the other leaves) owns 256
// score rows = (256 / G) consecutive new tokens x the G query heads that share
// a kv head, and walks the program's keys in tiles of 64 (four pages):
//
//   * K and V tiles go HBM -> LDS once per workgroup and serve all 256 rows.
//     The memory pipeline writes them into LDS itself (global_load_lds_dwordx4),
//     so staging takes no vector registers, no LDS store instructions and no
//     vector ALU work; a ring of four slots keeps a tile in flight for two
//     iterations, with one barrier per tile;
//   * every wave owns 32 rows and computes the TRANSPOSED scores S^T = K Q^T,
//     so that each lane holds one query row's scores in its accumulator
//     registers: the softmax needs one cross-lane exchange per tile, and the
//     exponentiated scores are already laid out as the B operand of
//     O^T = V^T P^T;
//   * V stays row-major in LDS; the A operand of O^T = V^T P^T (eight keys of one
//     dim per lane) is fetched by the transposing LDS read ds_read_b64_tr_b16;
//   * the running maximum is only raised (and O rescaled) when it grows by more
//     than 2^8, a wave-uniform and rare event after the first tile.
//
// With random operands the chip's power management, not the instruction mix,
// sets the pace of this kernel: the shader clock settles well below its
// nominal value as soon as the matrix cores are busy most of the time, and
// every byte fetched through the fabric costs clock as well.
#include <atomic>
#include <type_traits>

#include "ta_internal.h"

namespace ta {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kThreads = 512;        // eight waves, two per SIMD
constexpr int kRowsPerBlock = 256;   // score rows per workgroup
constexpr int kRB = 1;               // 32-row blocks per wave
constexpr int kTileKeys = 64;        // keys per LDS tile (4 pages)
constexpr float kRescaleThreshold = 8.0f;  // log2 units
#ifndef TA_PAIRS_IN_X
#define TA_PAIRS_IN_X 6
#endif
constexpr int kRing = 4;                   // LDS slots (tiles in flight); the slot arithmetic below is "& 3"
static_assert(kRing == 4, "slot indices are computed modulo four");
constexpr int kKAhead = 3;                 // LDS operand reads in flight ahead of their matrix instruction
constexpr int kVAhead = 4;

struct PrefillParams {
    const uint16_t* q;
    const char* k_pool;
    const char* v_pool;
    const int32_t* block_table;
    const int32_t* context_lens;
    const int32_t* cu_q_lens;
    const int32_t* tile_start;  // [batch + 1]
    const int2* tiles;          // (program, query tile)
    uint16_t* out;
    float* lse;
    // shared-prefix decode only: one item = (position of the group's first member in `order`,
    // members, chunk, first member); the members are order[position .. position + members)
    const int4* shared_items;
    const int32_t* order;
    int32_t* counts;             // counts[1] = number of shared items, counts[2] = next (item, kv head) pair to take,
                                 // counts[3] = pages per chunk (the plan kernel settles it)
    const int32_t* chunk_start;  // [batch + 1] first partial slot of each program
    float* part_ml;              // [slot][Hq][2]  reference maximum (log2 domain), sum
    float* part_o;               // [slot][Hq][128] unnormalised output
    int64_t stride_page_bytes;
    int64_t stride_head_bytes;
    int32_t block_table_stride;
    int32_t batch;
    int32_t num_q_heads;
    int32_t num_kv_heads;
    float scale_log2;
    float out_scale;             // append-prefill: multiplies the normalised output (the value scale of an FP8 cache, else 1)
    // append-prefill with the keys of every query tile cut into `split` chunks of chunk_tiles key
    // tiles (split = 1: not cut): a workgroup computes one chunk and writes the rows' partials to
    // part_ml / part_o at [row * split + chunk], row = token * Hq + head
    int32_t split;
    int32_t chunk_tiles;
    // tiles == nullptr (batches of up to 64 programs whose keys are cut into chunks): every wave works
    // the tile list out for itself from cu_q_lens, at most tiles_per_program_max tiles a program
    int32_t tiles_per_program_max;
};

// plan: query tiles of tile_tokens tokens per program, listed flat.  Workgroups are dispatched
// in list order and a tile's run time grows with its program's context, so for batches of up to
// 1024 programs the list starts with the longest contexts (the short ones fill the tail of the
// launch); the tiles of one program stay together, they share its K/V stream in L2.
__global__ __launch_bounds__(1024) void plan_tiles_kernel(const int32_t* __restrict__ cu_q_lens,
                                                          const int32_t* __restrict__ context_lens,
                                                          int32_t batch, int32_t tile_tokens,
                                                          int32_t max_per_program,
                                                          int32_t* __restrict__ tile_start,
                                                          int2* __restrict__ tiles) {
    __shared__ int32_t scan[1024];
    __shared__ int32_t order[1024];    // program at each list position
    __shared__ int32_t length[1024];   // its context length (sort key)
    __shared__ int32_t carry;
    const int tid = threadIdx.x;
    const int nt = blockDim.x;         // a power of two, 64 .. 1024, at least the batch when the batch is at most 1024
    auto tiles_of = [&](int b) {
        const int nq = cu_q_lens[b + 1] - cu_q_lens[b];
        const int n = nq > 0 ? (nq + tile_tokens - 1) / tile_tokens : 0;
        return n > max_per_program ? max_per_program : n;
    };
    if (tid == 0) carry = 0;
    const bool sorted = batch <= 1024;
    if (sorted) {
        order[tid] = tid;
        length[tid] = tid < batch ? context_lens[tid] : -1;
        __syncthreads();
        // bitonic sort, descending by length, ties by program index (a total order: deterministic)
        for (int k = 2; k <= nt; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                const int other = tid ^ j;
                if (other > tid) {
                    const int la = length[tid], lb = length[other], oa = order[tid], ob = order[other];
                    const bool a_first = la > lb || (la == lb && oa < ob);   // a belongs before b
                    const bool descending = (tid & k) == 0;
                    if (a_first != descending) {
                        length[tid] = lb; length[other] = la;
                        order[tid] = ob; order[other] = oa;
                    }
                }
                __syncthreads();
            }
        }
    }
    __syncthreads();
    for (int base = 0; base < batch; base += nt) {
        const int pos = base + tid;
        const int b = sorted ? order[tid] : pos;
        const int n = pos < batch ? tiles_of(b) : 0;
        scan[tid] = n;
        __syncthreads();
        for (int off = 1; off < nt; off <<= 1) {
            const int v = tid >= off ? scan[tid - off] : 0;
            __syncthreads();
            scan[tid] += v;
            __syncthreads();
        }
        const int first = carry + scan[tid] - n;
        if (pos < batch) {
            tile_start[b] = first;
            for (int c = 0; c < n; ++c) tiles[first + c] = make_int2(b, c);
        }
        __syncthreads();
        if (tid == nt - 1) carry += scan[nt - 1];
        __syncthreads();
    }
    if (tid == 0) tile_start[batch] = carry;
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    // round to nearest even; inputs are finite non-negative weights
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    const f32x2 v = {lo, hi};
    const bf16x2 r = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ uint16_t to_bf16_rne(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

// Maximum of a value over lanes l and l ^ 32 (the two lanes that hold one score row), on the
// vector ALU: v_permlane32_swap returns {old[0..31], src[0..31]} and {old[32..63], src[32..63]}.
__device__ __forceinline__ float max_across_halves(float x) {
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const u32x2 r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, r.x), __builtin_bit_cast(float, r.y));
}

// LDS holds a ring of kRing slots; a slot is the K tile followed by the V tile of 64 keys, both
// row-major (one key = 256 bytes) with their sixteen 16-byte chunks permuted per row so that the
// operand reads are free of bank conflicts:
//   K: chunk c of key k sits at chunk position c ^ (k & 15)        (16 lanes read 16 keys, same c)
//   V: chunk c of key k sits at chunk position c ^ ((k & 3) << 2)  (a transposing read touches
//      4 keys x 64 bytes)
// The tiles are written by the memory pipeline itself (global_load_lds_dwordx4: every lane names
// the 16 global bytes it wants, the wave's 64 pieces land in LDS in lane order), so staging costs
// no vector registers and no LDS store instructions; the permutation is applied on the global
// side, by choosing which chunk a lane fetches.
constexpr int kTileBytes = kTileKeys * kHeadDim * 2;   // 16 KiB
constexpr int kSlotBytes = 2 * kTileBytes;

typedef __attribute__((ext_vector_type(4))) short s16x4;
#define TA_LDS_PTR(T, ptr) ((__attribute__((address_space(3))) T*)(ptr))
#define TA_GLOBAL_PTR(ptr) ((const __attribute__((address_space(1))) void*)(ptr))

// SHARED = false: append-prefill, rows = (new token, head), causal, writes bf16 output.
// SHARED = true:  decode of a group of programs whose block tables begin with the same pages
//                 (forked agent branches): rows = (member program, head), keys = one chunk of
//                 the shared prefix, no mask, writes split-K partials for the decode merge.
//                 A group of one program is a private chunk (used when G = 8, where the
//                 vector-ALU decode kernel runs out of registers, and for large batches,
//                 which stream faster here): it may hold the end of the program's context,
//                 so its last tile is masked like a causal one.  At most 128 rows; the two
//                 waves of a row block split the keys of every tile.
// Waves none of whose 32 rows exist take part in the loads and barriers only.
template <int G, bool SHARED>
__global__ __launch_bounds__(kThreads, 1) void attention_tile_kernel(PrefillParams p) {
    constexpr int kTileTokens = kRowsPerBlock / G;   // new tokens per query tile (append-prefill)
    extern __shared__ __attribute__((aligned(16))) char lds[];   // [kRing][K tile | V tile]

    // Append-prefill is launched with one workgroup per (item, kv head) pair.  The decode side
    // is launched with a small resident grid (its item count is only known on the device, and is
    // zero unless programs share pages or G = 8) whose workgroups take the next pair from a
    // counter as they finish one: items differ in length by a factor of four, and a fixed
    // stride left the tail of the launch unbalanced.  Every item writes its own partial slots,
    // so the result does not depend on which workgroup ran it.
    // Append-prefill of a few programs is a short launch, and a plan kernel in front of it plus two
    // more dependent loads here (tile -> program -> its lengths) are a fifth of its time: there
    // lane l of every wave takes program l, and a scan over the wave gives the tile list.
    const bool plan_here = !SHARED && p.tiles == nullptr;
    __shared__ int plan_tiles[64], plan_tiles_through[64];   // tiles of program l; of programs 0 .. l
    int tiles_through_mine = 0;
    if (plan_here) {
        const int l = threadIdx.x & 63;
        int tiles_mine = 0;
        if (l < p.batch) {
            const int nq = p.cu_q_lens[l + 1] - p.cu_q_lens[l];
            tiles_mine = nq > 0 ? (nq + kTileTokens - 1) / kTileTokens : 0;
            tiles_mine = tiles_mine < p.tiles_per_program_max ? tiles_mine : p.tiles_per_program_max;
        }
        tiles_through_mine = tiles_mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int below = __shfl_up(tiles_through_mine, d);
            if (l >= d) tiles_through_mine += below;
        }
        if (threadIdx.x < 64) {          // kept in LDS: registers are what this kernel is short of
            plan_tiles[l] = tiles_mine;
            plan_tiles_through[l] = tiles_through_mine;
        }
        __syncthreads();
    }
    const int n_items = SHARED      ? p.counts[1]
                        : plan_here ? __builtin_amdgcn_readlane(tiles_through_mine, 63)
                                    : p.tile_start[p.batch];
    if (SHARED && n_items == 0) return;   // nothing shared in this batch (the usual case off the tile route): no trip to the counter
    const int tiles_per_chunk = SHARED ? p.counts[3] / 4 : 0;   // read once: the line it shares with the work counter is busy
    __shared__ int next_pair;
    auto take_pair = [&]() {
        if (threadIdx.x == 0) next_pair = atomicAdd(p.counts + 2, 1);
        __syncthreads();
        const int v = next_pair;
        __syncthreads();
        return v;
    };
    // (Claiming the next pair one item ahead hides the counter's round trip but costs more at the
    // end of the launch, where a claimed item waits for its owner: measured slower.)
    // Append-prefill with the keys cut into `split` chunks: a stream = (chunk of keys, kv head), read
    // by every query tile that reaches it.  Workgroups go to the eight XCDs in turn (workgroup i to
    // XCD i % 8), each XCD with an L2 of its own: stream s belongs to XCD s % 8, which runs the
    // stream's query tiles one after the other, so the stream comes out of memory once.  (Uncut,
    // the tiles of a program are neighbours in the same way when there are eight kv heads.)
    const int split = SHARED ? 1 : p.split;
    const int n_streams = p.num_kv_heads * split;
    const int blk_end = split > 1 ? ((n_streams + 7) >> 3) * 8 * n_items : n_items * p.num_kv_heads;
    int blk = SHARED ? take_pair() : int(blockIdx.x);
    while (blk < blk_end) {
    int part = 0, tile_id, g;
    if (split > 1) {
        const int turn = (blk >> 3) / n_items;
        const int stream = turn * 8 + (blk & 7);
        if (stream >= n_streams) { blk += int(gridDim.x); continue; }
        tile_id = (blk >> 3) - turn * n_items;
        part = stream / p.num_kv_heads;
        g = stream - part * p.num_kv_heads;
    } else {
        tile_id = blk / p.num_kv_heads;
        g = blk - tile_id * p.num_kv_heads;
    }
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hl = lane >> 5;                // which half of the wave
    const int l32 = lane & 31;
    // Append-prefill: wave w owns rows 32 w .. 32 w + 31 and computes on both 32-key blocks of
    // every tile.  Decode side: a workgroup has at most 128 rows; waves 2 j and 2 j + 1 both own
    // rows 32 j .. 32 j + 31 and split the keys, wave 2 j + kb taking block kb of every tile (the
    // two sit on different SIMDs); their results meet in LDS at the end of the item.  A private
    // chunk (eight rows) then keeps two matrix cores busy instead of one, and a tile is
    // consumed in half the time.
    const int row_block = SHARED ? (wave >> 1) : wave;
    const int kb_mine = wave & 1;

    int b, q0, nq, L, prefix, t0, t_begin, n_tiles, n_unmasked, members = 0, chunk = 0, first_pos = 0;
    if (SHARED) {
        const int4 it = p.shared_items[tile_id];
        first_pos = it.x;
        b = it.w;                      // the group's first program: its block table names the pages
        members = it.y;
        chunk = it.z;
        q0 = 0; nq = 0; prefix = 0; t0 = 0;
        t_begin = chunk * tiles_per_chunk;
        n_tiles = t_begin + tiles_per_chunk;
        n_unmasked = n_tiles;
        L = 0x7fffffff;                // every key of a shared chunk exists
        if (members == 1) {            // a private chunk ends where its program's context ends
            L = p.context_lens[b];
            const int last = (L + kTileKeys - 1) / kTileKeys;
            n_tiles = n_tiles < last ? n_tiles : last;
            n_unmasked = L / kTileKeys < n_tiles ? L / kTileKeys : n_tiles;
        }
    } else {
        int2 tl;
        if (plan_here) {
            // the program of the tile: the first whose tiles reach beyond it (programs without tiles are passed over)
            tl.x = __builtin_popcountll(__builtin_amdgcn_ballot_w64(plan_tiles_through[threadIdx.x & 63] <= tile_id));
            tl.y = tile_id - (plan_tiles_through[tl.x] - plan_tiles[tl.x]);
        } else {
            tl = p.tiles[tile_id];
        }
        b = tl.x;
        q0 = p.cu_q_lens[b];
        nq = p.cu_q_lens[b + 1] - q0;
        L = p.context_lens[b];
        prefix = L - nq;
        t0 = tl.y * kTileTokens;                         // first new token of this tile
        int t_end = t0 + kTileTokens;
        t_end = t_end > nq ? nq : t_end;
        const int keys_needed = prefix + t_end;          // largest visible count in the tile
        t_begin = 0;
        n_tiles = (keys_needed + kTileKeys - 1) / kTileKeys;
        n_unmasked = (prefix + t0 + 1) / kTileKeys;      // tiles every row sees completely
        if (split > 1) {                                 // this workgroup's chunk of them
            t_begin = part * p.chunk_tiles;
            if (t_begin >= n_tiles) {                    // the tile's keys end before this chunk: nothing to write
                blk += int(gridDim.x);
                continue;
            }
            n_tiles = n_tiles < t_begin + p.chunk_tiles ? n_tiles : t_begin + p.chunk_tiles;
            n_unmasked = n_unmasked < n_tiles ? n_unmasked : n_tiles;
        }
    }
    const int n_pages_b = (p.context_lens[b] + kPageSize - 1) / kPageSize;

    // ---- per-lane rows: one block of 32 rows per wave ----
    // row -> (token or member program, head): row = index * G + head
    int vis[kRB];            // visible keys of this lane's row in row block rb (0 = row does not exist)
    bf16x8 qf[kRB][8];       // B operands: q[row][16 ks + 8 hl .. + 7]
    int64_t out_row[kRB];    // element offset of the row in q / out, or -1
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
        const int row = row_block * (32 * kRB) + rb * 32 + l32;
        const int idx = t0 + row / G;
        const int head = g * G + row % G;
        const bool ok = SHARED ? (row / G < members) : (idx < nq);
        vis[rb] = ok ? (SHARED ? L : prefix + idx + 1) : 0;
        // a member's query row is its program's row; members sit side by side in `order`
        const int q_row = ok ? (SHARED ? p.order[first_pos + row / G] : q0 + idx) : 0;
        out_row[rb] = ok ? (int64_t(q_row) * p.num_q_heads + head) * kHeadDim : int64_t(-1);
        const uint16_t* qrow = p.q + (ok ? out_row[rb] : 0) + hl * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            u32x4 t = {0u, 0u, 0u, 0u};
            if (ok) t = *reinterpret_cast<const u32x4*>(qrow + ks * 16);
            qf[rb][ks] = __builtin_bit_cast(bf16x8, t);
        }
    }

    bool any_row = false;
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) any_row = any_row || vis[rb] > 0;
    const bool wave_active = __builtin_amdgcn_ballot_w64(any_row) != 0;   // wave-uniform

    // ---- staging: wave w brings in keys 8 w .. 8 w + 7 of every tile (half a page) ----
    // Two instructions for K and two for V; instruction q covers keys 8 w + 4 q + (0 .. 3), and
    // lane (lrow, l16) of it fills chunk position l16 of key 8 w + 4 q + lrow.
    const int l16 = lane & 15;
    const int lrow = lane >> 4;
    uint32_t dma_k[2], dma_v[2];    // byte offset inside the page of the chunk this lane fetches
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int row = 8 * (wave & 1) + 4 * q + lrow;            // row of the key in its page
        dma_k[q] = row * 256 + ((l16 ^ (row & 15)) << 4);
        dma_v[q] = row * 256 + ((l16 ^ ((row & 3) << 2)) << 4);
    }
    const char* k_head = p.k_pool + int64_t(g) * p.stride_head_bytes;
    const char* v_head = p.v_pool + int64_t(g) * p.stride_head_bytes;
    const int32_t* table = p.block_table + int64_t(b) * p.block_table_stride;
    const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(TA_LDS_PTR(char, lds)));

    // Page ids: lane l of every wave holds the id of page (64 g + l) of the current group of 64
    // pages (16 tiles), clamped to the program's last page; the next group is fetched one
    // group ahead, so no tile waits for a dependent id load.
    auto fetch_ids = [&](int group) -> int {
        int pg = group * 64 + lane;
        pg = pg < n_pages_b ? pg : n_pages_b - 1;
        return table[pg];
    };
    // byte offset of a page inside a pool, computed by all lanes at once when a group of ids
    // becomes current (their load was issued a group earlier)
    auto page_bytes = [&](int id) -> int64_t { return int64_t(id) * p.stride_page_bytes; };
    auto lane_value = [&](int64_t v, int idx) -> int64_t {
        const uint32_t lo = __builtin_amdgcn_readlane(static_cast<int>(v), idx);
        const uint32_t hi = __builtin_amdgcn_readlane(static_cast<int>(v >> 32), idx);
        return static_cast<int64_t>((uint64_t(hi) << 32) | lo);
    };
    int ids_group = t_begin >> 4;
    int64_t ids_cur = page_bytes(fetch_ids(ids_group));
    int ids_next = fetch_ids(ids_group + 1);

    // Starting the loads of one tile = the page offset out of the lanes + four instructions.
    // Exactly four per tile, always (tiles past the end re-read the last page): the waits below
    // count on it.
    auto plan_load = [&](int t) -> int64_t {
        // The ring runs three tiles ahead.  Past the item's last tile, append-prefill re-reads
        // that tile (still in L2) instead of pulling pages nobody will use through the fabric.
        // The decode side's loads do not stay in L2, so there the surplus loads all read the
        // pool's first page: one line set that every workgroup keeps warm.  (Nothing computes
        // on these tiles.)
        if (SHARED && t >= n_tiles) return 0;
        t = t < n_tiles ? t : n_tiles - 1;
        if ((t >> 4) != ids_group) {      // tiles are visited in order, so this is group + 1
            ids_group = t >> 4;
            ids_cur = page_bytes(ids_next);
            ids_next = fetch_ids(ids_group + 1);
        }
        return lane_value(ids_cur, (t & 15) * 4 + (wave >> 1));
    };
    auto load_step = [&](int64_t page_off, int slot, int i) __attribute__((always_inline)) {
        const uint32_t dst = lds_base + slot * kSlotBytes + (i >> 1) * kTileBytes + wave * 2048 + (i & 1) * 1024;
        // the page's address is the same for all lanes (scalar registers, scalar adds); a lane adds
        // only the 32-bit offset of its chunk, so starting a load takes no vector instruction
        const char* page = ((i >> 1) ? v_head : k_head) + page_off;
        const uint32_t chunk = (i >> 1) ? dma_v[i & 1] : dma_k[i & 1];
        // Written as assembly on purpose: for the builtin form the compiler assumes that every
        // later LDS read may touch the bytes in flight and waits for the load right away.  The
        // waits are placed by hand instead (finish_tile), one per tile.  The instruction takes
        // its LDS address from m0, which the compiler manages on its own and does not expect a
        // statement to change: the statement puts back the value it found.
        // On the decode side every K/V byte is used once by one workgroup: the loads carry the
        // non-temporal hint, like those of the other decode kernels.  Append-prefill re-reads
        // K/V from the L2 (the query tiles of a program run side by side) and keeps the default.
        uint32_t saved_m0;
        if constexpr (SHARED)
            asm volatile(
                "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3 nt\n\ts_mov_b32 m0, %0"
                : "=&s"(saved_m0)
                : "s"(dst), "v"(chunk), "s"(page)
                : "memory");
        else
            asm volatile(
                "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
                : "=&s"(saved_m0)
                : "s"(dst), "v"(chunk), "s"(page)
                : "memory");
    };
    auto load_tile = [&](int t, int slot) __attribute__((always_inline)) {
        const int64_t page_off = plan_load(t);
#pragma unroll
        for (int i = 0; i < 4; ++i) load_step(page_off, slot, i);
    };
    // Keys at or beyond the context length may hold anything (even NaN): their V rows are
    // zeroed once they have landed, because 0 * NaN inside the matrix core would poison O.
    // Every lane clears the pieces it fetched itself.
    auto scrub_tail = [&](int t, int slot) {
        if ((t + 1) * kTileKeys > L) {   // only the tile that holds the end of the context
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int key = t * kTileKeys + 8 * wave + 4 * q + lrow;
                if (key >= L)
                    *reinterpret_cast<u32x4*>(lds + slot * kSlotBytes + kTileBytes + wave * 2048 + q * 1024 + lane * 16) =
                        u32x4{0u, 0u, 0u, 0u};
            }
        }
    };

    // ---- accumulators ----
    f32x16 o[4][kRB];        // O^T blocks: [dim block][row block]
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][rb][r] = 0.0f;
    float m[kRB], lsum[kRB];   // reference maximum (log2 domain, scaled); this lane's share of the row sum
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) { m[rb] = kNegBig; lsum[rb] = 0.0f; }

    // ---- LDS operand reads: one per-lane offset each, the rest are compile-time offsets ----
    // K operand of (block kb, step ks): key l32 + 32 kb, dims 16 ks + 8 hl .. + 7 = chunk 2 ks + hl
    int k_rd[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        k_rd[ks] = l32 * 256 + (((2 * ks + hl) ^ (l32 & 15)) << 4) + (SHARED ? kb_mine * 32 * 256 : 0);
    // V operand of (block kb, step, dim block db): lane (l32, hl) needs dim 32 db + l32 of the keys
    // 32 kb + 16 step + 4 hl + {0..3, 8..11} (the keys whose weights sit in its B operand).  Two
    // transposing reads (ds_read_b64_tr_b16) fetch four keys each: in every group of 16 lanes,
    // lane s names the 8 bytes (4 dims) of key s / 4 at dims 4 (s % 4) .., and lane j receives
    // dim j of the four keys.
    int v_rd[4];
#pragma unroll
    for (int db = 0; db < 4; ++db) {
        const int key = 4 * hl + (l16 >> 2);                      // + 32 kb + 16 step + 8 half
        const int c = 4 * db + 2 * (lrow & 1) + ((lane & 3) >> 1);   // 16-byte chunk of the dims
        v_rd[db] = key * 256 + ((c ^ ((key & 3) << 2)) << 4) + (lane & 1) * 8 + (SHARED ? kb_mine * 32 * 256 : 0);
    }
    auto k_operand_at = [&](const char* kt, int kb, int ks) __attribute__((always_inline)) {
        return *reinterpret_cast<const bf16x8*>(kt + kb * 32 * 256 + k_rd[ks]);
    };
    auto v_operand_at = [&](const char* vt, int kb, int idx) __attribute__((always_inline)) {   // idx = 4 step + dim block
        const char* at = vt + (kb * 32 + (idx >> 2) * 16) * 256 + v_rd[idx & 3];
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(TA_LDS_PTR(s16x4, at));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(TA_LDS_PTR(s16x4, at + 8 * 256));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // The same reads for the pipelined body, where the slot is a compile-time value.  An LDS
    // instruction carries a 16-bit offset, and the ring is 128 KiB: for the upper two slots the
    // per-lane part lives in a second set of registers that already holds + 64 KiB, so that no
    // read needs a vector add for its address.  (The value is hidden from the compiler, which
    // would otherwise recompute it at every use, and masked so it is known to be non-negative,
    // which the offset folding requires.)
    int k_rd_hi[8], v_rd_hi[4];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        int x = k_rd[ks] + 65536;
        asm volatile("" : "+v"(x));
        k_rd_hi[ks] = x & 0x1ffff;
    }
#pragma unroll
    for (int db = 0; db < 4; ++db) {
        int x = v_rd[db] + 65536;
        asm volatile("" : "+v"(x));
        v_rd_hi[db] = x & 0x1ffff;
    }
    auto k_operand_in = [&](auto slot_tag, int kb, int ks) __attribute__((always_inline)) {
        constexpr int S = decltype(slot_tag)::value;
        const int lane_part = S >= 2 ? k_rd_hi[ks] : k_rd[ks];
        return *reinterpret_cast<const bf16x8*>(lds + (S & 1) * kSlotBytes + kb * 32 * 256 + lane_part);
    };
    auto v_operand_in = [&](auto slot_tag, int kb, int idx) __attribute__((always_inline)) {
        constexpr int S = decltype(slot_tag)::value;
        const int lane_part = S >= 2 ? v_rd_hi[idx & 3] : v_rd[idx & 3];
        const char* at = lds + (S & 1) * kSlotBytes + kTileBytes + (kb * 32 + (idx >> 2) * 16) * 256 + lane_part;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(TA_LDS_PTR(s16x4, at));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(TA_LDS_PTR(s16x4, at + 8 * 256));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    // ---- the four steps of one 32-key block ----
    // A: S^T block = K Q^T, 32 keys x 32 rows; register r of lane (l32, hl) holds
    //    key 8 (r / 4) + 4 hl + r % 4 of the block
    auto scores = [&](const char* kt, int kb, f32x16 (&s)[kRB]) {
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[rb][r] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 a = k_operand_at(kt, kb, ks);
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][ks], s[rb], 0, 0, 0);
        }
    };
    // causal mask of a block that straddles the diagonal
    auto mask_scores = [&](int key_base, f32x16 (&s)[kRB]) {
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key_base + 4 * hl + 8 * (r >> 2) + (r & 3);
                s[rb][r] = key < vis[rb] ? s[rb][r] : -INFINITY;
            }
    };
    // B1: row maxima; the reference is raised (and O, l rescaled) only when it would grow
    //     by more than the threshold, a wave-uniform and rare event
    auto rescale_if_needed = [&](const float (&cand)[kRB]) {
        bool grow = false;
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) grow = grow || cand[rb] > m[rb] + kRescaleThreshold;
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(grow) != 0, 0)) {
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                const float m_new = fmaxf(m[rb], cand[rb]);
                const float alpha = __builtin_amdgcn_exp2f(m[rb] - m_new);
                m[rb] = m_new;
                lsum[rb] *= alpha;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[db][rb][r] *= alpha;
            }
        }
    };
    auto raise_reference = [&](const f32x16 (&s)[kRB]) {
        float cand[kRB];
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
            float mx = fmaxf(fmaxf(s[rb][0], s[rb][1]), s[rb][2]);
#pragma unroll
            for (int r = 3; r < 15; r += 2) mx = fmaxf(fmaxf(mx, s[rb][r]), s[rb][r + 1]);
            mx = fmaxf(mx, s[rb][15]);
            mx = max_across_halves(mx);
            cand[rb] = mx * p.scale_log2;
        }
        rescale_if_needed(cand);
    };
    // B2: weights 2^(s c - m), row-sum share, packing into the B operands of the two k = 16 steps
    auto weights = [&](const f32x16 (&s)[kRB], bf16x8 (&pf)[kRB][2]) {
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
            const float bias = -m[rb];
            float pr[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) pr[r] = __builtin_amdgcn_exp2f(fmaf(s[rb][r], p.scale_log2, bias));
            // the row sum adds up the weights as computed (before rounding), in the same order
            // as the pipelined body
            float acc = lsum[rb];
#pragma unroll
            for (int step = 0; step < 2; ++step) {
                u32x4 w;
                w.x = pack_bf16(pr[8 * step + 0], pr[8 * step + 1]);
                w.y = pack_bf16(pr[8 * step + 2], pr[8 * step + 3]);
                w.z = pack_bf16(pr[8 * step + 4], pr[8 * step + 5]);
                w.w = pack_bf16(pr[8 * step + 6], pr[8 * step + 7]);
#pragma unroll
                for (int r = 0; r < 8; ++r) acc += pr[8 * step + r];
                pf[rb][step] = __builtin_bit_cast(bf16x8, w);
            }
            lsum[rb] = acc;
        }
    };
    // C: O^T += V^T P^T
    auto accumulate = [&](const char* vt, int kb, const bf16x8 (&pf)[kRB][2]) {
#pragma unroll
        for (int idx = 0; idx < 8; ++idx) {
            const bf16x8 a = v_operand_at(vt, kb, idx);
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb)
                o[idx & 3][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[rb][idx >> 2], o[idx & 3][rb], 0, 0, 0);
        }
    };

    // ---- the pipelined body's two regions, written slice by slice ----
    // Two waves share a SIMD; within a wave nothing hides latency except the order of its own
    // instructions, so the order is written out: every slice issues one matrix instruction, the
    // LDS read of an operand needed a few slices later, and a fixed share of the vector work; a
    // scheduling barrier closes the slice so the compiler keeps the interleaving.
    //
    // The LDS reads of a region's first operands are issued by the region before it (its last
    // slices call `prefetch_next`), so no region starts by waiting out an LDS round trip:
    // ka[0 .. kKAhead) and va[0 .. kVAhead) are always in flight or loaded on entry.
    //
    // Region X: scores of the next block (matrix core) with the weights of the current block
    // (vector ALU).  Turning a pair of scores into weights is seven vector instructions (two
    // multiply-adds, two exponentials, one packing conversion, two additions into the row sum).
    // All eight pairs in this region would be seven vector instructions per matrix instruction
    // here and nearly none in region Y, so this region converts pairs 0 .. kPairsInX - 1 and the
    // first slices of region Y, which otherwise only wait for the scores to leave the matrix
    // core, convert the rest; the matrix instructions that multiply with those come four slices
    // later.
    //
    // The row sum adds up the weights before they are rounded to bf16, with plain additions:
    // summing the rounded ones two at a time with the dot-product instruction was measured at
    // several times the cost of an addition (it does not overlap with matrix instructions).
    bf16x8 ka[8], va[8];
    constexpr int kPairsInX = TA_PAIRS_IN_X, kPairSteps = 7;
    uint32_t pw[kRB][8];          // packed weights of the current block, pair by pair
    float wf[kRB][8][2];          // a pair on its way through the steps
    auto weight_step = [&](const f32x16 (&s_old)[kRB], int rb, int j) __attribute__((always_inline)) {
        const int c = j / kPairSteps, part = j % kPairSteps;
        if (part < 2) {
            wf[rb][c][part] = fmaf(s_old[rb][2 * c + part], p.scale_log2, -m[rb]);
            asm volatile("" ::"v"(wf[rb][c][part]));
        } else if (part < 4) {
            wf[rb][c][part - 2] = __builtin_amdgcn_exp2f(wf[rb][c][part - 2]);
            asm volatile("" ::"v"(wf[rb][c][part - 2]));
        } else if (part == 4) {
            pw[rb][c] = pack_bf16(wf[rb][c][0], wf[rb][c][1]);
            asm volatile("" ::"v"(pw[rb][c]));
        } else {
            lsum[rb] += wf[rb][c][part - 5];
            asm volatile("" ::"v"(lsum[rb]));
        }
    };
    auto region_scores_weights = [&](auto&& read_k, f32x16 (&s_new)[kRB], const f32x16 (&s_old)[kRB],
                                     bf16x8 (&pf)[kRB][2], auto&& prefetch_next) __attribute__((always_inline)) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                s_new[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qf[rb][ks], ks == 0 ? zero : s_new[rb], 0, 0, 0);
                if (rb == 0 && ks + kKAhead < 8) ka[ks + kKAhead] = read_k(ks + kKAhead);
                if (rb == kRB - 1 && ks >= 8 - kVAhead) prefetch_next(ks - (8 - kVAhead));
                // an eighth of this region's share of the steps, in order
#pragma unroll
                for (int j = ks * (kPairSteps * kPairsInX) / 8; j < (ks + 1) * (kPairSteps * kPairsInX) / 8; ++j)
                    weight_step(s_old, rb, j);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
            const u32x4 w = {pw[rb][0], pw[rb][1], pw[rb][2], pw[rb][3]};
            pf[rb][0] = __builtin_bit_cast(bf16x8, w);
        }
    };
    // Region Y: O^T += V^T P^T (matrix core) with the last pairs of the current block's weights
    // (slices 0 .. 3) and the row maxima of the next block's scores (slices 4 .. 7, when those
    // scores have left the matrix core) on the vector ALU.
    auto region_accumulate_maxima = [&](auto&& read_v, bf16x8 (&pf)[kRB][2], const f32x16 (&s_old)[kRB],
                                        const f32x16 (&s_new)[kRB], bool use_new, auto&& staging_step,
                                        auto&& prefetch_next) __attribute__((always_inline)) {
        constexpr int kLeft = 8 - kPairsInX;    // pairs converted here
        float mx[kRB];
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) mx[rb] = -INFINITY;
#pragma unroll
        for (int idx = 0; idx < 8; ++idx) {
            const int step = idx >> 2, db = idx & 3;
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                if (idx == 4) {
                    const u32x4 w = {pw[rb][4], pw[rb][5], pw[rb][6], pw[rb][7]};
                    pf[rb][1] = __builtin_bit_cast(bf16x8, w);
                }
                o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[idx], pf[rb][step], o[db][rb], 0, 0, 0);
                if (rb == 0) {
                    if (idx + kVAhead < 8) va[idx + kVAhead] = read_v(idx + kVAhead);
                    if (idx >= 8 - kKAhead) prefetch_next(idx - (8 - kKAhead));
                }
                if (rb == kRB - 1) staging_step(idx);   // a share of the next tiles' HBM -> LDS traffic
                if (idx < 3) {          // the packed weights are complete one slice before their first use
#pragma unroll
                    for (int j = idx * (5 * kLeft) / 3; j < (idx + 1) * (5 * kLeft) / 3; ++j)
                        weight_step(s_old, rb, (kPairsInX + j / 5) * kPairSteps + j % 5);
                } else if (idx == 3) {  // their shares of the row sum
#pragma unroll
                    for (int c = kPairsInX; c < 8; ++c) {
                        weight_step(s_old, rb, c * kPairSteps + 5);
                        weight_step(s_old, rb, c * kPairSteps + 6);
                    }
                } else {                // four slices, four scores per slice
                    const int r0 = (idx - 4) * 4;
                    mx[rb] = fmaxf(fmaxf(mx[rb], s_new[rb][r0]), s_new[rb][r0 + 1]);
                    mx[rb] = fmaxf(fmaxf(mx[rb], s_new[rb][r0 + 2]), s_new[rb][r0 + 3]);
                    asm volatile("" ::"v"(mx[rb]));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        float cand[kRB];
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
            mx[rb] = max_across_halves(mx[rb]);
            // a look-ahead block that will be thrown away must not move the reference
            cand[rb] = use_new ? mx[rb] * p.scale_log2 : kNegBig;
        }
        rescale_if_needed(cand);
    };

    // ---- LDS ring of four slots; tile t lives in slot (t - t_begin) % 4 ----
    // Every iteration t: start the loads of tile t + 3 into the slot tile t - 1 left (last read
    // before the previous barrier), compute on tile t (the pipelined body also reads K of tile
    // t + 1), then wait until at most this iteration's four loads are in flight -- the memory
    // pipeline retires loads in order, so tile t + 2 has landed -- and meet at the barrier.
    // A tile is therefore requested two iterations before its first use.
    auto slot_ptr = [&](int slot) { return lds + slot * kSlotBytes; };
    auto finish_tile = [&](int t_landed, int slot_landed) __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        scrub_tail(t_landed, slot_landed);
        __syncthreads();
    };
    // The decode side reads nothing but tile t in iteration t, so it only needs tile t + 1 at the
    // barrier: two tiles (eight loads per wave) stay in flight across it, three while it computes.
    // Short iterations are bound by memory latency over tiles in flight, not by arithmetic.
    auto finish_tile_early = [&](int t_landed, int slot_landed) __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        scrub_tail(t_landed, slot_landed);
        __syncthreads();
    };
#pragma unroll
    for (int i = 0; i < 3; ++i) load_tile(t_begin + i, i);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int i = 0; i < 3; ++i) scrub_tail(t_begin + i, i);
    __syncthreads();

    // one pipelined iteration on tile t in slot S (a compile-time value: every LDS address of
    // the body is then a per-lane register plus an instruction offset)
    f32x16 sa[kRB], sb[kRB];
    bf16x8 pf[kRB][2];
    auto pipelined_tile = [&](int t, auto slot_tag) __attribute__((always_inline)) {
        constexpr int S = decltype(slot_tag)::value;
        const std::integral_constant<int, S> here{};
        const std::integral_constant<int, (S + 1) & 3> next{};
        const int64_t page_off = plan_load(t + 3);
        region_scores_weights([&](int i) { return k_operand_in(here, 1, i); }, sb, sa, pf,
                              [&](int i) { va[i] = v_operand_in(here, 0, i); });
        region_accumulate_maxima([&](int i) { return v_operand_in(here, 0, i); }, pf, sa, sb, true,
                                 [&](int i) { if (i < 4) load_step(page_off, (S + 3) & 3, i); },
                                 [&](int i) { ka[i] = k_operand_in(next, 0, i); });
        region_scores_weights([&](int i) { return k_operand_in(next, 0, i); }, sa, sb, pf,
                              [&](int i) { va[i] = v_operand_in(here, 1, i); });
        // the next tile's first region reads K of tile t + 1, block 1 (in LDS since the last barrier)
        region_accumulate_maxima([&](int i) { return v_operand_in(here, 1, i); }, pf, sb, sa, t + 1 < n_unmasked,
                                 [&](int) {}, [&](int i) { ka[i] = k_operand_in(next, 1, i); });
        finish_tile(t + 2, (S + 2) & 3);
    };

    int t = t_begin;
    if constexpr (SHARED) {
        // ---- decode side.  A private chunk (two waves at work) is bound by memory latency over
        // the tiles in flight: plain body, three tiles in flight.  A chunk that several programs
        // share keeps up to eight waves busy and is bound by their arithmetic: the same two
        // regions as append-prefill, one block per tile and wave, looking one tile ahead for
        // the scores (so two tiles in flight).  All waves of the workgroup follow the item's
        // cadence of waits, whether they have rows or not. ----
        const int pipe_end = members >= 2 ? t_begin + ((n_tiles - t_begin) & ~3) : t_begin;
        auto pipelined_half_tile = [&](int tt, auto slot_tag, f32x16 (&s_cur)[kRB], f32x16 (&s_nxt)[kRB])
                                       __attribute__((always_inline)) {
            constexpr int S = decltype(slot_tag)::value;
            const std::integral_constant<int, S> here{};
            const std::integral_constant<int, (S + 1) & 3> next{};
            const int64_t page_off = plan_load(tt + 3);
            // tile tt + 1 has landed with the barrier just passed: its first operands cannot be
            // asked for any earlier
#pragma unroll
            for (int i = 0; i < kKAhead; ++i) ka[i] = k_operand_in(next, 0, i);
            region_scores_weights([&](int i) { return k_operand_in(next, 0, i); }, s_nxt, s_cur, pf,
                                  [&](int i) { va[i] = v_operand_in(here, 0, i); });
            region_accumulate_maxima([&](int i) { return v_operand_in(here, 0, i); }, pf, s_cur, s_nxt, tt + 1 < n_tiles,
                                     [&](int i) { if (i < 4) load_step(page_off, (S + 3) & 3, i); }, [&](int) {});
            finish_tile(tt + 2, (S + 2) & 3);
        };
        if (!wave_active) {
            for (; t < n_tiles; ++t) {
                const int s = (t - t_begin) & 3;
                load_tile(t + 3, (s + 3) & 3);
                if (t < pipe_end) finish_tile(t + 2, (s + 2) & 3);
                else finish_tile_early(t + 1, (s + 1) & 3);
            }
        } else {
            if (pipe_end > t_begin) {
                scores(slot_ptr(0), 0, sa);          // the read offsets already point at this wave's block
                raise_reference(sa);
                for (; t < pipe_end; t += 4) {
                    pipelined_half_tile(t, std::integral_constant<int, 0>{}, sa, sb);
                    pipelined_half_tile(t + 1, std::integral_constant<int, 1>{}, sb, sa);
                    pipelined_half_tile(t + 2, std::integral_constant<int, 2>{}, sa, sb);
                    pipelined_half_tile(t + 3, std::integral_constant<int, 3>{}, sb, sa);
                }
            }
            int slot = 0;                            // the pipelined trips are whole turns of the ring
            for (; t < n_tiles; ++t) {
                load_tile(t + 3, (slot + 3) & 3);
                const char* kt = slot_ptr(slot);
                f32x16 s[kRB];
                scores(kt, 0, s);
                if (t >= n_unmasked) mask_scores(t * kTileKeys + kb_mine * 32, s);
                raise_reference(s);
                weights(s, pf);
                accumulate(kt + kTileBytes, 0, pf);
                finish_tile_early(t + 1, (slot + 1) & 3);
                slot = (slot + 1) & 3;
            }
        }
    } else {
        // ---- pipelined body, four tiles per trip: the tiles whose successor is also unmasked ----
        const int pipe_end = t_begin + ((n_unmasked - 1 - t_begin) & ~3);
        if (!wave_active) {
            // nothing to compute: keep the workgroup's loads and barriers going
            for (; t < n_tiles; ++t) {
                const int s = (t - t_begin) & 3;
                load_tile(t + 3, (s + 3) & 3);
                finish_tile(t + 2, (s + 2) & 3);
            }
        } else if (pipe_end > t_begin) {
            scores(slot_ptr(0), 0, sa);
            raise_reference(sa);
#pragma unroll
            for (int i = 0; i < kKAhead; ++i) ka[i] = k_operand_at(slot_ptr(0), 1, i);
            for (; t < pipe_end; t += 4) {
                pipelined_tile(t, std::integral_constant<int, 0>{});
                pipelined_tile(t + 1, std::integral_constant<int, 1>{});
                pipelined_tile(t + 2, std::integral_constant<int, 2>{});
                pipelined_tile(t + 3, std::integral_constant<int, 3>{});
            }
            // sa holds the first block of tile t, which the plain body below computes again
        }
        // ---- plain body: the last unmasked tiles and the tiles that straddle the diagonal ----
        int slot = 0;                                // (t - t_begin) % 4: the pipelined trips are whole turns
        for (; t < n_tiles; ++t) {
            load_tile(t + 3, (slot + 3) & 3);
            const char* kt = slot_ptr(slot);
            const char* vt = kt + kTileBytes;
            const bool masked = t >= n_unmasked;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                f32x16 s[kRB];
                scores(kt, kb, s);
                if (masked) mask_scores(t * kTileKeys + kb * 32, s);
                raise_reference(s);
                weights(s, pf);
                accumulate(vt, kb, pf);
            }
            finish_tile(t + 2, (slot + 2) & 3);
            slot = (slot + 1) & 3;
        }
    }

    if constexpr (SHARED) {
        // The two waves of a row block hold results over disjoint keys of the same rows, lane for
        // lane: wave 2 j + 1 hands its (m, l, O) to wave 2 j through the ring, which is idle now
        // (every load has landed, every operand read is done), laid out [value][lane].
        static_assert(kRB == 1, "one row block per wave");
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        float* xch = reinterpret_cast<float*>(lds) + row_block * (66 * 64) + lane;
        if (wave_active && kb_mine == 1) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) xch[(db * 16 + r) * 64] = o[db][0][r];
            xch[64 * 64] = m[0];
            xch[65 * 64] = lsum[0];
        }
        __syncthreads();
        if (wave_active && kb_mine == 0) {
            const float m_other = xch[64 * 64];
            const float m_new = fmaxf(m[0], m_other);
            const float mine = __builtin_amdgcn_exp2f(m[0] - m_new);
            const float other = __builtin_amdgcn_exp2f(m_other - m_new);
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][0][r] = o[db][0][r] * mine + xch[(db * 16 + r) * 64] * other;
            lsum[0] = lsum[0] * mine + xch[65 * 64] * other;
            m[0] = m_new;
        }
    }

    // ---- epilogue ----
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
        const float total = lsum[rb] + __shfl_xor(lsum[rb], 32);
        if (out_row[rb] < 0) continue;
        if (SHARED && kb_mine == 1) continue;      // its partner writes the merged result
        if (SHARED) {
            // split-K partial of (member program, head) for this chunk: unnormalised O, the
            // reference maximum it is relative to, and the sum of weights
            const int row = row_block * (32 * kRB) + rb * 32 + l32;
            const int head = g * G + row % G;
            const int program = static_cast<int>(out_row[rb] / (int64_t(p.num_q_heads) * kHeadDim));
            const int64_t rowid = int64_t(p.chunk_start[program] + chunk) * p.num_q_heads + head;
            float* orow = p.part_o + rowid * kHeadDim;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int dim = db * 32 + 8 * q4 + 4 * hl;
                    *reinterpret_cast<float4*>(orow + dim) = make_float4(o[db][rb][4 * q4], o[db][rb][4 * q4 + 1],
                                                                           o[db][rb][4 * q4 + 2], o[db][rb][4 * q4 + 3]);
                }
            if (hl == 0) {
                p.part_ml[rowid * 2 + 0] = m[rb];
                p.part_ml[rowid * 2 + 1] = total;
            }
        } else if (split > 1) {
            // the partial of this row over this chunk of keys (a row that sees none of them: an empty one)
            const int64_t rowid = (out_row[rb] / kHeadDim) * split + part;
            float* orow = p.part_o + rowid * kHeadDim;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int dim = db * 32 + 8 * q4 + 4 * hl;
                    *reinterpret_cast<float4*>(orow + dim) = make_float4(o[db][rb][4 * q4], o[db][rb][4 * q4 + 1],
                                                                           o[db][rb][4 * q4 + 2], o[db][rb][4 * q4 + 3]);
                }
            if (hl == 0) {
                p.part_ml[rowid * 2 + 0] = m[rb];
                p.part_ml[rowid * 2 + 1] = total;
            }
        } else {
            const float inv = total > 0.0f ? p.out_scale / total : 0.0f;
            uint16_t* orow = p.out + out_row[rb];
#pragma unroll
            for (int db = 0; db < 4; ++db) {
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    // registers 4 q4 .. 4 q4 + 3 are dims db 32 + 8 q4 + 4 hl + 0..3
                    const int dim = db * 32 + 8 * q4 + 4 * hl;
                    u32x2 w;
                    w.x = uint32_t(to_bf16_rne(o[db][rb][4 * q4 + 0] * inv)) |
                          (uint32_t(to_bf16_rne(o[db][rb][4 * q4 + 1] * inv)) << 16);
                    w.y = uint32_t(to_bf16_rne(o[db][rb][4 * q4 + 2] * inv)) |
                          (uint32_t(to_bf16_rne(o[db][rb][4 * q4 + 3] * inv)) << 16);
                    *reinterpret_cast<u32x2*>(orow + dim) = w;
                }
            }
            if (p.lse != nullptr && hl == 0)
                p.lse[out_row[rb] / kHeadDim] =
                    total > 0.0f ? (m[rb] + __builtin_amdgcn_logf(total)) * kLn2 : -INFINITY;
        }
    }
    // the next item reuses the LDS ring: no load may still be on its way into it
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    blk = SHARED ? take_pair() : blk + int(gridDim.x);
    }
}

// Append-prefill with the keys cut into chunks: one wave per output row adds up the row's partials
// (those of the chunks that its query tile reaches: the others were never written).
__global__ __launch_bounds__(256) void prefill_merge_kernel(PrefillParams p, int32_t total_q, int32_t tile_tokens) {
    const int lane = threadIdx.x & 63;
    const int64_t rid = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (rid >= int64_t(total_q) * p.num_q_heads) return;
    const int token = static_cast<int>(rid / p.num_q_heads);
    // the program of the token: the last b with cu_q_lens[b] <= token
    int lo = 0, hi = p.batch;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (p.cu_q_lens[mid] <= token) lo = mid; else hi = mid;
    }
    const int b = lo;
    const int q0 = p.cu_q_lens[b], nq = p.cu_q_lens[b + 1] - q0;
    const int prefix = p.context_lens[b] - nq;
    const int tile = (token - q0) / tile_tokens;
    int t_end = (tile + 1) * tile_tokens;
    t_end = t_end > nq ? nq : t_end;
    const int n_tiles = (prefix + t_end + kTileKeys - 1) / kTileKeys;
    const int n_chunks = (n_tiles + p.chunk_tiles - 1) / p.chunk_tiles;      // 1 .. split

    const float* ml = p.part_ml + rid * p.split * 2;
    const float* po = p.part_o + rid * p.split * kHeadDim;
    float mt = kNegBig;
    for (int c = lane; c < n_chunks; c += 64) mt = fmaxf(mt, ml[c * 2]);
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) mt = fmaxf(mt, __shfl_xor(mt, s));
    float lt = 0.0f, o0 = 0.0f, o1 = 0.0f;
#pragma unroll 4
    for (int c = 0; c < n_chunks; ++c) {
        const float wt = __builtin_amdgcn_exp2f(ml[c * 2] - mt);
        lt = fmaf(ml[c * 2 + 1], wt, lt);
        const float2 v = *reinterpret_cast<const float2*>(po + c * kHeadDim + 2 * lane);
        o0 = fmaf(v.x, wt, o0);
        o1 = fmaf(v.y, wt, o1);
    }
    const float inv = lt > 0.0f ? p.out_scale / lt : 0.0f;
    reinterpret_cast<uint32_t*>(p.out + rid * kHeadDim)[lane] =
        uint32_t(to_bf16_rne(o0 * inv)) | (uint32_t(to_bf16_rne(o1 * inv)) << 16);
    if (p.lse != nullptr && lane == 0)
        p.lse[rid] = lt > 0.0f ? (mt + __builtin_amdgcn_logf(lt)) * kLn2 : -INFINITY;
}

// 128 KiB of dynamic LDS is above the default 64 KiB limit: raised once per kernel instance and
// device (the attribute belongs to the device's copy of the kernel).
template <int G, bool SHARED>
int launch_instance(unsigned blocks, const PrefillParams& pp, hipStream_t stream) {
    const size_t lds_bytes = kRing * kSlotBytes;
    constexpr int kMaxDevices = 64;
    static std::atomic<bool> raised[kMaxDevices];
    int device = 0;
    TA_HIP_TRY(hipGetDevice(&device));
    if (device < 0 || device >= kMaxDevices) return TA_ERR_UNSUPPORTED;
    if (!raised[device].load(std::memory_order_acquire)) {
        TA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_tile_kernel<G, SHARED>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(lds_bytes)));
        raised[device].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((attention_tile_kernel<G, SHARED>), dim3(blocks), dim3(kThreads), lds_bytes, stream, pp);
    TA_HIP_TRY(hipGetLastError());
    return TA_OK;
}

template <bool SHARED>
int launch_tile_kernel(int group, unsigned blocks, const PrefillParams& pp, hipStream_t stream) {
    switch (group) {
        case 1: return launch_instance<1, SHARED>(blocks, pp, stream);
        case 2: return launch_instance<2, SHARED>(blocks, pp, stream);
        case 4: return launch_instance<4, SHARED>(blocks, pp, stream);
        case 8: return launch_instance<8, SHARED>(blocks, pp, stream);
        default: return TA_ERR_UNSUPPORTED;
    }
}

}  // namespace

int launch_prefill(const Geometry& g, const PrefillArgs& a, const WorkspaceLayout& w, char* workspace,
                   hipStream_t stream) {
    int32_t* tile_start = reinterpret_cast<int32_t*>(workspace + w.off_tile_start);
    int2* tiles = reinterpret_cast<int2*>(workspace + w.off_tiles);
    const int tile_tokens = kRowsPerBlock / g.group;
    const int32_t per_prog = (a.max_q_len + tile_tokens - 1) / tile_tokens;
    const int64_t max_tiles = int64_t(per_prog) * a.batch;
    if (max_tiles > w.max_tiles) return TA_ERR_INVALID_ARG;

    // (with the keys cut into chunks and up to 64 programs the tile kernel works the list out itself)
    const bool plan_in_tile_kernel = w.prefill_split > 1 && a.batch <= 64;
    if (!plan_in_tile_kernel) {
        // one workgroup, as small as the batch allows (its sort and scan are all barriers)
        unsigned plan_threads = 64;
        while (plan_threads < 1024 && plan_threads < static_cast<unsigned>(a.batch)) plan_threads <<= 1;
        hipLaunchKernelGGL(plan_tiles_kernel, dim3(1), dim3(plan_threads), 0, stream, a.cu_q_lens, a.context_lens,
                           a.batch, tile_tokens, per_prog, tile_start, tiles);
        TA_HIP_TRY(hipGetLastError());
    }

    PrefillParams pp{};
    pp.q = a.q;
    pp.k_pool = reinterpret_cast<const char*>(a.k_pool);
    pp.v_pool = reinterpret_cast<const char*>(a.v_pool);
    pp.block_table = a.block_table;
    pp.stride_page_bytes = g.stride_page_bytes;
    pp.stride_head_bytes = g.stride_head_bytes;
    pp.block_table_stride = a.block_table_stride;
    pp.scale_log2 = g.scale_log2;
    pp.out_scale = 1.0f;
    if (g.kv_fp8) {
        // an FP8 cache: the kernel reads the batch's pages from a widened copy (code values in bf16)
        char* wide_k = workspace + w.off_wide_k;
        char* wide_v = workspace + w.off_wide_v;
        int32_t* wide_table = reinterpret_cast<int32_t*>(workspace + w.off_wide_table);
        const int rc = launch_widen_pages(g, a.k_pool, a.v_pool, a.block_table, a.block_table_stride, a.context_lens,
                                          a.batch, w.wide_width, wide_k, wide_v, wide_table, stream);
        if (rc != TA_OK) return rc;
        pp.k_pool = wide_k;
        pp.v_pool = wide_v;
        pp.block_table = wide_table;
        pp.block_table_stride = w.wide_width;
        pp.stride_head_bytes = int64_t(kPageSize) * kHeadDim * 2;
        pp.stride_page_bytes = pp.stride_head_bytes * g.num_kv_heads;
        pp.scale_log2 = g.scale_log2 * g.k_scale;
        pp.out_scale = g.v_scale;
    }
    pp.context_lens = a.context_lens;
    pp.cu_q_lens = a.cu_q_lens;
    pp.tile_start = tile_start;
    pp.tiles = plan_in_tile_kernel ? nullptr : tiles;
    pp.tiles_per_program_max = per_prog;
    pp.out = a.out;
    pp.lse = a.lse;
    pp.batch = a.batch;
    pp.num_q_heads = g.num_q_heads;
    pp.num_kv_heads = g.num_kv_heads;

    pp.split = w.prefill_split;
    pp.chunk_tiles = w.prefill_chunk_tiles;
    if (pp.split > 1) {
        pp.part_ml = reinterpret_cast<float*>(workspace + w.off_part_ml);
        pp.part_o = reinterpret_cast<float*>(workspace + w.off_part_o);
    }

    const int64_t blocks = pp.split > 1 ? (int64_t(g.num_kv_heads) * pp.split + 7) / 8 * 8 * max_tiles
                                        : max_tiles * g.num_kv_heads;
    if (blocks > 0x7fffffff) return TA_ERR_INVALID_ARG;
    const ProfileEvents ev = profile_events();
    if (ev.start != nullptr) TA_HIP_TRY(hipEventRecord(ev.start, stream));
    const int rc = launch_tile_kernel<false>(g.group, static_cast<unsigned>(blocks), pp, stream);
    if (rc != TA_OK) return rc;
    if (ev.stop != nullptr) TA_HIP_TRY(hipEventRecord(ev.stop, stream));
    if (pp.split > 1) {
        const int64_t rows = int64_t(a.total_q) * g.num_q_heads;
        hipLaunchKernelGGL(prefill_merge_kernel, dim3(static_cast<unsigned>((rows + 3) / 4)), dim3(256), 0, stream, pp,
                           a.total_q, tile_tokens);
        TA_HIP_TRY(hipGetLastError());
    }
    return TA_OK;
}

int launch_shared_prefix(const Geometry& g, const SharedPrefixArgs& a, hipStream_t stream) {
    PrefillParams pp{};
    pp.q = a.q;
    pp.k_pool = reinterpret_cast<const char*>(a.k_pool);
    pp.v_pool = reinterpret_cast<const char*>(a.v_pool);
    pp.block_table = a.block_table;
    pp.context_lens = a.context_lens;
    pp.shared_items = reinterpret_cast<const int4*>(a.shared_items);
    pp.order = a.order;
    pp.counts = a.counts;
    pp.chunk_start = a.chunk_start;
    pp.part_ml = a.part_ml;
    pp.part_o = a.part_o;
    pp.stride_page_bytes = g.stride_page_bytes;
    pp.stride_head_bytes = g.stride_head_bytes;
    pp.block_table_stride = a.block_table_stride;
    pp.batch = a.batch;
    pp.num_q_heads = g.num_q_heads;
    pp.num_kv_heads = g.num_kv_heads;
    pp.scale_log2 = g.scale_log2;
    pp.out_scale = 1.0f;
    int64_t blocks = int64_t(a.max_items) * g.num_kv_heads;
    if (blocks <= 0) return TA_OK;
    // One workgroup fits per CU and they take items from a counter.  Twice the CU count keeps the
    // tail of a launch busy when every chunk of the batch runs here; when only shared chunks can
    // (usually none at all), one workgroup per CU is enough and an empty launch is over sooner.
    const int64_t cap = a.private_on_tiles ? 512 : 256;
    if (blocks > cap) blocks = cap;
    return launch_tile_kernel<true>(g.group, static_cast<unsigned>(blocks), pp, stream);
}

}  // namespace ta
