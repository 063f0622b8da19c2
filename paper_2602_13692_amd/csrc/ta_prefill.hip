// Append-prefill attention for gfx950: the n new tokens of a program attend
// causally to the retained prefix plus themselves (ThunderAgent Sec. 4.2, the
// incremental-prefill term of Eq. 3; Sec. 2.1, c_{t+1} extends c_t).
//
// Here q.K^T and p.V are dense contractions, so both run on the matrix cores
// (v_mfma_f32_32x32x16_bf16).  One workgroup of four waves owns 256 score rows
// = (256 / G) consecutive new tokens x the G query heads that share a kv head,
// and walks the program's keys in tiles of 64 (four pages):
//
//   * K and V tiles go HBM -> registers -> LDS once per workgroup, through a
//     ring of three tiles with one barrier per tile, and serve all 256 rows;
//   * every wave owns 64 rows and computes the TRANSPOSED scores S^T = K Q^T,
//     so that each lane holds one query row's scores in its accumulator
//     registers: the softmax needs one cross-lane exchange per tile, and the
//     exponentiated scores are already laid out as the B operand of
//     O^T = V^T P^T;
//   * V is written to LDS as [8-key octet][dim][8 keys] (an in-register
//     transpose at staging time), which makes the A operand of O^T = V^T P^T
//     one 16-byte LDS read per lane; LDS moves a fixed 64 bytes per cycle and CU
//     for 16-byte accesses and half that for 8-byte ones, and this kernel is
//     bound by exactly that, so every operand is read 16 bytes wide;
//   * the running maximum is only raised (and O rescaled) when it grows by more
//     than 2^8, a wave-uniform and rare event after the first tile.
#include "ta_internal.h"

namespace ta {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kThreads = 256;
constexpr int kRowsPerBlock = 256;  // score rows per workgroup
constexpr int kTileKeys = 64;       // keys per LDS tile (4 pages)
constexpr int kKTileBytes = kTileKeys * kHeadDim * 2;  // 16 KiB
constexpr int kVTileBytes = kTileKeys * kHeadDim * 2;  // 16 KiB
constexpr float kRescaleThreshold = 8.0f;  // log2 units
constexpr int kRing = 3;                   // LDS tiles in flight
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
    // shared-prefix decode only: one item = (first program of the group, members, chunk)
    const int4* shared_items;
    const int32_t* counts;       // counts[1] = number of shared items
    const int32_t* chunk_start;  // [batch + 1] first partial slot of each program
    float* part_ml;              // [slot][Hq][2]  reference maximum (log2 domain), sum
    float* part_o;               // [slot][Hq][128] unnormalised output
    int32_t tiles_per_chunk;
    int64_t stride_page_bytes;
    int64_t stride_head_bytes;
    int32_t block_table_stride;
    int32_t batch;
    int32_t num_q_heads;
    int32_t num_kv_heads;
    float scale_log2;
};

// plan: query tiles of tile_tokens tokens per program, listed flat
__global__ __launch_bounds__(1024) void plan_tiles_kernel(const int32_t* __restrict__ cu_q_lens,
                                                          int32_t batch, int32_t tile_tokens,
                                                          int32_t max_per_program,
                                                          int32_t* __restrict__ tile_start,
                                                          int2* __restrict__ tiles) {
    __shared__ int32_t scan[1024];
    __shared__ int32_t carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < batch; base += 1024) {
        const int b = base + tid;
        int n = 0;
        if (b < batch) {
            const int nq = cu_q_lens[b + 1] - cu_q_lens[b];
            n = nq > 0 ? (nq + tile_tokens - 1) / tile_tokens : 0;
            n = n > max_per_program ? max_per_program : n;
        }
        scan[tid] = n;
        __syncthreads();
        for (int off = 1; off < 1024; off <<= 1) {
            const int v = tid >= off ? scan[tid - off] : 0;
            __syncthreads();
            scan[tid] += v;
            __syncthreads();
        }
        const int first = carry + scan[tid] - n;
        if (b < batch) {
            tile_start[b] = first;
            for (int c = 0; c < n; ++c) tiles[first + c] = make_int2(b, c);
        }
        __syncthreads();
        if (tid == 1023) carry += scan[1023];
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

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b),
                                           acc, false);
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

// Staging registers of one thread for one 64-key tile: four 16-byte pieces of K
// (keys r16 + 16 i, chunk c16) and eight 8-byte pieces of V (the eight keys of one
// "octet", 4 dims).
struct Stage {
    u32x4 k[4];
    u32x2 v[8];
};

// V lives in LDS as [octet][dim][8 keys]: one 16-byte entry is exactly the A operand of one
// lane for O^T += V^T P^T.  Octet (kb, step, hl) of a 64-key tile holds the keys that lane half
// hl contracts in k = 16 step `step` of 32-key block kb: kb 32 + step 16 + hl 4 + {0..3, 8..11}.
// Byte offset of the entry of `dim` inside its octet (the 16-byte entries of a 64-byte run of
// four dims are XOR-swizzled so that the staging writes are bank-conflict free):
__device__ __forceinline__ int v_entry_offset(int dim) {
    const int chunk = dim >> 2;
    return chunk * 64 + (((dim & 3) ^ ((chunk >> 2) & 3)) << 4);
}

// SHARED = false: append-prefill, rows = (new token, head), causal, writes bf16 output.
// SHARED = true:  decode of a group of programs whose block tables begin with the same pages
//                 (forked agent branches): rows = (member program, head), keys = one chunk of
//                 the shared prefix, no mask, writes split-K partials for the decode merge.
template <int G, bool SHARED>
__global__ __launch_bounds__(kThreads, 1) void attention_tile_kernel(PrefillParams p) {
    constexpr int kTileTokens = kRowsPerBlock / G;   // programs per item when SHARED
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* k_lds = lds;                           // [kRing][kKTileBytes]
    char* v_lds = lds + kRing * kKTileBytes;     // [kRing][kVTileBytes]

    // Workgroups stride over the (item, kv head) pairs: append-prefill is launched with one
    // workgroup per pair, the shared-prefix decode with a small resident grid (its item count is
    // only known on the device and is usually zero).
    const int n_items = SHARED ? p.counts[1] : p.tile_start[p.batch];
    for (int blk = blockIdx.x; blk < n_items * p.num_kv_heads; blk += gridDim.x) {
    const int tile_id = blk / p.num_kv_heads;
    const int g = blk - tile_id * p.num_kv_heads;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hl = lane >> 5;                // which half of the wave
    const int l32 = lane & 31;

    int b, q0, nq, L, prefix, t0, t_begin, n_tiles, n_unmasked, members = 0, chunk = 0;
    if (SHARED) {
        const int4 it = p.shared_items[tile_id];
        b = it.x;                      // the group's first program: its block table names the pages
        members = it.y;
        chunk = it.z;
        q0 = 0; nq = 0; prefix = 0; t0 = 0;
        L = 0x7fffffff;                // every key of a shared chunk exists
        t_begin = chunk * p.tiles_per_chunk;
        n_tiles = t_begin + p.tiles_per_chunk;
        n_unmasked = n_tiles;
    } else {
        const int2 tl = p.tiles[tile_id];
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
    }
    const int n_pages_b = (p.context_lens[b] + kPageSize - 1) / kPageSize;

    // ---- per-lane rows: two blocks of 32 rows per wave ----
    // row -> (token or member program, head): row = index * G + head
    int vis[2];            // visible keys of this lane's row in row block rb (0 = row does not exist)
    bf16x8 qf[2][8];       // B operands: q[row][16 ks + 8 hl .. + 7]
    int64_t out_row[2];    // element offset of the row in q / out, or -1
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int row = wave * 64 + rb * 32 + l32;
        const int idx = t0 + row / G;
        const int head = g * G + row % G;
        const bool ok = SHARED ? (row / G < members) : (idx < nq);
        vis[rb] = ok ? prefix + idx + 1 : 0;
        out_row[rb] = ok ? (int64_t(SHARED ? b + row / G : q0 + idx) * p.num_q_heads + head) * kHeadDim : int64_t(-1);
        const uint16_t* qrow = p.q + (ok ? out_row[rb] : 0) + hl * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            u32x4 t = {0u, 0u, 0u, 0u};
            if (ok) t = *reinterpret_cast<const u32x4*>(qrow + ks * 16);
            // Q is only ever a matrix-instruction operand: parking it in accumulation registers
            // leaves the vector registers to the softmax and the operand prefetch
            asm volatile("" : "+a"(t));
            qf[rb][ks] = __builtin_bit_cast(bf16x8, t);
        }
    }

    // ---- staging addresses ----
    const int c16 = tid & 15;   // 16-byte chunk of a 256-byte row
    const int r16 = tid >> 4;   // 0..15
    const char* k_base = p.k_pool + int64_t(g) * p.stride_head_bytes + r16 * 256 + c16 * 16;
    // V: thread -> (octet oc = tid / 32, 8-byte chunk c32 of 4 dims); the octet's keys all lie in
    // page oc / 2 = wave of the tile, rows 4 hl + {0..3} and 8 + 4 hl + {0..3}
    const int c32 = tid & 31;
    const int oc = tid >> 5;
    const char* v_base = p.v_pool + int64_t(g) * p.stride_head_bytes + ((oc & 1) * 4) * 256 + c32 * 8;
    const int v_key0 = (oc >> 1) * 16 + (oc & 1) * 4;                // first key of the octet in the tile
    const int32_t* table = p.block_table + int64_t(b) * p.block_table_stride;
    const int k_lds_off = r16 * 256 + ((c16 ^ r16) << 4);           // + i * 4096 for key r16 + 16 i
    const int v_lds_off = oc * 2048 + c32 * 64;                     // entries at ((e ^ (c32 >> 2)) << 4)

    // Page ids: lane l of every wave holds the id of page (64 g + l) of the current group of 64
    // pages (16 tiles), clamped to the program's last page; the next group is fetched one
    // group ahead, so no tile waits for a dependent id load.
    auto fetch_ids = [&](int group) -> int {
        int pg = group * 64 + lane;
        pg = pg < n_pages_b ? pg : n_pages_b - 1;
        return table[pg];
    };
    int ids_group = t_begin >> 4;
    int ids_cur = fetch_ids(ids_group);
    int ids_next = fetch_ids(ids_group + 1);

    // Loading one tile = planning (page ids -> byte offsets, scalar) + 8 loads of 16 bytes;
    // storing it to LDS = 4 K writes + 4 V pieces (mask, 4x8 transpose, write).  Both are cut
    // into eight steps so that the pipelined body can spread them over its slices.
    struct LoadPlan {
        int64_t k_off[4];
        int64_t v_off;
    };
    auto plan_load = [&](int t) -> LoadPlan {
        if ((t >> 4) != ids_group) {      // tiles are visited in order, so this is group + 1
            ids_group = t >> 4;
            ids_cur = ids_next;
            ids_next = fetch_ids(ids_group + 1);
        }
        LoadPlan lp;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            lp.k_off[i] = int64_t(__builtin_amdgcn_readlane(ids_cur, (t & 15) * 4 + i)) * p.stride_page_bytes;
        // V: this thread's octet lies in page `wave` of the tile
        lp.v_off = int64_t(__builtin_amdgcn_readlane(ids_cur, (t & 15) * 4 + wave)) * p.stride_page_bytes;
        return lp;
    };
    auto load_step = [&](Stage& st, const LoadPlan& lp, int i) {
        if (i < 4) {
            st.k[i] = *reinterpret_cast<const u32x4*>(k_base + lp.k_off[i]);
        } else {   // octet rows 2 (i - 4) and 2 (i - 4) + 1; rows 4..7 sit 8 keys further
            const int j = 2 * (i - 4);
            const int row = (j & 3) + (j >> 2) * 8;
            st.v[j] = *reinterpret_cast<const u32x2*>(v_base + lp.v_off + row * 256);
            st.v[j + 1] = *reinterpret_cast<const u32x2*>(v_base + lp.v_off + (row + 1) * 256);
        }
    };
    auto load_tile = [&](Stage& st, int t) {
        const LoadPlan lp = plan_load(t);
#pragma unroll
        for (int i = 0; i < 8; ++i) load_step(st, lp, i);
    };
    auto store_step = [&](const Stage& st, int t, int slot, int i) {
        if (i < 4) {
            *reinterpret_cast<u32x4*>(k_lds + slot * kKTileBytes + k_lds_off + i * 4096) = st.k[i];
        } else {
            // entry e = the octet's eight keys at dim 4 c32 + e: an 8x1 column of the 8x4 block
            // this thread loaded.  Keys at or beyond the context length may hold anything (even
            // NaN): their V rows are zeroed, because 0 * NaN inside the matrix core would poison O.
            const int e = i - 4;
            uint32_t a[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int key = t * kTileKeys + v_key0 + (j & 3) + (j >> 2) * 8;
                a[j] = key < L ? st.v[j][e >> 1] : 0u;
            }
            const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;   // high or low halves
            u32x4 entry;
            entry.x = __builtin_amdgcn_perm(a[1], a[0], sel);
            entry.y = __builtin_amdgcn_perm(a[3], a[2], sel);
            entry.z = __builtin_amdgcn_perm(a[5], a[4], sel);
            entry.w = __builtin_amdgcn_perm(a[7], a[6], sel);
            *reinterpret_cast<u32x4*>(v_lds + slot * kVTileBytes + v_lds_off + ((e ^ ((c32 >> 2) & 3)) << 4)) = entry;
        }
    };
    auto store_tile = [&](const Stage& st, int t, int slot) {
#pragma unroll
        for (int i = 0; i < 8; ++i) store_step(st, t, slot, i);
    };

    // ---- accumulators ----
    f32x16 o[4][2];        // O^T blocks: [dim block][row block]
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][rb][r] = 0.0f;
    float m[2] = {kNegBig, kNegBig};   // reference maximum (log2 domain, scaled)
    float lsum[2] = {0.0f, 0.0f};      // this lane's share of the row sum

    // LDS read offsets
    int k_rd[2];   // K operand: key l32 + 32 kb, chunk (2 ks + hl) ^ (key & 15)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) k_rd[kb] = (kb * 32 + l32) * 256;
    const int k_swz = l32 & 15;
    int v_rd[4];   // V operand: entry of dim l32 + 32 db in octet (.., hl)
#pragma unroll
    for (int db = 0; db < 4; ++db) v_rd[db] = hl * 2048 + v_entry_offset(db * 32 + l32);

    // ---- the four steps of one 32-key block ----
    // A: S^T block = K Q^T, 32 keys x (2 x 32 rows); register r of lane (l32, hl) holds
    //    key 8 (r / 4) + 4 hl + r % 4 of the block
    auto scores = [&](const char* kt, int kb, f32x16 (&s)[2]) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[rb][r] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(kt + k_rd[kb] + (((2 * ks + hl) ^ k_swz) << 4));
            s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0][ks], s[0], 0, 0, 0);
            s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[1][ks], s[1], 0, 0, 0);
        }
    };
    // causal mask of a block that straddles the diagonal
    auto mask_scores = [&](int key_base, f32x16 (&s)[2]) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key_base + 4 * hl + 8 * (r >> 2) + (r & 3);
                s[rb][r] = key < vis[rb] ? s[rb][r] : -INFINITY;
            }
    };
    // B1: row maxima; the reference is raised (and O, l rescaled) only when it would grow
    //     by more than the threshold, a wave-uniform and rare event
    // The hand-written matrix instructions are invisible to the compiler's hazard checks:
    // before anything else reads O, let the matrix core finish (32 wait states cover the
    // 16-pass write-back latency).
    auto mfma_drain = [&]() { asm volatile("s_nop 15\n\ts_nop 15"); };
    auto rescale_if_needed = [&](const float (&cand)[2]) {
        const bool grow = cand[0] > m[0] + kRescaleThreshold || cand[1] > m[1] + kRescaleThreshold;
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(grow) != 0, 0)) {
            mfma_drain();
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                const float m_new = fmaxf(m[rb], cand[rb]);
                const float alpha = __builtin_amdgcn_exp2f(m[rb] - m_new);
                m[rb] = m_new;
                lsum[rb] *= alpha;
                // O lives in the accumulation registers the matrix core writes; scaling it there
                // (read, multiply, write back) keeps this rare path from forcing copies of O
                // into vector registers on the common path
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float x = o[db][rb][r];
                        float tmp;
                        asm volatile(
                            "v_accvgpr_read_b32 %1, %0\n\t"
                            "s_nop 1\n\t"
                            "v_mul_f32 %1, %1, %2\n\t"
                            "s_nop 1\n\t"
                            "v_accvgpr_write_b32 %0, %1"
                            : "+a"(x), "=&v"(tmp)
                            : "v"(alpha));
                        o[db][rb][r] = x;
                    }
            }
        }
    };
    auto raise_reference = [&](const f32x16 (&s)[2]) {
        float cand[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
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
    auto weights = [&](const f32x16 (&s)[2], bf16x8 (&pf)[2][2]) {
        const uint32_t ones = 0x3f803f80u;   // (1.0, 1.0) in bf16
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const float bias = -m[rb];
            float pr[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) pr[r] = __builtin_amdgcn_exp2f(fmaf(s[rb][r], p.scale_log2, bias));
            // the row sum adds up the ROUNDED weights (the ones the matrix core multiplies),
            // two per instruction
            float acc = lsum[rb];
#pragma unroll
            for (int step = 0; step < 2; ++step) {
                u32x4 w;
                w.x = pack_bf16(pr[8 * step + 0], pr[8 * step + 1]);
                w.y = pack_bf16(pr[8 * step + 2], pr[8 * step + 3]);
                w.z = pack_bf16(pr[8 * step + 4], pr[8 * step + 5]);
                w.w = pack_bf16(pr[8 * step + 6], pr[8 * step + 7]);
                acc = dot2_bf16(w.x, ones, acc);
                acc = dot2_bf16(w.y, ones, acc);
                acc = dot2_bf16(w.z, ones, acc);
                acc = dot2_bf16(w.w, ones, acc);
                pf[rb][step] = __builtin_bit_cast(bf16x8, w);
            }
            lsum[rb] = acc;
        }
    };
    // C: O^T += V^T P^T; the A operand of (block kb, step, lane half hl) is octet 4 kb + 2 step + hl
    auto accumulate = [&](const char* vt, int kb, const bf16x8 (&pf)[2][2]) {
#pragma unroll
        for (int step = 0; step < 2; ++step) {
            const char* vq = vt + (kb * 4 + step * 2) * 2048;
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(vq + v_rd[db]);
                o[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[0][step], o[db][0], 0, 0, 0);
                o[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[1][step], o[db][1], 0, 0, 0);
            }
        }
    };

    // ---- the pipelined body's two regions, written slice by slice ----
    // With one wave per SIMD nothing hides latency except the order of this wave's own
    // instructions, so the order is written out: every slice issues two matrix instructions,
    // the LDS read of the operand needed two slices later, and a fixed share of the vector
    // work; a scheduling barrier closes the slice so the compiler keeps the interleaving.
    //
    // Region X: scores of the next block (matrix core) with the weights of the current block
    // (vector ALU).  Slice ks turns scores 2 ks and 2 ks + 1 of both row blocks into weights.
    auto region_scores_weights = [&](const char* kt, int kb, f32x16 (&s_new)[2],
                                     const f32x16 (&s_old)[2], bf16x8 (&pf)[2][2]) {
        const uint32_t ones = 0x3f803f80u;   // (1.0, 1.0) in bf16
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        bf16x8 a[8];
        uint32_t pw[2][8];
        float acc[2] = {lsum[0], lsum[1]};
        const float bias[2] = {-m[0], -m[1]};
        auto k_operand = [&](int ks) {
            return *reinterpret_cast<const bf16x8*>(kt + k_rd[kb] + (((2 * ks + hl) ^ k_swz) << 4));
        };
#pragma unroll
        for (int i = 0; i < kKAhead; ++i) a[i] = k_operand(i);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            s_new[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], qf[0][ks], ks == 0 ? zero : s_new[0], 0, 0, 0);
            s_new[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], qf[1][ks], ks == 0 ? zero : s_new[1], 0, 0, 0);
            if (ks + kKAhead < 8) a[ks + kKAhead] = k_operand(ks + kKAhead);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(s_old[rb][2 * ks], p.scale_log2, bias[rb]));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(s_old[rb][2 * ks + 1], p.scale_log2, bias[rb]));
                pw[rb][ks] = pack_bf16(p0, p1);
                acc[rb] = dot2_bf16(pw[rb][ks], ones, acc[rb]);   // row sum of the ROUNDED weights
            }
            // the slice's vector results are "used" here, so instruction selection cannot let
            // them drift past the barrier to the end of the region
            asm volatile("" ::"v"(pw[0][ks]), "v"(pw[1][ks]), "v"(acc[0]), "v"(acc[1]));
            __builtin_amdgcn_sched_barrier(0);
        }
        lsum[0] = acc[0];
        lsum[1] = acc[1];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int step = 0; step < 2; ++step) {
                const u32x4 w = {pw[rb][4 * step], pw[rb][4 * step + 1], pw[rb][4 * step + 2], pw[rb][4 * step + 3]};
                pf[rb][step] = __builtin_bit_cast(bf16x8, w);
            }
    };
    // Region Y: O^T += V^T P^T (matrix core) with the row maxima of the next block's scores
    // (vector ALU).  The maxima start two slices in, when the scores have left the matrix core.
    auto region_accumulate_maxima = [&](const char* vt, int kb, const bf16x8 (&pf)[2][2],
                                        const f32x16 (&s_new)[2], bool use_new, auto&& staging_step) {
        bf16x8 av[8];
        auto v_operand = [&](int idx) {   // idx = 4 step + dim block
            return *reinterpret_cast<const bf16x8*>(vt + (kb * 4 + (idx >> 2) * 2) * 2048 + v_rd[idx & 3]);
        };
        float mx[2] = {-INFINITY, -INFINITY};
#pragma unroll
        for (int i = 0; i < kVAhead; ++i) av[i] = v_operand(i);
#pragma unroll
        for (int idx = 0; idx < 8; ++idx) {
            const int step = idx >> 2, db = idx & 3;
            // written as assembly so that O is pinned to accumulation registers ("+a") while the
            // scores, which the vector ALU reads, stay in vector registers; nothing reads O
            // again before mfma_drain()
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(o[db][0]) : "v"(av[idx]), "v"(pf[0][step]));
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(o[db][1]) : "v"(av[idx]), "v"(pf[1][step]));
            if (idx + kVAhead < 8) av[idx + kVAhead] = v_operand(idx + kVAhead);
            if (idx >= 4) {   // four slices, four scores of each row block per slice
                const int r0 = (idx - 4) * 4;
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    mx[rb] = fmaxf(fmaxf(mx[rb], s_new[rb][r0]), s_new[rb][r0 + 1]);
                    mx[rb] = fmaxf(fmaxf(mx[rb], s_new[rb][r0 + 2]), s_new[rb][r0 + 3]);
                }
                asm volatile("" ::"v"(mx[0]), "v"(mx[1]));
            }
            staging_step(idx);   // one eighth of the next tiles' HBM -> LDS traffic
            __builtin_amdgcn_sched_barrier(0);
        }
        float cand[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            mx[rb] = max_across_halves(mx[rb]);
            // a look-ahead block that will be thrown away must not move the reference
            cand[rb] = use_new ? mx[rb] * p.scale_log2 : kNegBig;
        }
        rescale_if_needed(cand);
    };

    // ---- LDS ring of three tiles; tile t lives in slot t % 3 ----
    // Every iteration t: compute on tile t (the pipelined body also reads K of tile t + 1),
    // write tile t + 2 (loaded two iterations ago) into the slot tile t - 1 left, start the
    // loads of tile t + 4 into the registers just freed, barrier.  Tile t - 1 was last read
    // before the previous barrier and tile t + 2 is first read after this one, so one barrier
    // per tile is enough.  Two register sets alternate: st0 holds tile t + 2, st1 tile t + 3.
    Stage st0, st1;
    load_tile(st0, t_begin);
    store_tile(st0, t_begin, 0);
    load_tile(st0, t_begin + 1);
    store_tile(st0, t_begin + 1, 1);
    load_tile(st0, t_begin + 2);
    load_tile(st1, t_begin + 3);
    __syncthreads();

    int slot = 0;                                // slot of tile t
    auto next_slot = [](int s) { return s == kRing - 1 ? 0 : s + 1; };
    auto prev_slot = [](int s) { return s == 0 ? kRing - 1 : s - 1; };

    // one pipelined iteration; st holds tile t + 2 on entry and tile t + 4 (in flight) on exit
    f32x16 sa[2], sb[2];
    bf16x8 pf[2][2];
    auto pipelined_tile = [&](int t, Stage& st) {
        const char* kt = k_lds + slot * kKTileBytes;
        const char* vt = v_lds + slot * kVTileBytes;
        const char* kt_next = k_lds + next_slot(slot) * kKTileBytes;
        const int s2 = prev_slot(slot);          // slot of tile t + 2 == slot of tile t - 1
        region_scores_weights(kt, 1, sb, sa, pf);
        region_accumulate_maxima(vt, 0, pf, sb, true, [&](int i) { store_step(st, t + 2, s2, i); });
        region_scores_weights(kt_next, 0, sa, sb, pf);
        const LoadPlan lp = plan_load(t + 4);
        region_accumulate_maxima(vt, 1, pf, sa, t + 1 < n_unmasked, [&](int i) { load_step(st, lp, i); });
        __syncthreads();
        slot = next_slot(slot);
    };

    int t = t_begin;
    // ---- pipelined body, two tiles per trip.  Append-prefill pipelines the tiles whose
    // successor is also unmasked; a shared chunk has no masked tile and is pipelined to its end
    // (the scores of the block after its last one are computed and thrown away). ----
    const int pipe_end = SHARED ? n_tiles : t_begin + ((n_unmasked - 1 - t_begin) & ~1);
    if (pipe_end > t_begin) {
        scores(k_lds + slot * kKTileBytes, 0, sa);
        raise_reference(sa);
        for (; t < pipe_end; t += 2) {
            pipelined_tile(t, st0);
            pipelined_tile(t + 1, st1);
        }
        // sa holds the first block of tile t, which the plain body below computes again
        mfma_drain();
    }
    // ---- plain body: the last unmasked tiles and the tiles that straddle the diagonal ----
    for (; t < n_tiles; ++t) {
        const char* kt = k_lds + slot * kKTileBytes;
        const char* vt = v_lds + slot * kVTileBytes;
        const bool masked = t >= n_unmasked;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            f32x16 s[2];
            scores(kt, kb, s);
            if (masked) mask_scores(t * kTileKeys + kb * 32, s);
            raise_reference(s);
            weights(s, pf);
            accumulate(vt, kb, pf);
        }
        store_tile(st0, t + 2, prev_slot(slot));
        load_tile(st0, t + 4);
        const Stage tmp = st0;                   // st0 must hold tile t + 3 next time round
        st0 = st1;
        st1 = tmp;
        __syncthreads();
        slot = next_slot(slot);
    }

    // ---- epilogue ----
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const float total = lsum[rb] + __shfl_xor(lsum[rb], 32);
        if (out_row[rb] < 0) continue;
        if (SHARED) {
            // split-K partial of (member program, head) for this chunk: unnormalised O, the
            // reference maximum it is relative to, and the sum of weights
            const int member = (wave * 64 + rb * 32 + l32) / G;
            const int head = g * G + (wave * 64 + rb * 32 + l32) % G;
            const int64_t rowid = int64_t(p.chunk_start[b + member] + chunk) * p.num_q_heads + head;
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
            const float inv = total > 0.0f ? 1.0f / total : 0.0f;
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
    __syncthreads();   // the next item reuses the LDS ring
    }
}

// 96 KiB of dynamic LDS is above the default 64 KiB limit: raised once per kernel instance.
template <int G, bool SHARED>
int launch_instance(unsigned blocks, const PrefillParams& pp, hipStream_t stream) {
    const size_t lds_bytes = kRing * (kKTileBytes + kVTileBytes);
    static const hipError_t lds_rc =
        hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_tile_kernel<G, SHARED>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, int(lds_bytes));
    TA_HIP_TRY(lds_rc);
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

    hipLaunchKernelGGL(plan_tiles_kernel, dim3(1), dim3(1024), 0, stream, a.cu_q_lens, a.batch,
                       tile_tokens, per_prog, tile_start, tiles);
    TA_HIP_TRY(hipGetLastError());

    PrefillParams pp{};
    pp.q = a.q;
    pp.k_pool = reinterpret_cast<const char*>(a.k_pool);
    pp.v_pool = reinterpret_cast<const char*>(a.v_pool);
    pp.block_table = a.block_table;
    pp.context_lens = a.context_lens;
    pp.cu_q_lens = a.cu_q_lens;
    pp.tile_start = tile_start;
    pp.tiles = tiles;
    pp.out = a.out;
    pp.lse = a.lse;
    pp.stride_page_bytes = g.stride_page_bytes;
    pp.stride_head_bytes = g.stride_head_bytes;
    pp.block_table_stride = a.block_table_stride;
    pp.batch = a.batch;
    pp.num_q_heads = g.num_q_heads;
    pp.num_kv_heads = g.num_kv_heads;
    pp.scale_log2 = g.scale_log2;

    const int64_t blocks = max_tiles * g.num_kv_heads;
    if (blocks > 0x7fffffff) return TA_ERR_INVALID_ARG;
    const ProfileEvents ev = profile_events();
    if (ev.start != nullptr) TA_HIP_TRY(hipEventRecord(ev.start, stream));
    const int rc = launch_tile_kernel<false>(g.group, static_cast<unsigned>(blocks), pp, stream);
    if (rc != TA_OK) return rc;
    if (ev.stop != nullptr) TA_HIP_TRY(hipEventRecord(ev.stop, stream));
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
    pp.counts = a.counts;
    pp.chunk_start = a.chunk_start;
    pp.part_ml = a.part_ml;
    pp.part_o = a.part_o;
    pp.tiles_per_chunk = a.tiles_per_chunk;
    pp.stride_page_bytes = g.stride_page_bytes;
    pp.stride_head_bytes = g.stride_head_bytes;
    pp.block_table_stride = a.block_table_stride;
    pp.batch = a.batch;
    pp.num_q_heads = g.num_q_heads;
    pp.num_kv_heads = g.num_kv_heads;
    pp.scale_log2 = g.scale_log2;
    int64_t blocks = int64_t(a.max_items) * g.num_kv_heads;
    if (blocks <= 0) return TA_OK;
    if (blocks > 512) blocks = 512;   // one workgroup fits per CU; they stride over the items
    return launch_tile_kernel<true>(g.group, static_cast<unsigned>(blocks), pp, stream);
}

}  // namespace ta
