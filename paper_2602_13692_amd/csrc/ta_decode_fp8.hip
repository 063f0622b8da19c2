// Paged decode over an FP8 KV cache for gfx950 (the paper serves its large models in FP8,
// ThunderAgent Sec. 5.1; decode is the term of Sec. 4.2, Eq. 3 whose bytes the format halves).
//
// Keys and values are 8-bit E4M3 codes (2 KiB per page and kv head) with one scale each per
// call; queries and outputs stay bf16.  With half the bytes per token the vector-ALU decode
// kernel would be compute-bound, so this kernel does both contractions on the matrix cores and
// keeps the vector ALUs for what only they can do: widening the codes (two per instruction,
// exact: every E4M3 value is a bf16 value) and the softmax.
//
// One workgroup of four waves per (item, kv head), the same items as the bf16 path (a bulk chunk
// or a piece of a program's leftover).  A wave walks 32-key blocks (two pages):
//   * S^T = K Q^T with v_mfma_f32_16x16x32_bf16: A = 16 keys x 32 dims of K straight from the
//     wave's global loads (the contraction index may be permuted freely, so lane (key, c) simply
//     owns dims 16 c .. and 16 (c + 4) .. of its key: two 16-byte loads per page), B = the
//     query heads of the group, padded to 16 columns, resident in registers.  A lane ends up
//     with the scores of ONE head for four keys of each page, so the softmax needs two
//     cross-lane exchanges per block and the weights are already laid out as the B operand of
//   * O^T = V^T P^T: the A operand wants eight keys of one dim per lane, a transposed view of
//     the row-major page.  V goes global -> registers -> bf16 -> a wave-private LDS tile and
//     comes back through the transposing read ds_read_b64_tr_b16.  No barrier: the tile belongs
//     to one wave.
// The key scale is folded into the softmax scale, the value scale into the final
// normalisation.  Per block a wave issues 16 matrix instructions and about 150 vector ones for
// 8 KiB of cache: the kernel is HBM-bound with the vector ALUs a third busy.
#include "ta_internal.h"

namespace ta {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
#define TA_LDS_PTR(T, ptr) ((__attribute__((address_space(3))) T*)(ptr))

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kPageBytes = kPageSize * kHeadDim;        // one (page, kv head) tile of codes: 2 KiB
constexpr int kStageBytes = 2 * kPageSize * kHeadDim * 2;   // a wave's V tile of 32 keys in bf16: 8 KiB
constexpr int kMaxGroup = 16;                           // columns of the score tile

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint16_t to_bf16_rne(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
}

// Two E4M3 codes (the low or the high half of a dword) -> two bf16 in one dword (exact; scale 1).
__device__ __forceinline__ uint32_t widen_lo(uint32_t codes) {
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes, 1.0f, false));
}
__device__ __forceinline__ uint32_t widen_hi(uint32_t codes) {
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes, 1.0f, true));
}
// Eight codes (two dwords) -> eight bf16.
__device__ __forceinline__ u32x4 widen8_bits(uint32_t c0, uint32_t c1) {
    return u32x4{widen_lo(c0), widen_hi(c0), widen_lo(c1), widen_hi(c1)};
}
__device__ __forceinline__ bf16x8 widen8(uint32_t c0, uint32_t c1) {
    return __builtin_bit_cast(bf16x8, widen8_bits(c0, c1));
}

// One 32-key block in flight: for each of its two pages, this lane's two 16-byte pieces of K
// (key lane % 16, dims 16 (lane / 16 + 4 i) ..) and of V (bytes 16 lane .. of each KiB: key
// 8 i + lane / 8, dims 16 (lane % 8) ..).
struct BlockRegs {
    u32x4 k[2][2];
    u32x4 v[2][2];
};

__device__ __forceinline__ void load_page(BlockRegs& r, int pg, const char* k_tile, const char* v_tile, int lane) {
    const u32x4* kp = reinterpret_cast<const u32x4*>(k_tile + (lane & 15) * kHeadDim + (lane >> 4) * 16);
    const u32x4* vp = reinterpret_cast<const u32x4*>(v_tile) + lane;
    r.k[pg][0] = __builtin_nontemporal_load(kp);
    r.k[pg][1] = __builtin_nontemporal_load(kp + 4);      // + 64 bytes
    r.v[pg][0] = __builtin_nontemporal_load(vp);
    r.v[pg][1] = __builtin_nontemporal_load(vp + 64);     // + 1 KiB
}

struct SoftmaxState {
    float m;          // reference maximum of the head (log2 domain), the same in the four lanes of a head
    float l;          // this lane's share of the sum of weights
    f32x4 o[8];       // O^T: dims 16 db + 4 (lane / 16) + 0..3 of head lane % 16
};

// One block of up to 32 keys.  valid = keys of the block that exist (32 unless MASKED).  SETS sets
// of sixteen columns (query heads) take their turn on every operand once it is in registers.
template <bool MASKED, int SETS>
__device__ __forceinline__ void process_block(const BlockRegs& r, const bf16x8 (&qop)[SETS][2][2], SoftmaxState (&st)[SETS],
                                              char* stage, float scale_log2, int lane, int valid) {
    const int r16 = lane & 15, c = lane >> 4;
    // ---- scores: 16 keys x 16 heads per page, contraction over the 128 dims in four steps ----
    f32x4 s[SETS][2];
#pragma unroll
    for (int pg = 0; pg < 2; ++pg) {
        f32x4 acc[SETS];
#pragma unroll
        for (int q = 0; q < SETS; ++q) acc[q] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const bf16x8 lo = widen8(r.k[pg][i].x, r.k[pg][i].y), hi = widen8(r.k[pg][i].z, r.k[pg][i].w);
#pragma unroll
            for (int q = 0; q < SETS; ++q) {
                acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo, qop[q][i][0], acc[q], 0, 0, 0);
                acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi, qop[q][i][1], acc[q], 0, 0, 0);
            }
        }
#pragma unroll
        for (int q = 0; q < SETS; ++q) s[q][pg] = acc[q];
    }
    // ---- V: widen and park it in this wave's LDS tile, row-major bf16, 16-byte chunks permuted
    // per row (chunk ch of key k at ch ^ 4 (k % 4)) so that the transposing reads below spread
    // over the banks ----
#pragma unroll
    for (int pg = 0; pg < 2; ++pg)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int key = 8 * i + (lane >> 3);
            u32x4 lo = widen8_bits(r.v[pg][i].x, r.v[pg][i].y);
            u32x4 hi = widen8_bits(r.v[pg][i].z, r.v[pg][i].w);
            if (MASKED && pg * kPageSize + key >= valid) {       // 0 * NaN inside the matrix core would poison O
                lo = u32x4{0u, 0u, 0u, 0u};
                hi = u32x4{0u, 0u, 0u, 0u};
            }
            const int ch = 2 * (lane & 7), swz = (key & 3) << 2;
            char* row = stage + pg * (kPageSize * kHeadDim * 2) + key * (kHeadDim * 2);
            *reinterpret_cast<u32x4*>(row + ((ch ^ swz) << 4)) = lo;
            *reinterpret_cast<u32x4*>(row + (((ch + 1) ^ swz) << 4)) = hi;
        }
    // ---- softmax: this lane holds head r16 of each set, keys 4 c .. 4 c + 3 of each page ----
    bf16x8 pf[SETS];
#pragma unroll
    for (int q = 0; q < SETS; ++q) {
        float t[2][4];
        float mx = -INFINITY;
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float x = s[q][pg][e] * scale_log2;
                if (MASKED) x = (pg * kPageSize + 4 * c + e) < valid ? x : -INFINITY;
                t[pg][e] = x;
                mx = fmaxf(mx, x);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        if (__builtin_amdgcn_ballot_w64(mx > st[q].m) != 0) {         // wave-uniform; rare after the first blocks
            const float m_new = fmaxf(st[q].m, mx);
            const float alpha = fast_exp2(st[q].m - m_new);
            st[q].m = m_new;
            st[q].l *= alpha;
#pragma unroll
            for (int db = 0; db < 8; ++db) st[q].o[db] *= alpha;
        }
        const uint32_t ones = 0x3f803f80u;   // (1.0, 1.0) in bf16
        u32x4 pw;
        pw.x = pack_bf16(fast_exp2(t[0][0] - st[q].m), fast_exp2(t[0][1] - st[q].m));
        pw.y = pack_bf16(fast_exp2(t[0][2] - st[q].m), fast_exp2(t[0][3] - st[q].m));
        pw.z = pack_bf16(fast_exp2(t[1][0] - st[q].m), fast_exp2(t[1][1] - st[q].m));
        pw.w = pack_bf16(fast_exp2(t[1][2] - st[q].m), fast_exp2(t[1][3] - st[q].m));
        // the sum adds up the ROUNDED weights, the ones the matrix core multiplies
        float l = st[q].l;
        l = dot2_bf16(pw.x, ones, l);
        l = dot2_bf16(pw.y, ones, l);
        l = dot2_bf16(pw.z, ones, l);
        l = dot2_bf16(pw.w, ones, l);
        st[q].l = l;
        pf[q] = __builtin_bit_cast(bf16x8, pw);
    }
    // ---- O^T += V^T P^T: for every block of 16 dims, eight keys of one dim per lane.  In each
    // group of 16 lanes, lane s names the 8 bytes (4 dims) of key 4 c + s / 4 at dims
    // 16 db + 4 (s % 4) .., and receives dim 16 db + s of the four keys 4 c .. 4 c + 3. ----
    const int key_s = 4 * c + (r16 >> 2);
    const char* rd = stage + key_s * (kHeadDim * 2) + (r16 & 1) * 8;
    const int swz_s = (r16 >> 2) << 2, half = (r16 & 3) >> 1;
#pragma unroll
    for (int db = 0; db < 8; ++db) {
        const char* at = rd + (((2 * db + half) ^ swz_s) << 4);
        const s16x4 a0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(TA_LDS_PTR(s16x4, at));
        const s16x4 a1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(TA_LDS_PTR(s16x4, at + kPageSize * kHeadDim * 2));
        const bf16x8 a = __builtin_bit_cast(bf16x8, __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
        for (int q = 0; q < SETS; ++q) st[q].o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pf[q], st[q].o[db], 0, 0, 0);
    }
}

// DIRECT: every program is one item (its whole context); the workgroup normalises and writes the
// bf16 output itself.
// SHARED: an item is a bulk chunk that `members` programs have in common (their block tables
// name the same pages there): two sets of sixteen columns hold the heads of all of them
// (column = member * group + head, up to 32 / group members), the pages are streamed once, every
// operand serves both sets while it is in registers, and every member gets its partial in its
// own slot.
template <bool DIRECT, bool SHARED, bool BEYOND_CAP>
__device__ __forceinline__ void decode_fp8_body(const ChunkParams& p, int32_t group) {
    constexpr int SETS = SHARED ? 2 : 1;
    // the waves' V tiles during the walk, the waves' results afterwards
    __shared__ __attribute__((aligned(16))) char smem[kWaves * kStageBytes];
    __shared__ float sm_m[kWaves][kMaxGroup];
    __shared__ float sm_l[kWaves][kMaxGroup];
    __shared__ int32_t sm_ids[kMaxItemPagesFp8];
    static_assert(kWaves * kStageBytes >= kWaves * kMaxGroup * kHeadDim * 4, "the merge reuses the V tiles' memory");

    const int g = blockIdx.x % p.num_kv_heads;
    // The launches are sized for the most items a batch could have under its bound on the context
    // length, often far more than it has (half a million workgroups that find nothing to do cost
    // 150 us).  Shared form: a bounded number of workgroups walks the list.  Private form: a launch
    // has at most kChunkGridCap workgroups, one item each; items beyond that number (very large
    // batches) belong to a second launch of as many workgroups, in the BEYOND_CAP form, which walks
    // the rest of the list.  (The walking form of the private kernel needs 226 registers instead
    // of 180 and streamed config 2 four per cent slower: hence two forms.)
    const int per_grid = int(gridDim.x) / p.num_kv_heads;
    const int item_step = (SHARED || BEYOND_CAP) ? per_grid : 0;
    for (int item = blockIdx.x / p.num_kv_heads + (BEYOND_CAP ? per_grid : 0);; item += item_step) {
        int b, page0, n_here, slot = 0, members = 1, chunk = 0, first_pos = 0;
        if (SHARED) {
            if (item >= p.counts[1]) return;
            const int4 it = p.shared_items[item];
            first_pos = it.x; members = it.y; chunk = it.z; b = it.w;
            n_here = p.counts[3];                      // a whole bulk chunk, every key of it exists
            page0 = chunk * n_here;
        } else if (DIRECT) {
            b = item;
            page0 = 0;
        } else {
            if (item >= p.counts[0]) return;
            const int4 it = p.items[item];
            b = it.x; page0 = it.y; n_here = it.z; slot = it.w;
        }
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const int r16 = lane & 15, c = lane >> 4;

        const int L = p.context_lens[b];
        int n_pages_b = L > 0 ? (L + kPageSize - 1) / kPageSize : 0;
        if (DIRECT) {
            n_pages_b = n_pages_b > p.max_pages ? p.max_pages : n_pages_b;
            n_here = n_pages_b;
        }
        const int tail_valid = L - (n_pages_b - 1) * kPageSize;           // 1..16 where the program's last page is reached
        const bool has_tail = !SHARED && n_here > 0 && (page0 + n_here == n_pages_b) && tail_valid < kPageSize;
        const int n_full_pages = has_tail ? n_here - 1 : n_here;
        const int full_blocks = n_full_pages >> 1;                         // blocks of two complete pages
        const int rest_pages = n_here - 2 * full_blocks;                   // 0, 1 or 2 pages in a last, masked block
        const int rest_valid = rest_pages == 0 ? 0 : (rest_pages - 1) * kPageSize + (has_tail ? tail_valid : kPageSize);

        // page ids of this item (up to 512: the start of an item costs its workgroup a microsecond
        // in which it streams nothing, so items are as long as the batch allows), kept in LDS
        {
            const int32_t* table = p.block_table + int64_t(b) * p.block_table_stride + page0;
            for (int i = threadIdx.x; i < n_here; i += kThreads) sm_ids[i] = table[i];
            __syncthreads();
        }
        auto page_off = [&](int idx) -> int64_t {                          // idx is wave-uniform
            return int64_t(__builtin_amdgcn_readfirstlane(sm_ids[idx])) * p.stride_page_bytes;
        };

        // B operands: column 16 q + r16 of set q is head (column % group) of member (column / group),
        // zero beyond the last member; dims 16 (c + 4 i) + 8 hf ..
        bf16x8 qop[SETS][2][2];
        SoftmaxState st[SETS];
#pragma unroll
        for (int q = 0; q < SETS; ++q) {
            const int col = 16 * q + r16;
            const bool head_ok = col < members * group;
            const int member = head_ok ? col / group : 0, head = head_ok ? col % group : 0;
            const int q_program = SHARED ? p.order[first_pos + member] : b;
            const uint16_t* qrow = p.q + (int64_t(q_program) * p.num_q_heads + g * group + head) * kHeadDim;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    u32x4 w = {0u, 0u, 0u, 0u};
                    if (head_ok) w = *reinterpret_cast<const u32x4*>(qrow + 16 * (c + 4 * i) + 8 * hf);
                    qop[q][i][hf] = __builtin_bit_cast(bf16x8, w);
                }
            st[q].m = kNegBig;
            st[q].l = 0.0f;
#pragma unroll
            for (int db = 0; db < 8; ++db) st[q].o[db] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        }

        const char* k_head = p.k_pool + int64_t(g) * p.stride_head_bytes;
        const char* v_head = p.v_pool + int64_t(g) * p.stride_head_bytes;
        char* stage = smem + wave * kStageBytes;

        // this wave's full blocks: wave, wave + 4, ...  Two block buffers: each is refilled right
        // after its block has been consumed and is consumed one block later; no load is issued for a
        // page that is not used.
        const int n_mine = full_blocks > wave ? (full_blocks - wave + kWaves - 1) / kWaves : 0;
        if (n_mine > 0) {
            auto load_block = [&](BlockRegs& r, int j) {
                const int blk = wave + kWaves * j;
                const int64_t o0 = page_off(2 * blk), o1 = page_off(2 * blk + 1);
                load_page(r, 0, k_head + o0, v_head + o0, lane);
                load_page(r, 1, k_head + o1, v_head + o1, lane);
            };
            BlockRegs bufA, bufB;
            load_block(bufA, 0);
            int j = 0;
            for (; j + 2 < n_mine; j += 2) {
                load_block(bufB, j + 1);
                __builtin_amdgcn_sched_barrier(0);
                process_block<false, SETS>(bufA, qop, st, stage, p.scale_log2, lane, 2 * kPageSize);
                load_block(bufA, j + 2);
                __builtin_amdgcn_sched_barrier(0);
                process_block<false, SETS>(bufB, qop, st, stage, p.scale_log2, lane, 2 * kPageSize);
            }
            if (j + 1 < n_mine) {
                load_block(bufB, j + 1);
                __builtin_amdgcn_sched_barrier(0);
                process_block<false, SETS>(bufA, qop, st, stage, p.scale_log2, lane, 2 * kPageSize);
                process_block<false, SETS>(bufB, qop, st, stage, p.scale_log2, lane, 2 * kPageSize);
            } else {
                process_block<false, SETS>(bufA, qop, st, stage, p.scale_log2, lane, 2 * kPageSize);
            }
        }
        if (rest_pages > 0 && (full_blocks & (kWaves - 1)) == wave) {
            BlockRegs t;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                t.k[1][i] = u32x4{0u, 0u, 0u, 0u};
                t.v[1][i] = u32x4{0u, 0u, 0u, 0u};
            }
            const int64_t o0 = page_off(2 * full_blocks);
            load_page(t, 0, k_head + o0, v_head + o0, lane);
            if (rest_pages > 1) {
                const int64_t o1 = page_off(2 * full_blocks + 1);
                load_page(t, 1, k_head + o1, v_head + o1, lane);
            }
            process_block<true, SETS>(t, qop, st, stage, p.scale_log2, lane, rest_valid);
        }

        // ---- the four lanes of a head add up their shares; the waves meet in LDS, one set of columns
        // at a time ----
        float* sm_o = reinterpret_cast<float*>(smem);      // [wave][column of the set][128]
#pragma unroll
        for (int q = 0; q < SETS; ++q) {
            const int cols_here = members * group - 16 * q < 16 ? members * group - 16 * q : 16;     // may be <= 0
            float lt = st[q].l;
            lt += __shfl_xor(lt, 16);
            lt += __shfl_xor(lt, 32);
            __syncthreads();                                   // every wave is done with its V tile (and with the set before)
            if (r16 < cols_here) {
                float* dst = sm_o + (wave * kMaxGroup + r16) * kHeadDim + 4 * c;
#pragma unroll
                for (int db = 0; db < 8; ++db) *reinterpret_cast<f32x4*>(dst + 16 * db) = st[q].o[db];
                if (c == 0) {
                    sm_m[wave][r16] = st[q].m;
                    sm_l[wave][r16] = lt;
                }
            }
            __syncthreads();

            // thread t owns two neighbouring dims of one head
            for (int idx = threadIdx.x; idx < cols_here * (kHeadDim / 2); idx += kThreads) {
                const int h = idx / (kHeadDim / 2);           // column of this set
                const int col = 16 * q + h;
                const int d0 = 2 * (idx % (kHeadDim / 2));
                float mt = sm_m[0][h];
#pragma unroll
                for (int w = 1; w < kWaves; ++w) mt = fmaxf(mt, sm_m[w][h]);
                float sum = 0.0f, a0 = 0.0f, a1 = 0.0f;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    const float wt = fast_exp2(sm_m[w][h] - mt);
                    sum = fmaf(sm_l[w][h], wt, sum);
                    const float2 v = *reinterpret_cast<const float2*>(sm_o + (w * kMaxGroup + h) * kHeadDim + d0);
                    a0 = fmaf(v.x, wt, a0);
                    a1 = fmaf(v.y, wt, a1);
                }
                if (DIRECT) {
                    const float inv = sum > 0.0f ? p.out_scale / sum : 0.0f;
                    const int64_t rid = int64_t(b) * p.num_q_heads + g * group + h;
                    *reinterpret_cast<uint32_t*>(p.out + rid * kHeadDim + d0) =
                        uint32_t(to_bf16_rne(a0 * inv)) | (uint32_t(to_bf16_rne(a1 * inv)) << 16);
                    if (p.lse != nullptr && d0 == 0)
                        p.lse[rid] = sum > 0.0f ? (mt + __builtin_amdgcn_logf(sum)) * kLn2 : -INFINITY;
                } else {
                    // (shared form: column col is head col % group of member col / group, whose partial of this chunk
                    // sits at its own first slot + chunk)
                    const int my_slot = SHARED ? p.chunk_start[p.order[first_pos + col / group]] + chunk : slot;
                    const int64_t rowid = int64_t(my_slot) * p.num_q_heads + g * group + (SHARED ? col % group : h);
                    *reinterpret_cast<float2*>(p.part_o + rowid * kHeadDim + d0) = make_float2(a0, a1);
                    if (d0 == 0) {
                        p.part_ml[rowid * 2 + 0] = mt;    // already in the log2 domain
                        p.part_ml[rowid * 2 + 1] = sum;
                    }
                }
            }
        }
        if (!SHARED && !BEYOND_CAP) break;
        __syncthreads();                               // the merge buffers are the next item's V tiles
    }
}

template <bool DIRECT, bool SHARED>
__global__ __launch_bounds__(kThreads) void decode_fp8_kernel(ChunkParams p, int32_t group) {
    decode_fp8_body<DIRECT, SHARED, false>(p, group);
}

__global__ __launch_bounds__(kThreads) void decode_fp8_beyond_cap_kernel(ChunkParams p, int32_t group) {
    decode_fp8_body<false, false, true>(p, group);
}

// Append-prefill over an FP8 cache runs the bf16 tile kernel on a widened copy of the batch's
// pages: the contraction there is bound by the matrix cores and their issue port, and widening
// every operand on the fly would add vector work to exactly that port, while one streaming pass
// (codes in, twice the bytes out) costs a few per cent of the prefill's time.  The copy holds
// code VALUES; the scales enter the softmax scale and the output as in the decode kernel.
__global__ __launch_bounds__(256) void widen_pages_kernel(
    const char* __restrict__ k_codes, const char* __restrict__ v_codes, const int32_t* __restrict__ block_table,
    int32_t block_table_stride, const int32_t* __restrict__ context_lens, int32_t width, int32_t num_kv_heads,
    int64_t stride_page_bytes, int64_t stride_head_bytes, char* __restrict__ wide_k, char* __restrict__ wide_v,
    int32_t* __restrict__ wide_table) {
    const int b = blockIdx.y, i = blockIdx.x;
    const int slot = b * width + i;
    if (threadIdx.x == 0) wide_table[slot] = slot;
    const int L = context_lens[b];
    int pages = L > 0 ? (L + kPageSize - 1) / kPageSize : 0;
    pages = pages < width ? pages : width;
    if (i >= pages) return;
    const int64_t src = int64_t(block_table[int64_t(b) * block_table_stride + i]) * stride_page_bytes;
    const int64_t dst = int64_t(slot) * num_kv_heads * (kPageBytes * 2);
    // a lane takes 16 codes (16 bytes in, 32 bytes out); a (page, kv head) tile is 128 such pieces
    for (int piece = threadIdx.x; piece < num_kv_heads * 128 * 2; piece += blockDim.x) {
        const int is_v = piece / (num_kv_heads * 128);
        const int rest = piece - is_v * num_kv_heads * 128;
        const int g = rest >> 7, c = rest & 127;
        const u32x4 codes = *reinterpret_cast<const u32x4*>((is_v ? v_codes : k_codes) + src + g * stride_head_bytes + c * 16);
        u32x4* out = reinterpret_cast<u32x4*>((is_v ? wide_v : wide_k) + dst + int64_t(g) * (kPageBytes * 2) + c * 32);
        out[0] = widen8_bits(codes.x, codes.y);
        out[1] = widen8_bits(codes.z, codes.w);
    }
}

}  // namespace

int launch_widen_pages(const Geometry& g, const void* k_codes, const void* v_codes, const int32_t* block_table,
                       int32_t block_table_stride, const int32_t* context_lens, int32_t batch, int32_t width,
                       void* wide_k, void* wide_v, int32_t* wide_table, hipStream_t stream) {
    if (batch < 1 || width < 1 || batch > 65535) return TA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(widen_pages_kernel, dim3(unsigned(width), unsigned(batch)), dim3(256), 0, stream,
                       static_cast<const char*>(k_codes), static_cast<const char*>(v_codes), block_table,
                       block_table_stride, context_lens, width, g.num_kv_heads, g.stride_page_bytes,
                       g.stride_head_bytes, static_cast<char*>(wide_k), static_cast<char*>(wide_v), wide_table);
    TA_HIP_TRY(hipGetLastError());
    return TA_OK;
}

int launch_fp8_items(const ChunkParams& p, int32_t group, bool direct, bool shared, unsigned blocks, hipStream_t stream) {
    if (group < 1 || group > kMaxGroup || (direct && shared)) return TA_ERR_UNSUPPORTED;
    if (shared) hipLaunchKernelGGL((decode_fp8_kernel<false, true>), dim3(blocks), dim3(kThreads), 0, stream, p, group);
    else if (direct) hipLaunchKernelGGL((decode_fp8_kernel<true, false>), dim3(blocks), dim3(kThreads), 0, stream, p, group);
    else {
        // at most kChunkGridCap workgroups, a whole number of kv-head sets (the kernel steps by grid / kv heads items)
        const unsigned sets = kChunkGridCap / unsigned(p.num_kv_heads) > 0 ? kChunkGridCap / unsigned(p.num_kv_heads) : 1u;
        const unsigned cap = sets * unsigned(p.num_kv_heads);
        hipLaunchKernelGGL((decode_fp8_kernel<false, false>), dim3(blocks < cap ? blocks : cap), dim3(kThreads), 0, stream, p, group);
        if (blocks > cap) {
            TA_HIP_TRY(hipGetLastError());
            hipLaunchKernelGGL(decode_fp8_beyond_cap_kernel, dim3(cap), dim3(kThreads), 0, stream, p, group);
        }
    }
    TA_HIP_TRY(hipGetLastError());
    return TA_OK;
}

}  // namespace ta
