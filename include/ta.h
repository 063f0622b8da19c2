/*
 * ta.h -- C ABI of the paged-KV attention hot path for AMD MI355X (gfx950).
 *
 * The paper this library serves (ThunderAgent) schedules long-lived agent
 * programs over inference backends.  Each program's context only grows and is
 * kept as a KV cache between turns (Sec. 2.1); a step prefills the new
 * tool-output tokens against the retained prefix and then decodes (the two
 * productive terms of the cost decomposition, Sec. 4.2, Eq. 3); a paused
 * program loses its pages and a restored one needs them back (Sec. 4.3,
 * Eq. 4-5; host offloading in App. A.2 and A.4).  The paper treats the backend
 * as a black box; this library is the device-side part of that backend:
 *
 *   ta_paged_decode      one new token per program attends to the program's
 *                        whole cached context;
 *   ta_append_prefill    n new tokens per program attend causally to prefix +
 *                        themselves;
 *   ta_kv_page_evict     pool pages are copied out to pinned host memory (Pause);
 *   ta_kv_append         the new tokens' keys and values are written to the tail
 *                        of their programs' pages;
 *   ta_kv_page_restore   pages held in pinned host memory are written back
 *                        into free slots of the device page pool.
 *
 * Common conventions
 *   - Every pointer is labelled DEVICE or HOST.  DEVICE pointers are HIP device
 *     allocations on the current device; the library never allocates or frees.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and the call returns without synchronising.
 *     HOST arrays are consumed before the call returns.
 *   - bf16 values are 16-bit patterns (upper half of an IEEE fp32).
 *   - Token j of program b lives in page block_table[b*stride + j/page_size],
 *     row j % page_size.  With the default pool layout [P][Hkv][page_size][d]
 *     one (page, kv head) tile is 4 KiB contiguous.  Query head h reads kv head
 *     h / (Hq/Hkv).  Pages may be shared between programs; the attention calls
 *     only read the pools.
 *   - Block-table entries beyond ceil(context_len/page_size) are ignored.  Rows
 *     of the last page beyond the context length are never read into a result.
 *   - Device-resident metadata is not validated: a block-table entry outside
 *     the pool or a context length beyond stride*page_size is undefined
 *     behaviour.  Everything the host can see is validated before any launch.
 *     In debug mode (ta_set_debug_checks(1), or the environment variable
 *     TA_DEBUG=1 when the library makes its first call) ta_paged_decode,
 *     ta_append_prefill and ta_kv_append first run a checking kernel and wait
 *     for it (the call then synchronises the stream; a call made while its stream
 *     is being captured into a graph goes unchecked): context lengths outside [0, max_context_len], block-table entries
 *     among the pages in use that are negative or, when the descriptor states
 *     pool_pages, not below it, and prefix sums (cu_q_lens, cu_new_lens) that do
 *     not start at 0, decrease, do not end at the stated total, or give a
 *     program more new tokens than max_q_len or than its context holds, make
 *     the call return TA_ERR_INVALID_ARG before any other kernel runs.
 *   - Return value: TA_OK (0) or a negative ta_status.  No exceptions, no
 *     aborts, nothing is printed.  batch == 0, total_q == 0 and n_pages == 0
 *     are valid and do nothing.
 */
#ifndef TA_H
#define TA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Exported symbols keep default visibility; everything else in the library is hidden. */
#define TA_API __attribute__((visibility("default")))

typedef enum ta_status {
    TA_OK = 0,
    TA_ERR_INVALID_ARG = -1, /* null pointer, negative size, Hq % Hkv != 0, workspace too small,
                                slot out of range or duplicated, ... */
    TA_ERR_UNSUPPORTED = -2, /* head_dim != 128, page_size != 16, group size not in {1,2,4,8},
                                token stride != head_dim, misaligned strides */
    TA_ERR_HIP = -3,         /* a HIP call failed; see ta_last_hip_error() */
    TA_ERR_TOO_LARGE = -4    /* ta_paged_decode_static: the call needs more scratch than
                                TA_STATIC_SCRATCH_BYTES; use ta_paged_decode with a workspace */
} ta_status;

typedef struct ta_attn_desc {
    int32_t num_q_heads;       /* Hq */
    int32_t num_kv_heads;      /* Hkv, divides Hq; Hq/Hkv in {1,2,4,8} */
    int32_t head_dim;          /* 128 */
    int32_t page_size;         /* 16 tokens */
    float scale;               /* multiplies q.k; 0.0f selects 1/sqrt(head_dim) */
    int32_t pool_pages;        /* pages in each pool, for the debug checks; 0 = not stated */
    int64_t pool_stride_page;  /* elements between pages;       0 selects Hkv*page_size*head_dim */
    int64_t pool_stride_head;  /* elements between kv heads;    0 selects page_size*head_dim */
    int64_t pool_stride_token; /* elements between token rows;  0 selects head_dim (only value supported) */
    int32_t decode_chunk_pages; /* split-K chunk of ta_paged_decode in pages: 0 lets the library choose
                                   the chunk and the kernel that streams the private chunks (the kernel by
                                   batch and the bound on the context length, confirmed on the device
                                   from the real lengths, which also settle the chunk), else 8, 16, 32, 64 or 128 (a bf16 cache with
                                   up to four query heads per kv head: on the vector-ALU kernel), or 256
                                   or 512 (a bf16 cache: on the matrix-core tile kernel; an FP8 cache:
                                   longer items of its one kernel).  The same value must be given to
                                   ta_workspace_bytes. */
    int32_t kv_format;         /* TA_KV_BF16 (0) or TA_KV_FP8_E4M3 (1), see below */
    float k_scale;             /* TA_KV_FP8_E4M3: a cached key element is code value * k_scale; > 0, finite */
    float v_scale;             /* TA_KV_FP8_E4M3: a cached value element is code value * v_scale; > 0, finite */
    int32_t prefill_key_chunks; /* ta_append_prefill: into how many chunks of even length the keys of every
                                   query tile are cut, one workgroup per (tile, kv head, chunk), the chunks'
                                   partial results merged by a second kernel.  0 lets the library choose
                                   (it cuts when the batch's query tiles alone would leave most compute
                                   units idle: few programs appending onto long contexts), 1 never cuts,
                                   2 .. 1024 asks for that many (fewer when a chunk would have less than
                                   four key tiles of 64 tokens).  The same value must be given to
                                   ta_workspace_bytes. */
} ta_attn_desc;

/*
 * Formats of the K and V pools.
 *   TA_KV_BF16      16-bit patterns, the upper half of an IEEE fp32 (k_scale, v_scale ignored).
 *   TA_KV_FP8_E4M3  8-bit codes of the OCP "E4M3" format: 1 sign bit, 4 exponent bits with
 *                   bias 7, 3 mantissa bits, no infinities, S.1111.111 = NaN, exponent field 0 =
 *                   subnormals m * 2^-9, largest value 448; one fp32 scale for all keys and one
 *                   for all values of the call.  (The paper serves its large models in FP8,
 *                   Sec. 5.1; it does not describe the cache, so format and scale granularity
 *                   are this library's reading.)  Pool strides count elements, i.e. bytes; a
 *                   (page, kv head) tile is 2 KiB.  Supported by ta_paged_decode and
 *                   ta_paged_decode_static (queries and outputs stay bf16: the output is
 *                   softmax(scale * k_scale * <q, K codes>) . (V codes) * v_scale), and by the
 *                   byte-wise ta_kv_page_restore / ta_kv_page_evict.  ta_kv_append writes such
 *                   a cache: the code of an element x is the E4M3 value nearest to x / scale
 *                   (the quotient in fp32, ties to the code with an even mantissa, anything
 *                   beyond the largest value becomes +-448, NaN stays NaN).
 *                   ta_append_prefill reads such a cache through a bf16 copy of the batch's
 *                   pages that it makes in the workspace first (exact: every code value is a
 *                   bf16 value), so ta_workspace_bytes then also counts
 *                   batch * ceil(max_context_len / 16) pages of Hkv * 8 KiB for K and V together.
 */
#define TA_KV_BF16 0
#define TA_KV_FP8_E4M3 1

/* Library version, major*10000 + minor*100 + patch. */
TA_API int32_t ta_version(void);

/* Text for a ta_status value (static storage). */
TA_API const char *ta_strerror(int status);

/* The hipError_t (as int) of the last failed HIP call on this thread, 0 if none. */
TA_API int ta_last_hip_error(void);

/*
 * Debug mode for the whole process: on != 0 makes the calls listed above check
 * their device-resident metadata first (and synchronise), 0 switches that off.
 * Until the first call of this function the mode is what the environment
 * variable TA_DEBUG said ("1" = on) when the library first looked.
 * Returns the previous mode (0 or 1).
 */
TA_API int ta_set_debug_checks(int on);

/*
 * Bytes of DEVICE workspace that ta_paged_decode (max_q_len <= 1) or
 * ta_append_prefill needs for `batch` programs, at most `max_q_len` query
 * tokens per program and at most `max_context_len` cached tokens per program.
 * Returns 0 for an invalid descriptor.  The workspace holds the work plan and
 * the split-K partial results (running max, sum and unnormalised output per
 * chunk of the key axis); its contents need not survive between calls.
 */
TA_API size_t ta_workspace_bytes(const ta_attn_desc *desc, int32_t batch, int32_t max_q_len,
                          int32_t max_context_len);

/*
 * Decode (Sec. 2.1: the emission is sampled conditioned on the whole context;
 * Sec. 4.3: context lengths keep growing during decoding).  For every program
 * b and query head h:
 *     out[b][h][:] = softmax_j(scale * <q[b][h], K_j>) . V_j,   j < context_lens[b]
 * computed with bf16 inputs, fp32 accumulation, bf16 output (round to nearest
 * even).  context_lens[b] counts every cached token including the newest one.
 * A program with context length 0 gets a zero row and lse = -inf.
 *
 *   q             DEVICE bf16 [batch][Hq][128]
 *   k_pool,v_pool DEVICE bf16 (or E4M3 codes, see kv_format), layout given by desc, read only,
 *                 16-byte aligned
 *   block_table   DEVICE int32 [batch][block_table_stride]
 *   context_lens  DEVICE int32 [batch]
 *   max_context_len  HOST upper bound on context_lens[]; sizes the launch, so no
 *                 device-to-host copy is needed.  Lengths above it are undefined.
 *   out           DEVICE bf16 [batch][Hq][128]
 *   lse           DEVICE fp32 [batch][Hq] natural-log sum of exponentials, or NULL
 *   workspace     DEVICE, at least ta_workspace_bytes(desc, batch, 1, max_context_len),
 *                 256-byte aligned
 */
TA_API int ta_paged_decode(const ta_attn_desc *desc, const void *q, const void *k_pool,
                    const void *v_pool, const int32_t *block_table, int32_t block_table_stride,
                    const int32_t *context_lens, int32_t batch, int32_t max_context_len,
                    void *out, float *lse, void *workspace, size_t workspace_bytes,
                    void *hip_stream);

/*
 * ta_paged_decode for callers that cannot allocate or hand over a workspace:
 * code under HIP graph capture that may not call an allocator, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * the same results as ta_paged_decode, without `workspace`: the split-K plan
 * and partial results live in an array of TA_STATIC_SCRATCH_BYTES that the
 * library holds in device memory on every GPU it runs on, from the first call
 * on that GPU until the process ends.  The call itself allocates and frees
 * nothing, on the host or on the device.
 *
 * Returns TA_ERR_TOO_LARGE (and enqueues nothing) when
 * ta_workspace_bytes(desc, batch, 1, max_context_len) exceeds
 * TA_STATIC_SCRATCH_BYTES; other errors as for ta_paged_decode.
 * All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams, or graphs replayed side by side) race; calls on
 * one stream are ordered and safe.  Nothing in the array needs to survive
 * between calls; every call writes what it later reads.
 */
#define TA_STATIC_SCRATCH_BYTES (64u << 20)
TA_API int ta_paged_decode_static(const ta_attn_desc *desc, const void *q, const void *k_pool,
                           const void *v_pool, const int32_t *block_table,
                           int32_t block_table_stride, const int32_t *context_lens, int32_t batch,
                           int32_t max_context_len, void *out, float *lse, void *hip_stream);

/*
 * Append-prefill (Sec. 4.2: incremental prefilling of tool-execution results,
 * as opposed to recomputation over the full context).  Program b owns
 * n_b = cu_q_lens[b+1] - cu_q_lens[b] new tokens whose keys and values are
 * ALREADY in its pages, so context_lens[b] = prefix_b + n_b.  New token i
 * (0-based) sees keys 0 .. prefix_b + i, itself included:
 *     out[cu_q_lens[b]+i][h][:] = softmax_j(scale * <q, K_j>) . V_j,  j <= prefix_b + i
 * bf16 inputs, fp32 accumulation on the matrix cores, bf16 output.
 *
 *   q             DEVICE bf16 [total_q][Hq][128], programs packed back to back
 *   cu_q_lens     DEVICE int32 [batch+1], non-decreasing, cu_q_lens[0] = 0
 *   total_q       HOST, equals cu_q_lens[batch]
 *   max_q_len     HOST upper bound on n_b
 *   max_context_len HOST upper bound on context_lens[]
 *   out           DEVICE bf16 [total_q][Hq][128]
 *   lse           DEVICE fp32 [total_q][Hq] or NULL
 *   workspace     DEVICE, at least ta_workspace_bytes(desc, batch, max_q_len, max_context_len)
 * Other arguments as for ta_paged_decode.
 * When the batch has few query tiles (batch * ceil(max_q_len / (256 / (Hq / Hkv))) * Hkv below about
 * 500) and long contexts, the keys of every tile are cut into chunks that run side by side and a
 * second kernel merges their partial results (desc->prefill_key_chunks); the result is the same
 * up to fp32 summation order.
 */
TA_API int ta_append_prefill(const ta_attn_desc *desc, const void *q, const int32_t *cu_q_lens,
                      const void *k_pool, const void *v_pool, const int32_t *block_table,
                      int32_t block_table_stride, const int32_t *context_lens, int32_t batch,
                      int32_t total_q, int32_t max_q_len, int32_t max_context_len, void *out,
                      float *lse, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Bytes of DEVICE staging that ta_kv_page_restore / ta_kv_page_evict need at
 * least (none: 0), and the size from which they switch from touching the
 * pinned host pages directly inside the scatter / gather kernel to staging
 * them through large copies over the host link.
 */
TA_API size_t ta_restore_staging_min_bytes(int32_t n_pages);
TA_API size_t ta_restore_staging_full_bytes(int32_t n_pages, size_t page_bytes);

/*
 * KV page restore (Sec. 4.3: Restore re-admits a paused program whose KV cache
 * was released; App. A.2/A.4: the pages come back from host memory over the
 * host link).  Bytes only, bit-exact:
 *     k_pool[dst_slots[i]] = host_k[i],  v_pool[dst_slots[i]] = host_v[i],  i < n_pages
 * Pages not named in dst_slots are left untouched.
 *
 *   k_pool,v_pool DEVICE, pool_pages pages of page_bytes each, contiguous
 *   page_bytes    bytes of one page of K over all kv heads (Hkv*16*128*2), multiple of 16,
 *                 below 2 GiB (else TA_ERR_UNSUPPORTED)
 *   host_k,host_v HOST, pinned (hipHostMalloc), [n_pages][page_bytes] contiguous;
 *                 must stay valid until the stream reaches the end of this call
 *   dst_slots     HOST int32 [n_pages] (pageable is fine), distinct, each in [0, pool_pages).
 *                 The list is read completely before the call returns (it travels inside
 *                 the kernel arguments, 960 slots per launch): the caller may free or reuse
 *                 it at once, and the call waits for nothing on the stream.
 *   staging       DEVICE scratch, 256-byte aligned, or NULL with staging_bytes == 0.
 *                 With at least ta_restore_staging_full_bytes() the pages travel as
 *                 large host-to-device copies into staging and a kernel scatters them;
 *                 with less, the scatter kernel reads the pinned host pages directly.
 *                 With staging for two rounds of at least 256 pages (4 * 256 * page_bytes)
 *                 and more pages than one round, the copies of one round (on hip_stream)
 *                 run beside the scatter of the round before, which goes to a stream of
 *                 the library's own (one per GPU, default priority, created at the first
 *                 such call); that stream starts after everything enqueued on hip_stream
 *                 before the call, and hip_stream has waited for it when it reaches the
 *                 end of the call: the ordering the caller sees is that of a single
 *                 stream.  (Not while hip_stream is being captured into a graph: then one
 *                 stream does it all.)
 *                 This is the route to take when attention runs on another stream
 *                 meanwhile: the host link stays busy while a scatter launch waits for
 *                 compute units.  Staged calls on one GPU enqueue one at a time (a lock).
 */
TA_API int ta_kv_page_restore(void *k_pool, void *v_pool, size_t page_bytes, const void *host_k,
                       const void *host_v, const int32_t *dst_slots, int32_t n_pages,
                       int32_t pool_pages, void *staging, size_t staging_bytes, void *hip_stream);

/*
 * KV page evict, the inverse of ta_kv_page_restore (Sec. 4.3: Pause releases a
 * program's KV cache; App. A.2/A.4: the pages are kept in host memory instead
 * of being recomputed later).  Bytes only, bit-exact:
 *     host_k[i] = k_pool[src_slots[i]],  host_v[i] = v_pool[src_slots[i]],  i < n_pages
 * The pools are only read; the caller frees the slots by forgetting them.
 *
 *   k_pool,v_pool DEVICE, pool_pages pages of page_bytes each, contiguous, only read
 *   host_k,host_v HOST, PINNED (hipHostMalloc), written: [n_pages][page_bytes], 16-byte aligned
 *   src_slots     HOST int32 [n_pages], each in [0, pool_pages); a slot may repeat.
 *                 Read completely before the call returns, as for ta_kv_page_restore.
 *   staging       DEVICE, 256-byte aligned, or NULL with staging_bytes == 0; from
 *                 ta_restore_staging_full_bytes on the pages are gathered into it and
 *                 leave through large device-to-host copies, below that the gather kernel
 *                 writes the pinned host pages itself.  With staging for two rounds the
 *                 gathers run on the library's own stream beside the copy of the round
 *                 before, as for ta_kv_page_restore.
 * host_k / host_v hold the pages once hip_stream has reached the end of the call.
 * Errors as for ta_kv_page_restore (nothing is enqueued when the slot list is bad).
 */
TA_API int ta_kv_page_evict(const void *k_pool, const void *v_pool, size_t page_bytes, void *host_k,
                     void *host_v, const int32_t *src_slots, int32_t n_pages, int32_t pool_pages,
                     void *staging, size_t staging_bytes, void *hip_stream);

/*
 * KV append (Sec. 2.1: the context c_{t+1} extends c_t, so a program's cache
 * grows at its tail; it is what makes the precondition of ta_append_prefill and
 * ta_paged_decode true: the new tokens' keys and values are in their pages).
 * Program b's n_b = cu_new_lens[b+1] - cu_new_lens[b] new tokens become its
 * tokens context_lens[b] - n_b .. context_lens[b] - 1 (context_lens counts them
 * already); bit patterns are copied:
 *     pool[block_table[b][t / 16]][g][t % 16][:] = new[cu_new_lens[b] + i][g][:],
 *     t = context_lens[b] - n_b + i,  for K and for V, every kv head g
 * (into a TA_KV_FP8_E4M3 cache: the E4M3 codes of new / k_scale and new / v_scale, see the
 * formats above).  The pages named by the block table must exist; no other byte changes.
 *
 *   new_k,new_v   DEVICE bf16 [total_new][Hkv][128], programs packed back to back
 *   cu_new_lens   DEVICE int32 [batch+1], non-decreasing, cu_new_lens[0] = 0
 *   k_pool,v_pool DEVICE, written; layout per desc
 *   total_new     HOST, equals cu_new_lens[batch]
 * Other arguments as for ta_paged_decode.  Two programs that share a tail page
 * and both write it race (forked programs share full prefix pages only).
 * Returns TA_ERR_INVALID_ARG for NULL or misaligned pointers or negative sizes.
 */
TA_API int ta_kv_append(const ta_attn_desc *desc, const void *new_k, const void *new_v,
                 const int32_t *cu_new_lens, void *k_pool, void *v_pool,
                 const int32_t *block_table, int32_t block_table_stride,
                 const int32_t *context_lens, int32_t batch, int32_t total_new, void *hip_stream);

/*
 * Instrumentation for benchmarks (no paper passage: it measures, it computes
 * nothing).  While both events are non-NULL, ta_paged_decode and
 * ta_append_prefill record start_event immediately before and stop_event
 * immediately after their dominant kernel (the split-K chunk kernel, the MFMA
 * tile kernel) on the call's stream, so that hipEventElapsedTime(start, stop)
 * is that kernel's duration.  The events are hipEvent_t passed as void*, owned
 * by the caller, and apply to the calling thread's next calls until replaced;
 * NULLs switch the recording off.
 */
TA_API void ta_profile_events(void *start_event, void *stop_event);

#ifdef __cplusplus
}
#endif
#endif /* TA_H */
