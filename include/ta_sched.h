/*
 * ta_sched.h -- C ABI of the program-aware scheduling tick (host code, no GPU).
 *
 * ThunderAgent decides every Delta-t which programs keep their KV cache on which
 * backend (Sec. 4.3).  This header carries that decision and nothing else: the
 * caller owns the program table and acts on the decisions (ta_kv_page_evict for
 * a Pause, ta_kv_page_restore or a re-prefill for a Restore; see ta.h).
 *
 * One tick, for B backends that each hold capacity_tokens tokens of KV cache:
 *   load(L) = sum of c_p over active reasoning programs on L
 *           + sum of c_q * f(t_q) over active acting programs on L,  f(t) = decay_base^(-t)
 *             (the decayed thrashing check of Sec. 4.3; decay_base = 2 in Sec. 5.1)
 *   Pause:   while load(L) > lambda_max * capacity_tokens, pause the active program
 *            on L with the largest S_pause = 1/c + [tau = Acting]   (ties: lower id)
 *   Restore: over all paused programs in descending S_restore = 1/c + [tau = Reasoning]
 *            (ties: lower id): bind the program to the backend with the most room below
 *            lambda_max * capacity_tokens among those with load < lambda_min * capacity_tokens
 *            (ties: lower index) if its weight (c, or c f(t) while acting) still fits below
 *            lambda_max * capacity_tokens there; otherwise it stays in the waiting queue
 *            (one global queue for all backends).
 * Loads are summed in table order in double precision; a program paused in this
 * tick may be restored on another backend in the same tick.
 */
#ifndef TA_SCHED_H
#define TA_SCHED_H

#include <stdint.h>

#include "ta.h"

#ifdef __cplusplus
extern "C" {
#endif

enum { TA_PHASE_REASONING = 0, TA_PHASE_ACTING = 1 };
enum { TA_STATUS_ACTIVE = 0, TA_STATUS_PAUSED = 1, TA_STATUS_TERMINATED = 2 };

/* The fields of the paper's program tuple <ID, c, T, L, tau, s> that the policy reads. */
typedef struct ta_program {
    int32_t id;         /* ID */
    int32_t context;    /* c: tokens in the context, >= 1 */
    int32_t backend;    /* L: backend index in [0, n_backends), or -1 when unbound */
    int32_t phase;      /* tau: TA_PHASE_* */
    int32_t status;     /* s: TA_STATUS_* */
    float acting_time;  /* t: time the current tool call has been running (read while acting), >= 0 */
} ta_program;

typedef struct ta_sched_config {
    double capacity_tokens;  /* C_total of one backend */
    double lambda_max;       /* high watermark (the paper runs with 1) */
    double lambda_min;       /* low watermark  (the paper runs with 1) */
    double decay_base;       /* f(t) = decay_base^(-t); >= 1; 1 switches the decay off */
} ta_sched_config;

/*
 * Runs one tick over the HOST table `programs` (n_programs entries), updating the
 * status and backend of the programs it pauses or restores.
 *
 *   paused_ids        HOST int32 [n_programs], receives the ids in pause order
 *   restored_ids      HOST int32 [n_programs], receives the ids in restore order
 *   restored_backends HOST int32 [n_programs], the backend each restored program was bound to
 *   n_paused, n_restored  HOST, receive the counts
 *
 * Returns TA_OK, or TA_ERR_INVALID_ARG (nothing modified) for NULL pointers, negative
 * counts, a non-finite or negative capacity or watermark, decay_base < 1, or a table
 * entry with context < 1, an unknown phase or status, an active program whose backend
 * is out of range, or a negative or non-finite acting time.
 */
TA_API int ta_sched_tick(const ta_sched_config *config, ta_program *programs, int32_t n_programs,
                         int32_t n_backends, int32_t *paused_ids, int32_t *n_paused,
                         int32_t *restored_ids, int32_t *restored_backends, int32_t *n_restored);

#ifdef __cplusplus
}
#endif
#endif /* TA_SCHED_H */
