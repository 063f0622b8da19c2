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

/*
 * ---------------------------------------------------------------------------
 * Trace-driven simulator of the policy over several backends (host code, no GPU).
 *
 * It owns what the paper's middleware owns (Sec. 4.1, 4.3; App. B): the program table, the
 * periodic decision (ta_sched_tick every Delta-t, here `steps_per_tick` decode steps), the
 * global waiting queue over n_backends backends, and in addition each backend's page
 * allocator, so that every decision comes out as an ordered list of events that a driver turns
 * into calls of ta.h on real page pools: a Pause is a ta_kv_page_evict of the program's pages,
 * a Restore a ta_kv_page_restore into the pages named, a tool result a ta_kv_append plus
 * ta_append_prefill of its tokens, a reasoning step a ta_kv_append plus ta_paged_decode.
 * The workflow of a program alternates reasoning turns and tool calls (Sec. 2.1); their
 * lengths, the tool latencies (heavy-tailed in the paper's traces, App. B) and the sizes of
 * the tool outputs are INPUTS, drawn by the caller: the simulator draws no random number, so
 * its decisions are a function of the trace alone.
 *
 * One tick, in this order:
 *   1. tools: every acting program's tool time grows by time_per_tick and its remaining
 *      latency drops by one tick; a tool that has returned makes its program reasoning again,
 *      with the tool's output waiting to be prefilled and the next turn's tokens to decode;
 *   2. the policy: ta_sched_tick over all backends; paused programs give up their pages
 *      (TA_SIM_EVICT), restored ones get pages on their new backend (TA_SIM_RESTORE);
 *   3. every active reasoning program with tool output waiting grows by it (TA_SIM_PREFILL);
 *   4. steps_per_tick decode steps: every active reasoning program with tokens left in its
 *      turn grows by one token per step (TA_SIM_DECODE, `tokens` = index of the step);
 *   5. a finished turn starts the next tool call, or ends the program when the trace is
 *      used up (TA_SIM_RELEASE: its pages are free again).
 * A program whose context would exceed max_context is released instead of growing.
 *
 * What the paper leaves to the backend: the decayed check counts an idle acting program for
 * less than the pages it still holds, in the expectation that the backend reclaims them when
 * it needs room (Sec. 4.3).  The simulator plays that part of the backend explicitly: when a
 * backend has no free page for a grant, it takes the pages of the active program on that
 * backend that is waiting for a tool, has the highest S_pause and is not being served in this
 * tick (TA_SIM_EVICT_FORCED; the program joins the waiting queue); if there is none, the
 * program asking is the one that leaves (a restore is simply not carried out).
 * ---------------------------------------------------------------------------
 */
typedef struct ta_sim ta_sim;

typedef struct ta_sim_config {
    int32_t n_programs;
    int32_t n_backends;
    int32_t n_turns;         /* reasoning turns per program in the trace */
    int32_t pool_pages;      /* physical pages (16 tokens each) of every backend */
    int32_t steps_per_tick;  /* decode steps between two scheduling decisions (the paper's Delta-t) */
    int32_t max_context;     /* tokens; a program that would grow beyond it is released */
    double time_per_tick;    /* Delta-t in the time unit of f(t) */
    ta_sched_config sched;   /* capacity_tokens is per backend */
} ta_sim_config;

enum {
    TA_SIM_EVICT = 1,         /* Pause: `slots` = the program's pages in logical order, now free */
    TA_SIM_EVICT_FORCED = 2,  /* the backend reclaimed an idle cache (see above); otherwise as EVICT */
    TA_SIM_RESTORE = 3,       /* `slots` = the pages the program's context goes into, in logical order */
    TA_SIM_PREFILL = 4,       /* `tokens` new tokens appended; `slots` = pages newly added at the tail */
    TA_SIM_DECODE = 5,        /* one new token in decode step `tokens`; `slots` = the page added, if any */
    TA_SIM_RELEASE = 6        /* the program ended; `slots` = its pages, now free (none if it was paused) */
};

typedef struct ta_sim_event {
    int32_t kind;        /* TA_SIM_* */
    int32_t program;     /* id = index into the trace arrays */
    int32_t backend;     /* the backend whose pool `slots` refer to */
    int32_t tokens;      /* see the kinds */
    int32_t context;     /* the program's context length after the event */
    int32_t first_slot;  /* range [first_slot, first_slot + n_slots) of the tick's slot array */
    int32_t n_slots;
} ta_sim_event;

/*
 * Creates a simulator (HOST allocation; the only calls of this library that allocate).  All
 * programs start paused in the waiting queue, reasoning, with initial_context tokens held on the
 * host and their first turn ahead.
 *   initial_context  HOST int32 [n_programs], each in [1, max_context]
 *   turn_tokens      HOST int32 [n_programs][n_turns], tokens decoded in each turn, >= 1
 *   tool_ticks       HOST int32 [n_programs][n_turns], latency of the tool call after each turn, >= 1
 *   tool_tokens      HOST int32 [n_programs][n_turns], tokens of that tool's output, >= 1
 * The arrays are copied.  Returns NULL for invalid arguments.
 */
TA_API ta_sim *ta_sim_create(const ta_sim_config *config, const int32_t *initial_context,
                             const int32_t *turn_tokens, const int32_t *tool_ticks,
                             const int32_t *tool_tokens);
TA_API void ta_sim_destroy(ta_sim *sim);

/*
 * Advances the simulation by one tick and keeps the tick's events until the next call.
 * n_events / n_slots receive their counts.  Returns TA_OK or TA_ERR_INVALID_ARG (NULL).
 */
TA_API int ta_sim_tick(ta_sim *sim, int32_t *n_events, int32_t *n_slots);

/* Copies the last tick's events and slot array (sizes from ta_sim_tick) to HOST buffers. */
TA_API int ta_sim_fetch(const ta_sim *sim, ta_sim_event *events, int32_t *slots);

/* Snapshot of the program table (HOST ta_program [n_programs]). */
TA_API int ta_sim_programs(const ta_sim *sim, ta_program *out);

/*
 * The pages of one program in logical order (empty while it is paused or ended).  Copies at
 * most max_pages entries to HOST `out`; returns the number of pages the program holds, or -1.
 */
TA_API int32_t ta_sim_page_table(const ta_sim *sim, int32_t program, int32_t *out, int32_t max_pages);

#ifdef __cplusplus
}
#endif
#endif /* TA_SCHED_H */
