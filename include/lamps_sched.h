/*
 * liblamps, host side: the LAMPS scheduler (arXiv 2410.18248, Algorithm 1).
 *
 * The paper ranks API-augmented requests by the memory they will hold over
 * time, given how their KV cache will be treated while an API call lasts
 * (Preserve / Discard / Swap, chosen before the request runs as the least of
 * the memory wastes of equations (1)-(3)), forms the running batch anew every
 * iteration, and moves requests that have waited too long to the head of the
 * queue.  This header exposes
 *   - the closed forms: equations (1)-(3), their argmin, and the
 *     memory-over-time rank function of Section 4.2 / 4.3;
 *   - a scheduler object that owns the requests' state machines and is
 *     stepped once per iteration: lamps_sched_next_batch() says which
 *     requests run and what each has to bring back first (swap-in, recompute),
 *     the caller executes the iteration on the GPU (lamps.h) or lets the cost
 *     model stand in for it, lamps_sched_commit() advances time and reports
 *     which requests reached an API call (and by which strategy they leave)
 *     or finished.  lamps_sched_run() loops the two on the cost model.
 *
 * Plain C ABI, host memory only, no GPU call anywhere in this header's
 * functions.  Every function that returns int returns a lamps_status
 * (lamps.h): LAMPS_OK, LAMPS_ERR_INVALID, LAMPS_ERR_RANGE, LAMPS_ERR_NOMEM.
 * A scheduler is not thread-safe.
 *
 * Units are the caller's: seconds and tokens in production; the paper's
 * worked example (Section 3.1) counts time in iterations (cost.unit = 1).
 *
 * Readings where the paper is silent:
 *   - A request is a list of segments: output tokens, then one API call
 *     (duration, response tokens); the last segment has no call
 *     (Section 4.2, "Multi-API").
 *   - "runningBatch is not full": fewer than max_batch requests and the
 *     memory the candidate needs is free.  At the start of a segment a
 *     request needs room for the whole segment (context to swap in or
 *     recompute, the API response, the segment's tokens); in the middle of
 *     one, room for one token (or one recompute chunk).  Memory is what
 *     requests hold now, not what they may come to hold.
 *   - Every unfinished request outside an API call is in the waiting queue
 *     at every iteration; a displaced request keeps its memory.
 *   - An iteration in which a request recomputes context or processes an API
 *     response yields no new token for it.
 *   - Rank ties: earlier arrival, then lower id.
 *   - If nothing can run while waiting requests hold memory, the worst-ranked
 *     of them is discarded (it recomputes later); if none holds memory the
 *     engine idles until the next arrival or API return.
 */
#ifndef LAMPS_SCHED_H
#define LAMPS_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lamps_sched lamps_sched; /* opaque, library-owned */

typedef enum { LAMPS_PRESERVE = 0, LAMPS_DISCARD = 1, LAMPS_SWAP = 2, LAMPS_HANDLING_AUTO = -1 } lamps_handling;

typedef enum {
    LAMPS_POLICY_FCFS = 0,      /* arrival order (the baseline the paper compares with)      */
    LAMPS_POLICY_SJF = 1,       /* remaining tokens to process                               */
    LAMPS_POLICY_SJF_TOTAL = 2, /* ... plus the remaining API time, in iterations            */
    LAMPS_POLICY_LAMPS = 3,     /* memory over time of the current segment (Section 4.3)     */
    LAMPS_POLICY_FIXED = 4      /* the priority given with the request                       */
} lamps_policy;

/* Times of the engine being scheduled:
 *   iteration = it_a + it_b * (context tokens of the running batch)
 *               + fwd_b * (tokens recomputed or first processed in it)
 *               + (sw_a + sw_b * tokens swapped in or out in it)   if swap_stalls
 *   T_fwd(C)  = fwd_a + fwd_b * C        T_swap(C) = sw_a + sw_b * C
 * unit != 0 (the worked example of Section 3.1): every iteration takes exactly 1,
 * recomputing a discarded context takes one iteration (T_fwd = 1) and swaps cost
 * nothing (T_swap = 0). */
typedef struct {
    double it_a, it_b, fwd_a, fwd_b, sw_a, sw_b;
    int32_t swap_stalls; /* the paper's substrate: a swap interrupts the forward pass (Section 4.3) */
    int32_t unit;
} lamps_cost_model;

typedef struct {
    int32_t policy;               /* lamps_policy                                            */
    int32_t max_batch;            /* requests per iteration                                  */
    int64_t memory_tokens;        /* KV budget, tokens                                       */
    int32_t starvation_threshold; /* iterations left out of the batch before a request goes
                                     to the head of the queue, in the iteration in which its
                                     counter gets there (Section 4.4; the paper uses 100)    */
    int32_t score_refresh;        /* iterations a cached score stays valid (Section 5: 1, or
                                     10 on ToolBench)                                        */
    int64_t recompute_chunk;      /* most tokens one request recomputes per iteration        */
    double c_other;               /* estimated context of the other requests in the batch,
                                     tokens (C_other of equation (2); C_batch = C_i + it)    */
    double bytes_per_token;       /* M of equations (1)-(3) (lamps_kv_bytes_per_token)       */
    lamps_cost_model cost;
} lamps_sched_config;

typedef struct {
    int32_t n_out;        /* tokens generated in this segment, >= 1                          */
    double api_duration;  /* the call that ends the segment; < 0: none (last segment only)   */
    int32_t api_response; /* tokens the call returns into the context                        */
    int32_t handling;     /* lamps_handling, or LAMPS_HANDLING_AUTO: least waste             */
} lamps_segment;

/* What a request of the running batch does in the iteration. */
typedef struct {
    int64_t id;
    int64_t swap_in;   /* tokens to bring back from host memory before it runs               */
    int64_t recompute; /* tokens to run through the model (discarded context, prompt, API
                          response); if > 0 the request generates no token this iteration   */
    int64_t context;   /* context tokens after the iteration                                 */
} lamps_batch_entry;

/* What happened to a request at the end of the iteration. */
typedef struct {
    int64_t id;
    int32_t what;      /* 0: reached an API call, 1: finished                                */
    int32_t handling;  /* what == 0: lamps_handling by which its cache leaves                */
    int64_t context;   /* its context tokens at that moment                                  */
} lamps_sched_event;

/* ---- closed forms ---- */

/* Equation (1): T_INT * C_i * M. */
double lamps_waste_preserve(double t_int, double c_i, double m);
/* Equation (2): T_fwd(C_i) * C_i * M + T_fwd(C_i) * C_other * M. */
double lamps_waste_discard(double t_fwd_ci, double c_i, double c_other, double m);
/* Equation (3): 2 * T_swap(C_i) * C_batch * M. */
double lamps_waste_swap(double t_swap_ci, double c_batch, double m);
/* The lamps_handling of least waste, C_batch = C_i + C_other; ties go to the
 * earlier of Preserve, Discard, Swap (Section 4.2). */
int lamps_handling_strategy(double t_int, double c_i, double c_other, double m, double t_fwd_ci,
                            double t_swap_ci);
/* Integral of a request's memory (tokens) over time (Section 4.2, the
 * memory-over-time figure): c0 tokens of context, n1 tokens generated (tau
 * each), an API call of t_int handled by `strategy` with C = c0 + n1 tokens of
 * context (Preserve: t_int * C; Discard: T_fwd(C) * C; Swap: 2 T_swap(C) * C),
 * rho tokens returned, n2 more generated. */
double lamps_memory_over_time(int strategy, int64_t c0, int64_t n1, double t_int, int64_t rho,
                              int64_t n2, double tau, double t_fwd_c, double t_swap_c);

/* ---- scheduler ---- */

int lamps_sched_create(const lamps_sched_config *cfg, lamps_sched **out);
int lamps_sched_destroy(lamps_sched *s);
/* Adds a request (before or between iterations).  segments are copied.
 * Errors: INVALID (null, n_segments < 1, a middle segment without a call, the
 * last one with a call, n_out < 1, negative sizes), DUP (id already added). */
int lamps_sched_add(lamps_sched *s, int64_t id, double arrival, int32_t prompt_tokens,
                    const lamps_segment *segments, int32_t n_segments, double priority);

/* Steps 1-6 of an iteration of Algorithm 1 at the current time: arrivals and
 * finished API calls enter the waiting queue, scores, sort, batch formation,
 * starvation counters (a request that reaches the threshold is tagged and the
 * batch formed once more with it at the head).  If nothing can run, the worst-ranked waiting request
 * that holds memory is discarded, or, if none does, time moves to the next
 * arrival or API return; then the steps repeat.
 * Writes the batch (<= cap entries; cap >= max_batch) and *n.  *n == 0 means
 * every request has finished.  Errors: INVALID, RANGE (cap too small), NOMEM
 * (a request needs more memory than the whole budget). */
int lamps_sched_next_batch(lamps_sched *s, lamps_batch_entry *batch, int32_t cap, int32_t *n);
/* Ends the iteration started by lamps_sched_next_batch: requests generate
 * their token (or have recomputed), time advances by `iteration_time`
 * (measured by the caller), or by the cost model's if iteration_time < 0;
 * requests that reached an API call leave by their handling strategy, finished
 * ones are retired.  Writes what happened (<= cap events; cap >= max_batch).
 * Errors: INVALID (no batch pending), RANGE. */
int lamps_sched_commit(lamps_sched *s, double iteration_time, lamps_sched_event *events,
                       int32_t cap, int32_t *n);
/* Requests that lamps_sched_next_batch discarded because nothing fitted (their
 * cache is to be dropped; they recompute it when they run again), oldest first;
 * each is reported once.  Writes at most cap ids and *n.  A caller that executes
 * the iterations for real drains this after every lamps_sched_next_batch. */
int lamps_sched_take_discards(lamps_sched *s, int64_t *ids, int32_t cap, int32_t *n);
/* next_batch / commit on the cost model until every request has finished. */
int lamps_sched_run(lamps_sched *s);

double lamps_sched_now(const lamps_sched *s);
/* Completion and first-token times (absolute), and the handling strategy chosen
 * for each of its segments' calls (n_handling entries written at most).
 * A time is < 0 while it has not happened.  Errors: INVALID, RANGE (unknown id). */
int lamps_sched_result(const lamps_sched *s, int64_t id, double *completion, double *first_token,
                       int32_t *handling, int32_t n_handling);
/* iterations executed, peak memory held (tokens), out-of-memory discards. */
int lamps_sched_stats(const lamps_sched *s, int64_t *iterations, int64_t *peak_memory,
                      int64_t *preemptions);

#ifdef __cplusplus
}
#endif
#endif /* LAMPS_SCHED_H */
