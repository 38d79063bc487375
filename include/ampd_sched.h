/*
 * ampd_sched.h -- C ABI of libampd_sched: the two online scheduling decisions that consume the
 * cost model of the attention path (host code only, no GPU).
 *
 *   ampd_route    adaptive routing of one prefill task (paper Section 4.1, Algorithm 1, with the
 *                 local / remote cost estimates of Eq. 1 and Eq. 2)
 *   ampd_reorder  TTFT-aware reordering of the head window of a prefill queue (Section 4.2,
 *                 Algorithm 2, Eq. 3 and Eq. 4)
 *
 * All pointers are HOST memory, read during the call only.  Times are seconds (any unit works as
 * long as it is the same everywhere).  Random choices are inputs: the caller draws the visiting
 * order of Algorithm 1's first loop.
 *
 * Readings where the paper leaves a choice open: ties in the final arg-min of Algorithm 1 go to
 * the first of {local, remote_0, remote_1, ...}; Algorithm 2 enumerates orderings in
 * lexicographic order of window positions, identity first, and keeps the first ordering that
 * reaches the best count; a task counts as "postponed" by an ordering when it is placed later
 * than its current position in the queue.
 */
#ifndef AMPD_SCHED_H
#define AMPD_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct { int32_t l_hist, l_incr; } ampd_task;     /* history length, incremental length */

/* T_pre(l_hist, l_incr) of one worker: one line alpha + beta * l_hist per l_incr bucket (ascending,
 * n >= 1); between buckets the two neighbouring lines are interpolated linearly in log(l_incr),
 * outside them the nearest line is used. */
typedef struct {
    int32_t n;
    const double *l_incr, *alpha, *beta;
} ampd_tpre_model;

typedef struct { double alpha, beta; } ampd_tkv_model;   /* T_kv(l_ctx) = alpha + beta * l_ctx for one (source, destination) pair */

double ampd_t_pre(const ampd_tpre_model *m, int32_t l_hist, int32_t l_incr);

typedef struct {
    int32_t n_prefill_workers;             /* >= 0 */
    const double *ttft_hat;                /* [n] windowed TTFT statistic of every prefill worker */
    double itl_hat;                        /* windowed ITL statistic of the task's decode worker */
    double ttft_thres, itl_thres;          /* SLO thresholds */
    double alpha, beta;                    /* slack factors (paper default 0.9, 0.85) */
    const int32_t *visit_order;            /* [n] permutation of 0..n-1: the random order of the first loop */
    const ampd_tpre_model *decode_model;   /* theta_d */
    const ampd_tpre_model *prefill_models; /* [n] theta_{p_i} */
    const ampd_tkv_model *kv_d2p;          /* [n] history KV, decode worker -> prefill worker i */
    const ampd_tkv_model *kv_p2d;          /* [n] incremental KV, prefill worker i -> decode worker */
    const ampd_task *local_queue;          /* prefill queue of the decode worker */
    int32_t local_queue_len;
    const ampd_task *const *remote_queues; /* [n] prefill queue of every prefill worker */
    const int32_t *remote_queue_len;       /* [n] */
} ampd_route_input;

#define AMPD_ROUTE_LOCAL (-1)
#define AMPD_ROUTE_ERROR (-2)

/* Returns AMPD_ROUTE_LOCAL, the index i of the chosen prefill worker, or AMPD_ROUTE_ERROR on invalid
 * input.  costs (optional, [n + 1]) receives t_local (Eq. 1) followed by every t_remote_i (Eq. 2); they are
 * computed on every valid call, whichever rule decides; *reason (optional) gets 0 = TTFT slack, 1 = ITL slack, 2 = cost. */
int32_t ampd_route(const ampd_route_input *in, ampd_task task, double *costs, int32_t *reason);

typedef struct {
    double t_pre;            /* estimated execution time of the task */
    double enqueue_time;
    int32_t postponed;       /* postponement counter */
    int32_t reserved;
} ampd_queued_task;

#define AMPD_MAX_WINDOW 8

/* window: the first n <= w <= AMPD_MAX_WINDOW tasks of the queue, in queue order.  Writes the chosen
 * ordering to perm (perm[k] = window index of the task placed k-th; perm[0] is dequeued next), the
 * updated counters to postponed_out, and the predicted number of TTFT-satisfying tasks to *satisfied.
 * Returns 0, or -1 on invalid input. */
int32_t ampd_reorder(const ampd_queued_task *window, int32_t n, int32_t w, double now, double ttft_thres,
                     int32_t *perm, int32_t *postponed_out, int32_t *satisfied);

#ifdef __cplusplus
}
#endif
#endif
