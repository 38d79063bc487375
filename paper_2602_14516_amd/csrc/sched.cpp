// Host-side scheduling decisions that consume the attention cost model (see include/ampd_sched.h).
#include "ampd_sched.h"

#include <algorithm>
#include <cmath>
#include <numeric>

extern "C" {

double ampd_t_pre(const ampd_tpre_model* m, int32_t l_hist, int32_t l_incr) {
    if (!m || m->n <= 0) return NAN;
    const double q = std::log(std::max<double>(l_incr, 1e-30));
    int hi = 0;
    while (hi < m->n && std::log(m->l_incr[hi]) < q) ++hi;            // first bucket >= l_incr
    if (hi == 0) return m->alpha[0] + m->beta[0] * l_hist;
    if (hi == m->n) return m->alpha[m->n - 1] + m->beta[m->n - 1] * l_hist;
    const int lo = hi - 1;
    const double a = std::log(m->l_incr[lo]), b = std::log(m->l_incr[hi]);
    const double w = b > a ? (q - a) / (b - a) : 0.0;
    const double t_lo = m->alpha[lo] + m->beta[lo] * l_hist, t_hi = m->alpha[hi] + m->beta[hi] * l_hist;
    return (1.0 - w) * t_lo + w * t_hi;
}

// Adaptive routing (Algorithm 1 with the cost estimates of Eq. 1 and Eq. 2), in three parts: check the
// whole input, cost every candidate placement once, then decide.  The decision prefers, in this order, a prefill
// worker whose windowed TTFT leaves slack (first in the caller's visiting order), the decode worker itself when
// its windowed ITL leaves slack, and otherwise the cheapest candidate.
namespace {

double queue_time(const ampd_tpre_model* m, const ampd_task* q, int32_t len) {
    double t = 0.0;
    for (int32_t k = 0; k < len; ++k) t += ampd_t_pre(m, q[k].l_hist, q[k].l_incr);
    return t;
}

bool route_input_ok(const ampd_route_input* in) {
    if (!in || in->n_prefill_workers < 0 || !in->decode_model) return false;
    const int n = in->n_prefill_workers;
    if (n > 0 && (!in->ttft_hat || !in->visit_order || !in->prefill_models || !in->kv_d2p || !in->kv_p2d ||
                  !in->remote_queues || !in->remote_queue_len))
        return false;
    if (in->local_queue_len < 0 || (in->local_queue_len > 0 && !in->local_queue)) return false;
    for (int i = 0; i < n; ++i) {
        if (in->visit_order[i] < 0 || in->visit_order[i] >= n) return false;
        if (in->remote_queue_len[i] < 0 || (in->remote_queue_len[i] > 0 && !in->remote_queues[i])) return false;
    }
    return true;
}

}  // namespace

int32_t ampd_route(const ampd_route_input* in, ampd_task task, double* costs, int32_t* reason) {
    if (!route_input_ok(in)) return AMPD_ROUTE_ERROR;
    const int n = in->n_prefill_workers;

    // candidate 0 = local (Eq. 1: the task plus everything queued on the decode worker); candidate 1 + i = prefill
    // worker i (Eq. 2: the task there, its history KV over, its incremental KV back, and that worker's queue)
    int32_t cheapest = AMPD_ROUTE_LOCAL;
    double cheapest_t = ampd_t_pre(in->decode_model, task.l_hist, task.l_incr) +
                        queue_time(in->decode_model, in->local_queue, in->local_queue_len);
    if (costs) costs[0] = cheapest_t;
    for (int i = 0; i < n; ++i) {
        const ampd_tpre_model* m = &in->prefill_models[i];
        const double t = ampd_t_pre(m, task.l_hist, task.l_incr) + in->kv_d2p[i].alpha + in->kv_d2p[i].beta * task.l_hist +
                         in->kv_p2d[i].alpha + in->kv_p2d[i].beta * task.l_incr +
                         queue_time(m, in->remote_queues[i], in->remote_queue_len[i]);
        if (costs) costs[1 + i] = t;
        if (t < cheapest_t) {                         // strict: ties stay with the earlier candidate
            cheapest_t = t;
            cheapest = i;
        }
    }

    int32_t why = 2, choice = cheapest;
    if (in->itl_hat <= in->beta * in->itl_thres) {
        why = 1;
        choice = AMPD_ROUTE_LOCAL;
    }
    for (int k = n - 1; k >= 0; --k) {                // the first worker with slack in visiting order wins
        const int i = in->visit_order[k];
        if (in->ttft_hat[i] <= in->alpha * in->ttft_thres) {
            why = 0;
            choice = i;
        }
    }
    if (reason) *reason = why;
    return choice;
}

// Algorithm 2 with Eq. 3 (completion time of the k-th task of an ordering = prefix sum of the
// estimated execution times) and Eq. 4 (count of tasks whose waiting time so far plus completion
// time stays within the TTFT threshold).
int32_t ampd_reorder(const ampd_queued_task* window, int32_t n, int32_t w, double now, double ttft_thres,
                     int32_t* perm, int32_t* postponed_out, int32_t* satisfied) {
    if (!window || !perm || n < 0 || w < 1 || n > w || w > AMPD_MAX_WINDOW) return -1;
    int idx[AMPD_MAX_WINDOW];
    std::iota(idx, idx + n, 0);
    int best[AMPD_MAX_WINDOW];
    int best_s = -1;
    do {
        bool feasible = true;                         // no task with an exhausted counter moves back
        for (int k = 0; k < n && feasible; ++k)
            if (k > idx[k] && window[idx[k]].postponed >= w) feasible = false;
        if (!feasible) continue;
        double c = 0.0;
        int s = 0;
        for (int k = 0; k < n; ++k) {
            c += window[idx[k]].t_pre;
            if ((now - window[idx[k]].enqueue_time) + c <= ttft_thres) ++s;
        }
        if (s > best_s) {
            best_s = s;
            std::copy(idx, idx + n, best);
        }
    } while (std::next_permutation(idx, idx + n));
    for (int k = 0; k < n; ++k) perm[k] = best[k];
    if (postponed_out) {
        for (int i = 0; i < n; ++i) postponed_out[i] = window[i].postponed;
        for (int k = 0; k < n; ++k)
            if (k > best[k]) ++postponed_out[best[k]];
    }
    if (satisfied) *satisfied = std::max(best_s, 0);
    return 0;
}

}  // extern "C"
