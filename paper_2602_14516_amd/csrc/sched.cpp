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

// Algorithm 1.  Lines 1-3: a prefill worker with TTFT slack, in the given random order.  Lines 4-5:
// local execution if the decode worker has ITL slack.  Lines 6-9: the cheaper of Eq. 1 and Eq. 2.
int32_t ampd_route(const ampd_route_input* in, ampd_task task, double* costs, int32_t* reason) {
    if (!in || in->n_prefill_workers < 0 || !in->decode_model) return AMPD_ROUTE_ERROR;
    const int n = in->n_prefill_workers;
    if (n > 0 && (!in->ttft_hat || !in->visit_order || !in->prefill_models || !in->kv_d2p || !in->kv_p2d ||
                  !in->remote_queues || !in->remote_queue_len))
        return AMPD_ROUTE_ERROR;
    if (in->local_queue_len < 0 || (in->local_queue_len > 0 && !in->local_queue)) return AMPD_ROUTE_ERROR;
    for (int k = 0; k < n; ++k) {
        const int i = in->visit_order[k];
        if (i < 0 || i >= n) return AMPD_ROUTE_ERROR;
        if (in->ttft_hat[i] <= in->alpha * in->ttft_thres) {
            if (reason) *reason = 0;
            return i;
        }
    }
    if (in->itl_hat <= in->beta * in->itl_thres) {
        if (reason) *reason = 1;
        return AMPD_ROUTE_LOCAL;
    }
    // Eq. 1: the task itself plus everything queued on the decode worker
    double t_local = ampd_t_pre(in->decode_model, task.l_hist, task.l_incr);
    for (int k = 0; k < in->local_queue_len; ++k)
        t_local += ampd_t_pre(in->decode_model, in->local_queue[k].l_hist, in->local_queue[k].l_incr);
    if (costs) costs[0] = t_local;
    int32_t best = AMPD_ROUTE_LOCAL;
    double best_t = t_local;
    for (int i = 0; i < n; ++i) {
        // Eq. 2: prefill + history KV there + incremental KV back + queue
        double t = ampd_t_pre(&in->prefill_models[i], task.l_hist, task.l_incr);
        t += in->kv_d2p[i].alpha + in->kv_d2p[i].beta * task.l_hist;
        t += in->kv_p2d[i].alpha + in->kv_p2d[i].beta * task.l_incr;
        if (in->remote_queue_len[i] < 0 || (in->remote_queue_len[i] > 0 && !in->remote_queues[i])) return AMPD_ROUTE_ERROR;
        for (int k = 0; k < in->remote_queue_len[i]; ++k)
            t += ampd_t_pre(&in->prefill_models[i], in->remote_queues[i][k].l_hist, in->remote_queues[i][k].l_incr);
        if (costs) costs[1 + i] = t;
        if (t < best_t) {
            best_t = t;
            best = i;
        }
    }
    if (reason) *reason = 2;
    return best;
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
