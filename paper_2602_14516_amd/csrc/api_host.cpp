// C ABI of libampd (see include/ampd.h), host half: argument validation, work planning and the entry points that
// are pure host computation.  Nothing here includes or calls HIP.
#include "api_host.h"

#include <cmath>
#include <vector>

namespace ampd {
namespace host {

int log2_exact(int x) {
    int l = 0;
    while ((1 << l) < x) ++l;
    return (1 << l) == x ? l : -1;
}

// ---- validation ------------------------------------------------------------------------------

ampd_status validate(const ampd_kv_cache* c, const ampd_batch* b, bool need_pools) {
    if (!c || !b) return AMPD_ERR_INVALID_ARG;
    if (c->num_q_heads <= 0 || c->num_kv_heads <= 0 || c->num_q_heads % c->num_kv_heads != 0) return AMPD_ERR_INVALID_ARG;
    if (c->num_kv_heads > 255 || c->num_q_heads / c->num_kv_heads > 64) return AMPD_ERR_UNSUPPORTED;
    if (c->head_dim != 64 && c->head_dim != 128) return AMPD_ERR_UNSUPPORTED;
    if (c->page_size != 16 && c->page_size != 32 && c->page_size != 64) return AMPD_ERR_UNSUPPORTED;
    if (c->kv_dtype != AMPD_KV_BF16 && c->kv_dtype != AMPD_KV_FP8_E4M3) return AMPD_ERR_UNSUPPORTED;
    if (c->reserved != 0 || c->reserved2 != 0) return AMPD_ERR_INVALID_ARG;
    if (c->num_pages <= 0) return AMPD_ERR_INVALID_ARG;
    if (!(c->softmax_scale > 0.0f) || !std::isfinite(c->softmax_scale)) return AMPD_ERR_INVALID_ARG;
    if (need_pools) {
        if (!c->k_pool || !c->v_pool) return AMPD_ERR_INVALID_ARG;
        if (c->kv_dtype == AMPD_KV_FP8_E4M3 && (!c->k_scale || !c->v_scale)) return AMPD_ERR_INVALID_ARG;
    }
    if (b->num_reqs < 0 || b->max_pages_per_req < 0) return AMPD_ERR_INVALID_ARG;
    if (b->num_reqs > 0 && (!b->h_ctx_len || !b->h_incr_len)) return AMPD_ERR_INVALID_ARG;
    if (need_pools && b->num_reqs > 0 && !b->d_block_table) return AMPD_ERR_INVALID_ARG;
    int64_t sumL = 0;
    for (int r = 0; r < b->num_reqs; ++r) {
        const int64_t C = b->h_ctx_len[r], L = b->h_incr_len[r];
        if (C < 0 || L < 0) return AMPD_ERR_INVALID_ARG;
        const int64_t T = C + L;
        if (T > (int64_t)1 << 30) return AMPD_ERR_UNSUPPORTED;
        const int64_t need = (T + c->page_size - 1) / c->page_size;
        if (L > 0 && need > b->max_pages_per_req) return AMPD_ERR_INVALID_ARG;
        sumL += L;
        if (sumL > (int64_t)1 << 30) return AMPD_ERR_UNSUPPORTED;
    }
    if (b->h_block_table) {
        for (int r = 0; r < b->num_reqs; ++r) {
            if (b->h_incr_len[r] == 0) continue;
            const int64_t T = (int64_t)b->h_ctx_len[r] + b->h_incr_len[r];
            const int64_t need = (T + c->page_size - 1) / c->page_size;
            const int32_t* row = b->h_block_table + (int64_t)r * b->max_pages_per_req;
            for (int64_t i = 0; i < need; ++i)
                if (row[i] < 0 || row[i] >= c->num_pages) return AMPD_ERR_PAGE_RANGE;
        }
    }
    return AMPD_OK;
}

// The last plan built on this thread is kept: a caller sizes its workspace with ampd_workspace_bytes and then issues
// the call with the same lengths, and a serving loop often repeats a batch shape; both then plan once.
namespace {
struct PlanKey {
    int32_t Hq = 0, Hkv = 0, D = 0, P = 0, splits = 0;
    bool append_items = false;
    std::vector<int32_t> ctx, incr;
    bool operator==(const PlanKey& o) const {
        return Hq == o.Hq && Hkv == o.Hkv && D == o.D && P == o.P && splits == o.splits && append_items == o.append_items &&
               ctx == o.ctx && incr == o.incr;
    }
};
thread_local PlanKey t_key;
thread_local Plan t_plan;
thread_local bool t_plan_valid = false;
}  // namespace

ampd_status make_plan(const ampd_kv_cache* c, const ampd_batch* b, const ampd_plan_options* o, bool with_append, const Plan** plan) {
    PlanOptions po;
    po.append_items = with_append && c->kv_dtype == AMPD_KV_BF16;
    if (o) {
        if (o->force_kv_splits < 0) return AMPD_ERR_INVALID_ARG;
        for (int i = 0; i < 7; ++i)
            if (o->reserved[i] != 0) return AMPD_ERR_INVALID_ARG;
        po.force_kv_splits = o->force_kv_splits;
    }
    PlanKey key;
    key.Hq = c->num_q_heads; key.Hkv = c->num_kv_heads; key.D = c->head_dim; key.P = c->page_size;
    key.splits = po.force_kv_splits;
    key.append_items = po.append_items;
    key.ctx.assign(b->h_ctx_len, b->h_ctx_len + b->num_reqs);
    key.incr.assign(b->h_incr_len, b->h_incr_len + b->num_reqs);
    if (!(t_plan_valid && key == t_key)) {
        t_plan_valid = false;
        Shape s{c->num_q_heads, c->num_kv_heads, c->head_dim, c->page_size};
        build_plan(s, b->num_reqs, b->h_ctx_len, b->h_incr_len, po, t_plan);
        t_key = std::move(key);
        t_plan_valid = true;
    }
    if (t_plan.partial_floats > 0x7fffffff || t_plan.items.size() > 0x7fffffffu) return AMPD_ERR_UNSUPPORTED;
    *plan = &t_plan;
    return AMPD_OK;
}

}  // namespace host
}  // namespace ampd

using namespace ampd;
using namespace ampd::host;

extern "C" {

size_t ampd_workspace_bytes_opts(const ampd_kv_cache* cache, const ampd_batch* batch, const ampd_plan_options* opts) {
    if (validate(cache, batch, false) != AMPD_OK) return 0;
    const Plan* plan = nullptr;
    if (make_plan(cache, batch, opts, true, &plan) != AMPD_OK) return 0;
    return (size_t)plan->total_bytes;
}

size_t ampd_workspace_bytes(const ampd_kv_cache* cache, const ampd_batch* batch) {
    return ampd_workspace_bytes_opts(cache, batch, nullptr);
}

ampd_status ampd_plan_describe(const ampd_kv_cache* cache, const ampd_batch* batch, const ampd_plan_options* opts,
                               ampd_plan_info* info) {
    if (!info) return AMPD_ERR_INVALID_ARG;
    ampd_status vs = validate(cache, batch, false);
    if (vs != AMPD_OK) return vs;
    const Plan* planp = nullptr;
    vs = make_plan(cache, batch, opts, true, &planp);
    if (vs != AMPD_OK) return vs;
    const Plan& plan = *planp;
    info->num_items = (int64_t)plan.items.size();
    info->num_wide_items = plan.num_wide;
    info->num_narrow_items = plan.num_narrow;
    info->num_combine_items = (int64_t)plan.combs.size();
    info->num_append_items = plan.num_append;
    info->num_append_launches = plan.num_append > 0 ? 0 : (batch->num_reqs + APPEND_MAX_REQS - 1) / APPEND_MAX_REQS;
    info->partial_bytes = plan.partial_floats * 4;
    info->plan_bytes = plan.plan_bytes;
    info->num_workgroups = plan.grid;
    return AMPD_OK;
}

int64_t ampd_plan_items(const ampd_kv_cache* cache, const ampd_batch* batch, const ampd_plan_options* opts,
                        int32_t* h_items, int64_t max_items) {
    ampd_status vs = validate(cache, batch, false);
    if (vs != AMPD_OK) return vs;
    const Plan* planp = nullptr;
    vs = make_plan(cache, batch, opts, true, &planp);
    if (vs != AMPD_OK) return vs;
    const Plan& plan = *planp;
    const int64_t n = (int64_t)plan.items.size();
    for (int64_t i = 0; i < n && i < max_items && h_items; ++i) {
        const Item& it = plan.items[i];
        int32_t* o = h_items + i * 10;
        o[0] = it.req;
        o[1] = (it.heads >> 24) & 0xff;
        o[2] = it.heads & 0xff;
        o[3] = (it.heads >> 8) & 0xff;
        o[4] = (it.heads >> 16) & 0xff;
        o[5] = it.q0;
        o[6] = it.nq;
        o[7] = it.kv_begin;
        o[8] = it.kv_end;
        o[9] = it.part_off;
    }
    return n;
}

const char* ampd_status_string(ampd_status s) {
    switch (s) {
        case AMPD_OK: return "ok";
        case AMPD_ERR_INVALID_ARG: return "invalid argument";
        case AMPD_ERR_UNSUPPORTED: return "unsupported configuration";
        case AMPD_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case AMPD_ERR_PAGE_RANGE: return "block table entry out of range";
        case AMPD_ERR_HIP: return "HIP runtime error";
        case AMPD_ERR_NOT_INITIALISED: return "ampd_init has not been called on this device";
    }
    return "unknown status";
}

const char* ampd_version(void) { return "libampd 0.2 (gfx950)"; }

}  // extern "C"
