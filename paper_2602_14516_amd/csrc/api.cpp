// C ABI of libampd (see include/ampd.h): argument validation, work planning, the pinned
// staging ring that carries the work list to the device, and the kernel launches.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "ampd.h"
#include "kernels.h"
#include "plan.h"

namespace {

using namespace ampd;

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

ampd_status make_plan(const ampd_kv_cache* c, const ampd_batch* b, const ampd_plan_options* o, Plan& plan) {
    PlanOptions po;
    if (o) {
        if (o->force_kv_splits < 0) return AMPD_ERR_INVALID_ARG;
        for (int i = 0; i < 7; ++i)
            if (o->reserved[i] != 0) return AMPD_ERR_INVALID_ARG;
        po.force_kv_splits = o->force_kv_splits;
    }
    Shape s{c->num_q_heads, c->num_kv_heads, c->head_dim, c->page_size};
    build_plan(s, b->num_reqs, b->h_ctx_len, b->h_incr_len, po, plan);
    if (plan.partial_floats > 0x7fffffff || plan.items.size() > 0x7fffffffu) return AMPD_ERR_UNSUPPORTED;
    return AMPD_OK;
}

// ---- pinned staging ring ---------------------------------------------------------------------
// The work list is built on the host in pinned memory and copied to the caller's workspace by
// a small upload kernel that reads the pinned buffer directly.  Each call takes the next ring slot; a slot is reused
// only after the event recorded behind its copy has completed.

struct Slot {
    void* host = nullptr;
    size_t cap = 0;
    hipEvent_t ev = nullptr;
    bool pending = false;
};
constexpr int RING = 16;
std::mutex g_mu;
Slot g_ring[RING];
int g_next = 0;

bool g_timing = false;
thread_local hipEvent_t t_ev[4] = {nullptr, nullptr, nullptr, nullptr};   // append0, attn0, attn1, comb1
thread_local bool t_valid = false, t_has_append = false;

hipError_t take_slot(size_t bytes, Slot** out) {
    static bool primed = false;
    if (!primed) {                            // allocate the whole ring once, not one slot per call
        primed = true;
        for (int i = 0; i < RING; ++i) {
            if (hipHostMalloc(&g_ring[i].host, 1 << 20, hipHostMallocDefault) != hipSuccess) {
                g_ring[i].host = nullptr;
                break;
            }
            g_ring[i].cap = 1 << 20;
        }
    }
    Slot& s = g_ring[g_next];
    g_next = (g_next + 1) % RING;
    hipError_t e;
    if (s.pending) {
        e = hipEventSynchronize(s.ev);
        if (e != hipSuccess) return e;
        s.pending = false;
    }
    if (s.cap < bytes) {
        if (s.host) {
            e = hipHostFree(s.host);
            if (e != hipSuccess) return e;
            s.host = nullptr;
            s.cap = 0;
        }
        size_t cap = 1 << 20;                 // 1 MiB covers ~30 k work items: regrowth is rare
        while (cap < bytes) cap <<= 1;
        e = hipHostMalloc(&s.host, cap, hipHostMallocDefault);
        if (e != hipSuccess) return e;
        s.cap = cap;
    }
    if (!s.ev) {
        e = hipEventCreateWithFlags(&s.ev, hipEventDisableTiming);
        if (e != hipSuccess) return e;
    }
    *out = &s;
    return hipSuccess;
}

#define HIP_TRY(x)                              \
    do {                                        \
        if ((x) != hipSuccess) return AMPD_ERR_HIP; \
    } while (0)

ampd_status ensure_timing_events() {
    for (int i = 0; i < 4; ++i)
        if (!t_ev[i]) HIP_TRY(hipEventCreate(&t_ev[i]));
    return AMPD_OK;
}

// ---- launches --------------------------------------------------------------------------------

// A work list staged in pinned host memory that still has to reach the workspace.
struct PendingUpload {
    const void* src = nullptr;
    void* dst = nullptr;
    size_t bytes = 0;
};

// mode 0: append (all heads);  1: unpack rows of heads [h0, h0+hn) into pages;  2: pack pages into rows.
// up (mode 0 only): rides on the first launch that is actually made; bytes is set to 0 once it is on its way.
ampd_status do_append(const ampd_kv_cache* c, const ampd_batch* b, const void* k_new, const void* v_new, hipStream_t st,
                      int mode = 0, int h0 = 0, int hn = -1, PendingUpload* up = nullptr) {
    const int logP = log2_exact(c->page_size);
    if (hn < 0) hn = c->num_kv_heads;
    int64_t row_off = 0;
    for (int r0 = 0; r0 < b->num_reqs; r0 += APPEND_MAX_REQS) {
        const int n = std::min(APPEND_MAX_REQS, b->num_reqs - r0);
        AppendParams p;
        std::memset(&p, 0, sizeof(p));
        p.k_new = k_new;
        p.v_new = v_new;
        p.k_pool = c->k_pool;
        p.v_pool = c->v_pool;
        p.k_scale = c->k_scale;
        p.v_scale = c->v_scale;
        p.block_table = b->d_block_table;
        p.Hkv = c->num_kv_heads;
        p.D = c->head_dim;
        p.P = c->page_size;
        p.logP = logP;
        p.max_pages = b->max_pages_per_req;
        p.req0 = r0;
        p.h0 = h0;
        p.hn = hn;
        int max_touched = 0;
        for (int i = 0; i < n; ++i) {
            const int C = b->h_ctx_len[r0 + i], L = b->h_incr_len[r0 + i];
            p.C[i] = C;
            p.L[i] = L;
            p.row_off[i] = (int32_t)row_off;
            row_off += L;
            if (L > 0) max_touched = std::max(max_touched, (C + L - 1) / c->page_size - C / c->page_size + 1);
        }
        if (mode == 0) {
            if (up && up->bytes > 0 && max_touched > 0) {
                p.up_src = up->src;
                p.up_dst = up->dst;
                p.up_n16 = (int32_t)((up->bytes + 15) / 16);
                up->bytes = 0;
            }
            HIP_TRY(launch_append(p, c->kv_dtype == AMPD_KV_FP8_E4M3 ? KV_FP8 : KV_BF16, max_touched, n, st));
        } else
            HIP_TRY(launch_kv_move(p, mode == 2, max_touched, n, st));
    }
    return AMPD_OK;
}

ampd_status check_workspace(const Plan& plan, const void* workspace, size_t workspace_bytes) {
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < (size_t)plan.total_bytes)
        return AMPD_ERR_WORKSPACE;
    return AMPD_OK;
}

// Stage the work list in a pinned ring slot (the caller holds g_mu and, once the launch that reads the slot
// is enqueued, records the slot's event and marks it pending).
ampd_status stage_plan(const Plan& plan, void* workspace, Slot** slot, PendingUpload* up) {
    HIP_TRY(take_slot((size_t)plan.plan_bytes, slot));
    char* h = static_cast<char*>((*slot)->host);
    std::memcpy(h + plan.off_reqs, plan.reqs.data(), plan.reqs.size() * sizeof(ReqInfo));
    std::memcpy(h + plan.off_items, plan.items.data(), plan.items.size() * sizeof(Item));
    if (!plan.combs.empty()) std::memcpy(h + plan.off_combs, plan.combs.data(), plan.combs.size() * sizeof(CombItem));
    up->src = h;
    up->dst = workspace;
    up->bytes = (size_t)plan.plan_bytes;
    return AMPD_OK;
}

// plan: already built and checked against the workspace.  append: the K/V rows to append first (or null).
ampd_status do_attn(const ampd_kv_cache* c, const ampd_batch* b, const Plan& plan, const void* q, void* out,
                    void* workspace, hipStream_t st, const void* k_new = nullptr, const void* v_new = nullptr) {
    if (plan.items.empty()) return k_new ? do_append(c, b, k_new, v_new, st) : AMPD_OK;

    {
        std::lock_guard<std::mutex> lk(g_mu);
        Slot* s = nullptr;
        PendingUpload up;
        ampd_status vs = stage_plan(plan, workspace, &s, &up);
        if (vs != AMPD_OK) return vs;
        if (k_new) {
            vs = do_append(c, b, k_new, v_new, st, 0, 0, -1, &up);     // the work list rides on the append launch
            if (vs != AMPD_OK) return vs;
        }
        if (up.bytes > 0) HIP_TRY(launch_upload(up.src, up.dst, up.bytes, st));
        HIP_TRY(hipEventRecord(s->ev, st));
        s->pending = true;
    }

    char* ws = static_cast<char*>(workspace);
    AttnParams p;
    std::memset(&p, 0, sizeof(p));
    p.q = q;
    p.out = out;
    p.k_pool = c->k_pool;
    p.v_pool = c->v_pool;
    p.k_scale = c->k_scale;
    p.v_scale = c->v_scale;
    p.block_table = b->d_block_table;
    p.reqs = reinterpret_cast<const ReqInfo*>(ws + plan.off_reqs);
    p.items = reinterpret_cast<const Item*>(ws + plan.off_items);
    p.combs = reinterpret_cast<const CombItem*>(ws + plan.off_combs);
    p.partial = reinterpret_cast<float*>(ws + plan.off_partial);
    p.Hq = c->num_q_heads;
    p.Hkv = c->num_kv_heads;
    p.P = c->page_size;
    p.logP = log2_exact(c->page_size);
    p.max_pages = b->max_pages_per_req;
    p.c_log2 = c->softmax_scale * 1.44269504088896340736f;
    const int kvt = c->kv_dtype == AMPD_KV_FP8_E4M3 ? KV_FP8 : KV_BF16;

    if (g_timing) HIP_TRY(hipEventRecord(t_ev[1], st));
    HIP_TRY(launch_attn(p, c->head_dim, kvt, (int)plan.items.size(), st));
    if (g_timing) HIP_TRY(hipEventRecord(t_ev[2], st));
    int comb_rows = 0;
    for (const CombItem& ci : plan.combs) comb_rows = std::max(comb_rows, ci.nq * ((ci.heads >> 16) & 0xff));
    HIP_TRY(launch_combine(p, c->head_dim, (int)plan.combs.size(), comb_rows, st));
    if (g_timing) {
        HIP_TRY(hipEventRecord(t_ev[3], st));
        t_valid = true;
    }
    return AMPD_OK;
}

ampd_status append_then_attend(const ampd_kv_cache* c, const ampd_batch* b, const void* q, const void* k_new,
                               const void* v_new, void* out, void* workspace, size_t workspace_bytes, void* stream,
                               const ampd_plan_options* opts) {
    ampd_status vs = validate(c, b, true);
    if (vs != AMPD_OK) return vs;
    int64_t sumL = 0;
    for (int r = 0; r < b->num_reqs; ++r) sumL += b->h_incr_len[r];
    if (sumL == 0) return AMPD_OK;
    if (!q || !k_new || !v_new || !out) return AMPD_ERR_INVALID_ARG;
    // check the workspace before anything is enqueued
    Plan plan;
    vs = make_plan(c, b, opts, plan);
    if (vs != AMPD_OK) return vs;
    vs = check_workspace(plan, workspace, workspace_bytes);
    if (vs != AMPD_OK) return vs;
    hipStream_t st = static_cast<hipStream_t>(stream);
    t_valid = false;
    t_has_append = false;
    if (g_timing) {
        vs = ensure_timing_events();
        if (vs != AMPD_OK) return vs;
        HIP_TRY(hipEventRecord(t_ev[0], st));
        t_has_append = true;
    }
    return do_attn(c, b, plan, q, out, workspace, st, k_new, v_new);
}

}  // namespace

extern "C" {

size_t ampd_workspace_bytes_opts(const ampd_kv_cache* cache, const ampd_batch* batch, const ampd_plan_options* opts) {
    if (validate(cache, batch, false) != AMPD_OK) return 0;
    Plan plan;
    if (make_plan(cache, batch, opts, plan) != AMPD_OK) return 0;
    return (size_t)plan.total_bytes;
}

size_t ampd_workspace_bytes(const ampd_kv_cache* cache, const ampd_batch* batch) {
    return ampd_workspace_bytes_opts(cache, batch, nullptr);
}

ampd_status ampd_kv_append(const ampd_kv_cache* cache, const ampd_batch* batch, const void* k_new, const void* v_new,
                           void* stream) {
    ampd_status vs = validate(cache, batch, true);
    if (vs != AMPD_OK) return vs;
    int64_t sumL = 0;
    for (int r = 0; r < batch->num_reqs; ++r) sumL += batch->h_incr_len[r];
    if (sumL == 0) return AMPD_OK;
    if (!k_new || !v_new) return AMPD_ERR_INVALID_ARG;
    return do_append(cache, batch, k_new, v_new, static_cast<hipStream_t>(stream));
}

static ampd_status kv_move(const ampd_kv_cache* cache, const ampd_batch* batch, int32_t head_begin, int32_t head_count,
                           const void* k_rows, const void* v_rows, void* stream, int mode) {
    ampd_status vs = validate(cache, batch, true);
    if (vs != AMPD_OK) return vs;
    if (cache->kv_dtype != AMPD_KV_BF16) return AMPD_ERR_UNSUPPORTED;
    if (head_begin < 0 || head_count <= 0 || head_begin + head_count > cache->num_kv_heads) return AMPD_ERR_INVALID_ARG;
    int64_t sumL = 0;
    for (int r = 0; r < batch->num_reqs; ++r) sumL += batch->h_incr_len[r];
    if (sumL == 0) return AMPD_OK;
    if (!k_rows || !v_rows) return AMPD_ERR_INVALID_ARG;
    return do_append(cache, batch, k_rows, v_rows, static_cast<hipStream_t>(stream), mode, head_begin, head_count);
}

ampd_status ampd_kv_pack(const ampd_kv_cache* cache, const ampd_batch* batch, int32_t head_begin, int32_t head_count,
                         void* k_out, void* v_out, void* stream) {
    return kv_move(cache, batch, head_begin, head_count, k_out, v_out, stream, 2);
}

ampd_status ampd_kv_unpack(const ampd_kv_cache* cache, const ampd_batch* batch, int32_t head_begin, int32_t head_count,
                           const void* k_in, const void* v_in, void* stream) {
    return kv_move(cache, batch, head_begin, head_count, k_in, v_in, stream, 1);
}

ampd_status ampd_incr_prefill_attn_opts(const ampd_kv_cache* cache, const ampd_batch* batch, const void* q,
                                        const void* k_new, const void* v_new, void* out, void* workspace,
                                        size_t workspace_bytes, void* stream, const ampd_plan_options* opts) {
    return append_then_attend(cache, batch, q, k_new, v_new, out, workspace, workspace_bytes, stream, opts);
}

ampd_status ampd_incr_prefill_attn(const ampd_kv_cache* cache, const ampd_batch* batch, const void* q,
                                   const void* k_new, const void* v_new, void* out, void* workspace,
                                   size_t workspace_bytes, void* stream) {
    return append_then_attend(cache, batch, q, k_new, v_new, out, workspace, workspace_bytes, stream, nullptr);
}

// A mixed batch goes through the same planner: rows with few query rows (decode rows) become
// narrow items, prefill rows become wide tiles, and both kinds sit in one work list that a
// single attention launch consumes.
ampd_status ampd_mixed_batch_attn_opts(const ampd_kv_cache* cache, const ampd_batch* batch, const void* q,
                                       const void* k_new, const void* v_new, void* out, void* workspace,
                                       size_t workspace_bytes, void* stream, const ampd_plan_options* opts) {
    return append_then_attend(cache, batch, q, k_new, v_new, out, workspace, workspace_bytes, stream, opts);
}

ampd_status ampd_mixed_batch_attn(const ampd_kv_cache* cache, const ampd_batch* batch, const void* q,
                                  const void* k_new, const void* v_new, void* out, void* workspace,
                                  size_t workspace_bytes, void* stream) {
    return append_then_attend(cache, batch, q, k_new, v_new, out, workspace, workspace_bytes, stream, nullptr);
}

ampd_status ampd_paged_attn(const ampd_kv_cache* cache, const ampd_batch* batch, const void* q, void* out,
                            void* workspace, size_t workspace_bytes, void* stream, const ampd_plan_options* opts) {
    ampd_status vs = validate(cache, batch, true);
    if (vs != AMPD_OK) return vs;
    Plan plan;
    vs = make_plan(cache, batch, opts, plan);
    if (vs != AMPD_OK) return vs;
    if (plan.items.empty()) return AMPD_OK;
    if (!q || !out) return AMPD_ERR_INVALID_ARG;
    vs = check_workspace(plan, workspace, workspace_bytes);
    if (vs != AMPD_OK) return vs;
    t_valid = false;
    t_has_append = false;
    if (g_timing) {
        vs = ensure_timing_events();
        if (vs != AMPD_OK) return vs;
    }
    return do_attn(cache, batch, plan, q, out, workspace, static_cast<hipStream_t>(stream));
}

ampd_status ampd_plan_describe(const ampd_kv_cache* cache, const ampd_batch* batch, const ampd_plan_options* opts,
                               ampd_plan_info* info) {
    if (!info) return AMPD_ERR_INVALID_ARG;
    ampd_status vs = validate(cache, batch, false);
    if (vs != AMPD_OK) return vs;
    Plan plan;
    vs = make_plan(cache, batch, opts, plan);
    if (vs != AMPD_OK) return vs;
    info->num_items = (int64_t)plan.items.size();
    info->num_wide_items = plan.num_wide;
    info->num_narrow_items = plan.num_narrow;
    info->num_combine_items = (int64_t)plan.combs.size();
    info->num_append_launches = (batch->num_reqs + APPEND_MAX_REQS - 1) / APPEND_MAX_REQS;
    info->partial_bytes = plan.partial_floats * 4;
    info->plan_bytes = plan.plan_bytes;
    return AMPD_OK;
}

int64_t ampd_plan_items(const ampd_kv_cache* cache, const ampd_batch* batch, const ampd_plan_options* opts,
                        int32_t* h_items, int64_t max_items) {
    ampd_status vs = validate(cache, batch, false);
    if (vs != AMPD_OK) return vs;
    Plan plan;
    vs = make_plan(cache, batch, opts, plan);
    if (vs != AMPD_OK) return vs;
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

void ampd_set_timing(int enabled) { g_timing = enabled != 0; }

ampd_status ampd_last_timing(float* attn_ms, float* combine_ms, float* append_ms) {
    if (!t_valid) return AMPD_ERR_INVALID_ARG;
    float a = 0.f, c = 0.f, ap = 0.f;
    HIP_TRY(hipEventElapsedTime(&a, t_ev[1], t_ev[2]));
    HIP_TRY(hipEventElapsedTime(&c, t_ev[2], t_ev[3]));
    if (t_has_append) HIP_TRY(hipEventElapsedTime(&ap, t_ev[0], t_ev[1]));
    if (attn_ms) *attn_ms = a;
    if (combine_ms) *combine_ms = c;
    if (append_ms) *append_ms = ap;
    return AMPD_OK;
}

const char* ampd_status_string(ampd_status s) {
    switch (s) {
        case AMPD_OK: return "ok";
        case AMPD_ERR_INVALID_ARG: return "invalid argument";
        case AMPD_ERR_UNSUPPORTED: return "unsupported configuration";
        case AMPD_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case AMPD_ERR_PAGE_RANGE: return "block table entry out of range";
        case AMPD_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char* ampd_version(void) { return "libampd 0.1 (gfx950)"; }

}  // extern "C"
