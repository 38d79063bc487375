// C ABI of libampd (see include/ampd.h), device half: the pinned staging ring that carries the work list to the
// device, the static workspace, and the kernel launches.  Argument validation and the entry points that never
// touch a GPU live in api_host.cpp.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cmath>
#include <cstring>
#include <mutex>
#include <thread>
#include <vector>

#include "ampd.h"
#include "api_host.h"
#include "kernels.h"
#include "plan.h"

namespace {

using namespace ampd;
using namespace ampd::host;

// ---- per-device state: pinned staging ring, static workspace ------------------------------------
// The work list is built on the host in pinned memory and copied to the workspace by the GPU reading the pinned
// buffer directly.  Every call takes a ring slot that no enqueued copy still reads: a slot becomes free once the
// attention launch of its call has started, which that launch reports by storing the call's sequence number into a
// flag word behind the slot (polled, never waited for; no HIP event sits between the launches of a call, where a
// record costs ~4 us of GPU time per call).  When every slot is busy the ring grows, so the depth of the ring follows
// the number of calls the caller keeps in flight; only a call that may not allocate (the static-workspace entry
// point) waits for the oldest slot instead.

// Device memory that the static-workspace entry point uses in place of a caller-provided workspace.  On the host
// this name is only a handle for hipGetSymbolAddress: the address that kernels and copies take is the one
// that call returns on each device.
static __device__ __align__(256) unsigned char g_static_workspace[AMPD_STATIC_WORKSPACE_BYTES];

struct Slot {
    void* host = nullptr;
    size_t cap = 0;
    uint32_t* flag = nullptr;          // in the same pinned allocation, behind the cap bytes; written by the GPU
    uint32_t seq = 0;                  // value the flag takes once the slot is free again
    bool pending = false;
};
struct DeviceState {
    bool ready = false;
    void* static_ws = nullptr;         // device address of g_static_workspace on this device
    std::vector<Slot> ring;
    size_t next = 0;
    uint32_t seq = 0;                  // sequence number of the last call that took a slot
};
constexpr int MAX_DEVICES = 64;
constexpr size_t SLOT_BYTES = 256u << 10;      // ~5 000 work items; larger plans get a slot of their own size
constexpr size_t FLAG_BYTES = 256;
constexpr size_t RING_INITIAL = 32;
constexpr size_t RING_MAX = 4096;              // beyond this many calls in flight a call waits for the oldest
std::mutex g_mu;
DeviceState g_dev[MAX_DEVICES];

thread_local bool t_timing = false;
thread_local hipEvent_t t_ev[4] = {nullptr, nullptr, nullptr, nullptr};   // append0, attn0, attn1, comb1
thread_local bool t_valid = false, t_has_append = false;

hipError_t new_slot(size_t bytes, Slot* s) {
    size_t cap = SLOT_BYTES;
    while (cap < bytes) cap <<= 1;
    // coherent (fine-grained) host memory: the GPU's store to the flag must become visible while later work still runs
    const hipError_t e = hipHostMalloc(&s->host, cap + FLAG_BYTES, hipHostMallocCoherent);
    if (e != hipSuccess) return e;
    s->cap = cap;
    s->flag = reinterpret_cast<uint32_t*>(static_cast<char*>(s->host) + cap);
    *s->flag = 0;
    s->seq = 0;
    return hipSuccess;
}

bool slot_released(const Slot& s) { return __atomic_load_n(s.flag, __ATOMIC_ACQUIRE) == s.seq; }

// Set-up of the device that is current on the calling thread (g_mu held): resolve the static workspace and pin the
// initial ring.  Runs once per device.
hipError_t ensure_device(DeviceState** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    DeviceState& d = g_dev[dev];
    if (!d.ready) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_workspace));
        if (e != hipSuccess) return e;
        d.static_ws = p;
        d.ring.reserve(RING_INITIAL);
        while (d.ring.size() < RING_INITIAL) {
            Slot s;
            e = new_slot(SLOT_BYTES, &s);
            if (e != hipSuccess) return e;
            d.ring.push_back(s);
        }
        d.ready = true;
    }
    *out = &d;
    return hipSuccess;
}

// A slot of at least `bytes` that no copy still reads (g_mu held).
hipError_t take_slot(DeviceState& d, size_t bytes, bool may_allocate, Slot** out) {
    const size_t n = d.ring.size();
    for (size_t k = 0; k < n; ++k) {                   // oldest first: in the steady state the first probe hits
        Slot& s = d.ring[(d.next + k) % n];
        if (s.cap < bytes) continue;
        if (s.pending) {
            if (!slot_released(s)) continue;
            s.pending = false;
        }
        d.next = (d.next + k + 1) % n;
        *out = &s;
        return hipSuccess;
    }
    if (may_allocate && n < RING_MAX) {
        Slot s;
        const hipError_t e = new_slot(bytes, &s);
        if (e != hipSuccess) return e;
        d.ring.push_back(s);
        *out = &d.ring.back();
        return hipSuccess;
    }
    for (size_t k = 0; k < n; ++k) {                   // no allocation allowed (or the ring is at its cap): wait
        Slot& s = d.ring[(d.next + k) % n];
        if (s.cap < bytes) continue;
        // for the oldest slot's launch to start; if that takes seconds, for the device: a flag still unset after that
        // belongs to a call whose attention launch was never made (its enqueue failed)
        const auto t0 = std::chrono::steady_clock::now();
        while (!slot_released(s)) {
            std::this_thread::yield();
            if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(2)) {
                const hipError_t e = hipDeviceSynchronize();
                if (e != hipSuccess) return e;
                break;
            }
        }
        s.pending = false;
        d.next = (d.next + k + 1) % n;
        *out = &s;
        return hipSuccess;
    }
    return hipErrorOutOfMemory;                        // no slot of this size exists and none may be made
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

// Stage the work list in a pinned ring slot of the current device (the caller holds g_mu and, once the launch that
// reads the slot is enqueued, gives the slot its sequence number and marks it pending).
ampd_status stage_plan(DeviceState& d, const Plan& plan, void* workspace, bool may_allocate, Slot** slot, PendingUpload* up) {
    HIP_TRY(take_slot(d, (size_t)plan.plan_bytes, may_allocate, slot));
    char* h = static_cast<char*>((*slot)->host);
    std::memcpy(h + plan.off_reqs, plan.reqs.data(), plan.reqs.size() * sizeof(ReqInfo));
    std::memcpy(h + plan.off_items, plan.items.data(), plan.items.size() * sizeof(Item));
    if (!plan.combs.empty()) std::memcpy(h + plan.off_combs, plan.combs.data(), plan.combs.size() * sizeof(CombItem));
    std::memcpy(h + plan.off_queues, plan.queue_heads, sizeof(plan.queue_heads));
    up->src = h;
    up->dst = workspace;
    up->bytes = (size_t)plan.plan_bytes;
    return AMPD_OK;
}

// plan: already built and checked against the workspace.  append: the K/V rows to append first (or null).
// workspace == nullptr selects the static workspace of the current device; that path allocates nothing (the
// device must have been set up by ampd_init) and records no timing events.
ampd_status do_attn(const ampd_kv_cache* c, const ampd_batch* b, const Plan& plan, const void* q, void* out,
                    void* workspace, hipStream_t st, const void* k_new = nullptr, const void* v_new = nullptr) {
    if (plan.items.empty()) return k_new ? do_append(c, b, k_new, v_new, st) : AMPD_OK;
    const bool use_static = workspace == nullptr;
    const bool timing = t_timing && !use_static;
    // bf16 cache: the page writes are append items of the attention launch (the plan holds them), and the attention
    // items read the new tokens from k_new / v_new; 8-bit cache: a quantising append launch goes first
    const bool fused_append = k_new && plan.num_append > 0;
    uint32_t* slot_flag = nullptr;     // the attention launch below releases the staging slot through these
    uint32_t slot_seq = 0;

    {
        std::lock_guard<std::mutex> lk(g_mu);
        DeviceState* d = nullptr;
        if (use_static) {
            int dev = -1;
            HIP_TRY(hipGetDevice(&dev));
            if (dev < 0 || dev >= MAX_DEVICES || !g_dev[dev].ready) return AMPD_ERR_NOT_INITIALISED;
            d = &g_dev[dev];
            workspace = d->static_ws;
        } else {
            HIP_TRY(ensure_device(&d));
        }
        Slot* s = nullptr;
        PendingUpload up;
        ampd_status vs = stage_plan(*d, plan, workspace, !use_static, &s, &up);
        if (vs != AMPD_OK) return vs;
        if (k_new && !fused_append) {
            vs = do_append(c, b, k_new, v_new, st, 0, 0, -1, &up);     // the work list rides on the append launch
            if (vs != AMPD_OK) return vs;
        }
        if (up.bytes > 0) HIP_TRY(launch_upload(up.src, up.dst, up.bytes, st));
        s->seq = ++d->seq;
        s->pending = true;
        slot_flag = s->flag;
        slot_seq = s->seq;
    }

    char* ws = static_cast<char*>(workspace);
    AttnParams p;
    std::memset(&p, 0, sizeof(p));
    p.q = q;
    p.out = out;
    p.k_new = fused_append ? k_new : nullptr;
    p.v_new = fused_append ? v_new : nullptr;
    p.k_pool = c->k_pool;
    p.v_pool = c->v_pool;
    p.k_scale = c->k_scale;
    p.v_scale = c->v_scale;
    p.block_table = b->d_block_table;
    p.reqs = reinterpret_cast<const ReqInfo*>(ws + plan.off_reqs);
    p.items = reinterpret_cast<const Item*>(ws + plan.off_items);
    p.combs = reinterpret_cast<const CombItem*>(ws + plan.off_combs);
    p.partial = reinterpret_cast<float*>(ws + plan.off_partial);
    p.queue_heads = reinterpret_cast<int32_t*>(ws + plan.off_queues);
    p.nitems = (int32_t)plan.items.size();
    p.Hq = c->num_q_heads;
    p.Hkv = c->num_kv_heads;
    p.P = c->page_size;
    p.logP = log2_exact(c->page_size);
    p.max_pages = b->max_pages_per_req;
    p.c_log2 = c->softmax_scale * 1.44269504088896340736f;
    p.slot_flag = slot_flag;
    p.slot_seq = slot_seq;
    const int kvt = c->kv_dtype == AMPD_KV_FP8_E4M3 ? KV_FP8 : KV_BF16;

    if (timing) HIP_TRY(hipEventRecord(t_ev[1], st));
    HIP_TRY(launch_attn(p, c->head_dim, kvt, plan.grid, st));
    if (timing) HIP_TRY(hipEventRecord(t_ev[2], st));
    int comb_rows = 0, comb_splits = 0;
    for (const CombItem& ci : plan.combs) {
        comb_rows = std::max(comb_rows, ci.nq * ((ci.heads >> 16) & 0xff));
        comb_splits = std::max(comb_splits, (int)ci.nsplit);
    }
    HIP_TRY(launch_combine(p, c->head_dim, (int)plan.combs.size(), comb_rows, comb_splits, st));
    if (timing) {
        HIP_TRY(hipEventRecord(t_ev[3], st));
        t_valid = true;
    }
    return AMPD_OK;
}

// use_static: take the static workspace of the current device instead of (workspace, workspace_bytes)
ampd_status append_then_attend(const ampd_kv_cache* c, const ampd_batch* b, const void* q, const void* k_new,
                               const void* v_new, void* out, void* workspace, size_t workspace_bytes, void* stream,
                               const ampd_plan_options* opts, bool use_static = false) {
    ampd_status vs = validate(c, b, true);
    if (vs != AMPD_OK) return vs;
    int64_t sumL = 0;
    for (int r = 0; r < b->num_reqs; ++r) sumL += b->h_incr_len[r];
    if (sumL == 0) return AMPD_OK;
    if (!q || !k_new || !v_new || !out) return AMPD_ERR_INVALID_ARG;
    // check the workspace before anything is enqueued
    const Plan* planp = nullptr;
    vs = make_plan(c, b, opts, true, &planp);
    if (vs != AMPD_OK) return vs;
    const Plan& plan = *planp;
    if (use_static) {
        if ((size_t)plan.total_bytes > (size_t)AMPD_STATIC_WORKSPACE_BYTES || (size_t)plan.plan_bytes > SLOT_BYTES)
            return AMPD_ERR_WORKSPACE;
        workspace = nullptr;
    } else {
        vs = check_workspace(plan, workspace, workspace_bytes);
        if (vs != AMPD_OK) return vs;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    t_valid = false;
    t_has_append = false;
    if (t_timing && !use_static) {
        vs = ensure_timing_events();
        if (vs != AMPD_OK) return vs;
        HIP_TRY(hipEventRecord(t_ev[0], st));
        t_has_append = true;
    }
    return do_attn(c, b, plan, q, out, workspace, st, k_new, v_new);
}

}  // namespace

extern "C" {

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

ampd_status ampd_init(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    DeviceState* d = nullptr;
    HIP_TRY(ensure_device(&d));
    return AMPD_OK;
}

size_t ampd_static_workspace_limit(void) { return (size_t)AMPD_STATIC_WORKSPACE_BYTES; }

ampd_status ampd_mixed_batch_attn_static(const ampd_kv_cache* cache, const ampd_batch* batch, const void* q,
                                         const void* k_new, const void* v_new, void* out, void* stream) {
    return append_then_attend(cache, batch, q, k_new, v_new, out, nullptr, 0, stream, nullptr, true);
}

ampd_status ampd_paged_attn(const ampd_kv_cache* cache, const ampd_batch* batch, const void* q, void* out,
                            void* workspace, size_t workspace_bytes, void* stream, const ampd_plan_options* opts) {
    ampd_status vs = validate(cache, batch, true);
    if (vs != AMPD_OK) return vs;
    const Plan* planp = nullptr;
    vs = make_plan(cache, batch, opts, false, &planp);
    if (vs != AMPD_OK) return vs;
    const Plan& plan = *planp;
    if (plan.items.empty()) return AMPD_OK;
    if (!q || !out) return AMPD_ERR_INVALID_ARG;
    vs = check_workspace(plan, workspace, workspace_bytes);
    if (vs != AMPD_OK) return vs;
    t_valid = false;
    t_has_append = false;
    if (t_timing) {
        vs = ensure_timing_events();
        if (vs != AMPD_OK) return vs;
    }
    return do_attn(cache, batch, plan, q, out, workspace, static_cast<hipStream_t>(stream));
}

void ampd_set_timing(int enabled) { t_timing = enabled != 0; }

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


}  // extern "C"
