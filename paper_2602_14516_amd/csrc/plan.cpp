// Host-side work planner (see plan.h).  Pure integer host code: no HIP calls.
#include "plan.h"

#include <algorithm>

namespace ampd {

namespace {

constexpr int KV_TILE = 64;          // keys per LDS tile of a wide item; split points are multiples of it
constexpr int MIN_NARROW_CHUNK = 256;
constexpr int MIN_WIDE_CHUNK = 1024;

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

struct QBlock {            // a query block before splitting
    int32_t req, heads, q0, nq, nkeys, rows, kind;
};

}  // namespace

void build_plan(const Shape& s, int num_reqs, const int32_t* ctx_len, const int32_t* incr_len,
                const PlanOptions& opt, Plan& out) {
    out = Plan();
    const int G = s.Hq / s.Hkv;
    const int nhb = (G + 31) / 32;                 // head blocks of at most 32 heads per KV head
    out.reqs.resize(num_reqs);
    int64_t off = 0;
    for (int r = 0; r < num_reqs; ++r) {
        out.reqs[r] = ReqInfo{ctx_len[r], incr_len[r], (int32_t)off, 0};
        off += incr_len[r];
    }
    out.sum_L = off;

    // 1. query blocks
    std::vector<QBlock> qb;
    int64_t narrow_keys = 0;
    int64_t n_wide = 0;
    for (int r = 0; r < num_reqs; ++r) {
        const int C = ctx_len[r], L = incr_len[r];
        if (L <= 0) continue;
        for (int kvh = 0; kvh < s.Hkv; ++kvh) {
            for (int hb = 0; hb < nhb; ++hb) {
                const int g0 = hb * 32;
                const int gn = std::min(32, G - g0);
                const int tq_wave = 32 / gn;                   // tokens per wave (>= 1)
                if ((int64_t)L * gn <= 32) {
                    qb.push_back(QBlock{r, pack_heads(kvh, g0, gn, KIND_NARROW), 0, L, C + L, L * gn, KIND_NARROW});
                    narrow_keys += C + L;
                } else {
                    const int tq = ATTN_WAVES * tq_wave;
                    for (int q0 = 0; q0 < L; q0 += tq) {
                        const int nq = std::min(tq, L - q0);
                        qb.push_back(QBlock{r, pack_heads(kvh, g0, gn, KIND_WIDE), q0, nq, C + q0 + nq, nq * gn, KIND_WIDE});
                        ++n_wide;
                    }
                }
            }
        }
    }

    // 2. split policy (chunk sizes in keys, multiples of KV_TILE)
    int64_t narrow_chunk = 1 << 30, wide_chunk = 1 << 30;
    if (opt.force_kv_splits <= 0) {
        if (narrow_keys > 0) {
            // aim at ~8 items per resident workgroup slot so that the tail is short
            narrow_chunk = std::max<int64_t>(MIN_NARROW_CHUNK, round_up(ceil_div(narrow_keys, 8 * (int64_t)opt.wg_slots), KV_TILE));
        }
        if (n_wide > 0 && n_wide < 2 * (int64_t)opt.wg_slots) {
            int64_t max_keys = 0;
            for (const QBlock& b : qb)
                if (b.kind == KIND_WIDE) max_keys = std::max<int64_t>(max_keys, b.nkeys);
            const int64_t want = ceil_div(2 * (int64_t)opt.wg_slots, n_wide);
            wide_chunk = std::max<int64_t>(MIN_WIDE_CHUNK, round_up(ceil_div(max_keys, want), KV_TILE));
        }
    }

    // 3. items
    struct Cost { int64_t cost; int32_t idx; };
    std::vector<Cost> order;
    for (const QBlock& b : qb) {
        int64_t chunk;
        if (opt.force_kv_splits > 0)
            chunk = std::max<int64_t>(KV_TILE, round_up(ceil_div(b.nkeys, opt.force_kv_splits), KV_TILE));
        else
            chunk = b.kind == KIND_WIDE ? wide_chunk : narrow_chunk;
        const int nsplit = (int)ceil_div(b.nkeys, chunk);
        const int32_t slot = b.rows * (s.D + 2);                // floats per partial slot
        int64_t part0 = -1;
        if (nsplit > 1) {
            part0 = out.partial_floats;
            out.partial_floats += (int64_t)slot * nsplit;
            out.combs.push_back(CombItem{b.req, b.heads, b.q0, b.nq, (int32_t)part0, nsplit, slot, 0});
        }
        for (int sp = 0; sp < nsplit; ++sp) {
            Item it;
            it.req = b.req;
            it.heads = b.heads;
            it.q0 = b.q0;
            it.nq = b.nq;
            it.kv_begin = (int32_t)(sp * chunk);
            it.kv_end = (int32_t)std::min<int64_t>(b.nkeys, (sp + 1) * chunk);
            it.part_off = nsplit > 1 ? (int32_t)(part0 + (int64_t)sp * slot) : -1;
            it.pad = 0;
            const int64_t keys = it.kv_end - it.kv_begin;
            const int64_t cost = b.kind == KIND_WIDE ? keys * 4 : keys;
            order.push_back(Cost{cost, (int32_t)out.items.size()});
            out.items.push_back(it);
            if (b.kind == KIND_WIDE) ++out.num_wide; else ++out.num_narrow;
        }
    }

    // 4. launch order: longest first within each kind (stable, so the order is a function of the
    //    lengths only).  In a mixed batch the two kinds are interleaved in proportion to their
    //    total cost, so that at any time some CUs run compute-bound tiles while others stream
    //    decode rows, instead of one phase after the other.
    std::stable_sort(order.begin(), order.end(), [](const Cost& a, const Cost& b) { return a.cost > b.cost; });
    std::vector<int32_t> wide_ix, narrow_ix;
    double wide_cost = 0, narrow_cost = 0;
    for (const Cost& c : order) {
        const bool is_wide = ((out.items[c.idx].heads >> 24) & 0xff) == KIND_WIDE;
        (is_wide ? wide_ix : narrow_ix).push_back(c.idx);
        (is_wide ? wide_cost : narrow_cost) += (double)c.cost;
    }
    std::vector<Item> sorted;
    sorted.reserve(out.items.size());
    {
        size_t iw = 0, in = 0;
        double dw = 0, dn = 0;                     // cost already emitted per kind
        while (iw < wide_ix.size() || in < narrow_ix.size()) {
            bool take_wide;
            if (iw >= wide_ix.size()) take_wide = false;
            else if (in >= narrow_ix.size()) take_wide = true;
            else take_wide = dw * narrow_cost <= dn * wide_cost;      // the kind that lags behind its share
            const int32_t idx = take_wide ? wide_ix[iw++] : narrow_ix[in++];
            const Item& it = out.items[idx];
            const double keys = it.kv_end - it.kv_begin;
            (take_wide ? dw : dn) += take_wide ? keys * 4 : keys;
            sorted.push_back(it);
        }
    }
    out.items.swap(sorted);

    // 5. byte layout
    out.off_reqs = 0;
    out.off_items = round_up((int64_t)out.reqs.size() * sizeof(ReqInfo), 256);
    out.off_combs = out.off_items + round_up((int64_t)out.items.size() * sizeof(Item), 256);
    out.plan_bytes = out.off_combs + round_up((int64_t)out.combs.size() * sizeof(CombItem), 256);
    out.off_partial = out.plan_bytes;
    out.total_bytes = out.off_partial + round_up(out.partial_floats * 4, 256);
    if (out.total_bytes == 0) out.total_bytes = 256;
}

}  // namespace ampd
