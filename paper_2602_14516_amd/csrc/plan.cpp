// Host-side work planner (see plan.h).  Pure integer host code: no HIP calls.
#include "plan.h"

#include <algorithm>
#include <utility>

namespace ampd {

namespace {

constexpr int KV_TILE = 64;          // keys per LDS tile of a wide item; split points are multiples of it
constexpr int MIN_NARROW_CHUNK = 256;
constexpr int NARROW_ITEM_KEYS = 512;  // fixed cost of a narrow item (item, Q, page ids, first block, merge), in keys streamed
constexpr int MIN_WIDE_CHUNK = 512;          // tiles of a launch without decode rows
constexpr int MIN_WIDE_CHUNK_MIXED = 1024;   // ... of a mixed launch
constexpr int WIDE_STAGE_KEYS = 128;   // a tile works through its keys in stages of 128: part of a stage costs a whole one
constexpr int WIDE_ITEM_KEYS = 128;    // fixed cost of a tile (item, Q, first stage, output), in keys of a tile
constexpr int WIDE_SPLIT_KEYS = 1408;  // a piece of a cut tile also writes a partial result of up to 256 rows that the
                                       // combine pass reads again (fitted to single-request latencies, like the others)
constexpr int NUM_XCD = NUM_QUEUES;   // accelerator dies; workgroup i is dispatched to die i % NUM_XCD

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
    // (keys, number of blocks with that many): what the split policy needs to know of the blocks; noted for KV head 0
    // and multiplied by the number of KV heads afterwards
    std::vector<std::pair<int32_t, int32_t>> narrow_runs, wide_runs;
    auto note = [](std::vector<std::pair<int32_t, int32_t>>& runs, int32_t keys) {
        if (!runs.empty() && runs.back().first == keys)
            ++runs.back().second;
        else
            runs.emplace_back(keys, 1);
    };
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
                    if (kvh == 0) note(narrow_runs, C + L);
                } else {
                    // A tile that is not full costs its workgroup nearly as much per key as a full one, so the
                    // remainder of the row goes into the FIRST tile, which sees the fewest keys.
                    const int tq = ATTN_WAVES * tq_wave;
                    const int first = L % tq ? L % tq : tq;
                    for (int q0 = 0; q0 < L; q0 += q0 ? tq : first) {
                        const int nq = q0 ? tq : first;
                        qb.push_back(QBlock{r, pack_heads(kvh, g0, gn, KIND_WIDE), q0, nq, C + q0 + nq, nq * gn, KIND_WIDE});
                        ++n_wide;
                        if (kvh == 0) note(wide_runs, C + q0 + nq);
                    }
                }
            }
        }
    }

    for (auto& r : narrow_runs) r.second *= s.Hkv;
    for (auto& r : wide_runs) r.second *= s.Hkv;

    // 2. split policy (chunk sizes in keys, multiples of KV_TILE)
    // An item costs a few microseconds around its key range (item, Q, page ids and first block before the first key;
    // merge of the waves or the store of a partial result after the last), and a CU runs one item at a time, so
    // nothing hides that: few, long items win as long as the slots (resident workgroups) stay evenly loaded.
    // Candidates are the smallest chunks whose items fit ONE round on all, half or a quarter of the slots, the chunks
    // that give ~2, 3, 4 items per slot, and (tiles) no cut at all.  One round lasts as long as its longest piece; several rounds about a slot's
    // share of the keys plus half a longest piece; every item adds its fixed cost (item_keys, in keys streamed), and
    // every piece of a cut block the cost of its partial result (split_keys: written, and read again by the combine pass).
    int64_t narrow_chunk = 1 << 30, wide_chunk = 1 << 30;
    auto choose_chunk = [&](const std::vector<std::pair<int32_t, int32_t>>& runs, int64_t slots, int64_t granule,
                            int64_t min_chunk, int64_t item_keys, int64_t split_keys) {
        auto count_items = [&](int64_t chunk, int64_t* pieces_of_cut_blocks = nullptr) {
            int64_t n = 0, cut = 0;
            for (const auto& r : runs) {
                const int64_t pieces = ceil_div(r.first, chunk);
                n += pieces * r.second;
                if (pieces > 1) cut += pieces * r.second;
            }
            if (pieces_of_cut_blocks) *pieces_of_cut_blocks = cut;
            return n;
        };
        int64_t n_blocks = 0, max_len = 0, keys = 0;
        for (const auto& r : runs) {
            n_blocks += r.second;
            max_len = std::max<int64_t>(max_len, r.first);
            keys += (int64_t)r.first * r.second;
        }
        const int64_t base = ceil_div(keys, slots);
        int64_t best_cost = -1, best = 1 << 30;
        auto consider = [&](int64_t chunk) {
            int64_t cut = 0;
            const int64_t n = count_items(chunk, &cut);
            const int64_t piece = std::min(chunk, max_len);
            const int64_t cost = (n <= slots ? piece + item_keys : base + piece / 2 + ceil_div(item_keys * n, slots)) +
                                 ceil_div(split_keys * cut, slots);
            if (best_cost < 0 || cost < best_cost) {
                best_cost = cost;
                best = chunk;
            }
        };
        // one round on all, half or a quarter of the slots: the smallest chunk whose items fit
        for (int64_t target = slots; target >= slots / 4 && target >= n_blocks; target /= 2) {
            int64_t lo = min_chunk / granule - 1, hi = std::max<int64_t>(min_chunk / granule, ceil_div(max_len, granule));
            while (lo + 1 < hi) {                          // count(hi) = n_blocks <= target
                const int64_t mid = (lo + hi) / 2;
                (count_items(mid * granule) > target ? lo : hi) = mid;
            }
            consider(hi * granule);
        }
        // ~2, 3, 4 items per slot
        for (int per_slot = n_blocks <= slots ? 2 : 1; per_slot <= 4; ++per_slot) {
            const int64_t chunk = std::max<int64_t>(min_chunk, round_up(ceil_div(base, per_slot), granule));
            consider(chunk);
            if (chunk == min_chunk) break;                 // (smaller chunks are not allowed)
        }
        if (split_keys > 0) consider(round_up(max_len, granule));    // whole blocks
        return best;
    };
    if (opt.force_kv_splits <= 0) {
        const int64_t slots = opt.wg_slots;
        if (narrow_keys > 0) {
            // Two or more rows per slot: whole rows balance well by themselves (longest first); only a row longer
            // than a slot's share of the keys is cut.
            int64_t n_blocks = 0;
            for (const auto& r : narrow_runs) n_blocks += r.second;
            if (n_blocks >= 2 * slots)
                narrow_chunk = std::max<int64_t>(MIN_NARROW_CHUNK, round_up(ceil_div(narrow_keys, slots), KV_TILE));
            else
                narrow_chunk = choose_chunk(narrow_runs, slots, KV_TILE, MIN_NARROW_CHUNK, NARROW_ITEM_KEYS, 0);
        }
        // tiles: cut only when fewer than two per slot exist
        if (n_wide > 0 && n_wide < 2 * slots) {
            if (narrow_keys == 0) {
                wide_chunk = choose_chunk(wide_runs, slots, WIDE_STAGE_KEYS, MIN_WIDE_CHUNK, WIDE_ITEM_KEYS, WIDE_SPLIT_KEYS);
            } else {
                // next to decode rows (a mixed batch) the tiles are not alone on the slots and the estimate above does
                // not hold; measured best there: about two pieces per slot, cut by the longest tile, at least 1024 keys
                int64_t max_keys = 0;
                for (const auto& r : wide_runs) max_keys = std::max<int64_t>(max_keys, r.first);
                const int64_t want = ceil_div(2 * slots, n_wide);
                wide_chunk = std::max<int64_t>(MIN_WIDE_CHUNK_MIXED, round_up(ceil_div(max_keys, want), KV_TILE));
            }
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
            it.C = out.reqs[b.req].C;
            it.row_off = out.reqs[b.req].row_off;
            it.pad[0] = it.pad[1] = it.pad[2] = 0;
            const int64_t keys = it.kv_end - it.kv_begin;
            const int64_t cost = b.kind == KIND_WIDE ? keys * 4 : keys;
            order.push_back(Cost{cost, (int32_t)out.items.size()});
            out.items.push_back(it);
            if (b.kind == KIND_WIDE) ++out.num_wide; else ++out.num_narrow;
        }
    }

    // 4. launch order.  Workgroup i runs on XCD i % NUM_XCD, and each XCD has its own L2, so the position of
    //    an item in the launch order decides which L2 its K/V stream passes through.  Wide items that read
    //    the same stream (same request and KV head: the query tiles of one prefill chunk, which all start at
    //    key 0 and advance at the same rate) are therefore queued on the same XCD, next to each other, so
    //    that the stream is fetched from HBM once and the other tiles hit in L2:
    //      a. streams are dealt to the XCDs longest-processing-time first (a stream that is a large part of
    //         one XCD's share is first cut into pieces, tile by tile);
    //      b. inside an XCD, streams run longest keys first, and tiles of a stream longest first, so the
    //         last workgroups of the launch are the short ones;
    //         (then single items move from the heaviest queue to the lightest until they are level);
    //      c. the XCD queues are interleaved position by position; null items pad a queue that is shorter
    //         than the others.
    //    Narrow items stream their key range exactly once, so they only need balance: longest first.  In a
    //    mixed batch the two kinds alternate in runs of NUM_XCD in proportion to their total cost, so that at
    //    any time some CUs run compute-bound tiles while others stream decode rows.
    //    Everything is stable and depends on the lengths only.
    std::vector<int32_t> wide_ix, narrow_ix;
    double wide_cost = 0, narrow_cost = 0;
    {
        std::vector<Cost> nar;
        struct Stream { int64_t cost = 0; int64_t max_keys = 0; std::vector<Cost> items; };
        std::vector<Stream> streams;
        std::vector<int32_t> stream_of((size_t)num_reqs * s.Hkv, -1);
        for (const Cost& c : order) {
            const Item& it = out.items[c.idx];
            if (((it.heads >> 24) & 0xff) != KIND_WIDE) {
                nar.push_back(c);
                narrow_cost += (double)c.cost;
                continue;
            }
            wide_cost += (double)c.cost;
            int32_t& sid = stream_of[(size_t)it.req * s.Hkv + (it.heads & 0xff)];
            if (sid < 0) {
                sid = (int32_t)streams.size();
                streams.emplace_back();
            }
            Stream& st = streams[sid];
            st.cost += c.cost;
            st.max_keys = std::max<int64_t>(st.max_keys, it.kv_end);
            st.items.push_back(c);
        }
        std::stable_sort(nar.begin(), nar.end(), [](const Cost& a, const Cost& b) { return a.cost > b.cost; });
        for (const Cost& c : nar) narrow_ix.push_back(c.idx);

        // a. pieces well below one XCD's share, dealt to the least loaded XCD, heaviest first
        const int64_t share = std::max<int64_t>(1, ceil_div((int64_t)wide_cost, NUM_XCD));
        std::vector<Stream> pieces;
        for (Stream& st : streams) {
            std::stable_sort(st.items.begin(), st.items.end(), [](const Cost& a, const Cost& b) { return a.cost > b.cost; });
            // pieces of a quarter share let the dies mix long and short streams, but a piece keeps at least 8
            // tiles so that a die still reuses what it fetched; a power of two, so that equal streams deal evenly
            const int64_t want = std::max<int64_t>(1, std::min<int64_t>(ceil_div(4 * st.cost, share), (int64_t)st.items.size() / 8));
            int np = 1;
            while (2 * np <= want && np < NUM_XCD) np *= 2;
            const size_t base = pieces.size();
            pieces.resize(base + np);
            for (size_t i = 0; i < st.items.size(); ++i) {         // deal the tiles round-robin: equal pieces
                Stream& pc = pieces[base + i % np];
                pc.items.push_back(st.items[i]);
                pc.cost += st.items[i].cost;
                pc.max_keys = st.max_keys;
            }
        }
        std::vector<int32_t> by_cost(pieces.size());
        for (size_t i = 0; i < pieces.size(); ++i) by_cost[i] = (int32_t)i;
        std::stable_sort(by_cost.begin(), by_cost.end(), [&](int32_t a, int32_t b) { return pieces[a].cost > pieces[b].cost; });
        std::vector<int32_t> bin_pieces[NUM_XCD];
        int64_t bin_cost[NUM_XCD] = {0};
        for (int32_t pi : by_cost) {
            int best = 0;
            for (int x = 1; x < NUM_XCD; ++x)
                if (bin_cost[x] < bin_cost[best]) best = x;
            bin_pieces[best].push_back(pi);
            bin_cost[best] += pieces[pi].cost;
        }
        // b. queue of every XCD
        std::vector<Cost> queue[NUM_XCD];
        for (int x = 0; x < NUM_XCD; ++x) {
            std::stable_sort(bin_pieces[x].begin(), bin_pieces[x].end(),
                             [&](int32_t a, int32_t b) { return pieces[a].max_keys > pieces[b].max_keys; });
            for (int32_t pi : bin_pieces[x])
                for (const Cost& c : pieces[pi].items) queue[x].push_back(c);
        }
        //    level the queues: the heaviest queue hands its last (shortest) item to the lightest one while that
        //    lowers the maximum.  The result is kept only if the launch gets shorter when every queue is
        //    replayed on the CUs of one XCD, which also sees the granularity of a few long items per CU.
        const int cus = std::max(1, opt.wg_slots / NUM_XCD);
        std::vector<int64_t> cu_free;
        auto finish_time = [&](const std::vector<Cost>& q) {
            cu_free.assign(cus, 0);                                 // min-heap of the CUs' free times
            auto later = [](int64_t a, int64_t b) { return a > b; };
            int64_t last = 0;
            for (const Cost& c : q) {
                std::pop_heap(cu_free.begin(), cu_free.end(), later);
                cu_free.back() += c.cost;
                last = std::max(last, cu_free.back());
                std::push_heap(cu_free.begin(), cu_free.end(), later);
            }
            return last;
        };
        auto launch_time = [&](const std::vector<Cost>* q) {
            int64_t t = 0;
            for (int x = 0; x < NUM_XCD; ++x) t = std::max(t, finish_time(q[x]));
            return t;
        };
        {
            std::vector<Cost> trial[NUM_XCD];
            int64_t sum[NUM_XCD];
            for (int x = 0; x < NUM_XCD; ++x) {
                trial[x] = queue[x];
                sum[x] = bin_cost[x];
            }
            bool moved = false;
            for (size_t moves = 0; moves < out.items.size(); ++moves) {
                int hi = 0, lo = 0;
                for (int x = 1; x < NUM_XCD; ++x) {
                    if (sum[x] > sum[hi]) hi = x;
                    if (sum[x] < sum[lo]) lo = x;
                }
                if (trial[hi].empty()) break;
                const Cost c = trial[hi].back();
                if (sum[lo] + c.cost >= sum[hi]) break;
                trial[hi].pop_back();
                trial[lo].push_back(c);
                sum[hi] -= c.cost;
                sum[lo] += c.cost;
                moved = true;
            }
            if (moved && launch_time(trial) < launch_time(queue))
                for (int x = 0; x < NUM_XCD; ++x) queue[x].swap(trial[x]);
        }
        // c. interleave; -1 stands for a null item that pads a shorter queue
        size_t longest = 0;
        for (int x = 0; x < NUM_XCD; ++x) longest = std::max(longest, queue[x].size());
        for (size_t j = 0; j < longest; ++j)
            for (int x = 0; x < NUM_XCD; ++x) wide_ix.push_back(j < queue[x].size() ? queue[x][j].idx : -1);
        while (!wide_ix.empty() && wide_ix.back() < 0) wide_ix.pop_back();
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
            for (int k = 0; k < NUM_XCD; ++k) {
                if (take_wide ? iw >= wide_ix.size() : in >= narrow_ix.size()) break;
                const int32_t idx = take_wide ? wide_ix[iw++] : narrow_ix[in++];
                if (idx < 0) {
                    sorted.push_back(Item{-1, pack_heads(0, 0, 0, KIND_NULL), 0, 0, 0, 0, -1, 0, 0, {0, 0, 0}});
                    continue;
                }
                const Item& it = out.items[idx];
                const double keys = it.kv_end - it.kv_begin;
                (take_wide ? dw : dn) += take_wide ? keys * 4 : keys;
                sorted.push_back(it);
            }
        }
    }
    out.items.swap(sorted);

    // 4b. append items: consecutive runs of packed rows, whatever request they belong to (a decode batch of 96
    //     rows is two items, not 96); each names the request and token its first row belongs to.
    if (opt.append_items) {
        int r = 0;
        for (int64_t row = 0; row < out.sum_L; row += APPEND_ITEM_ROWS) {
            while (row >= (int64_t)out.reqs[r].row_off + out.reqs[r].L) ++r;
            Item it{r, pack_heads(0, 0, 0, KIND_APPEND), (int32_t)(row - out.reqs[r].row_off),
                    (int32_t)std::min<int64_t>(APPEND_ITEM_ROWS, out.sum_L - row), 0, 0, -1, out.reqs[r].C, out.reqs[r].row_off,
                    {0, 0, 0}};
            out.items.push_back(it);
            ++out.num_append;
        }
    }

    // 5. byte layout
    out.off_reqs = 0;
    out.off_items = round_up((int64_t)out.reqs.size() * sizeof(ReqInfo), 256);
    out.off_combs = out.off_items + round_up((int64_t)out.items.size() * sizeof(Item), 256);
    out.off_queues = out.off_combs + round_up((int64_t)out.combs.size() * sizeof(CombItem), 256);
    out.plan_bytes = out.off_queues + 256;
    // persistent workgroups pay off where tiles are in the launch (the dies finish together: -1.2 % on configuration 2, -3.5 % on
    // the fused mixed launch of configuration 3); a launch of decode rows alone gains nothing from them (+-1 %)
    out.grid = (int32_t)(out.num_wide > 0 ? std::min<int64_t>((int64_t)out.items.size(), opt.wg_slots) : (int64_t)out.items.size());
    for (int q = 0; q < NUM_QUEUES; ++q) out.queue_heads[q] = out.grid > q ? (out.grid - q + NUM_QUEUES - 1) / NUM_QUEUES : 0;
    out.off_partial = out.plan_bytes;
    out.total_bytes = out.off_partial + round_up(out.partial_floats * 4, 256);
    if (out.total_bytes == 0) out.total_bytes = 256;
}

}  // namespace ampd
