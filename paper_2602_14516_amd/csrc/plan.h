// Host-side work planner: cuts a batch of (C_r, L_r) rows into GPU work items.
//
// A prefill task is described to the scheduler by its history length and incremental
// length only (paper Section 3, T_pre(l_hist, l_incr)); a decode step by one token per
// request (T_dec).  From these lengths alone the planner derives, per request and KV head:
//   * wide items   -- tiles of up to 256 query rows (tokens x grouped heads) whose 8 waves
//                     share K/V tiles staged in LDS (compute-bound prefill work), and
//   * narrow items -- blocks of at most 32 query rows (decode rows, very short chunks)
//                     whose 8 waves split the key range (bandwidth-bound work),
//   * append items -- (bf16 cache, append-then-attend calls) runs of packed new rows to be copied into
//                     their pages by the same launch; they close the work list, where they fill the CUs
//                     that run out of attention work first,
// optionally cutting an item's key range into pieces (split-KV) that a combine pass merges.
// Workgroup i of a launch runs on accelerator die (XCD) i % 8, each with its own L2, so the
// launch order also decides which L2 a K/V stream passes through; null items (no work) pad the
// per-die queues to equal length.
// Everything is computed from logical positions, never from physical page ids, so results
// are bitwise independent of where pages live in the pool.
#pragma once
#include <cstdint>
#include <vector>

namespace ampd {

enum : int32_t { KIND_WIDE = 0, KIND_NARROW = 1, KIND_NULL = 2, KIND_APPEND = 3 };

constexpr int ATTN_WAVES = 8;      // waves of an attention workgroup (one workgroup per CU)
constexpr int NUM_QUEUES = 8;      // accelerator dies (XCDs): workgroup i of a launch is dispatched to die i % 8
constexpr int APPEND_MAX_REQS = 128;   // requests per append launch (their lengths travel as kernel arguments)

struct ReqInfo {          // 16 B, one per request, device-visible
    int32_t C, L, row_off, pad;
};

struct Item {             // 48 B, one per attention workgroup, device-visible
    int32_t req;          // -1 for a null item
    int32_t heads;        // kvh | g0 << 8 | gn << 16 | kind << 24
    int32_t q0, nq;       // first new-token index and token count of this item
    int32_t kv_begin, kv_end;   // key range [begin, end) in logical positions
    int32_t part_off;     // float offset of this item's partial slot, or -1: write final output
    int32_t C;            // context length of the request and the first row of its packed q / out rows:
    int32_t row_off;      // copies of its ReqInfo, so that a workgroup starts with one dependent load less
    int32_t pad[3];
};
static_assert(sizeof(Item) == 48, "device layout");

struct CombItem {         // 32 B, one per query tile whose key range was split
    int32_t req;
    int32_t heads;
    int32_t q0, nq;
    int32_t part_off;     // float offset of split 0
    int32_t nsplit;
    int32_t part_stride;  // floats between consecutive splits
    int32_t pad;
};

inline int32_t pack_heads(int kvh, int g0, int gn, int kind) {
    return kvh | (g0 << 8) | (gn << 16) | (kind << 24);
}

struct Shape {
    int Hq, Hkv, D, P;
};

constexpr int APPEND_ITEM_ROWS = 64;   // packed rows (new tokens, all heads, K and V) that one append item moves

struct PlanOptions {
    int force_kv_splits = 0;
    int wg_slots = 256;   // workgroups resident at once: one per CU
    bool append_items = false;   // the page writes of the call ride in the attention launch (bf16 cache): append items
                                 // of APPEND_ITEM_ROWS packed rows each close the work list
};

struct Plan {
    std::vector<ReqInfo> reqs;
    std::vector<Item> items;
    std::vector<CombItem> combs;
    int64_t num_wide = 0, num_narrow = 0, num_append = 0;
    int64_t partial_floats = 0;
    int64_t sum_L = 0;
    // A launch with tiles in it and more items than workgroup slots runs `grid` persistent workgroups (otherwise grid = the
    // number of items, one workgroup each): workgroup i starts with item i
    // and then takes items from the queue of its die (queue q = items q, q + NUM_QUEUES, ...; queue_heads[q] = the
    // queue's position of the first item nobody has started), helping out on other queues when its own is empty.
    int32_t grid = 0;
    int32_t queue_heads[NUM_QUEUES] = {0, 0, 0, 0, 0, 0, 0, 0};
    // byte layout of the device copy: [reqs][items][combs][queue heads], each 256 B aligned
    int64_t off_reqs = 0, off_items = 0, off_combs = 0, off_queues = 0, plan_bytes = 0;
    int64_t off_partial = 0, total_bytes = 0;
};

// ctx_len / incr_len must already be validated (non-negative, no overflow).
void build_plan(const Shape& s, int num_reqs, const int32_t* ctx_len, const int32_t* incr_len,
                const PlanOptions& opt, Plan& out);

}  // namespace ampd
