// Kernel parameter blocks and launcher declarations shared by kernels.hip and api.cpp.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.h"

namespace ampd {

enum : int { KV_BF16 = 0, KV_FP8 = 1 };

struct AttnParams {
    const void* q;             // bf16 [sum L][Hq][D]
    void* out;                 // bf16 [sum L][Hq][D]
    const void* k_new;         // bf16 [sum L][Hkv][D]: the new tokens of this call when their page writes ride in the
    const void* v_new;         //   attention launch (bf16 cache; keys >= C are then read from here), else null
    const void* k_pool;        // [pages][Hkv][P][D]
    const void* v_pool;
    const float* k_scale;      // [pages][Hkv] (8-bit cache) or null
    const float* v_scale;
    const int32_t* block_table;
    const ReqInfo* reqs;
    const Item* items;
    const CombItem* combs;
    float* partial;
    int32_t Hq, Hkv, P, logP, max_pages;
    float c_log2;              // softmax_scale * log2(e)
    // The host's pinned staging slot this call's work list came from may be reused once this launch runs (every copy
    // out of the slot precedes it in stream order): the first workgroup stores slot_seq to *slot_flag (pinned host memory).
    uint32_t* slot_flag;
    uint32_t slot_seq;
    // Persistent launch (more items than workgroups): per-die queue heads in the workspace, see Plan::queue_heads.
    int32_t* queue_heads;
    int32_t nitems;
};

struct AppendParams {
    const void* k_new;         // bf16 [sum L][Hkv][D]
    const void* v_new;
    void* k_pool;
    void* v_pool;
    float* k_scale;
    float* v_scale;
    const int32_t* block_table;
    int32_t Hkv, D, P, logP, max_pages, req0;
    int32_t h0, hn;            // KV heads [h0, h0 + hn) of the pool; the packed rows hold hn heads
    // Optional rider: the work list of the attention launch that follows, copied from pinned host memory
    // into the workspace by one extra z-slice of this launch (up_n16 16-byte vectors; 0: none).
    const void* up_src;
    void* up_dst;
    int32_t up_n16;
    int32_t C[APPEND_MAX_REQS], L[APPEND_MAX_REQS], row_off[APPEND_MAX_REQS];
};

// h_src: pinned, device-visible host memory; bytes is rounded up to 16
hipError_t launch_upload(const void* h_src, void* d_dst, size_t bytes, hipStream_t st);
hipError_t launch_attn(const AttnParams& p, int D, int kvt, int grid, hipStream_t st);
// max_rows: the largest nq * heads among the split tiles (sizes the second grid dimension)
hipError_t launch_combine(const AttnParams& p, int D, int ncombs, int max_rows, int max_splits, hipStream_t st);
hipError_t launch_append(const AppendParams& p, int kvt, int max_pages_touched, int nreq, hipStream_t st);
// bf16 only: pack = pages -> packed rows (k_new / v_new are written), otherwise packed rows -> pages
hipError_t launch_kv_move(const AppendParams& p, bool pack, int max_pages_touched, int nreq, hipStream_t st);

}  // namespace ampd
