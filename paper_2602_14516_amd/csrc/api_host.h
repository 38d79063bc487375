// Host half of the C ABI: argument validation and work planning, shared by api.cpp (which enqueues GPU work) and
// api_host.cpp (the entry points that never touch a GPU).  No HIP types: this half also builds with a plain host
// compiler, which is how it is run under the address / undefined-behaviour sanitizers.
#pragma once
#include "ampd.h"
#include "plan.h"

namespace ampd {
namespace host {

int log2_exact(int x);                                   // log2 of a power of two, -1 otherwise
// need_pools: also require the device pointers an entry point that enqueues work dereferences
ampd_status validate(const ampd_kv_cache* c, const ampd_batch* b, bool need_pools);
// with_append: plan an append-then-attend call; for a bf16 cache the page writes then ride in the attention launch
// as append items (an 8-bit cache quantises in a launch of its own first)
// *plan points at a plan owned by the calling thread: valid until that thread's next make_plan
ampd_status make_plan(const ampd_kv_cache* c, const ampd_batch* b, const ampd_plan_options* o, bool with_append, const Plan** plan);

}  // namespace host
}  // namespace ampd
