// Host-only planner of the data-swapping engine: decides which saved tensors
// leave the device between their last forward use and their first backward
// use (Sections 3.1-3.3), from sizes, op indices, a device budget, a
// look-ahead distance and include / exclude tags.  Pure integer work.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <vector>

namespace mi3d {

struct PlanTensor {
    int id = -1;
    size_t bytes = 0;
    int produce_op = 0, last_fwd_use_op = 0, bwd_first_use_op = 0, bwd_last_use_op = 0;
    unsigned tags = 0;
    bool planned = false;
    int prefetch_op = 0;     // op at whose launch the swap-in is issued (valid if planned)
    size_t host_offset = 0;  // slot in the pinned pool (valid if planned)
};

struct PlanParams {
    size_t budget_bytes = 0;
    size_t host_pool_bytes = 0;  // 0 = do not check
    int lookahead = 1;
    int policy = 0;
    int n_tensors = -1;
    unsigned exclude_tags = 0, include_tags = 0;
    int n_fwd_ops = 0, n_ops = 0;
    // optional measured op durations (ms, one per op) and host-link rate: with them the swap-ins are scheduled by
    // time (see plan_swaps), with `lookahead` as the minimum distance in ops
    const std::vector<float>* op_ms = nullptr;
    float link_gbs = 0.f;
};

struct PlanResult {
    uint64_t planned_peak = 0, unswapped_peak = 0;
    int n_planned = 0;
    size_t host_bytes = 0;
};

// Resident bytes at `op`: transients plus every tensor that is on the device
// then.  A tensor that is not swapped lives from produce_op to
// bwd_last_use_op; a swapped one from produce_op to last_fwd_use_op and again
// from prefetch_op to bwd_last_use_op.
uint64_t plan_bytes_at(const std::vector<PlanTensor>& ts, const std::vector<size_t>& transient, int op, bool ignore_plan);

// Fills planned / prefetch_op / host_offset.  Returns 0, MI3D_ERR_OVER_BUDGET
// or MI3D_ERR_HOST_POOL (the plan is filled in either way), or
// MI3D_ERR_INVALID_ARG for an inconsistent timeline.
int plan_swaps(std::vector<PlanTensor>& ts, const std::vector<size_t>& transient, const PlanParams& p, PlanResult* res);

}  // namespace mi3d
