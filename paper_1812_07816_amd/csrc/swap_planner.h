// Host-only planner of the data-swapping engine: decides which saved tensors
// leave the device between their last forward use and their first backward
// use (Sections 3.1-3.3), from sizes, op indices, a device budget, a
// look-ahead distance and include / exclude tags.  A tensor that leaves is
// either copied to the host and back (swapped) or dropped and computed again
// from tensors that are on the device (the re-computation method the paper
// compares with in Section 5, and the mix of the two it proposes there for
// slow host links).
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
    bool planned = false;    // swapped
    int prefetch_op = 0;     // op at whose launch the swap-in is issued (valid if planned)
    size_t host_offset = 0;  // slot in the pinned pool (valid if planned)
    // re-computation: cost of producing the tensor again (ms, < 0 = not possible) and the tensors that must be on
    // the device for it (-1 = none)
    float recompute_ms = -1.f;
    int dep[2] = {-1, -1};
    bool recompute = false;      // dropped after its last forward use, produced again at bwd_first_use_op
    int bwd_first_use_reg = -1;  // bwd_first_use_op as registered (the plan lowers it for tensors a re-computation reads)
    // static placement in the device arena: offset of the tensor's first stay on the device (from its production) and,
    // for a tensor that leaves and comes back, of its second stay (from its swap-in or re-computation)
    size_t arena_off[2] = {0, 0};
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
    int eviction = 0;            // MI3D_EVICT_SWAP / _RECOMPUTE / _HYBRID
};

struct PlanResult {
    uint64_t planned_peak = 0, unswapped_peak = 0;
    int n_planned = 0;
    size_t host_bytes = 0;
    int n_recompute = 0;
    double recompute_ms = 0.0;   // sum of the costs of the chosen re-computations
    uint64_t static_arena_bytes = 0;   // extent of the static placement (place_static)
};

// Resident bytes at `op`: transients plus every tensor that is on the device
// then.  A tensor that is not swapped lives from produce_op to
// bwd_last_use_op; a swapped one from produce_op to last_fwd_use_op and again
// from prefetch_op to bwd_last_use_op; a re-computed one from produce_op to
// last_fwd_use_op and again from bwd_first_use_op to bwd_last_use_op.
uint64_t plan_bytes_at(const std::vector<PlanTensor>& ts, const std::vector<size_t>& transient, int op, bool ignore_plan);

// Static placement of the saved tensors in one arena, from their lifetimes under the current plan: every stay of a tensor on
// the device (one for a tensor that is kept, two for one that is swapped or re-computed) is an interval of ops and gets a
// fixed offset, largest tensors first, each at the lowest offset where it overlaps no stay already placed that it shares an
// op with.  The first stay of a swapped tensor lasts until its copy to the host has finished: with op times that is
// modelled (the copies leave one after the other in production order at the link rate), else one op of grace is added.
// Sizes count in units of 256 bytes.  Fills arena_off and returns the extent of the arena.
uint64_t place_static(std::vector<PlanTensor>& ts, const PlanParams& p);

// Fills planned / prefetch_op / host_offset.  Returns 0, MI3D_ERR_OVER_BUDGET
// or MI3D_ERR_HOST_POOL (the plan is filled in either way), or
// MI3D_ERR_INVALID_ARG for an inconsistent timeline.
int plan_swaps(std::vector<PlanTensor>& ts, const std::vector<size_t>& transient, const PlanParams& p, PlanResult* res);

}  // namespace mi3d
