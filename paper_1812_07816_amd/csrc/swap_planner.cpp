#include "swap_planner.h"

#include <algorithm>

#include "../../include/mi3d.h"

namespace mi3d {

static bool resident(const PlanTensor& t, int op, bool ignore_plan) {
    if (op < t.produce_op || op > t.bwd_last_use_op) return false;
    if (ignore_plan) return true;
    if (t.recompute) return op <= t.last_fwd_use_op || op >= t.bwd_first_use_op;
    if (!t.planned) return true;
    return op <= t.last_fwd_use_op || op >= t.prefetch_op;
}

uint64_t plan_bytes_at(const std::vector<PlanTensor>& ts, const std::vector<size_t>& transient, int op, bool ignore_plan) {
    uint64_t b = (op >= 0 && op < (int)transient.size()) ? transient[op] : 0;
    for (const PlanTensor& t : ts)
        if (resident(t, op, ignore_plan)) b += t.bytes;
    return b;
}

static uint64_t peak(const std::vector<PlanTensor>& ts, const std::vector<size_t>& tr, int n_ops, bool ignore_plan, int* at) {
    uint64_t best = 0;
    int where = 0;
    for (int op = 0; op < n_ops; ++op) {
        uint64_t b = plan_bytes_at(ts, tr, op, ignore_plan);
        if (b > best) { best = b; where = op; }
    }
    if (at) *at = where;
    return best;
}

// Prefetch op by op count: `lookahead` ops before the first backward use, but never before the backward pass
// starts or the forward use ends.
static int prefetch_by_ops(const PlanTensor& t, const PlanParams& p) {
    int pf = t.bwd_first_use_op - p.lookahead;
    pf = std::max(pf, p.n_fwd_ops);
    pf = std::max(pf, t.last_fwd_use_op + 1);
    return std::min(pf, t.bwd_first_use_op);
}

// Prefetch ops by time for the planned tensors: the swap-ins share one copy stream, so they are laid out back
// to back, latest use first: a copy must end by the start of its tensor's first backward use and by the start
// of the copy scheduled after it; its duration is bytes / link rate plus 15 % and 50 us; it is issued at the
// latest op that starts no later than that.  Never later than the op-count rule.
static void prefetch_by_time(std::vector<PlanTensor>& ts, const PlanParams& p, int n_ops) {
    const std::vector<float>& ms = *p.op_ms;
    std::vector<double> extra(n_ops + 1, 0.0);   // re-computations run at the first backward use of their tensor
    for (const PlanTensor& t : ts)
        if (t.recompute && t.bwd_first_use_op >= 0 && t.bwd_first_use_op < n_ops) extra[t.bwd_first_use_op] += t.recompute_ms;
    std::vector<double> start(n_ops + 1, 0.0);
    for (int op = 0; op < n_ops; ++op) start[op + 1] = start[op] + (op < (int)ms.size() ? (double)ms[op] : 0.0) + extra[op];
    std::vector<int> order;
    for (int i = 0; i < (int)ts.size(); ++i)
        if (ts[i].planned) order.push_back(i);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return ts[a].bwd_first_use_op > ts[b].bwd_first_use_op; });
    double next_start = 1e300;
    for (int i : order) {
        PlanTensor& t = ts[i];
        const double dur = (double)t.bytes / ((double)p.link_gbs * 1e6) * 1.15 + 0.05;
        const double finish = std::min(start[std::min(t.bwd_first_use_op, n_ops)], next_start);
        const double begin = finish - dur;
        next_start = begin;
        int pf = prefetch_by_ops(t, p);
        while (pf > 0 && start[pf] > begin) --pf;
        pf = std::max(pf, p.n_fwd_ops);
        pf = std::max(pf, t.last_fwd_use_op + 1);
        t.prefetch_op = std::min(pf, t.bwd_first_use_op);
    }
}

// A re-computation reads its dependencies at its tensor's first backward use: they must be on the device by
// then, so their own first backward use is lowered to that op (transitively: a dependency that is re-computed
// itself is produced first, from its own dependencies).  Resets the prefetch ops to the op-count rule.
static void apply_deps(std::vector<PlanTensor>& ts, const PlanParams& p) {
    for (PlanTensor& t : ts) t.bwd_first_use_op = t.bwd_first_use_reg;
    bool changed = true;
    for (size_t guard = 0; changed && guard < ts.size() + 2; ++guard) {
        changed = false;
        for (const PlanTensor& t : ts) {
            if (!t.recompute) continue;
            for (int d : t.dep) {
                if (d < 0) continue;
                for (PlanTensor& u : ts)
                    if (u.id == d && u.bwd_first_use_op > t.bwd_first_use_op) {
                        u.bwd_first_use_op = t.bwd_first_use_op;
                        changed = true;
                    }
            }
        }
    }
    for (PlanTensor& t : ts) t.prefetch_op = prefetch_by_ops(t, p);
}

uint64_t place_static(std::vector<PlanTensor>& ts, const PlanParams& p) {
    int n_ops = p.n_ops;
    for (const PlanTensor& t : ts) n_ops = std::max(n_ops, t.bwd_last_use_op + 1);
    const bool timed = p.op_ms && !p.op_ms->empty() && p.link_gbs > 0.f;
    // start time of every op (ms) for the copy model
    std::vector<double> start(n_ops + 1, 0.0);
    if (timed)
        for (int op = 0; op < n_ops; ++op) start[op + 1] = start[op] + (op < (int)p.op_ms->size() ? (double)(*p.op_ms)[op] : 0.0);
    // end of the first stay of the swapped tensors: the copies share one stream and leave in production order
    std::vector<int> fwd_end(ts.size());
    std::vector<int> order(ts.size());
    for (size_t i = 0; i < ts.size(); ++i) order[i] = (int)i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return ts[a].produce_op < ts[b].produce_op; });
    double link_free = 0.0;
    for (int i : order) {
        const PlanTensor& t = ts[i];
        fwd_end[i] = t.last_fwd_use_op;
        if (!t.planned) continue;
        if (!timed) { fwd_end[i] = std::min(t.last_fwd_use_op + 1, std::max(t.prefetch_op - 1, t.last_fwd_use_op)); continue; }
        const double begin = std::max(start[std::min(t.produce_op + 1, n_ops)], link_free);
        const double finish = begin + (double)t.bytes / ((double)p.link_gbs * 1e6) * 1.15 + 0.05;
        link_free = finish;
        int e = t.last_fwd_use_op;
        while (e + 1 < t.prefetch_op && start[e + 1] < finish) ++e;   // ops that start while the copy still reads the block
        fwd_end[i] = e;
    }
    struct Stay { int tensor, which, from, to; size_t size, off; };
    std::vector<Stay> stays;
    for (size_t i = 0; i < ts.size(); ++i) {
        const PlanTensor& t = ts[i];
        const size_t sz = (t.bytes + 255) & ~(size_t)255;
        if (!t.planned && !t.recompute) {
            stays.push_back({(int)i, 0, t.produce_op, t.bwd_last_use_op, sz, 0});
        } else {
            stays.push_back({(int)i, 0, t.produce_op, fwd_end[i], sz, 0});
            stays.push_back({(int)i, 1, t.recompute ? t.bwd_first_use_op : t.prefetch_op, t.bwd_last_use_op, sz, 0});
        }
    }
    std::vector<int> by_size(stays.size());
    for (size_t i = 0; i < stays.size(); ++i) by_size[i] = (int)i;
    std::stable_sort(by_size.begin(), by_size.end(), [&](int a, int b) {
        return stays[a].size != stays[b].size ? stays[a].size > stays[b].size : stays[a].from < stays[b].from;
    });
    std::vector<int> placed;
    uint64_t extent = 0;
    for (int si : by_size) {
        Stay& s = stays[si];
        // the stays already placed that share an op with this one, by offset
        std::vector<std::pair<size_t, size_t>> busy;
        for (int pi : placed) {
            const Stay& q = stays[pi];
            if (q.from <= s.to && s.from <= q.to) busy.emplace_back(q.off, q.off + q.size);
        }
        std::sort(busy.begin(), busy.end());
        size_t off = 0;
        for (const auto& b : busy) {
            if (off + s.size <= b.first) break;
            off = std::max(off, b.second);
        }
        s.off = off;
        extent = std::max<uint64_t>(extent, off + s.size);
        placed.push_back(si);
    }
    for (const Stay& s : stays) ts[s.tensor].arena_off[s.which] = s.off;
    return extent;
}

int plan_swaps(std::vector<PlanTensor>& ts, const std::vector<size_t>& transient, const PlanParams& p, PlanResult* res) {
    int n_ops = p.n_ops;
    for (const PlanTensor& t : ts) n_ops = std::max(n_ops, t.bwd_last_use_op + 1);
    if (p.n_fwd_ops < 0 || p.n_fwd_ops > n_ops || p.lookahead < 0) return MI3D_ERR_INVALID_ARG;
    if (p.eviction != MI3D_EVICT_SWAP && p.eviction != MI3D_EVICT_RECOMPUTE && p.eviction != MI3D_EVICT_HYBRID) return MI3D_ERR_INVALID_ARG;
    const bool timed = p.op_ms && !p.op_ms->empty() && p.link_gbs > 0.f;
    for (PlanTensor& t : ts) {
        if (t.bwd_first_use_reg < 0) t.bwd_first_use_reg = t.bwd_first_use_op;
        t.bwd_first_use_op = t.bwd_first_use_reg;
        if (t.produce_op > t.last_fwd_use_op || t.last_fwd_use_op >= t.bwd_first_use_op ||
            t.bwd_first_use_op > t.bwd_last_use_op || t.produce_op < 0)
            return MI3D_ERR_INVALID_ARG;
        t.planned = false;
        t.recompute = false;
        t.prefetch_op = prefetch_by_ops(t, p);
        t.host_offset = 0;
    }
    // a re-computation is possible if every dependency is a known tensor that is still alive at that op
    std::vector<char> recomputable(ts.size(), 0);
    for (size_t i = 0; i < ts.size(); ++i) {
        const PlanTensor& t = ts[i];
        bool ok = t.recompute_ms >= 0.f;
        for (int d : t.dep) {
            if (d < 0 || !ok) continue;
            bool found = false;
            for (const PlanTensor& u : ts)
                if (u.id == d && u.id != t.id && u.produce_op < t.produce_op + 1 && u.bwd_last_use_op >= t.bwd_first_use_op) found = true;
            ok = found;
        }
        recomputable[i] = ok;
    }
    const bool can_swap = p.eviction != MI3D_EVICT_RECOMPUTE;
    // hybrid: a copy that hides behind compute costs nothing, a re-computation always costs its compute time.  With
    // measured op times the plan is first made with swapping alone; it stands if it meets the budget and its copies fit
    // into the shorter of the two passes (swap-outs ride under the forward pass, swap-ins under the backward pass; 90 %
    // of it: the copies do not pack perfectly).  Otherwise, and without op times, a tensor is re-computed where that
    // costs less compute time than its swap-in alone would take on the link.  (Filling the link first and re-computing
    // only the rest was tried: under tight budgets the swapped tensors, which come back early and leave late, cost
    // more footprint than the re-computed ones and the plans no longer met the budgets the per-tensor rule meets.)
    const double link_rate = p.link_gbs > 0.f ? (double)p.link_gbs : 50.0;
    auto copy_ms = [&](int i) { return (double)ts[i].bytes / (link_rate * 1e6); };
    double link_room_ms = 0.0;
    if (timed) {
        double fwd = 0.0, bwd = 0.0;
        for (int op = 0; op < n_ops && op < (int)p.op_ms->size(); ++op) (op < p.n_fwd_ops ? fwd : bwd) += (double)(*p.op_ms)[op];
        link_room_ms = 0.9 * std::min(fwd, bwd);
    }
    bool swap_only = false;      // first attempt of the hybrid with op times
    auto wants_recompute = [&](int i) {
        if (p.eviction == MI3D_EVICT_SWAP || !recomputable[i] || swap_only) return false;
        if (!can_swap) return true;
        return (double)ts[i].recompute_ms < copy_ms(i);
    };
    auto plan_swap = [&](int i) { ts[i].planned = true; };
    auto dep_recomputed = [&](int i) {
        for (int d : ts[i].dep)
            for (const PlanTensor& u : ts)
                if (d >= 0 && u.id == d && u.recompute) return true;
        return false;
    };
    // the residency model with the current choice; with op times the chosen tensors come back earlier
    auto reschedule = [&]() {
        apply_deps(ts, p);
        if (timed) prefetch_by_time(ts, p, n_ops);
    };
    res->unswapped_peak = peak(ts, transient, n_ops, true, nullptr);

    auto eligible = [&](const PlanTensor& t) {
        if (t.tags & p.exclude_tags) return false;
        if (p.include_tags && !(t.tags & p.include_tags)) return false;
        return true;
    };
    // production order, the order in which swap-outs would be issued
    std::vector<int> order;
    for (int i = 0; i < (int)ts.size(); ++i)
        if (eligible(ts[i])) order.push_back(i);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return ts[a].produce_op < ts[b].produce_op; });

    if (p.policy != MI3D_SWAP_ALL && p.policy != MI3D_SWAP_FIRST_N && p.policy != MI3D_SWAP_BUDGET) return MI3D_ERR_INVALID_ARG;
    const int attempts = (p.eviction == MI3D_EVICT_HYBRID && timed) ? 2 : 1;
    for (int attempt = 0; attempt < attempts; ++attempt) {
    swap_only = attempts == 2 && attempt == 0;
    for (PlanTensor& t : ts) {
        t.planned = false;
        t.recompute = false;
        t.bwd_first_use_op = t.bwd_first_use_reg;
        t.prefetch_op = prefetch_by_ops(t, p);
    }
    if (p.policy == MI3D_SWAP_ALL || p.policy == MI3D_SWAP_FIRST_N) {
        int n = (int)order.size();
        if (p.policy == MI3D_SWAP_FIRST_N && p.n_tensors >= 0) n = std::min<int>(p.n_tensors, n);
        for (int k = 0; k < n; ++k) {
            const int i = order[k];
            // re-computing a tensor from one that is re-computed itself would bring the whole chain back at
            // once: such a tensor is swapped instead (or kept, where swapping is not allowed)
            if (wants_recompute(i) && !dep_recomputed(i)) ts[i].recompute = true;
            else if (can_swap) plan_swap(i);
        }
        reschedule();
    } else if (p.policy == MI3D_SWAP_BUDGET) {
        std::vector<int> chosen;
        for (;;) {
            int at = 0;
            uint64_t pk = peak(ts, transient, n_ops, false, &at);
            if (pk <= p.budget_bytes) break;
            // candidates: tensors idle at the peak op.  Prefer the longest idle
            // interval (early feature maps live longest), then the earlier
            // producer, then the larger tensor.
            int best = -1, best_gap = 0;
            for (int i : order) {
                const PlanTensor& t = ts[i];
                if (t.planned || t.recompute) continue;
                const bool rc = wants_recompute(i);
                if (!rc && !can_swap) continue;
                const int back = rc ? t.bwd_first_use_op : t.prefetch_op;
                if (at <= t.last_fwd_use_op || at >= back) continue;
                const int gap = back - t.last_fwd_use_op;
                if (best >= 0) {
                    const PlanTensor& b = ts[best];
                    if (!(gap != best_gap ? gap > best_gap : (t.produce_op != b.produce_op ? t.produce_op < b.produce_op : t.bytes > b.bytes))) continue;
                }
                best = i;
                best_gap = gap;
            }
            if (best < 0) break;  // nothing more can lower this peak
            if (wants_recompute(best)) ts[best].recompute = true;
            else plan_swap(best);
            apply_deps(ts, p);
            chosen.push_back(best);
        }
        // drop tensors that later choices made unnecessary (less traffic, less re-computation)
        if (peak(ts, transient, n_ops, false, nullptr) <= p.budget_bytes) {
            for (int k = (int)chosen.size() - 1; k >= 0; --k) {
                PlanTensor& t = ts[chosen[k]];
                const bool was_planned = t.planned, was_recompute = t.recompute;
                t.planned = t.recompute = false;
                apply_deps(ts, p);
                if (peak(ts, transient, n_ops, false, nullptr) > p.budget_bytes) {
                    t.planned = was_planned;
                    t.recompute = was_recompute;
                    apply_deps(ts, p);
                }
            }
        }
    }

    // The swap set is chosen with the op-count rule (least residency, least traffic); only then are its swap-ins
    // moved earlier by time.  The budget comes before the hiding: where that lifts the model over the budget,
    // the tensors that are resident early at the peak are moved later again (at most back to the op-count rule).
    if (timed && p.policy == MI3D_SWAP_BUDGET) {
        reschedule();
        for (int guard = 0; guard < 4 * n_ops * (int)ts.size() + 16; ++guard) {
            int at = 0;
            if (peak(ts, transient, n_ops, false, &at) <= p.budget_bytes) break;
            int pick = -1;
            for (int i : order) {
                const PlanTensor& t = ts[i];
                if (!t.planned || at < t.prefetch_op || at >= prefetch_by_ops(t, p)) continue;
                if (pick < 0 || t.bwd_first_use_op > ts[pick].bwd_first_use_op) pick = i;   // needed last: least urgent
            }
            if (pick < 0) break;
            ts[pick].prefetch_op = std::min(at + 1, prefetch_by_ops(ts[pick], p));
        }
    }
    if (swap_only) {
        // does swapping alone do, hidden?  Else the second attempt decides tensor by tensor.
        double load = 0.0;
        for (int i = 0; i < (int)ts.size(); ++i)
            if (ts[i].planned) load += 1.15 * copy_ms(i);
        if (load <= link_room_ms && peak(ts, transient, n_ops, false, nullptr) <= p.budget_bytes) break;
    }
    }   // attempts

    size_t off = 0;
    int n = 0;
    for (int i : order) {
        if (!ts[i].planned) continue;
        ts[i].host_offset = off;
        off += (ts[i].bytes + 4095) & ~(size_t)4095;
        ++n;
    }
    res->n_planned = n;
    res->host_bytes = off;
    res->n_recompute = 0;
    res->recompute_ms = 0.0;
    for (const PlanTensor& t : ts)
        if (t.recompute) {
            ++res->n_recompute;
            res->recompute_ms += t.recompute_ms;
        }
    res->planned_peak = peak(ts, transient, n_ops, false, nullptr);
    res->static_arena_bytes = place_static(ts, p);
    if (p.host_pool_bytes && off > p.host_pool_bytes) return MI3D_ERR_HOST_POOL;
    if (res->planned_peak > p.budget_bytes) return MI3D_ERR_OVER_BUDGET;
    return MI3D_OK;
}

}  // namespace mi3d
