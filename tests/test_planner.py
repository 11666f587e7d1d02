"""Host-only tests of the swap planner (Sections 3.2-3.3 knobs): run on CPU."""
import itertools

import numpy as np
import pytest

from paper_1812_07816_amd import swap as sw
from paper_1812_07816_amd._lib import Mi3dError


def unet_like(levels=4, base=1024):
    """Encoder tensors shrink 8x per level; decoder mirrors it.  Returns
    (n_fwd, n_ops, tensors) with tensors = (id, bytes, produce, last_fwd, bwd_first, bwd_last, tag)."""
    n_fwd = 2 * levels
    n_ops = 2 * n_fwd
    ts = []
    for l in range(levels):       # encoder op l produces e_l, used by op l+1 and (skip) decoder op n_fwd-1-l
        ts.append((l, base >> (3 * l) if base >> (3 * l) else 1, l, n_fwd - 1 - l, n_fwd + l, n_ops - 1 - l, sw.TAG_ENCODER))
    for l in range(levels):       # decoder op levels+l produces d_l used by next op
        op = levels + l
        size = base >> (3 * (levels - 1 - l)) or 1
        ts.append((levels + l, size, op, min(op + 1, n_fwd - 1), n_ops - 1 - op, n_ops - 1 - op, sw.TAG_DECODER))
    return n_fwd, n_ops, ts


def chain(n_layers, sizes):
    """Plain chain: op i produces tensor i, op i+1 reads it, backward op
    n_ops-1-i reads it again."""
    n_fwd, n_ops = n_layers, 2 * n_layers
    return n_fwd, n_ops, [(i, sizes[i], i, min(i + 1, n_fwd - 1), n_ops - 1 - i, n_ops - 1 - i, sw.TAG_ENCODER)
                          for i in range(n_layers)]


def make(ts, n_fwd, n_ops, **kw):
    e = sw.SwapEngine(**kw)
    e.set_timeline(n_fwd, n_ops)
    for t in ts:
        e.register(*t)
    return e


def brute_bytes(ts, planned, prefetch, op):
    b = 0
    for (i, size, prod, lf, bf, bl, _tag) in ts:
        if op < prod or op > bl:
            continue
        if i in planned and lf < op < prefetch[i]:
            continue
        b += size
    return b


def test_accounting_equals_brute_force_sweep():
    n_fwd, n_ops, ts = chain(6, [600, 500, 400, 300, 200, 100])
    e = make(ts, n_fwd, n_ops, budget_bytes=1500, lookahead=1)
    e.plan()
    planned = {t[0] for t in ts if e.is_planned(t[0])}
    pre = {t[0]: e.prefetch_op(t[0]) for t in ts}
    assert planned
    sweep = [brute_bytes(ts, planned, pre, op) for op in range(n_ops)]
    assert sweep == [e.planned_bytes_at(op) for op in range(n_ops)]
    st = e.stats()
    assert st["planned_peak_bytes"] == max(sweep) <= 1500
    assert st["unswapped_peak_bytes"] == 2100
    assert st["n_planned"] == len(planned)


def test_budget_policy_picks_early_long_lived_tensors_first():
    n_fwd, n_ops, ts = chain(6, [600, 500, 400, 300, 200, 100])
    e = make(ts, n_fwd, n_ops, budget_bytes=1600, lookahead=1)
    e.plan()
    assert [e.is_planned(i) for i in range(6)] == [True, False, False, False, False, False]
    # nothing is swapped when everything fits
    e2 = make(ts, n_fwd, n_ops, budget_bytes=2100, lookahead=1)
    e2.plan()
    assert not any(e2.is_planned(i) for i in range(6))
    assert e2.stats()["n_planned"] == 0


def test_budget_plan_is_minimal_under_removal():
    n_fwd, n_ops, ts = unet_like()
    sizes = {t[0]: t[1] for t in ts}
    for budget in (1400, 1200, 1100):
        e = make(ts, n_fwd, n_ops, budget_bytes=budget, lookahead=1)
        st = e.plan(allow_over_budget=True)
        if st != 0:
            continue
        planned = [i for i in sizes if e.is_planned(i)]
        pre = {t[0]: e.prefetch_op(t[0]) for t in ts}
        for drop in planned:   # removing any one chosen tensor breaks the budget
            rest = set(planned) - {drop}
            assert max(brute_bytes(ts, rest, pre, op) for op in range(n_ops)) > budget


def test_infeasible_budget_is_reported():
    n_fwd, n_ops, ts = chain(4, [100, 100, 100, 100])
    e = make(ts, n_fwd, n_ops, budget_bytes=150, lookahead=1)
    with pytest.raises(Mi3dError) as ei:
        e.plan()
    assert ei.value.status == -6
    assert e.plan(allow_over_budget=True) == -6
    # the plan is still inspectable
    assert e.stats()["planned_peak_bytes"] > 150


def test_transients_count_against_the_budget():
    n_fwd, n_ops, ts = chain(4, [100, 100, 100, 100])
    e = make(ts, n_fwd, n_ops, budget_bytes=400, lookahead=1)
    e.plan()
    assert e.stats()["n_planned"] == 0
    e.set_transient(3, 150)
    e.plan()
    assert e.stats()["n_planned"] >= 1 and e.stats()["planned_peak_bytes"] <= 400


def test_policy_all_and_first_n_and_tags():
    n_fwd, n_ops, ts = unet_like()
    e = make(ts, n_fwd, n_ops, budget_bytes=1 << 40, policy=sw.POLICY_ALL)
    e.plan()
    assert all(e.is_planned(t[0]) for t in ts)                       # "n_tensors = -1"
    e = make(ts, n_fwd, n_ops, budget_bytes=1 << 40, policy=sw.POLICY_FIRST_N, n_tensors=3)
    e.plan()
    by_prod = sorted(ts, key=lambda t: t[2])
    assert [e.is_planned(t[0]) for t in by_prod] == [True] * 3 + [False] * (len(ts) - 3)
    e = make(ts, n_fwd, n_ops, budget_bytes=1 << 40, policy=sw.POLICY_ALL, exclude_tags=sw.TAG_DECODER)
    e.plan()                                                          # excl_scopes = synthesis path
    assert all(e.is_planned(t[0]) == (t[6] == sw.TAG_ENCODER) for t in ts)
    e = make(ts, n_fwd, n_ops, budget_bytes=1 << 40, policy=sw.POLICY_ALL, include_tags=sw.TAG_DECODER)
    e.plan()                                                          # incl_scopes
    assert all(e.is_planned(t[0]) == (t[6] == sw.TAG_DECODER) for t in ts)


def test_fewer_swapped_tensors_never_lower_the_modelled_peak():
    # Table 1's structure: the all-swapped configuration has the lowest peak
    n_fwd, n_ops, ts = unet_like()
    peaks = []
    for n in (len(ts), 5, 3, 1, 0):
        e = make(ts, n_fwd, n_ops, budget_bytes=1 << 40, policy=sw.POLICY_FIRST_N, n_tensors=n)
        e.plan()
        peaks.append(e.stats()["planned_peak_bytes"])
    assert peaks == sorted(peaks)


def test_lookahead_moves_prefetch_earlier_and_clamps():
    n_fwd, n_ops, ts = chain(6, [100] * 6)
    prev = None
    for lb in (0, 1, 2, 4, 20):
        e = make(ts, n_fwd, n_ops, budget_bytes=1 << 40, policy=sw.POLICY_ALL, lookahead=lb)
        e.plan()
        pre = [e.prefetch_op(i) for i in range(6)]
        for (i, _s, _p, lf, bf, _bl, _t), p in zip(ts, pre):
            assert p == min(bf, max(bf - lb, n_fwd, lf + 1))     # never before the backward pass starts
        if prev is not None:
            assert all(a <= b for a, b in zip(pre, prev))        # larger lb => earlier (or equal)
        prev = pre


def test_bad_registrations_and_states():
    e = sw.SwapEngine(budget_bytes=100)
    e.set_timeline(2, 4)
    e.register(0, 10, 0, 1, 2, 3)
    for args in [(0, 10, 0, 1, 2, 3), ]:
        with pytest.raises(Mi3dError) as ei:
            e.register(*args)
        assert ei.value.status == -7          # duplicate id
    for args in [(1, 0, 0, 1, 2, 3), (-1, 10, 0, 1, 2, 3), (2, 10, 1, 0, 2, 3), (3, 10, 0, 2, 2, 3), (4, 10, 0, 1, 3, 2)]:
        with pytest.raises(Mi3dError) as ei:
            e.register(*args)
        assert ei.value.status == -1
    with pytest.raises(Mi3dError) as ei:
        e.is_planned(0)                        # no plan yet
    assert ei.value.status == -7
    e.plan()
    with pytest.raises(Mi3dError) as ei:
        e.is_planned(99)                       # unknown id
    assert ei.value.status == -7
    # a planner-only engine (no pinned pool) refuses to copy, without touching HIP
    for call in (lambda: e.swap_out(0, 4096), lambda: e.swap_in(0, 4096), lambda: e.release(0),
                 lambda: e.wait_in(0), lambda: e.done(0), lambda: e.alloc(16)):
        with pytest.raises(Mi3dError) as ei:
            call()
        assert ei.value.status == -7
    with pytest.raises(Mi3dError) as ei:
        sw.SwapEngine(budget_bytes=1, lookahead=-1)
    assert ei.value.status == -1


def test_host_pool_capacity_is_checked_at_plan_time():
    # host_pool_bytes > 0 would allocate pinned memory (needs a GPU); the
    # capacity rule itself is visible through the planned set's size
    n_fwd, n_ops, ts = chain(4, [5000, 5000, 5000, 5000])
    e = make(ts, n_fwd, n_ops, budget_bytes=1 << 40, policy=sw.POLICY_ALL)
    e.plan()
    assert e.stats()["n_planned"] == 4


def test_prefetch_by_time_lays_copies_out_back_to_back():
    # chain of 6 layers, every op 1 ms; link 1 GB/s -> a tensor of b bytes takes b / 1e6 * 1.15 + 0.05 ms
    sizes = [3_000_000, 2_000_000, 1_000_000, 500_000, 100_000, 50_000]
    n_fwd, n_ops, ts = chain(6, sizes)
    e = make(ts, n_fwd, n_ops, budget_bytes=1 << 40, policy=sw.POLICY_ALL, lookahead=1)
    e.plan()
    by_ops = [e.prefetch_op(i) for i in range(6)]
    e.set_op_times([1.0] * n_ops, 1.0)
    e.plan()
    pf = [e.prefetch_op(i) for i in range(6)]
    dur = [b / 1e6 * 1.15 + 0.05 for b in sizes]
    use = [n_ops - 1 - i for i in range(6)]          # first backward use; with 1 ms ops the start time equals the op index
    # latest use first: tensor 0 (used last) must end by its use; the copy before it must end when that one starts
    end = float("inf")
    for i in range(6):
        finish = min(use[i], end)
        begin = finish - dur[i]
        lower = max(n_fwd, ts[i][3] + 1)
        assert pf[i] <= by_ops[i]
        assert pf[i] <= max(begin, lower) + 1e-9, (i, pf[i], begin)          # issued early enough ...
        assert pf[i] == lower or pf[i] + 1 > begin - 1e-9, (i, pf[i], begin)   # ... and at the latest such op
        end = begin
    # back to the op-count rule
    e.set_op_times([], 0.0)
    e.plan()
    assert [e.prefetch_op(i) for i in range(6)] == by_ops
    e.close()


def test_op_times_count_in_the_budget_model():
    # earlier swap-ins keep tensors resident longer; the budget has priority over the hiding
    sizes = [4000, 3000, 2000, 1000, 500, 250]
    n_fwd, n_ops, ts = chain(6, sizes)
    total = sum(sizes)
    for frac, expect_earlier in ((0.7, False), (0.9, True)):
        budget = int(total * frac)
        e = make(ts, n_fwd, n_ops, budget_bytes=budget, lookahead=1)
        e.plan()
        by_ops = {i: e.prefetch_op(i) for i in range(6) if e.is_planned(i)}
        e.set_op_times([1.0] * n_ops, 4e-3)              # 4 MB/s: a 4000-byte tensor takes 1.2 ms, more than one op
        assert e.plan(allow_over_budget=True) == 0
        planned = {i for i in range(6) if e.is_planned(i)}
        prefetch = {i: e.prefetch_op(i) for i in planned}
        assert planned and all(prefetch[i] <= by_ops.get(i, 10 ** 9) for i in planned)
        assert any(prefetch[i] < by_ops.get(i, 10 ** 9) for i in planned) == expect_earlier
        for op in range(n_ops):
            assert brute_bytes(ts, planned, prefetch, op) == e.planned_bytes_at(op) <= budget
        e.close()
    e = make(ts, n_fwd, n_ops, budget_bytes=total, lookahead=1)
    with pytest.raises(Mi3dError):
        e.set_op_times([1.0, -1.0], 1.0)
    e.close()


# ---- re-computation and the hybrid (Section 5) ------------------------------------------------------------------
def real_chain(sizes):
    """Chain of layers: op i produces tensor i from tensor i-1; backward op of layer i (n_ops-1-i) reads tensor i and
    tensor i-1, so tensor i is first needed again at the backward op of layer i+1."""
    n = len(sizes)
    n_ops = 2 * n
    ts = []
    for i in range(n):
        bwd_own, bwd_next = n_ops - 1 - i, n_ops - 1 - (i + 1)
        first = bwd_next if i + 1 < n else bwd_own
        ts.append((i, sizes[i], i, min(i + 1, n - 1), first, bwd_own, sw.TAG_ENCODER))
    return n, n_ops, ts


def closure_first_use(ts, recomputed, deps):
    first = {t[0]: t[4] for t in ts}
    for _ in range(len(ts) + 2):
        for i in recomputed:
            for d in deps.get(i, ()):
                first[d] = min(first[d], first[i])
    return first


def brute_bytes_hybrid(ts, planned, recomputed, prefetch, first, op):
    b = 0
    for (i, size, prod, lf, _bf, bl, _tag) in ts:
        if op < prod or op > bl:
            continue
        if i in recomputed and lf < op < first[i]:
            continue
        if i in planned and lf < op < prefetch[i]:
            continue
        b += size
    return b


def plan_state(e, ts):
    ids = [t[0] for t in ts]
    return ({i for i in ids if e.is_planned(i)}, {i for i in ids if e.is_recomputed(i)},
            {i: e.prefetch_op(i) for i in ids}, {i: e.first_use_op(i) for i in ids})


@pytest.mark.parametrize("eviction", [sw.EVICT_RECOMPUTE, sw.EVICT_HYBRID])
def test_recompute_accounting_matches_brute_force_on_random_chains(eviction):
    rng = np.random.default_rng(7)
    seen_recompute = seen_swap = 0
    for trial in range(60):
        n = int(rng.integers(3, 9))
        sizes = [int(v) for v in rng.integers(50, 900, size=n)]
        n_fwd, n_ops, ts = real_chain(sizes)
        total = sum(sizes)
        budget = int(total * rng.uniform(0.45, 0.95))
        e = make(ts, n_fwd, n_ops, budget_bytes=budget, lookahead=int(rng.integers(1, 3)))
        e.set_eviction(eviction)
        deps = {}
        for i in range(1, n):
            if rng.uniform() < 0.8:
                # cost 0 ms is cheaper than any copy, 1e3 ms dearer than any: the hybrid re-computes the former only
                e.set_recompute(i, 0.0 if rng.uniform() < 0.6 else 1e3, i - 1)
                deps[i] = (i - 1,)
        st = e.plan(allow_over_budget=True)
        planned, recomputed, prefetch, first = plan_state(e, ts)
        assert first == closure_first_use(ts, recomputed, deps)
        assert not (planned & recomputed)
        if eviction == sw.EVICT_RECOMPUTE:
            assert not planned and recomputed <= set(deps)
        sweep = [brute_bytes_hybrid(ts, planned, recomputed, prefetch, first, op) for op in range(n_ops)]
        assert sweep == [e.planned_bytes_at(op) for op in range(n_ops)]
        s = e.stats()
        assert s["planned_peak_bytes"] == max(sweep) and s["n_recompute"] == len(recomputed) and s["n_planned"] == len(planned)
        assert (st == 0) == (max(sweep) <= budget)
        for i in planned:
            assert first[i] - 2 <= prefetch[i] <= first[i]
        seen_recompute += len(recomputed)
        seen_swap += len(planned)
        e.close()
    assert seen_recompute > 10 and (eviction == sw.EVICT_RECOMPUTE or seen_swap > 5)


def test_hybrid_recomputes_cheap_tensors_and_swaps_dear_ones():
    n_fwd, n_ops, ts = real_chain([100, 600, 500, 400, 300, 200])
    for cost, expect_recompute in ((0.0, True), (1e3, False)):
        e = make(ts, n_fwd, n_ops, budget_bytes=1600, lookahead=1)
        e.set_eviction(sw.EVICT_HYBRID)
        for i in range(1, 6):
            e.set_recompute(i, cost, i - 1)
        e.plan()
        planned, recomputed, _, _ = plan_state(e, ts)
        assert (recomputed, planned) == (({1}, set()) if expect_recompute else (set(), {1}))
        assert e.stats()["planned_peak_bytes"] <= 1600
        e.close()
    # with measured op times and link rate: 600 bytes at 1e-3 GB/s take 0.6 ms.  Where that hides behind the passes
    # (6 ops of 1 ms each way) the tensor is swapped whatever its re-computation costs; where the passes are too short
    # to hide it (6 ops of 0.05 ms), the comparison is cost against bytes / rate
    for op_ms, cost, expect in ((1.0, 0.5, False), (1.0, 0.0, False), (0.05, 0.5, True), (0.05, 0.7, False)):
        e = make(ts, n_fwd, n_ops, budget_bytes=1600, lookahead=1)
        e.set_eviction(sw.EVICT_HYBRID)
        e.set_op_times([op_ms] * n_ops, 1e-3)
        e.set_recompute(1, cost, 0)
        e.plan(allow_over_budget=True)
        assert e.is_recomputed(1) == expect and e.is_planned(1) == (not expect), (op_ms, cost)
        e.close()


def test_hybrid_swaps_everything_where_the_link_hides_it_and_decides_per_tensor_where_not():
    """Seven equal tensors that all have to go, all but the first cheaper to re-compute than to copy.  Seven copies
    of 1.15 x 0.9 ms fit into 90 % of a 14 ms pass: swapping alone stands.  They do not fit into 90 % of a 7 ms pass:
    every other tensor is re-computed (one whose source is re-computed itself is swapped)."""
    n_fwd, n_ops, ts = real_chain([900] * 7)
    for op_ms, want_planned, want_recomputed in ((2.0, {0, 1, 2, 3, 4, 5, 6}, set()), (1.0, {0, 2, 4, 6}, {1, 3, 5})):
        e = make(ts, n_fwd, n_ops, budget_bytes=900 * 3, lookahead=1, policy=sw.POLICY_ALL)
        e.set_eviction(sw.EVICT_HYBRID)
        e.set_op_times([op_ms] * n_ops, 1e-3)
        for i in range(1, 7):
            e.set_recompute(i, 0.1, i - 1)
        e.plan(allow_over_budget=True)
        planned, recomputed, _, _ = plan_state(e, ts)
        assert planned == want_planned and recomputed == want_recomputed, (op_ms, planned, recomputed)
        e.close()


def test_recompute_only_never_evicts_tensors_without_the_option():
    n_fwd, n_ops, ts = real_chain([600, 500, 400, 300, 200, 100])
    e = make(ts, n_fwd, n_ops, budget_bytes=100, lookahead=1, policy=sw.POLICY_ALL)
    e.set_eviction(sw.EVICT_RECOMPUTE)
    e.set_recompute(2, 0.1, 1)
    e.set_recompute(4, 0.1, 3)
    assert e.plan(allow_over_budget=True) != 0        # cannot be met
    planned, recomputed, _, first = plan_state(e, ts)
    assert not planned and recomputed == {2, 4}
    s = e.stats()
    assert s["n_recompute"] == 2 and abs(s["recompute_ms"] - 0.2) < 1e-6
    # the inputs of the re-computations are needed one op earlier than their own backward use
    assert first[1] == first[2] and first[3] == first[4]
    e.close()


def test_policy_all_with_recomputation_keeps_every_other_tensor_of_a_chain():
    n_fwd, n_ops, ts = real_chain([100] * 7)
    e = make(ts, n_fwd, n_ops, budget_bytes=10 ** 9, lookahead=1, policy=sw.POLICY_ALL)
    e.set_eviction(sw.EVICT_RECOMPUTE)
    for i in range(1, 7):
        e.set_recompute(i, 0.1, i - 1)
    e.plan()
    _, recomputed, _, _ = plan_state(e, ts)
    # no tensor is re-computed from a re-computed one (that would bring the whole chain back at once)
    assert recomputed and all(i - 1 not in recomputed for i in recomputed)
    assert len(recomputed) == 3
    e.close()
    # the hybrid swaps the ones in between
    e = make(ts, n_fwd, n_ops, budget_bytes=10 ** 9, lookahead=1, policy=sw.POLICY_ALL)
    e.set_eviction(sw.EVICT_HYBRID)
    for i in range(1, 7):
        e.set_recompute(i, 0.0, i - 1)
    e.plan()
    planned, recomputed, _, _ = plan_state(e, ts)
    assert len(recomputed) == 3 and planned | recomputed == set(range(7))
    e.close()


def test_recompute_argument_checks():
    n_fwd, n_ops, ts = real_chain([100, 100, 100])
    e = make(ts, n_fwd, n_ops, budget_bytes=1000)
    with pytest.raises(Mi3dError):
        e.set_eviction(7)
    with pytest.raises(Mi3dError):
        e.set_recompute(1, -1.0, 0)
    with pytest.raises(Mi3dError):
        e.set_recompute(1, 0.1, 1)          # depends on itself
    with pytest.raises(Mi3dError):
        e.set_recompute(1, 0.1, 42)         # unknown dependency
    with pytest.raises(Mi3dError):
        e.set_recompute(42, 0.1, 0)         # unknown tensor
    with pytest.raises(Mi3dError):
        e.is_recomputed(1)                  # no plan yet
    e.close()


def _stays(e, ts):
    """(from op, to op, offset, size) of every stay of every tensor under the engine's plan, op intervals as the
    placement reads them without op times: a swapped tensor's first stay gets one op of grace for its copy-out."""
    out = []
    for (i, size, prod, lf, bf, bl, _tag) in ts:
        sz = (size + 255) // 256 * 256
        if e.is_planned(i):
            pf = e.prefetch_op(i)
            out.append((prod, min(lf + 1, max(pf - 1, lf)), e.planned_offset(i, 0), sz))
            out.append((pf, bl, e.planned_offset(i, 1), sz))
        elif e.is_recomputed(i):
            out.append((prod, lf, e.planned_offset(i, 0), sz))
            out.append((e.first_use_op(i), bl, e.planned_offset(i, 1), sz))
        else:
            out.append((prod, bl, e.planned_offset(i, 0), sz))
    return out


@pytest.mark.parametrize("seed", range(12))
def test_static_placement_never_overlaps_two_tensors_that_share_an_op(seed):
    rng = np.random.default_rng(seed)
    levels = int(rng.integers(2, 6))
    n_fwd, n_ops, ts = unet_like(levels, base=int(rng.integers(1, 9)) * 4096)
    # ragged sizes, so that the 256-byte rounding matters
    ts = [(i, size + int(rng.integers(0, 300)), a, b, c, d, tag) for (i, size, a, b, c, d, tag) in ts]
    total = sum(t[1] for t in ts)
    policy = [sw.POLICY_BUDGET, sw.POLICY_ALL, sw.POLICY_FIRST_N][seed % 3]
    e = make(ts, n_fwd, n_ops, budget_bytes=int(total * (0.5 + 0.05 * (seed % 7))), lookahead=1 + seed % 3, policy=policy, n_tensors=levels)
    e.plan(allow_over_budget=True)
    stays = _stays(e, ts)
    for a in range(len(stays)):
        for b in range(a + 1, len(stays)):
            fa, ta, oa, sa = stays[a]
            fb, tb, ob, sb = stays[b]
            if fa <= tb and fb <= ta:                       # the two stays share an op ...
                assert oa + sa <= ob or ob + sb <= oa, (stays[a], stays[b])   # ... so they may not share a byte
    extent = e.stats()["static_arena_bytes"]
    assert extent == max(o + s for _, _, o, s in stays)
    # never less than the bytes that are on the device together, never more than everything side by side
    live = max(sum(s for f, t, _, s in stays if f <= op <= t) for op in range(n_ops))
    assert live <= extent <= sum((t[1] + 255) // 256 * 256 for t in ts)


def test_static_placement_reuses_the_space_of_swapped_tensors():
    # a chain of equal tensors, everything swapped: two places are enough for the forward pass (one being produced,
    # one being read) plus the grace op of the copy-out, whatever the depth
    n_fwd, n_ops, ts = chain(10, [4096] * 10)
    e = make(ts, n_fwd, n_ops, budget_bytes=1, policy=sw.POLICY_ALL)
    e.plan(allow_over_budget=True)
    assert e.stats()["static_arena_bytes"] <= 4 * 4096
    e2 = make(ts, n_fwd, n_ops, budget_bytes=1 << 40)
    e2.plan()
    assert e2.stats()["static_arena_bytes"] == 10 * 4096     # nothing leaves: everything side by side
