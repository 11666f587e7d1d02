// Run-time half of the data-swapping engine (Sections 3.1 and 3.3): pinned
// host pool, one side stream per copy direction, events that order copies
// against the compute stream, an event-aware device arena, and counters.
#include <algorithm>
#include <cstring>
#include <map>
#include <memory>
#include <new>
#include <vector>

#include "mi3d_internal.h"
#include "swap_planner.h"

using namespace mi3d;

namespace {

enum State { ST_NEW = 0, ST_OUT_ISSUED, ST_HOST, ST_IN_ISSUED, ST_BACK, ST_DONE };

struct Copy {
    hipEvent_t start = nullptr, done = nullptr;
    bool issued = false;
};

struct Tensor {
    PlanTensor plan;
    int allocs = 0;     // placements handed out by mi3d_swap_alloc_tensor in this step (0: first stay, 1: second)
    State state = ST_NEW;
    const void* dev_src = nullptr;
    Copy out, in;
};

// An event a freed block waits for.  copy: recorded on one of the engine's copy streams (behind a swap-out that
// still reads the block); such a wait can take a whole transfer, a wait on a compute-stream event is free for
// the next kernel of that stream.
struct Pending {
    std::shared_ptr<void> ev;
    bool copy;
};

struct ArenaBlock {
    size_t off, size;
    bool free;
    std::vector<Pending> pending;  // events that must fire before reuse
};

#if defined(__HIPCC__)
// 64-bit checksum of a device buffer: sum over its 8-byte words of word * (2 * index + 1) mod 2^64 (a trailing piece of
// fewer than 8 bytes counts as a zero-extended word).  Integer arithmetic: the value does not depend on the order of
// the additions, so any grid gives the same bits; the odd, position-dependent factor makes it notice flipped bits as
// well as words that changed places.
constexpr int CK_BLOCKS = 256;
__global__ void __launch_bounds__(256) checksum_partial_kernel(const unsigned char* __restrict__ p, size_t bytes, unsigned long long* __restrict__ part) {
    __shared__ unsigned long long red[256];
    const size_t words = bytes / 8;
    unsigned long long acc = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256)
        acc += ((const unsigned long long*)p)[i] * (2ull * i + 1ull);
    if (blockIdx.x == 0 && threadIdx.x == 0 && (bytes & 7)) {
        unsigned long long last = 0;
        for (size_t b = 0; b < (bytes & 7); ++b) last |= (unsigned long long)p[words * 8 + b] << (8 * b);
        acc += last * (2ull * words + 1ull);
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) part[blockIdx.x] = red[0];
}
__global__ void __launch_bounds__(64) checksum_final_kernel(const unsigned long long* __restrict__ part, int n, unsigned long long* __restrict__ out) {
    if (threadIdx.x == 0) {
        unsigned long long a = 0;
        for (int i = 0; i < n; ++i) a += part[i];
        *out = a;
    }
}
// enqueues the checksum of [p, p + bytes) on `s`; scratch: CK_BLOCKS words of device memory; out: device-writable
int enqueue_checksum(const void* p, size_t bytes, unsigned long long* scratch, unsigned long long* out, hipStream_t s) {
    checksum_partial_kernel<<<CK_BLOCKS, 256, 0, s>>>((const unsigned char*)p, bytes, scratch);
    int st = check_launch();
    if (st) return st;
    checksum_final_kernel<<<1, 64, 0, s>>>(scratch, CK_BLOCKS, out);
    return check_launch();
}
#endif

}  // namespace

struct mi3d_swap_engine {
    mi3d_swap_config cfg;
    std::map<int, Tensor> tensors;
    std::vector<size_t> transient;
    std::vector<float> op_ms;   // measured op durations (optional): swap-ins are then scheduled by time
    float link_gbs = 0.f;
    int eviction = MI3D_EVICT_SWAP;
    int n_fwd_ops = 0, n_ops = 0;
    bool have_plan = false;
    PlanResult plan_res;

    bool live = false;  // owns HIP objects
    int device = 0;
    char* host_pool = nullptr;
    hipStream_t s_out = nullptr, s_in = nullptr;
    hipEvent_t base = nullptr;
    std::vector<hipEvent_t> free_events_timed, free_events_plain;

    std::vector<ArenaBlock> blocks;
    // arena_used: bytes handed out.  arena_occupied_peak / arena_hwm: peak of the bytes, and highest end offset, of
    // blocks that are handed out OR freed but still read by a swap-out in flight (that memory is not yet reusable).
    // arena_cap: bytes the saved tensors occupy at the peak of the plan's residency model; allocations stay below
    // this offset as long as any block there can serve them (arena_overflow counts those that could not).
    size_t arena_used = 0, arena_occupied_peak = 0, arena_hwm = 0, arena_cap = 0;
    int arena_overflow = 0;

    uint64_t bytes_out = 0, bytes_in = 0;
    int n_out = 0, n_in = 0;

    // checksum mode: per tensor slot two words in pinned host memory (before the swap-out, after the swap-in) and
    // CK_BLOCKS words of device scratch per copy direction
    bool verify = false;
    unsigned long long* sums_host = nullptr;     // [slot][2]
    unsigned long long* sums_scratch = nullptr;  // device, [2][CK_BLOCKS]
    int sums_slots = 0;
    std::map<int, int> sum_slot;                 // tensor id -> slot (assigned at its swap-out)
};

namespace {

#define HIP_TRY(expr)                         \
    do {                                      \
        hipError_t err__ = (expr);            \
        if (err__ != hipSuccess) {            \
            note_hip_error(err__);            \
            return MI3D_ERR_HIP;              \
        }                                     \
    } while (0)

int get_event(mi3d_swap_engine* e, bool timed, hipEvent_t* ev) {
    std::vector<hipEvent_t>& pool = timed ? e->free_events_timed : e->free_events_plain;
    if (!pool.empty()) {
        *ev = pool.back();
        pool.pop_back();
        return MI3D_OK;
    }
    HIP_TRY(hipEventCreateWithFlags(ev, timed ? hipEventDefault : hipEventDisableTiming));
    return MI3D_OK;
}

// plain (untimed) event recorded on `s`, handed back to the pool when the
// last holder lets go
int record_shared(mi3d_swap_engine* e, hipStream_t s, std::shared_ptr<void>* out) {
    hipEvent_t ev;
    int st = get_event(e, false, &ev);
    if (st) return st;
    HIP_TRY(hipEventRecord(ev, s));
    *out = std::shared_ptr<void>((void*)ev, [e](void* p) { e->free_events_plain.push_back((hipEvent_t)p); });
    return MI3D_OK;
}

Tensor* find(mi3d_swap_engine* e, int id) {
    auto it = e->tensors.find(id);
    return it == e->tensors.end() ? nullptr : &it->second;
}

bool in_arena(const mi3d_swap_engine* e, const void* p) {
    const char* b = (const char*)e->cfg.dev_arena;
    return b && (const char*)p >= b && (const char*)p < b + e->cfg.arena_bytes;
}

bool waits_for_copy(const ArenaBlock& b) {
    for (const Pending& p : b.pending)
        if (p.copy) return true;
    return false;
}

// Merges neighbouring free blocks.  A block that still waits for a copy is kept apart, so that an allocation
// from its neighbour does not inherit that wait; it is merged once the copy's event has fired (see alloc).
void coalesce(mi3d_swap_engine* e) {
    std::vector<ArenaBlock>& bl = e->blocks;
    for (size_t i = 0; i + 1 < bl.size();) {
        if (bl[i].free && bl[i + 1].free && !waits_for_copy(bl[i]) && !waits_for_copy(bl[i + 1])) {
            bl[i].size += bl[i + 1].size;
            for (auto& ev : bl[i + 1].pending) bl[i].pending.push_back(ev);
            bl.erase(bl.begin() + i + 1);
        } else {
            ++i;
        }
    }
}

// Merges every run of neighbouring free blocks, also across blocks that wait for a copy (the merged block then
// waits for it as a whole).  Used when nothing fits without such a wait.
void coalesce_all(mi3d_swap_engine* e) {
    std::vector<ArenaBlock>& bl = e->blocks;
    for (size_t i = 0; i + 1 < bl.size();) {
        if (bl[i].free && bl[i + 1].free) {
            bl[i].size += bl[i + 1].size;
            for (auto& ev : bl[i + 1].pending) bl[i].pending.push_back(ev);
            bl.erase(bl.begin() + i + 1);
        } else {
            ++i;
        }
    }
}

int arena_free(mi3d_swap_engine* e, const void* ptr, std::vector<Pending> pending) {
    size_t off = (const char*)ptr - (const char*)e->cfg.dev_arena;
    for (ArenaBlock& b : e->blocks) {
        if (b.off == off && !b.free) {
            b.free = true;
            b.pending = std::move(pending);
            e->arena_used -= b.size;
            coalesce(e);
            return MI3D_OK;
        }
    }
    return MI3D_ERR_BAD_STATE;
}

// blocks whose memory is in use: handed out, or freed behind a copy that has not finished
void note_occupancy(mi3d_swap_engine* e) {
    size_t occ = 0, hwm = 0;
    for (const ArenaBlock& b : e->blocks)
        if (!b.free || waits_for_copy(b)) {
            occ += b.size;
            hwm = std::max(hwm, b.off + b.size);
        }
    e->arena_occupied_peak = std::max(e->arena_occupied_peak, occ);
    e->arena_hwm = std::max(e->arena_hwm, hwm);
}

void reset_step_state(mi3d_swap_engine* e) {
    for (auto& kv : e->tensors) {
        Tensor& t = kv.second;
        for (Copy* c : {&t.out, &t.in}) {
            if (c->start) e->free_events_timed.push_back(c->start);
            if (c->done) e->free_events_timed.push_back(c->done);
            *c = Copy();
        }
        t.state = ST_NEW;
        t.dev_src = nullptr;
        t.allocs = 0;
    }
    e->bytes_out = e->bytes_in = 0;
    e->n_out = e->n_in = 0;
    e->arena_occupied_peak = e->arena_hwm = 0;
    e->arena_overflow = 0;
    e->sum_slot.clear();
}

}  // namespace

extern "C" {

int mi3d_swap_create(const mi3d_swap_config* cfg, mi3d_swap_engine** out) {
    if (!cfg || !out) return MI3D_ERR_INVALID_ARG;
    if (cfg->lookahead < 0 || cfg->policy < MI3D_SWAP_BUDGET || cfg->policy > MI3D_SWAP_FIRST_N) return MI3D_ERR_INVALID_ARG;
    if ((cfg->dev_arena == nullptr) != (cfg->arena_bytes == 0)) return MI3D_ERR_INVALID_ARG;
    if (cfg->dev_arena && ((uintptr_t)cfg->dev_arena & 255)) return MI3D_ERR_INVALID_ARG;
    mi3d_swap_engine* e = new (std::nothrow) mi3d_swap_engine();
    if (!e) return MI3D_ERR_INVALID_ARG;
    e->cfg = *cfg;
    if (cfg->arena_bytes) e->blocks.push_back(ArenaBlock{0, cfg->arena_bytes & ~(size_t)255, true, {}});
    if (cfg->host_pool_bytes) {
        hipError_t err = hipGetDevice(&e->device);
        if (err == hipSuccess) err = hipHostMalloc((void**)&e->host_pool, cfg->host_pool_bytes, hipHostMallocDefault);
        // touch every page once: the first DMA into untouched pinned pages runs at a fraction of link speed
        if (err == hipSuccess) memset(e->host_pool, 0, cfg->host_pool_bytes);
        if (err == hipSuccess) err = hipStreamCreateWithFlags(&e->s_out, hipStreamNonBlocking);
        if (err == hipSuccess) err = hipStreamCreateWithFlags(&e->s_in, hipStreamNonBlocking);
        if (err == hipSuccess) err = hipEventCreate(&e->base);
        if (err == hipSuccess) err = hipEventRecord(e->base, e->s_out);
        if (err != hipSuccess) {
            note_hip_error(err);
            if (e->base) (void)hipEventDestroy(e->base);
            if (e->s_in) (void)hipStreamDestroy(e->s_in);
            if (e->s_out) (void)hipStreamDestroy(e->s_out);
            if (e->host_pool) (void)hipHostFree(e->host_pool);
            delete e;
            return MI3D_ERR_HIP;
        }
        e->live = true;
    }
    *out = e;
    return MI3D_OK;
}

int mi3d_swap_destroy(mi3d_swap_engine* e) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    int st = MI3D_OK;
    if (e->live) {
        if (hipStreamSynchronize(e->s_out) != hipSuccess) st = MI3D_ERR_HIP;
        if (hipStreamSynchronize(e->s_in) != hipSuccess) st = MI3D_ERR_HIP;
    }
    // (an engine without a pinned pool still records events when its arena is used)
    e->blocks.clear();  // drops shared events into the free lists
    reset_step_state(e);
    for (hipEvent_t ev : e->free_events_timed) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : e->free_events_plain) (void)hipEventDestroy(ev);
#if defined(__HIPCC__)
    if (e->sums_host) (void)hipHostFree(e->sums_host);
    if (e->sums_scratch) (void)hipFree(e->sums_scratch);
#endif
    if (e->live) {
        (void)hipEventDestroy(e->base);
        (void)hipStreamDestroy(e->s_out);
        (void)hipStreamDestroy(e->s_in);
        (void)hipHostFree(e->host_pool);
    }
    delete e;
    return st;
}

int mi3d_swap_set_timeline(mi3d_swap_engine* e, int n_fwd_ops, int n_ops) {
    if (!e || n_fwd_ops < 0 || n_ops < n_fwd_ops) return MI3D_ERR_INVALID_ARG;
    e->n_fwd_ops = n_fwd_ops;
    e->n_ops = n_ops;
    e->transient.resize(n_ops, 0);
    e->have_plan = false;
    return MI3D_OK;
}

int mi3d_swap_register(mi3d_swap_engine* e, int id, size_t bytes, int produce_op, int last_fwd_use_op,
                       int bwd_first_use_op, int bwd_last_use_op, unsigned tags) {
    if (!e || id < 0 || bytes == 0) return MI3D_ERR_INVALID_ARG;
    if (produce_op < 0 || produce_op > last_fwd_use_op || last_fwd_use_op >= bwd_first_use_op || bwd_first_use_op > bwd_last_use_op)
        return MI3D_ERR_INVALID_ARG;
    if (e->tensors.count(id)) return MI3D_ERR_BAD_STATE;
    Tensor t;
    t.plan.id = id;
    t.plan.bytes = bytes;
    t.plan.produce_op = produce_op;
    t.plan.last_fwd_use_op = last_fwd_use_op;
    t.plan.bwd_first_use_op = bwd_first_use_op;
    t.plan.bwd_last_use_op = bwd_last_use_op;
    t.plan.tags = tags;
    e->tensors[id] = t;
    e->have_plan = false;
    return MI3D_OK;
}

int mi3d_swap_set_transient(mi3d_swap_engine* e, int op, size_t bytes) {
    if (!e || op < 0) return MI3D_ERR_INVALID_ARG;
    if (op >= (int)e->transient.size()) e->transient.resize(op + 1, 0);
    e->transient[op] = bytes;
    e->have_plan = false;
    return MI3D_OK;
}

int mi3d_swap_set_op_times(mi3d_swap_engine* e, const float* ms, int n, float link_gbs) {
    if (!e || n < 0 || (n > 0 && (!ms || !(link_gbs > 0.f)))) return MI3D_ERR_INVALID_ARG;
    for (int i = 0; i < n; ++i)
        if (!(ms[i] >= 0.f)) return MI3D_ERR_INVALID_ARG;
    e->op_ms.assign(ms, ms + n);
    e->link_gbs = link_gbs;
    e->have_plan = false;
    return MI3D_OK;
}

int mi3d_swap_plan(mi3d_swap_engine* e) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    std::vector<PlanTensor> ts;
    for (auto& kv : e->tensors) ts.push_back(kv.second.plan);
    PlanParams p;
    p.budget_bytes = e->cfg.budget_bytes;
    p.host_pool_bytes = e->cfg.host_pool_bytes;
    p.lookahead = e->cfg.lookahead;
    p.op_ms = &e->op_ms;
    p.link_gbs = e->link_gbs;
    p.policy = e->cfg.policy;
    p.n_tensors = e->cfg.n_tensors;
    p.exclude_tags = e->cfg.exclude_tags;
    p.include_tags = e->cfg.include_tags;
    p.eviction = e->eviction;
    p.n_fwd_ops = e->n_fwd_ops;
    p.n_ops = std::max<int>(e->n_ops, (int)e->transient.size());
    int st = plan_swaps(ts, e->transient, p, &e->plan_res);
    if (st == MI3D_ERR_INVALID_ARG) return st;
    for (const PlanTensor& t : ts) e->tensors[t.id].plan = t;
    // a swap set that does not fit the pinned pool is not executable: its host slots lie beyond the pool
    e->have_plan = st != MI3D_ERR_HOST_POOL;
    // bytes of saved tensors at the peak of the residency model, each rounded up as the arena rounds them (the limit
    // mi3d_swap_alloc tries to stay under; mi3d_swap_alloc_tensor uses the static placement instead)
    e->arena_cap = 0;
    if (e->have_plan) {
        std::vector<PlanTensor> rounded = ts;
        for (PlanTensor& t : rounded) t.bytes = (t.bytes + 255) & ~(size_t)255;
        const std::vector<size_t> none;
        for (int op = 0; op < p.n_ops; ++op) e->arena_cap = std::max<size_t>(e->arena_cap, plan_bytes_at(rounded, none, op, false));
    }
    return st;
}

int mi3d_swap_set_eviction(mi3d_swap_engine* e, int eviction) {
    if (!e || (eviction != MI3D_EVICT_SWAP && eviction != MI3D_EVICT_RECOMPUTE && eviction != MI3D_EVICT_HYBRID)) return MI3D_ERR_INVALID_ARG;
    e->eviction = eviction;
    e->have_plan = false;
    return MI3D_OK;
}

int mi3d_swap_set_recompute(mi3d_swap_engine* e, int id, float cost_ms, int dep0, int dep1) {
    if (!e || !(cost_ms >= 0.f) || dep0 == id || dep1 == id) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t) return MI3D_ERR_BAD_STATE;
    for (int d : {dep0, dep1})
        if (d >= 0 && !find(e, d)) return MI3D_ERR_BAD_STATE;
    t->plan.recompute_ms = cost_ms;
    t->plan.dep[0] = dep0 >= 0 ? dep0 : -1;
    t->plan.dep[1] = dep1 >= 0 ? dep1 : -1;
    e->have_plan = false;
    return MI3D_OK;
}

int mi3d_swap_is_recomputed(mi3d_swap_engine* e, int id) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t || !e->have_plan) return MI3D_ERR_BAD_STATE;
    return t->plan.recompute ? 1 : 0;
}

int mi3d_swap_first_use_op(mi3d_swap_engine* e, int id) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t || !e->have_plan) return MI3D_ERR_BAD_STATE;
    return t->plan.bwd_first_use_op;
}

int mi3d_swap_is_planned(mi3d_swap_engine* e, int id) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t || !e->have_plan) return MI3D_ERR_BAD_STATE;
    return t->plan.planned ? 1 : 0;
}

int mi3d_swap_prefetch_op(mi3d_swap_engine* e, int id) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t || !e->have_plan) return MI3D_ERR_BAD_STATE;
    return t->plan.prefetch_op;
}

int mi3d_swap_planned_bytes_at(mi3d_swap_engine* e, int op, uint64_t* bytes) {
    if (!e || !bytes || op < 0) return MI3D_ERR_INVALID_ARG;
    if (!e->have_plan) return MI3D_ERR_BAD_STATE;
    std::vector<PlanTensor> ts;
    for (auto& kv : e->tensors) ts.push_back(kv.second.plan);
    *bytes = plan_bytes_at(ts, e->transient, op, false);
    return MI3D_OK;
}

int mi3d_swap_alloc(mi3d_swap_engine* e, size_t bytes, void* stream, void** dev_ptr) {
    if (!e || !dev_ptr || bytes == 0) return MI3D_ERR_INVALID_ARG;
    if (!e->cfg.dev_arena) return MI3D_ERR_BAD_STATE;
    size_t need = (bytes + 255) & ~(size_t)255;
    // drop events that have already fired, so that idle blocks cost no wait
    for (ArenaBlock& b : e->blocks) {
        if (!b.free) continue;
        auto& pv = b.pending;
        pv.erase(std::remove_if(pv.begin(), pv.end(), [](const Pending& p) { return hipEventQuery((hipEvent_t)p.ev.get()) == hipSuccess; }), pv.end());
    }
    coalesce(e);
    // First fit, in this order: (0) below the plan's peak of saved bytes, among blocks that do not wait for a copy
    // (the host runs ahead of the device, so most freed blocks still carry an unfired compute-stream event: that
    // wait costs nothing); (1) below that peak, a block behind a swap-out in flight: the allocating stream stalls
    // for the rest of that transfer, which is what a device of the budget's size would have to do; (2) anywhere:
    // only when fragmentation leaves no block below the peak (counted as an overflow).  Without a plan the whole
    // arena is fair game.
    const size_t cap = e->have_plan && e->arena_cap ? e->arena_cap : e->cfg.arena_bytes;
    const bool from_top = false;   // (placement runs upwards from the bottom of the arena)
    int pick = -1;
    size_t at = 0;   // offset of the allocation inside the picked block
    for (int pass = 0; pass < 4 && pick < 0; ++pass) {
        if (pass == 1) coalesce_all(e);   // from here on a wait for a copy is accepted: free space counts as one piece
        const int n = (int)e->blocks.size();
        for (int k = 0; k < n; ++k) {
            const int i = from_top ? n - 1 - k : k;
            const ArenaBlock& b = e->blocks[i];
            if (!b.free || b.size < need) continue;
            if ((pass == 0 || pass == 2) && waits_for_copy(b)) continue;
            size_t off = 0;
            if (from_top) {   // the highest position inside the block that stays below the cap (passes 0, 1)
                size_t end = b.off + b.size;
                if (pass < 2 && end > cap) end = cap;
                if (end < b.off + need) continue;
                off = end - need - b.off;
            } else if (pass < 2 && b.off + need > cap) {
                continue;
            }
            pick = i;
            at = off;
            break;
        }
    }
    if (pick < 0) return MI3D_ERR_OVER_BUDGET;
    if (e->blocks[pick].off + at + need > cap) e->arena_overflow++;
    for (auto& p : e->blocks[pick].pending) HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)p.ev.get(), 0));
    {
        // split the picked block into [before | allocation | after]; the free parts keep the pending events
        ArenaBlock b = e->blocks[pick];
        std::vector<ArenaBlock> parts;
        if (at > 0) parts.push_back(ArenaBlock{b.off, at, true, b.pending});
        parts.push_back(ArenaBlock{b.off + at, need, false, {}});
        if (at + need < b.size) parts.push_back(ArenaBlock{b.off + at + need, b.size - at - need, true, b.pending});
        e->blocks.erase(e->blocks.begin() + pick);
        e->blocks.insert(e->blocks.begin() + pick, parts.begin(), parts.end());
        if (at > 0) ++pick;
    }
    ArenaBlock& a = e->blocks[pick];
    e->arena_used += need;
    note_occupancy(e);
    *dev_ptr = (char*)e->cfg.dev_arena + a.off;
    return MI3D_OK;
}

int mi3d_swap_set_budget(mi3d_swap_engine* e, size_t budget_bytes) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    e->cfg.budget_bytes = budget_bytes;
    e->have_plan = false;
    return MI3D_OK;
}

int mi3d_swap_set_arena(mi3d_swap_engine* e, void* dev_arena, size_t arena_bytes) {
    if (!e || (dev_arena == nullptr) != (arena_bytes == 0) || ((uintptr_t)dev_arena & 255)) return MI3D_ERR_INVALID_ARG;
    for (const ArenaBlock& b : e->blocks)
        if (!b.free) return MI3D_ERR_BAD_STATE;   // blocks of the old arena are still handed out
    e->blocks.clear();
    e->cfg.dev_arena = dev_arena;
    e->cfg.arena_bytes = arena_bytes;
    e->arena_used = 0;
    if (arena_bytes) e->blocks.push_back(ArenaBlock{0, arena_bytes & ~(size_t)255, true, {}});
    return MI3D_OK;
}

int mi3d_swap_static_arena_bytes(mi3d_swap_engine* e, uint64_t* bytes) {
    if (!e || !bytes) return MI3D_ERR_INVALID_ARG;
    if (!e->have_plan) return MI3D_ERR_BAD_STATE;
    *bytes = e->plan_res.static_arena_bytes;
    return MI3D_OK;
}

int mi3d_swap_planned_offset(mi3d_swap_engine* e, int id, int stay, uint64_t* offset) {
    if (!e || !offset || stay < 0 || stay > 1) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t || !e->have_plan) return MI3D_ERR_BAD_STATE;
    if (stay == 1 && !t->plan.planned && !t->plan.recompute) return MI3D_ERR_BAD_STATE;   // a kept tensor stays once
    *offset = t->plan.arena_off[stay];
    return MI3D_OK;
}

int mi3d_swap_alloc_tensor(mi3d_swap_engine* e, int id, void* stream, void** dev_ptr) {
    if (!e || !dev_ptr) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t || !e->have_plan || !e->cfg.dev_arena) return MI3D_ERR_BAD_STATE;
    const size_t need = (t->plan.bytes + 255) & ~(size_t)255;
    const bool leaves = t->plan.planned || t->plan.recompute;
    const int stay = leaves && t->allocs > 0 ? 1 : 0;
    const size_t off = t->plan.arena_off[stay];
    t->allocs++;
    // every block the planned range touches must be free; the range then waits for whatever still uses those blocks
    bool fits = off + need <= (e->cfg.arena_bytes & ~(size_t)255);
    for (const ArenaBlock& b : e->blocks)
        if (fits && b.off < off + need && off < b.off + b.size && !b.free) fits = false;
    if (!fits) {   // the step did not follow the plan's lifetimes (or the arena is smaller than the placement): any free block
        e->arena_overflow++;
        return mi3d_swap_alloc(e, t->plan.bytes, stream, dev_ptr);
    }
    for (ArenaBlock& b : e->blocks) {   // drop events that have fired
        if (!b.free) continue;
        auto& pv = b.pending;
        pv.erase(std::remove_if(pv.begin(), pv.end(), [](const Pending& p) { return hipEventQuery((hipEvent_t)p.ev.get()) == hipSuccess; }), pv.end());
    }
    std::vector<ArenaBlock> out;
    bool placed = false;
    for (const ArenaBlock& b : e->blocks) {
        if (!(b.off < off + need && off < b.off + b.size)) { out.push_back(b); continue; }
        for (const Pending& p : b.pending) HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)p.ev.get(), 0));
        if (b.off < off) out.push_back(ArenaBlock{b.off, off - b.off, true, b.pending});
        if (!placed) { out.push_back(ArenaBlock{off, need, false, {}}); placed = true; }
        if (b.off + b.size > off + need) out.push_back(ArenaBlock{off + need, b.off + b.size - (off + need), true, b.pending});
    }
    e->blocks.swap(out);
    e->arena_used += need;
    note_occupancy(e);
    *dev_ptr = (char*)e->cfg.dev_arena + off;
    return MI3D_OK;
}

int mi3d_swap_free(mi3d_swap_engine* e, void* dev_ptr, void* stream) {
    if (!e || !dev_ptr) return MI3D_ERR_INVALID_ARG;
    if (!in_arena(e, dev_ptr)) return MI3D_ERR_BAD_STATE;
    std::shared_ptr<void> ev;
    int st = record_shared(e, (hipStream_t)stream, &ev);
    if (st) return st;
    return arena_free(e, dev_ptr, {Pending{ev, false}});
}

int mi3d_swap_out(mi3d_swap_engine* e, int id, const void* dev_src, void* producer_stream) {
    if (!e || !dev_src) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t || !e->have_plan || !t->plan.planned || t->state != ST_NEW || !e->live) return MI3D_ERR_BAD_STATE;
    if (t->plan.host_offset + t->plan.bytes > e->cfg.host_pool_bytes) return MI3D_ERR_HOST_POOL;
    hipEvent_t dep;
    int st = get_event(e, false, &dep);
    if (st) return st;
    HIP_TRY(hipEventRecord(dep, (hipStream_t)producer_stream));
    HIP_TRY(hipStreamWaitEvent(e->s_out, dep, 0));
    e->free_events_plain.push_back(dep);  // the enqueued wait refers to the record above; the handle may be re-recorded
    if ((st = get_event(e, true, &t->out.start)) || (st = get_event(e, true, &t->out.done))) return st;
#if defined(__HIPCC__)
    if (e->verify) {   // what leaves the device (the side stream is already behind the producer)
        if ((int)e->sum_slot.size() >= e->sums_slots) return MI3D_ERR_BAD_STATE;
        const int slot = (int)e->sum_slot.size();
        e->sum_slot[id] = slot;
        e->sums_host[2 * slot] = 0;
        e->sums_host[2 * slot + 1] = 1;   // differs from the first word until the swap-in has been checked
        if ((st = enqueue_checksum(dev_src, t->plan.bytes, e->sums_scratch, e->sums_host + 2 * slot, e->s_out))) return st;
    }
#endif
    HIP_TRY(hipEventRecord(t->out.start, e->s_out));
    HIP_TRY(hipMemcpyAsync(e->host_pool + t->plan.host_offset, dev_src, t->plan.bytes, hipMemcpyDeviceToHost, e->s_out));
    HIP_TRY(hipEventRecord(t->out.done, e->s_out));
    t->out.issued = true;
    t->dev_src = dev_src;
    t->state = ST_OUT_ISSUED;
    e->bytes_out += t->plan.bytes;
    e->n_out++;
    return MI3D_OK;
}

int mi3d_swap_release(mi3d_swap_engine* e, int id, void* last_consumer_stream) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t || t->state != ST_OUT_ISSUED) return MI3D_ERR_BAD_STATE;
    if (in_arena(e, t->dev_src)) {
        std::shared_ptr<void> consumer, copy;
        int st = record_shared(e, (hipStream_t)last_consumer_stream, &consumer);
        if (st) return st;
        if ((st = record_shared(e, e->s_out, &copy))) return st;  // s_out is in order: fires after this tensor's copy
        if ((st = arena_free(e, t->dev_src, {Pending{consumer, false}, Pending{copy, true}}))) return st;
    } else {
        HIP_TRY(hipStreamWaitEvent((hipStream_t)last_consumer_stream, t->out.done, 0));
    }
    t->dev_src = nullptr;
    t->state = ST_HOST;
    return MI3D_OK;
}

int mi3d_swap_in(mi3d_swap_engine* e, int id, void* dev_dst, void* consumer_stream) {
    if (!e || !dev_dst) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t || t->state != ST_HOST || !e->live) return MI3D_ERR_BAD_STATE;
    if (t->plan.host_offset + t->plan.bytes > e->cfg.host_pool_bytes) return MI3D_ERR_HOST_POOL;
    hipEvent_t dep;
    int st = get_event(e, false, &dep);
    if (st) return st;
    HIP_TRY(hipEventRecord(dep, (hipStream_t)consumer_stream));
    HIP_TRY(hipStreamWaitEvent(e->s_in, dep, 0));
    e->free_events_plain.push_back(dep);
    HIP_TRY(hipStreamWaitEvent(e->s_in, t->out.done, 0));  // the host copy must be complete
    if ((st = get_event(e, true, &t->in.start)) || (st = get_event(e, true, &t->in.done))) return st;
    HIP_TRY(hipEventRecord(t->in.start, e->s_in));
    HIP_TRY(hipMemcpyAsync(dev_dst, e->host_pool + t->plan.host_offset, t->plan.bytes, hipMemcpyHostToDevice, e->s_in));
    HIP_TRY(hipEventRecord(t->in.done, e->s_in));
#if defined(__HIPCC__)
    if (e->verify) {   // what arrived back on the device (behind the done event: the consumer does not wait for it)
        auto it = e->sum_slot.find(id);
        if (it == e->sum_slot.end()) return MI3D_ERR_BAD_STATE;
        if ((st = enqueue_checksum(dev_dst, t->plan.bytes, e->sums_scratch + CK_BLOCKS, e->sums_host + 2 * it->second + 1, e->s_in))) return st;
    }
#endif
    t->in.issued = true;
    t->state = ST_IN_ISSUED;
    e->bytes_in += t->plan.bytes;
    e->n_in++;
    return MI3D_OK;
}

int mi3d_swap_wait_in(mi3d_swap_engine* e, int id, void* consumer_stream) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t || (t->state != ST_IN_ISSUED && t->state != ST_BACK)) return MI3D_ERR_BAD_STATE;
    HIP_TRY(hipStreamWaitEvent((hipStream_t)consumer_stream, t->in.done, 0));
    t->state = ST_BACK;
    return MI3D_OK;
}

int mi3d_swap_done(mi3d_swap_engine* e, int id) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    Tensor* t = find(e, id);
    if (!t || t->state != ST_BACK) return MI3D_ERR_BAD_STATE;
    t->state = ST_DONE;
    return MI3D_OK;
}

int mi3d_swap_set_verify(mi3d_swap_engine* e, int on) {
    if (!e) return MI3D_ERR_INVALID_ARG;
#if defined(__HIPCC__)
    if (!e->live) return MI3D_ERR_BAD_STATE;
    if (on && !e->sums_host) {
        const int slots = (int)e->tensors.size() > 0 ? (int)e->tensors.size() : 1;
        HIP_TRY(hipHostMalloc((void**)&e->sums_host, (size_t)slots * 2 * sizeof(unsigned long long), hipHostMallocDefault));
        HIP_TRY(hipMalloc((void**)&e->sums_scratch, 2 * CK_BLOCKS * sizeof(unsigned long long)));
        e->sums_slots = slots;
    } else if (on && (int)e->tensors.size() > e->sums_slots) {
        return MI3D_ERR_BAD_STATE;   // tensors were registered after the mode was switched on
    }
    e->verify = on != 0;
    return MI3D_OK;
#else
    (void)on;
    return MI3D_ERR_UNSUPPORTED;
#endif
}

int mi3d_checksum64(const void* dev, size_t bytes, uint64_t* value, void* stream) {
    if (!dev || !value || ((uintptr_t)dev & 7)) return MI3D_ERR_INVALID_ARG;
#if defined(__HIPCC__)
    unsigned long long* scratch = nullptr;
    HIP_TRY(hipMalloc((void**)&scratch, (CK_BLOCKS + 1) * sizeof(unsigned long long)));
    int st = enqueue_checksum(dev, bytes, scratch, scratch + CK_BLOCKS, (hipStream_t)stream);
    hipError_t err = hipSuccess;
    if (!st) err = hipMemcpyAsync(value, scratch + CK_BLOCKS, sizeof(unsigned long long), hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (!st && err == hipSuccess) err = hipStreamSynchronize((hipStream_t)stream);
    (void)hipFree(scratch);
    if (err != hipSuccess) { note_hip_error(err); return MI3D_ERR_HIP; }
    return st;
#else
    (void)bytes; (void)stream;
    return MI3D_ERR_UNSUPPORTED;
#endif
}

int mi3d_swap_sync(mi3d_swap_engine* e) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    if (!e->live) return MI3D_OK;
    HIP_TRY(hipStreamSynchronize(e->s_out));
    HIP_TRY(hipStreamSynchronize(e->s_in));
    return MI3D_OK;
}

int mi3d_swap_reset_step(mi3d_swap_engine* e) {
    if (!e) return MI3D_ERR_INVALID_ARG;
    int st = mi3d_swap_sync(e);
    if (st) return st;
    // blocks a step that ended early never returned: nothing says which stream still uses them, so the device is
    // drained before they go back (a step that ran to its end has freed everything and pays nothing here)
    bool leaked = false;
    for (const ArenaBlock& b : e->blocks) leaked = leaked || !b.free;
    if (leaked) {
        HIP_TRY(hipDeviceSynchronize());
        for (ArenaBlock& b : e->blocks) {
            if (b.free) continue;
            b.free = true;
            b.pending.clear();
            e->arena_used -= b.size;
        }
        coalesce(e);
    }
    reset_step_state(e);
    if (e->live) HIP_TRY(hipEventRecord(e->base, e->s_out));
    return MI3D_OK;
}

int mi3d_swap_stats(mi3d_swap_engine* e, mi3d_swap_stats_t* out) {
    if (!e || !out) return MI3D_ERR_INVALID_ARG;
    *out = mi3d_swap_stats_t();
    out->bytes_out = e->bytes_out;
    out->bytes_in = e->bytes_in;
    out->peak_arena_bytes = e->arena_occupied_peak;
    out->arena_high_water_bytes = e->arena_hwm;
    out->planned_arena_bytes = e->have_plan ? e->arena_cap : 0;
    out->static_arena_bytes = e->have_plan ? e->plan_res.static_arena_bytes : 0;
    out->n_arena_overflow = e->arena_overflow;
    out->planned_peak_bytes = e->have_plan ? e->plan_res.planned_peak : 0;
    out->unswapped_peak_bytes = e->have_plan ? e->plan_res.unswapped_peak : 0;
    out->n_registered = (int)e->tensors.size();
    out->n_planned = e->have_plan ? e->plan_res.n_planned : 0;
    out->n_swapped_out = e->n_out;
    out->n_swapped_in = e->n_in;
    out->n_recompute = e->have_plan ? e->plan_res.n_recompute : 0;
    out->recompute_ms = e->have_plan ? e->plan_res.recompute_ms : 0.0;
    if (!e->live) return MI3D_OK;
    int st = mi3d_swap_sync(e);
    if (st) return st;
    std::vector<std::pair<float, float>> iv;
    for (auto& kv : e->tensors) {
        Tensor& t = kv.second;
        for (int dir = 0; dir < 2; ++dir) {
            Copy& c = dir ? t.in : t.out;
            if (!c.issued) continue;
            float t0 = 0.f, t1 = 0.f;
            HIP_TRY(hipEventElapsedTime(&t0, e->base, c.start));
            HIP_TRY(hipEventElapsedTime(&t1, e->base, c.done));
            (dir ? out->copy_ms_in : out->copy_ms_out) += (double)(t1 - t0);
            iv.emplace_back(t0, t1);
        }
    }
    for (auto& kv : e->sum_slot) {   // (both side streams are idle here)
        Tensor* t = find(e, kv.first);
        if (!t || !t->in.issued) continue;
        out->n_checksummed++;
        if (e->sums_host[2 * kv.second] != e->sums_host[2 * kv.second + 1]) out->n_checksum_mismatch++;
    }
    std::sort(iv.begin(), iv.end());
    double busy = 0.0;
    float cur0 = 0.f, cur1 = -1.f;
    for (auto& p : iv) {
        if (cur1 < cur0 || p.first > cur1) {
            if (cur1 >= cur0) busy += cur1 - cur0;
            cur0 = p.first;
            cur1 = p.second;
        } else {
            cur1 = std::max(cur1, p.second);
        }
    }
    if (cur1 >= cur0) busy += cur1 - cur0;
    out->busy_ms = busy;
    return MI3D_OK;
}

}  // extern "C"
