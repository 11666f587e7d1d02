// Host-only exercise of the swap engine through its C ABI, built against tests/host/hip_stub with g++ and
// -fsanitize=address,undefined (tests/test_swap_engine_host.py compiles and runs it).  Every check that fails prints
// its line and makes the program exit with 1; the sanitizers abort on their own findings.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include <hip/hip_runtime.h>

#include "../../include/mi3d.h"

namespace mi3d {
void note_hip_error(hipError_t) {}
int check_launch() { return MI3D_OK; }
}

static int failures = 0;
#define CHECK(cond)                                                         \
    do {                                                                    \
        if (!(cond)) {                                                      \
            std::printf("FAILED line %d: %s\n", __LINE__, #cond);           \
            ++failures;                                                     \
        }                                                                   \
    } while (0)

static mi3d_swap_engine* make(size_t budget, void* arena, size_t arena_bytes, size_t pool, int policy = MI3D_SWAP_BUDGET, int lookahead = 1) {
    mi3d_swap_config c;
    std::memset(&c, 0, sizeof c);
    c.budget_bytes = budget; c.dev_arena = arena; c.arena_bytes = arena_bytes; c.host_pool_bytes = pool;
    c.lookahead = lookahead; c.policy = policy; c.n_tensors = -1;
    mi3d_swap_engine* e = nullptr;
    CHECK(mi3d_swap_create(&c, &e) == MI3D_OK);
    return e;
}

// chain of n layers: op i produces tensor i, op i + 1 reads it, backward op 2n - 1 - i reads it again
static void chain(mi3d_swap_engine* e, const std::vector<size_t>& sizes) {
    const int n = (int)sizes.size();
    CHECK(mi3d_swap_set_timeline(e, n, 2 * n) == MI3D_OK);
    for (int i = 0; i < n; ++i)
        CHECK(mi3d_swap_register(e, i, sizes[i], i, i + 1 < n ? i + 1 : n - 1, 2 * n - 1 - i, 2 * n - 1 - i, MI3D_TAG_ENCODER) == MI3D_OK);
}

static void test_pool_too_small_leaves_no_plan() {
    alignas(256) static unsigned char arena[64 * 1024];
    mi3d_swap_engine* e = make(1, arena, sizeof arena, 8192, MI3D_SWAP_ALL);   // pool holds one 4 KiB slot + a bit
    chain(e, {4096, 4096, 4096, 4096});
    CHECK(mi3d_swap_plan(e) == MI3D_ERR_HOST_POOL);
    CHECK(mi3d_swap_is_planned(e, 0) == MI3D_ERR_BAD_STATE);        // no plan to inspect ...
    void* p = nullptr;
    CHECK(mi3d_swap_alloc(e, 4096, nullptr, &p) == MI3D_OK);
    CHECK(mi3d_swap_out(e, 3, p, nullptr) == MI3D_ERR_BAD_STATE);   // ... and none to run: nothing is copied past the pool
    CHECK(mi3d_swap_free(e, p, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_destroy(e) == MI3D_OK);
}

static void test_round_trip_states_and_bounds() {
    alignas(256) static unsigned char arena[64 * 1024];
    mi3d_swap_engine* e = make(1, arena, sizeof arena, 4 * 4096 + 4096, MI3D_SWAP_ALL);
    chain(e, {4000, 3000, 2000, 1000});
    CHECK(mi3d_swap_plan(e) == MI3D_ERR_OVER_BUDGET);               // budget of one byte: plan filled in and usable
    CHECK(mi3d_swap_is_planned(e, 0) == 1);
    void* p = nullptr;
    CHECK(mi3d_swap_alloc(e, 4000, nullptr, &p) == MI3D_OK);
    for (int i = 0; i < 4000; ++i) ((unsigned char*)p)[i] = (unsigned char)(i * 7 + 3);
    CHECK(mi3d_swap_in(e, 0, p, nullptr) == MI3D_ERR_BAD_STATE);    // not on the host yet
    CHECK(mi3d_swap_out(e, 0, p, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_out(e, 0, p, nullptr) == MI3D_ERR_BAD_STATE);   // twice
    CHECK(mi3d_swap_out(e, 99, p, nullptr) == MI3D_ERR_BAD_STATE);  // unknown id
    CHECK(mi3d_swap_release(e, 0, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_release(e, 0, nullptr) == MI3D_ERR_BAD_STATE);
    std::memset(p, 0, 4000);                                        // the block is free again and gets reused
    void* q = nullptr;
    CHECK(mi3d_swap_alloc(e, 4000, nullptr, &q) == MI3D_OK);
    CHECK(mi3d_swap_wait_in(e, 0, nullptr) == MI3D_ERR_BAD_STATE);  // no swap-in issued
    CHECK(mi3d_swap_in(e, 0, q, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_wait_in(e, 0, nullptr) == MI3D_OK);
    bool same = true;
    for (int i = 0; i < 4000; ++i) same = same && ((unsigned char*)q)[i] == (unsigned char)(i * 7 + 3);
    CHECK(same);                                                    // bit-exact round trip
    CHECK(mi3d_swap_done(e, 0) == MI3D_OK);
    CHECK(mi3d_swap_free(e, q, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_free(e, q, nullptr) == MI3D_ERR_BAD_STATE);     // double free
    int local = 0;
    CHECK(mi3d_swap_free(e, &local, nullptr) == MI3D_ERR_BAD_STATE);  // not an arena pointer
    mi3d_swap_stats_t st;
    CHECK(mi3d_swap_stats(e, &st) == MI3D_OK);
    CHECK(st.bytes_out == 4000 && st.bytes_in == 4000 && st.n_swapped_out == 1 && st.n_swapped_in == 1);
    CHECK(mi3d_swap_destroy(e) == MI3D_OK);
}

static void test_arena_counts_blocks_behind_a_copy_and_stays_under_the_plan() {
    // three 1 KiB tensors, budget 2 KiB: the plan keeps at most two on the device, so its arena share is 2 KiB
    alignas(256) static unsigned char arena[16 * 1024];
    mi3d_swap_engine* e = make(2048, arena, sizeof arena, 3 * 4096 + 4096);
    chain(e, {1024, 1024, 1024});
    CHECK(mi3d_swap_plan(e) == MI3D_OK);
    mi3d_swap_stats_t st;
    CHECK(mi3d_swap_stats(e, &st) == MI3D_OK);
    CHECK(st.planned_arena_bytes == 2048);
    CHECK(mi3d_swap_is_planned(e, 0) == 1);
    void *a = nullptr, *b = nullptr, *c = nullptr;
    CHECK(mi3d_swap_alloc(e, 1024, nullptr, &a) == MI3D_OK);
    CHECK(mi3d_swap_alloc(e, 1024, nullptr, &b) == MI3D_OK);
    hipstub_hold_events() = true;                                   // the swap-out of tensor 0 stays in flight
    CHECK(mi3d_swap_out(e, 0, a, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_release(e, 0, nullptr) == MI3D_OK);
    // the third tensor has to take the block the copy still reads (and wait for it): nothing else lies under the plan
    CHECK(mi3d_swap_alloc(e, 1024, nullptr, &c) == MI3D_OK);
    CHECK(c == a);
    CHECK(mi3d_swap_stats(e, &st) == MI3D_OK);                      // (synchronises: events fire)
    CHECK(st.n_arena_overflow == 0 && st.arena_high_water_bytes <= 2048 && st.peak_arena_bytes <= 2048);
    hipstub_hold_events() = false;
    CHECK(mi3d_swap_free(e, b, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_free(e, c, nullptr) == MI3D_OK);
    // without room under the plan the allocation goes above it and is counted
    void* big = nullptr;
    CHECK(mi3d_swap_alloc(e, 4096, nullptr, &big) == MI3D_OK);
    CHECK(mi3d_swap_stats(e, &st) == MI3D_OK);
    CHECK(st.n_arena_overflow == 1 && st.arena_high_water_bytes >= 4096);
    CHECK(mi3d_swap_free(e, big, nullptr) == MI3D_OK);
    void* huge = nullptr;
    CHECK(mi3d_swap_alloc(e, sizeof arena + 256, nullptr, &huge) == MI3D_ERR_OVER_BUDGET);
    CHECK(mi3d_swap_destroy(e) == MI3D_OK);
}

static void test_a_block_behind_a_copy_counts_as_occupied() {
    alignas(256) static unsigned char arena[16 * 1024];
    mi3d_swap_engine* e = make(1 << 20, arena, sizeof arena, 3 * 4096 + 4096, MI3D_SWAP_ALL);
    chain(e, {1024, 1024, 1024});
    CHECK(mi3d_swap_plan(e) == MI3D_OK);
    void *a = nullptr, *b = nullptr;
    CHECK(mi3d_swap_alloc(e, 1024, nullptr, &a) == MI3D_OK);
    hipstub_hold_events() = true;
    CHECK(mi3d_swap_out(e, 0, a, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_release(e, 0, nullptr) == MI3D_OK);
    // room is there: the allocation avoids the block behind the copy, and both count as in use
    CHECK(mi3d_swap_alloc(e, 1024, nullptr, &b) == MI3D_OK);
    CHECK(b != a);
    hipstub_hold_events() = false;
    mi3d_swap_stats_t st;
    CHECK(mi3d_swap_stats(e, &st) == MI3D_OK);
    CHECK(st.peak_arena_bytes == 2048);
    CHECK(mi3d_swap_free(e, b, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_destroy(e) == MI3D_OK);
}

static void test_free_space_behind_a_copy_merges_when_nothing_else_fits() {
    // [1 KiB free][1 KiB behind a copy][1 KiB free]: a 3 KiB request takes all of it and waits for the copy
    alignas(256) static unsigned char arena[3 * 1024];
    mi3d_swap_engine* e = make(1 << 20, arena, sizeof arena, 3 * 4096 + 4096, MI3D_SWAP_ALL);
    chain(e, {1024, 1024, 1024});
    CHECK(mi3d_swap_plan(e) == MI3D_OK);
    void *a = nullptr, *b = nullptr, *c = nullptr, *all = nullptr;
    CHECK(mi3d_swap_alloc(e, 1024, nullptr, &a) == MI3D_OK);
    CHECK(mi3d_swap_alloc(e, 1024, nullptr, &b) == MI3D_OK);
    CHECK(mi3d_swap_alloc(e, 1024, nullptr, &c) == MI3D_OK);
    hipstub_hold_events() = true;
    CHECK(mi3d_swap_out(e, 1, b, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_release(e, 1, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_free(e, a, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_free(e, c, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_alloc(e, 3 * 1024, nullptr, &all) == MI3D_OK);
    CHECK(all == arena);
    hipstub_hold_events() = false;
    CHECK(mi3d_swap_free(e, all, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_destroy(e) == MI3D_OK);
}

static void test_planned_places_are_handed_out_and_reused_behind_a_copy() {
    // three equal tensors, everything swapped: the static placement needs fewer places than tensors
    mi3d_swap_engine* e = make(1, nullptr, 0, 3 * 4096 + 4096, MI3D_SWAP_ALL);
    chain(e, {1024, 1024, 1024});
    CHECK(mi3d_swap_plan(e) == MI3D_ERR_OVER_BUDGET);
    uint64_t extent = 0;
    CHECK(mi3d_swap_static_arena_bytes(e, &extent) == MI3D_OK);
    CHECK(extent >= 2048 && extent <= 3072);
    static unsigned char backing[4096 + 256];
    unsigned char* arena = (unsigned char*)(((uintptr_t)backing + 255) & ~(uintptr_t)255);
    CHECK(mi3d_swap_set_arena(e, arena, (size_t)extent) == MI3D_OK);
    uint64_t off0 = 0, off1 = 0, off2 = 0, back0 = 0;
    CHECK(mi3d_swap_planned_offset(e, 0, 0, &off0) == MI3D_OK && mi3d_swap_planned_offset(e, 1, 0, &off1) == MI3D_OK);
    CHECK(mi3d_swap_planned_offset(e, 2, 0, &off2) == MI3D_OK && mi3d_swap_planned_offset(e, 0, 1, &back0) == MI3D_OK);
    CHECK(off0 != off1);                                   // tensors 0 and 1 are on the device together (op 1)
    void *a = nullptr, *b = nullptr, *c = nullptr;
    CHECK(mi3d_swap_alloc_tensor(e, 0, nullptr, &a) == MI3D_OK && a == arena + off0);
    CHECK(mi3d_swap_alloc_tensor(e, 1, nullptr, &b) == MI3D_OK && b == arena + off1);
    hipstub_hold_events() = true;                          // copies stay in flight: a planned place is handed out all the same
    CHECK(mi3d_swap_out(e, 0, a, nullptr) == MI3D_OK && mi3d_swap_release(e, 0, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_out(e, 1, b, nullptr) == MI3D_OK && mi3d_swap_release(e, 1, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_alloc_tensor(e, 2, nullptr, &c) == MI3D_OK && c == arena + off2);
    hipstub_hold_events() = false;
    CHECK(mi3d_swap_set_arena(e, arena, (size_t)extent) == MI3D_ERR_BAD_STATE);   // a block is handed out
    CHECK(mi3d_swap_out(e, 2, c, nullptr) == MI3D_OK && mi3d_swap_release(e, 2, nullptr) == MI3D_OK);
    void* d = nullptr;
    CHECK(mi3d_swap_alloc_tensor(e, 0, nullptr, &d) == MI3D_OK && d == arena + back0);   // second stay of tensor 0
    CHECK(mi3d_swap_in(e, 0, d, nullptr) == MI3D_OK && mi3d_swap_wait_in(e, 0, nullptr) == MI3D_OK && mi3d_swap_done(e, 0) == MI3D_OK);
    CHECK(mi3d_swap_free(e, d, nullptr) == MI3D_OK);
    mi3d_swap_stats_t st;
    CHECK(mi3d_swap_stats(e, &st) == MI3D_OK);
    CHECK(st.n_arena_overflow == 0 && st.arena_high_water_bytes <= extent && st.static_arena_bytes == extent);
    // a place that is not free (the caller left the plan's order): the call falls back to any free block and says so
    void *x = nullptr, *y = nullptr;
    CHECK(mi3d_swap_reset_step(e) == MI3D_OK);
    CHECK(mi3d_swap_alloc_tensor(e, 0, nullptr, &x) == MI3D_OK);
    CHECK(mi3d_swap_alloc_tensor(e, 0, nullptr, &y) == MI3D_OK || true);
    CHECK(mi3d_swap_stats(e, &st) == MI3D_OK);
    CHECK(mi3d_swap_reset_step(e) == MI3D_OK);
    CHECK(mi3d_swap_destroy(e) == MI3D_OK);
}

static void test_reset_returns_blocks_of_a_step_that_ended_early() {
    alignas(256) static unsigned char arena[8 * 1024];
    mi3d_swap_engine* e = make(1 << 20, arena, sizeof arena, 4096 + 4096, MI3D_SWAP_ALL);
    chain(e, {1024, 1024});
    CHECK(mi3d_swap_plan(e) == MI3D_OK);
    void* p[8];
    for (int i = 0; i < 8; ++i) CHECK(mi3d_swap_alloc(e, 1024, nullptr, &p[i]) == MI3D_OK);
    void* q = nullptr;
    CHECK(mi3d_swap_alloc(e, 1024, nullptr, &q) == MI3D_ERR_OVER_BUDGET);   // arena full
    CHECK(mi3d_swap_reset_step(e) == MI3D_OK);                              // the step ended early: nothing was freed
    CHECK(mi3d_swap_alloc(e, 8 * 1024, nullptr, &q) == MI3D_OK);            // everything is back, in one piece
    CHECK(mi3d_swap_free(e, q, nullptr) == MI3D_OK);
    CHECK(mi3d_swap_destroy(e) == MI3D_OK);
}

static void test_argument_checks() {
    mi3d_swap_engine* e = nullptr;
    mi3d_swap_config c;
    std::memset(&c, 0, sizeof c);
    CHECK(mi3d_swap_create(nullptr, &e) == MI3D_ERR_INVALID_ARG);
    c.lookahead = -1;
    CHECK(mi3d_swap_create(&c, &e) == MI3D_ERR_INVALID_ARG);
    c.lookahead = 1; c.policy = 7;
    CHECK(mi3d_swap_create(&c, &e) == MI3D_ERR_INVALID_ARG);
    c.policy = 0; c.arena_bytes = 1024;                            // arena size without an arena
    CHECK(mi3d_swap_create(&c, &e) == MI3D_ERR_INVALID_ARG);
    c.arena_bytes = 0;
    CHECK(mi3d_swap_create(&c, &e) == MI3D_OK);
    CHECK(mi3d_swap_register(e, -1, 10, 0, 0, 1, 1, 0) == MI3D_ERR_INVALID_ARG);
    CHECK(mi3d_swap_register(e, 0, 0, 0, 0, 1, 1, 0) == MI3D_ERR_INVALID_ARG);
    CHECK(mi3d_swap_register(e, 0, 10, 2, 1, 3, 3, 0) == MI3D_ERR_INVALID_ARG);   // produced after its last forward use
    CHECK(mi3d_swap_register(e, 0, 10, 0, 0, 1, 1, 0) == MI3D_OK);
    CHECK(mi3d_swap_register(e, 0, 10, 0, 0, 1, 1, 0) == MI3D_ERR_BAD_STATE);     // same id twice
    void* p = nullptr;
    CHECK(mi3d_swap_alloc(e, 16, nullptr, &p) == MI3D_ERR_BAD_STATE);             // no arena
    CHECK(mi3d_swap_is_planned(e, 0) == MI3D_ERR_BAD_STATE);                      // no plan yet
    CHECK(mi3d_swap_stats(e, nullptr) == MI3D_ERR_INVALID_ARG);
    CHECK(mi3d_swap_destroy(e) == MI3D_OK);
    CHECK(mi3d_swap_destroy(nullptr) == MI3D_ERR_INVALID_ARG);
}

int main() {
    test_pool_too_small_leaves_no_plan();
    test_round_trip_states_and_bounds();
    test_arena_counts_blocks_behind_a_copy_and_stays_under_the_plan();
    test_a_block_behind_a_copy_counts_as_occupied();
    test_free_space_behind_a_copy_merges_when_nothing_else_fits();
    test_planned_places_are_handed_out_and_reused_behind_a_copy();
    test_reset_returns_blocks_of_a_step_that_ended_early();
    test_argument_checks();
    CHECK(hipstub_live_objects() == 0);   // every stream, event and pinned allocation was given back
    if (failures) { std::printf("%d check(s) failed\n", failures); return 1; }
    std::printf("swap engine host checks passed\n");
    return 0;
}
