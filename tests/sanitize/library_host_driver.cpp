// Calls the host-side logic of the HIP library under the sanitizers (built by
// tests/test_sanitizers.py from csrc/distsim.hip, host code only; no GPU, no kernel launch):
// size queries, the carving of workspaces and of distsim_events, argument checks that return
// before any HIP call.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <initializer_list>

#include "distsim.h"

#define CHECK(x) do { if (!(x)) { std::printf("FAILED %s:%d %s\n", __FILE__, __LINE__, #x); return 1; } } while (0)

int main() {
    for (int L : {1, 7, 64, 255})
        for (int V : {1, 4, 16})
            for (int64_t C : {(int64_t)0, (int64_t)1, (int64_t)1000, (int64_t)1 << 20, (int64_t)0x7fffffff}) {
                const size_t w = distsim_workspace_bytes(L, V, C);
                CHECK(w > 0 && w % 256 == 0);
                distsim_costs co{};
                co.L = L; co.V = V;
                const int64_t cap = distsim_stage_entries(C > 4096 ? 4096 : C);
                const size_t a = distsim_events_bytes(&co, C, cap, 0), b = distsim_events_bytes(&co, C, cap, 1);
                CHECK(a >= w && b > a);
                distsim_events ev;
                std::memset(&ev, 0x5a, sizeof ev);
                CHECK(distsim_events_bind(&ev, (void*)(uintptr_t)(1u << 20), b, &co, C, cap, 1) == DISTSIM_OK);
                CHECK(ev.workspace_bytes == w && ev.stage_cap == cap && ev.L == L && ev.V == V && ev.num_candidates == 0);
                CHECK((uintptr_t)ev.stage_layers + (size_t)(cap > 0 ? cap : 1) * 4 <= (1u << 20) + b);
                CHECK(distsim_events_bind(&ev, (void*)(uintptr_t)(1u << 20), b - 1, &co, C, cap, 1) == DISTSIM_EINVAL);
            }
    CHECK(distsim_workspace_bytes(0, 1, 1) == 0 && distsim_workspace_bytes(256, 1, 1) == 0 && distsim_workspace_bytes(4, 17, 1) == 0);
    CHECK(distsim_workspace_bytes(4, 1, -1) == 0 && distsim_workspace_bytes(4, 1, (int64_t)1 << 31) == 0);
    CHECK(distsim_events_bytes(nullptr, 1, 1, 0) == 0);
    CHECK(distsim_stage_entries(-5) == 0 && distsim_stage_entries(10) == 10 * 64 + 448);
    CHECK(distsim_search_scratch_bytes(0) > 0 && distsim_search_scratch_bytes((int64_t)1 << 40) == distsim_search_scratch_bytes(1));
    CHECK(distsim_dedup_workspace_bytes(-1) == 0 && distsim_dedup_workspace_bytes(((int64_t)1 << 28) + 1) == 0);
    for (int64_t n : {(int64_t)0, (int64_t)1, (int64_t)63, (int64_t)100000, (int64_t)1 << 28}) CHECK(distsim_dedup_workspace_bytes(n) > 0);
    for (int k = -2; k <= DISTSIM_K_COUNT + 1; k++) CHECK(distsim_kernel_name(k) != nullptr && std::strlen(distsim_kernel_name(k)) > 0);
    // a null context is refused before anything else is looked at
    distsim_cluster cl{};
    distsim_costs co{};
    distsim_candidates ca{};
    distsim_events ev{};
    int64_t x[2];
    CHECK(distsim_build_events(nullptr, &co, &cl, &ca, 1, &ev, nullptr) == DISTSIM_EINVAL);
    CHECK(distsim_simulate(nullptr, &cl, &ca, &ev, 1, x, x, x, nullptr, nullptr) == DISTSIM_EINVAL);
    CHECK(distsim_search(nullptr, x, nullptr, 1, 0, x, x, nullptr) == DISTSIM_EINVAL);
    CHECK(distsim_search_static(nullptr, x, nullptr, 1, 0, x, nullptr) == DISTSIM_EINVAL);
    CHECK(distsim_timeline(nullptr, &cl, &ca, &ev, 1, x, x, x, x, x, x, nullptr) == DISTSIM_EINVAL);
    CHECK(distsim_bubbles(nullptr, &ca, &ev, 1, x, x, x, x, x, nullptr) == DISTSIM_EINVAL);
    CHECK(distsim_timing_enable(nullptr, 1) == DISTSIM_EINVAL);
    CHECK(std::strcmp(distsim_last_error(nullptr), "null context") == 0);
    distsim_destroy(nullptr);
    CHECK(distsim_create(nullptr, 0) == DISTSIM_EINVAL);
    std::printf("library host checks passed\n");
    return 0;
}
