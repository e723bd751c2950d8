// Drives the host-only logic of libjupiter_stage (argument validation, cache bookkeeping, the planner's dynamic
// programs) from a program whose jup_api and jup_plan objects are built with -fsanitize=address,undefined.  No
// kernel is launched and no device is needed: device pointers are fake and never dereferenced on the host.
// Every expectation is checked; the first failure prints its line and exits non-zero.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "jupiter_plan.h"
#include "jupiter_stage.h"

#define EXPECT(cond)                                                                  \
    do {                                                                              \
        if (!(cond)) {                                                                \
            std::fprintf(stderr, "host_driver.cpp:%d: %s  [%s]\n", __LINE__, #cond, jup_last_error()); \
            std::exit(1);                                                             \
        }                                                                             \
    } while (0)

static void* const FAKE = (void*)0x700000000000ull;  // 256-byte aligned, never touched

static jup_stage_config_t cfg_7b(int dtype) { return {8, 4096, 32, 128, 11008, 1e-5f, 1e4f, dtype, 0}; }
static jup_stage_config_t cfg_tiny() { return {2, 256, 4, 64, 688, 1e-5f, 1e4f, JUP_F32, 0}; }

static void stage_and_cache_validation() {
    jup_stage_config_t c = cfg_7b(JUP_BF16), t = cfg_tiny();
    EXPECT(jup_stage_packed_bytes(&c) > 0 && jup_stage_workspace_bytes(&c, 512) > 0);
    EXPECT(jup_stage_packed_bytes(nullptr) == 0 && jup_stage_workspace_bytes(&t, 0) == 0);
    jup_stage_config_t bad = t;
    bad.n_heads = 3;
    EXPECT(jup_stage_packed_bytes(&bad) == 0 && jup_kv_bytes(&bad, 8) == 0);

    std::vector<jup_layer_weights_t> layers(8);
    for (auto& w : layers) {
        w.wq = w.wk = w.wv = w.wo = w.w_gate = w.w_up = w.w_down = w.g_attn = w.g_mlp = FAKE;
        w.sq = w.sk = w.sv = w.so = w.s_gate = w.s_up = w.s_down = nullptr;
    }
    jup_stage_t* st = nullptr;
    const size_t pb = jup_stage_packed_bytes(&c), wb = jup_stage_workspace_bytes(&c, 32);
    EXPECT(jup_stage_create(&c, layers.data(), FAKE, pb - 1, FAKE, wb, 32, nullptr, &st) == JUP_EINVAL && !st);
    EXPECT(jup_stage_create(&c, layers.data(), FAKE, pb, FAKE, wb - 1, 32, nullptr, &st) == JUP_EINVAL);
    EXPECT(jup_stage_create(&c, layers.data(), nullptr, pb, FAKE, wb, 32, nullptr, &st) == JUP_EINVAL);
    EXPECT(jup_stage_create(&c, layers.data(), (char*)FAKE + 8, pb, FAKE, wb, 32, nullptr, &st) == JUP_EINVAL);
    EXPECT(jup_stage_create(&c, layers.data(), FAKE, pb, FAKE, wb, 0, nullptr, &st) == JUP_EINVAL);
    EXPECT(jup_stage_create(nullptr, layers.data(), FAKE, pb, FAKE, wb, 32, nullptr, &st) == JUP_EINVAL);
    EXPECT(jup_stage_create(&c, layers.data(), FAKE, pb, FAKE, wb, 32, nullptr, nullptr) == JUP_EINVAL);
    layers[5].w_up = nullptr;
    EXPECT(jup_stage_create(&c, layers.data(), FAKE, pb, FAKE, wb, 32, nullptr, &st) == JUP_EINVAL);
    layers[5].w_up = (char*)FAKE + 2;  // not 16-byte aligned
    EXPECT(jup_stage_create(&c, layers.data(), FAKE, pb, FAKE, wb, 32, nullptr, &st) == JUP_EINVAL);
    layers[5].w_up = FAKE;
    jup_stage_config_t w4 = cfg_7b(JUP_BF16_W4);
    EXPECT(jup_stage_create(&w4, layers.data(), FAKE, jup_stage_packed_bytes(&w4), FAKE, wb, 32, nullptr, &st) ==
           JUP_EINVAL);  // scales missing

    // cache bookkeeping (Sec. IV-A.2 position rules; Sec. V-A truncate; Sec. V-B fork)
    jup_kv_t *kv = nullptr, *fork = nullptr, *fork2 = nullptr;
    const size_t kb = jup_kv_bytes(&t, 48);
    EXPECT(jup_kv_create(&t, 48, FAKE, kb - 1, &kv) == JUP_EINVAL && !kv);
    EXPECT(jup_kv_create(&t, 0, FAKE, kb, &kv) == JUP_EINVAL);
    EXPECT(jup_kv_create(&t, 48, nullptr, kb, &kv) == JUP_EINVAL);
    EXPECT(jup_kv_create(&t, 48, FAKE, kb, &kv) == JUP_OK && kv);
    EXPECT(jup_kv_len(kv) == 0 && jup_kv_capacity(kv) == 48 && jup_kv_len(nullptr) == -1);
    EXPECT(jup_kv_check_append(kv, 32, 0) == JUP_OK);
    EXPECT(jup_kv_check_append(kv, 32, 1) == JUP_EPOS);
    EXPECT(jup_kv_check_append(kv, 49, 0) == JUP_ECAP);
    EXPECT(jup_kv_check_append(kv, -1, 0) == JUP_EINVAL && jup_kv_check_append(kv, 1, -1) == JUP_EINVAL);
    EXPECT(jup_kv_check_append(kv, INT32_MAX, 0) == JUP_ECAP);
    EXPECT(jup_kv_truncate(kv, 1) == JUP_EPOS && jup_kv_truncate(kv, 0) == JUP_OK);
    // an empty chunk is accepted without a device and moves the length (pos_offset <= length)
    EXPECT(jup_stage_prefill_chunk(nullptr, FAKE, 0, 0, kv, FAKE, nullptr) == JUP_EINVAL);
    EXPECT(jup_kv_fork_bytes(kv, 0, 16) > 0 && jup_kv_fork_bytes(kv, 4, 4) == 0 && jup_kv_fork_bytes(nullptr, 0, 4) == 0);
    EXPECT(jup_kv_fork(kv, 1, 16, FAKE, 1 << 30, &fork) == JUP_EPOS);  // parent holds 0 positions
    EXPECT(jup_kv_fork(kv, 0, 16, FAKE, jup_kv_fork_bytes(kv, 0, 16), &fork) == JUP_OK && fork);
    EXPECT(jup_kv_fork(fork, 0, 8, FAKE, 1 << 30, &fork2) == JUP_EINVAL);  // a fork of a fork
    EXPECT(jup_kv_destroy(kv) == JUP_EINVAL);                               // forks alive
    EXPECT(jup_kv_len(fork) == 0 && jup_kv_reset(fork) == JUP_OK);
    int32_t slots[4] = {0, 1, 2, 3};
    EXPECT(jup_kv_keep(fork, 0, 1, slots, nullptr) == JUP_EPOS);           // nothing cached behind base_len
    EXPECT(jup_kv_keep(fork, 0, 0, nullptr, nullptr) == JUP_OK);           // all rejected = truncate, no launch
    EXPECT(jup_kv_keep(fork, 0, 65, slots, nullptr) == JUP_EINVAL);
    EXPECT(jup_kv_keep(fork, 1, 0, nullptr, nullptr) == JUP_EPOS);
    EXPECT(jup_kv_destroy(fork) == JUP_OK && jup_kv_destroy(kv) == JUP_OK && jup_kv_destroy(nullptr) == JUP_OK);

    // calls that need a stage are refused before anything else is looked at
    int32_t chunks[3] = {4, 0, 4}, pos[2] = {0, 0}, parents[3] = {-1, 0, 1};
    EXPECT(jup_stage_prefill_chunks(nullptr, FAKE, 3, chunks, 0, nullptr, FAKE, nullptr) == JUP_EINVAL);
    EXPECT(jup_stage_prefill_branches(nullptr, 2, FAKE, 4, pos, nullptr, FAKE, nullptr) == JUP_EINVAL);
    EXPECT(jup_stage_prefill_tree(nullptr, FAKE, 3, 0, parents, nullptr, FAKE, nullptr) == JUP_EINVAL);
    EXPECT(jup_stage_trace(nullptr, 0, 4) == JUP_EINVAL && jup_stage_trace_read(nullptr, nullptr, nullptr, nullptr) == JUP_EINVAL);
    EXPECT(jup_stage_enable_overlap(nullptr, 2, FAKE, 1 << 20) == JUP_EINVAL);
    jup_stage_destroy(nullptr);
    EXPECT(jup_last_error()[0] != '\0');
}

static void planner() {
    // Eq. 1: 7 layers on 3 devices with a memory budget that forbids the otherwise best cut
    const int L = 7, D = 3;
    std::vector<double> time((size_t)D * L), mem(L, 1.0), budget = {3.0, 2.0, 4.0};
    for (int n = 0; n < D; ++n)
        for (int l = 0; l < L; ++l) time[(size_t)n * L + l] = 1.0 + 0.25 * n + 0.1 * l;
    int32_t last[3];
    double slowest = 0;
    EXPECT(jup_plan_layers(L, D, time.data(), mem.data(), budget.data(), last, &slowest) == JUP_OK);
    EXPECT(last[2] == L && last[0] >= 1 && last[0] < last[1] && last[1] < last[2] && slowest > 0);
    EXPECT(last[0] <= 3 && last[1] - last[0] <= 2 && last[2] - last[1] <= 4);
    EXPECT(jup_plan_layers(2, 3, time.data(), mem.data(), budget.data(), last, &slowest) == JUP_ECAP);
    budget[1] = 0.5;
    EXPECT(jup_plan_layers(L, D, time.data(), mem.data(), budget.data(), last, &slowest) == JUP_ECAP);
    EXPECT(jup_plan_layers(L, D, nullptr, mem.data(), budget.data(), last, &slowest) == JUP_EINVAL);

    // Eq. 2-4 on a grid that neither starts at 1 nor at 0, queried inside, on and outside the grid
    const int32_t xs[3] = {16, 64, 256}, ys[2] = {128, 512};
    const double q[6] = {1.0, 1.5, 1.2, 2.0, 3.0, 5.0};
    jup_seq_plan_t* plan = nullptr;
    EXPECT(jup_seq_plan_create(xs, 3, ys, 2, q, 8, 4, 700, &plan) == JUP_OK && plan);
    for (int x = 1; x <= 2000; x += 13)
        for (int y = 0; y <= 3000; y += 97) EXPECT(jup_seq_plan_q(plan, x, y) >= 1.0);
    EXPECT(std::isnan(jup_seq_plan_q(plan, 0, 0)) && std::isnan(jup_seq_plan_q(nullptr, 1, 1)));
    std::vector<int32_t> lens(16);
    double w = 0, total = 0, lat = 0;
    int32_t k = 0;
    for (int y = 1; y <= 700; y += 7) {
        const jup_status_t rc = jup_seq_plan_best(plan, y, &k, lens.data(), &lat);
        if (y < 8) {
            EXPECT(rc == JUP_ECAP);
            continue;
        }
        EXPECT(rc == JUP_OK && k >= 1 && k <= 16 && lat > 0);
        int sum = 0;
        for (int i = 0; i < k; ++i) {
            EXPECT(lens[i] >= 8);
            sum += lens[i];
        }
        EXPECT(sum == y);
        EXPECT(jup_seq_plan_partition(plan, y, k, lens.data(), &w, &total) == JUP_OK && std::fabs(lat - (total + 3 * w)) < 1e-9);
    }
    EXPECT(jup_seq_plan_partition(plan, 700, 17, lens.data(), &w, &total) == JUP_EINVAL);
    EXPECT(jup_seq_plan_partition(plan, 701, 2, lens.data(), &w, &total) == JUP_EINVAL);
    EXPECT(jup_seq_plan_partition(plan, 20, 3, lens.data(), &w, &total) == JUP_ECAP);
    jup_seq_plan_destroy(plan);
    jup_seq_plan_destroy(nullptr);
    const int32_t bad_xs[2] = {16, 16};
    EXPECT(jup_seq_plan_create(bad_xs, 2, ys, 2, q, 8, 4, 64, &plan) == JUP_EINVAL && !plan);
    const double bad_q[6] = {1.0, -1.0, 1.0, 1.0, 1.0, 1.0};
    EXPECT(jup_seq_plan_create(xs, 3, ys, 2, bad_q, 8, 4, 64, &plan) == JUP_EINVAL);
    EXPECT(jup_seq_plan_create(xs, 3, ys, 2, q, 8, 65, 64, &plan) == JUP_EINVAL);
}

int main() {
    stage_and_cache_validation();
    planner();
    std::printf("host_driver ok\n");
    return 0;
}
