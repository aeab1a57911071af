// Runs the host path of every entry point of the library (with the launchers stubbed out) so that a sanitizer
// can watch it: plans of 1, 5 and 64 stages in both storage types, every kind of step, pushes, ring state,
// error paths, and the pipeline planner on random layer tables with its worker threads.  Device pointers are
// fake, aligned integers; nothing dereferences them.
//
//   host_driver all       everything, single-threaded host code (AddressSanitizer + UndefinedBehaviorSanitizer)
//   host_driver planner   the planner only, on 8 worker threads (ThreadSanitizer)
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "ferret.h"
#include "ferret_planner.h"

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s (%s)\n", __LINE__, #cond, ferret_last_error()); ++failures; } } while (0)

static void *fake(uintptr_t off) { return reinterpret_cast<void *>(uintptr_t(0x10000000) + off); }

static void steps_and_pushes(ferret_precision prec, int32_t n_stages, int32_t n_iters, const ferret_tuning *tuning) {
    std::vector<ferret_tensor> tensors;
    std::vector<int32_t> tau(n_stages), zeros(n_stages, 0), full(n_stages, 6), active(n_stages), mode(n_stages), stale(n_stages);
    for (int32_t j = 0; j < n_stages; ++j) {
        tensors.push_back({1000 + 8 * j, j, 0});
        if (j % 4 == 0) tensors.push_back({3, j, 0});
        tau[j] = j % 7 < 5 ? j % 7 : 5;
        active[j] = j % 2;
        mode[j] = j % 3;
        stale[j] = tau[j] / 2;
    }
    ferret_plan *plan = nullptr;
    CHECK(ferret_plan_buckets_tuned(tensors.data(), (int32_t)tensors.size(), n_stages, tau.data(), n_iters, 6, prec, 0,
                                    tuning, &plan) == FERRET_OK);
    if (!plan) return;
    float *master = prec == FERRET_BF16_MASTER_F32 ? static_cast<float *>(fake(0x1000000)) : nullptr;
    float *norms = static_cast<float *>(fake(0x200));
    // warm-up: one version each, then a full ring
    CHECK(ferret_push_version(plan, fake(0), master, -1, fake(0x900), nullptr) == FERRET_OK);
    CHECK(ferret_compensate_step(plan, fake(0), fake(0x100), master, 0.5f, 0.01f, norms, fake(0x300), fake(0x400), nullptr) == FERRET_OK);
    CHECK(ferret_push_version(plan, fake(0), nullptr, -1, nullptr, nullptr) == FERRET_OK);
    CHECK(ferret_push_version(plan, fake(0), nullptr, -1, nullptr, nullptr) == FERRET_ESTATE);       // nothing left to commit
    CHECK(ferret_plan_set_state(plan, zeros.data(), full.data()) == FERRET_OK);
    std::vector<int32_t> heads(n_stages), valid(n_stages), slots(8);
    CHECK(ferret_plan_get_state(plan, heads.data(), valid.data()) == FERRET_OK);
    for (int32_t j = 0; j < n_stages; ++j) {
        const int32_t n = ferret_plan_stage_read_slots(plan, j, slots.data(), 8);
        CHECK(n == ferret_plan_stage_effective_iters(plan, j) + 1);
        CHECK(ferret_plan_stage_write_slot(plan, j) == 1 && ferret_plan_stage_chunk_elems(plan, j) % 1024 == 0);
    }
    CHECK(ferret_plan_step_bytes(plan) > 0 && ferret_plan_workspace_bytes(plan) >= (size_t)ferret_plan_n_chunks(plan) * 20);
    CHECK(ferret_compensate_step(plan, fake(0), fake(0x100), master, 0.5f, 0.01f, norms, fake(0x300), fake(0x400), nullptr) == FERRET_OK);
    CHECK(ferret_compensate_step_noalloc(plan, fake(0), fake(0x100), master, 0.5f, 0.01f, norms, nullptr, nullptr) == FERRET_OK);
    CHECK(ferret_compensate_stages(plan, fake(0), fake(0x100), master, active.data(), 0.5f, 0.01f, norms, nullptr, fake(0x400), nullptr) == FERRET_OK);
    CHECK(ferret_compensate_stages(plan, fake(0), fake(0x100), master, zeros.data(), 0.5f, 0.01f, norms, nullptr, fake(0x400), nullptr) == FERRET_OK);
    for (int32_t fused = 0; fused < 2 && n_iters != 0; ++fused) {
        ferret_adaptive ad = {static_cast<float *>(fake(0x500)), static_cast<float *>(fake(0x600)),
                              static_cast<float *>(fake(0x700)), 0.9f, 1e-3f, fused, 0};
        CHECK(ferret_compensate_step_adaptive(plan, fake(0), fake(0x100), master, &ad, 0.01f, norms, nullptr, fake(0x400), nullptr) == FERRET_OK);
        CHECK(ferret_compensate_stages_adaptive(plan, fake(0), fake(0x100), master, active.data(), &ad, 0.01f, nullptr, nullptr, fake(0x400), nullptr) == FERRET_OK);
        ferret_accumulate acc = {static_cast<float *>(fake(0x800)), 0.5f, mode.data(), stale.data()};
        CHECK(ferret_accumulate_step_adaptive(plan, fake(0), fake(0x100), master, &acc, &ad, 0.01f, norms, nullptr, fake(0x400), nullptr) == FERRET_OK);
    }
    ferret_accumulate acc = {static_cast<float *>(fake(0x800)), 0.5f, mode.data(), stale.data()};
    CHECK(ferret_accumulate_step(plan, fake(0), fake(0x100), master, &acc, 0.5f, 0.01f, norms, nullptr, fake(0x400), nullptr) == FERRET_OK);
    acc.staleness = nullptr;
    CHECK(ferret_accumulate_step(plan, fake(0), fake(0x100), master, &acc, 0.5f, 0.01f, nullptr, nullptr, nullptr, nullptr) == FERRET_OK);
    CHECK(ferret_penalized_step(plan, fake(0), fake(0x100), master, nullptr, nullptr, 0.01f, norms, nullptr, fake(0x400), nullptr) == FERRET_OK);
    std::vector<float> scale(n_stages, 1.0f), inv_c(n_stages, 2.0f);
    CHECK(ferret_penalized_step(plan, fake(0), fake(0x100), master, scale.data(), inv_c.data(), 0.01f, nullptr, nullptr, nullptr, nullptr) == FERRET_OK);
    inv_c[0] = -1.0f;
    CHECK(ferret_penalized_step(plan, fake(0), fake(0x100), master, scale.data(), inv_c.data(), 0.01f, nullptr, nullptr, nullptr, nullptr) == FERRET_EINVAL);
    CHECK(ferret_push_version(plan, fake(0), nullptr, n_stages - 1, fake(0x900), nullptr) == FERRET_OK);
    CHECK(ferret_push_version(plan, fake(0), nullptr, n_stages, fake(0x900), nullptr) == FERRET_EINVAL);
    // a stage without a version may sit a call out, but not take part
    valid[0] = 0;
    CHECK(ferret_plan_set_state(plan, zeros.data(), valid.data()) == FERRET_OK);
    CHECK(ferret_compensate_step(plan, fake(0), fake(0x100), master, 0.5f, 0.01f, nullptr, nullptr, nullptr, nullptr) == FERRET_ESTATE);
    if (n_stages > 1) {
        std::vector<int32_t> rest(n_stages, 1);
        rest[0] = 0;
        CHECK(ferret_compensate_stages(plan, fake(0), fake(0x100), master, rest.data(), 0.5f, 0.01f, nullptr, nullptr, nullptr, nullptr) == FERRET_OK);
        rest[0] = 1;
        CHECK(ferret_compensate_stages(plan, fake(0), fake(0x100), master, rest.data(), 0.5f, 0.01f, nullptr, nullptr, nullptr, nullptr) == FERRET_ESTATE);
    }
    CHECK(ferret_stream_mix(fake(0x100000), fake(0), 4096, 3, 4096, 2, nullptr) == FERRET_OK);
    CHECK(ferret_copy_bytes(fake(0x100000), fake(0), 4096, nullptr) == FERRET_OK);
    CHECK(ferret_read_bytes(fake(0), 4096, fake(0x100000), nullptr) == FERRET_OK);
    ferret_plan_destroy(plan);
}

static void bad_plans() {
    const ferret_tensor t[2] = {{100, 0, 0}, {100, 1, 0}};
    const int32_t tau[3] = {1, 0, 0};
    ferret_plan *plan = nullptr;
    CHECK(ferret_plan_buckets(nullptr, 2, 2, tau, 1, 2, FERRET_F32, 0, &plan) == FERRET_EINVAL);
    CHECK(ferret_plan_buckets(t, 2, 3, tau, 1, 2, FERRET_F32, 0, &plan) == FERRET_EINVAL);          // a stage without tensors
    CHECK(ferret_plan_buckets(t, 2, 2, tau, 1, 1, FERRET_F32, 0, &plan) == FERRET_EINVAL);          // staleness needs depth 2
    CHECK(ferret_plan_buckets(t, 2, 2, tau, -2, 2, FERRET_F32, 0, &plan) == FERRET_EINVAL);
    CHECK(ferret_plan_buckets(t, 2, 2, tau, 1, 2, FERRET_F32, 1000, &plan) == FERRET_EINVAL);       // chunk not a multiple of 1024
    CHECK(ferret_plan_buckets(t, 2, FERRET_MAX_STAGES + 1, tau, 1, 2, FERRET_F32, 0, &plan) == FERRET_EINVAL);
    CHECK(plan == nullptr);
    int32_t n = 0;
    float ms[4];
    CHECK(ferret_profile_begin(0) == FERRET_EINVAL);
    CHECK(ferret_profile_begin(4) == FERRET_OK && ferret_profile_end(ms, 4, &n) == FERRET_OK && n == 0);
}

static void planner(unsigned seed, int n_layers, bool threaded) {
    std::srand(seed);
    std::vector<ferret_layer> layers(n_layers);
    double mem = 0;
    for (auto &l : layers) {
        l.t_f = 0.5 + (std::rand() % 100) / 50.0;
        l.t_b = 2.0 * l.t_f;
        l.n_params = 100.0 + std::rand() % 5000;
        l.n_acts = 10.0 + std::rand() % 500;
        mem += l.n_params;
    }
    if (threaded) setenv("FERRET_PLANNER_THREADS", "8", 1);
    for (double budget : {mem * 100.0, mem * 4.0, mem * 1.5}) {
        ferret_pipeline *p = nullptr;
        CHECK(ferret_pipeline_plan(layers.data(), n_layers, 1.0, budget, 0.01, 1.0, &p) == FERRET_OK);
        if (!p) continue;
        const int32_t P = ferret_pipeline_n_stages(p), N = ferret_pipeline_n_workers(p);
        CHECK(P >= 1 && ferret_pipeline_stage_begin(p, P) == n_layers);
        for (int32_t n = 0; n < N; ++n)
            for (int32_t j = 0; j < P; ++j)
                CHECK(ferret_pipeline_worker_accum(p, n, j) >= 1 && ferret_pipeline_stage_versions(p, n, j) >= 0);
        for (int32_t k = 0; k < ferret_pipeline_n_moves(p); ++k) {
            int32_t wkr, kind, stage;
            CHECK(ferret_pipeline_move(p, k, &wkr, &kind, &stage) == FERRET_OK && kind >= 2 && kind <= 4);
        }
        if (ferret_pipeline_feasible(p)) CHECK(ferret_pipeline_memory(p) <= budget * (1 + 1e-12));
        // the search alone on the partition the plan chose reproduces the plan
        std::vector<int32_t> L(P + 1);
        for (int32_t j = 0; j <= P; ++j) L[j] = ferret_pipeline_stage_begin(p, j);
        ferret_pipeline *q = nullptr;
        CHECK(ferret_pipeline_search(layers.data(), n_layers, L.data(), P, 1.0, budget, 0.01, 1.0, &q) == FERRET_OK);
        if (q) CHECK(ferret_pipeline_rate(q) == ferret_pipeline_rate(p));
        ferret_pipeline_destroy(q);
        ferret_pipeline_destroy(p);
    }
}

int main(int argc, char **argv) {
    const bool planner_only = argc > 1 && std::strcmp(argv[1], "planner") == 0;
    if (!planner_only) {
        ferret_tuning tuned;
        std::memset(&tuned, 0, sizeof tuned);
        tuned.chunk_bytes = 20000;
        tuned.resident_cap = 3;
        tuned.cache_policy = 2;
        tuned.xcd_group = 5;
        tuned.slot_align_elems = 1024;
        tuned.slot_skew_elems = 40;
        for (ferret_precision prec : {FERRET_F32, FERRET_BF16_MASTER_F32})
            for (int32_t n_stages : {1, 5, FERRET_MAX_STAGES})
                for (int32_t n_iters : {FERRET_ITERS_FULL, 0, 2}) {
                    steps_and_pushes(prec, n_stages, n_iters, nullptr);
                    steps_and_pushes(prec, n_stages, n_iters, &tuned);
                }
        bad_plans();
        planner(1, 6, false);
        planner(2, 9, false);
        // two threads, each with its own plan and its own last-error buffer
        std::thread a(steps_and_pushes, FERRET_F32, 7, 2, nullptr), b(steps_and_pushes, FERRET_BF16_MASTER_F32, 9, -1, nullptr);
        a.join();
        b.join();
    } else {
        planner(3, 10, true);
        planner(4, 12, true);
    }
    std::printf("failures %d\n", failures);
    return failures ? 1 : 0;
}
