/*
 * A plain C99 consumer of include/ferret.h and include/ferret_planner.h: compiled with gcc -std=c99 -pedantic
 * -Wall -Werror by tests/test_c_consumer.py and linked against libferret.so.  It makes host-only calls (no
 * device work: planning, queries, ring state, argument errors, the pipeline planner on a tiny layer table)
 * and prints
 *     layout <struct> sizeof <n>
 *     layout <struct>.<field> offset <n> size <n>
 *     value <name> <n>
 * lines, which the test compares with the ctypes mirrors of the Python binding and with the values the
 * binding reports for the same calls.  Exit status 0 = every check in here held.
 */
#include <stddef.h>
#include <stdio.h>
#include <string.h>

#include "ferret.h"
#include "ferret_planner.h"

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)
#define FIELD(type, field) printf("layout %s.%s offset %lu size %lu\n", #type, #field, \
                                  (unsigned long)offsetof(type, field), (unsigned long)sizeof(((type *)0)->field))
#define SIZE(type) printf("layout %s sizeof %lu\n", #type, (unsigned long)sizeof(type))

int main(void) {
    /* ---- struct layouts ---- */
    SIZE(ferret_tensor);
    FIELD(ferret_tensor, numel); FIELD(ferret_tensor, stage); FIELD(ferret_tensor, reserved);
    SIZE(ferret_tuning);
    FIELD(ferret_tuning, slot_align_elems); FIELD(ferret_tuning, slot_skew_elems); FIELD(ferret_tuning, chunk_bytes);
    FIELD(ferret_tuning, blocks_per_cu); FIELD(ferret_tuning, resident_cap); FIELD(ferret_tuning, newest_from_master);
    FIELD(ferret_tuning, cache_policy); FIELD(ferret_tuning, xcd_group); FIELD(ferret_tuning, reserved);
    SIZE(ferret_adaptive);
    FIELD(ferret_adaptive, lambda); FIELD(ferret_adaptive, v_r); FIELD(ferret_adaptive, v_a);
    FIELD(ferret_adaptive, alpha); FIELD(ferret_adaptive, eta_lambda); FIELD(ferret_adaptive, fused);
    FIELD(ferret_adaptive, reserved);
    SIZE(ferret_accumulate);
    FIELD(ferret_accumulate, accum); FIELD(ferret_accumulate, scale); FIELD(ferret_accumulate, mode);
    FIELD(ferret_accumulate, staleness);
    SIZE(ferret_layer);
    FIELD(ferret_layer, t_f); FIELD(ferret_layer, t_b); FIELD(ferret_layer, n_params); FIELD(ferret_layer, n_acts);
    printf("value FERRET_OK %d\nvalue FERRET_EINVAL %d\nvalue FERRET_ESTATE %d\nvalue FERRET_ENOMEM %d\nvalue FERRET_EDEVICE %d\n",
           (int)FERRET_OK, (int)FERRET_EINVAL, (int)FERRET_ESTATE, (int)FERRET_ENOMEM, (int)FERRET_EDEVICE);
    printf("value FERRET_F32 %d\nvalue FERRET_BF16_MASTER_F32 %d\n", (int)FERRET_F32, (int)FERRET_BF16_MASTER_F32);
    printf("value FERRET_MAX_STAGES %d\nvalue FERRET_ALIGN_ELEMS %d\nvalue FERRET_ITERS_FULL %d\n", FERRET_MAX_STAGES,
           FERRET_ALIGN_ELEMS, FERRET_ITERS_FULL);
    printf("value FERRET_RING_DEPTH_MINIMAL %d\nvalue FERRET_NOALLOC_MAX_CHUNKS %d\n", FERRET_RING_DEPTH_MINIMAL,
           FERRET_NOALLOC_MAX_CHUNKS);

    /* ---- a plan: three stages, five tensors, staleness 2,1,0, K = 2, ring depth 3, fp32 ---- */
    const ferret_tensor tensors[5] = {{5000, 0, 0}, {33, 0, 0}, {2048, 1, 0}, {7, 2, 0}, {4096, 2, 0}};
    const int32_t staleness[3] = {2, 1, 0};
    ferret_plan *plan = NULL;
    CHECK(ferret_plan_buckets(tensors, 5, 3, staleness, 2, 3, FERRET_F32, 0, &plan) == FERRET_OK);
    CHECK(plan != NULL);
    CHECK(ferret_plan_n_stages(plan) == 3 && ferret_plan_n_tensors(plan) == 5);
    CHECK(ferret_plan_precision(plan) == (int32_t)FERRET_F32 && ferret_plan_n_iters(plan) == 2);
    CHECK(ferret_plan_total_params(plan) == 5000 + 33 + 2048 + 7 + 4096);
    CHECK(ferret_plan_stage_params(plan, 0) == 5033 && ferret_plan_stage_numel(plan, 0) == 5040);  /* padded to 8 */
    CHECK(ferret_plan_tensor_offset(plan, 1) == 5000 && ferret_plan_tensor_offset(plan, 4) == 8);
    CHECK(ferret_plan_stage_staleness(plan, 1) == 1 && ferret_plan_stage_ring_depth(plan, 2) == 3);
    CHECK(ferret_plan_ring_bytes(plan) == (size_t)ferret_plan_ring_elems(plan) * 4);
    CHECK(ferret_plan_grad_bytes(plan) == (size_t)ferret_plan_flat_elems(plan) * 4);
    CHECK(ferret_plan_workspace_bytes(plan) >= (size_t)ferret_plan_n_chunks(plan) * 20);
    printf("value n_chunks %ld\nvalue flat_elems %ld\nvalue ring_elems %ld\nvalue workspace_bytes %lu\n",
           (long)ferret_plan_n_chunks(plan), (long)ferret_plan_flat_elems(plan), (long)ferret_plan_ring_elems(plan),
           (unsigned long)ferret_plan_workspace_bytes(plan));
    for (int32_t j = 0; j < 3; ++j)
        printf("value stage%d_flat_offset %ld\nvalue stage%d_ring_offset %ld\nvalue stage%d_slot_stride %ld\n"
               "value stage%d_chunk_elems %ld\nvalue stage%d_n_chunks %ld\n",
               j, (long)ferret_plan_stage_flat_offset(plan, j), j, (long)ferret_plan_stage_ring_offset(plan, j), j,
               (long)ferret_plan_stage_slot_stride(plan, j), j, (long)ferret_plan_stage_chunk_elems(plan, j), j,
               (long)ferret_plan_stage_n_chunks(plan, j));

    /* ring state: nothing held yet; a step is refused, so is a commit; then adopt a full ring */
    int32_t heads[3], valid[3];
    CHECK(ferret_plan_get_state(plan, heads, valid) == FERRET_OK);
    CHECK(heads[0] == 0 && valid[0] == 0 && valid[2] == 0);
    char fake[64];                       /* never dereferenced: every call below fails before any device work */
    void *aligned = (void *)(((size_t)fake + 15u) & ~(size_t)15u);
    CHECK(ferret_compensate_step(plan, aligned, aligned, NULL, 0.5f, 0.01f, NULL, NULL, NULL, NULL) == FERRET_ESTATE);
    CHECK(strstr(ferret_last_error(), "no weight version") != NULL);
    CHECK(ferret_push_version(plan, aligned, NULL, -1, NULL, NULL) == FERRET_ESTATE);
    const int32_t new_heads[3] = {2, 0, 1}, new_valid[3] = {3, 2, 1};
    CHECK(ferret_plan_set_state(plan, new_heads, new_valid) == FERRET_OK);
    CHECK(ferret_plan_stage_effective_staleness(plan, 0) == 2 && ferret_plan_stage_effective_staleness(plan, 1) == 1);
    CHECK(ferret_plan_stage_effective_iters(plan, 0) == 2 && ferret_plan_stage_effective_iters(plan, 2) == 0);
    int32_t slots[4] = {-1, -1, -1, -1};
    CHECK(ferret_plan_stage_read_slots(plan, 0, slots, 4) == 3);       /* V[0], V[1], V[2] = slots 0, 1, 2 */
    CHECK(slots[0] == 0 && slots[1] == 1 && slots[2] == 2 && ferret_plan_stage_write_slot(plan, 0) == 0);
    CHECK(ferret_plan_step_bytes(plan) == 4 * ((2 + 3) * 5033 + (1 + 3) * 2048 + (0 + 3) * 4103));
    const int32_t bad_heads[3] = {3, 0, 0};
    CHECK(ferret_plan_set_state(plan, bad_heads, new_valid) == FERRET_EINVAL);
    /* argument errors of the step: null, misaligned, master on an fp32 plan, norms without workspace */
    CHECK(ferret_compensate_step(NULL, aligned, aligned, NULL, 0.5f, 0.01f, NULL, NULL, NULL, NULL) == FERRET_EINVAL);
    CHECK(ferret_compensate_step(plan, (char *)aligned + 4, aligned, NULL, 0.5f, 0.01f, NULL, NULL, NULL, NULL) == FERRET_EINVAL);
    CHECK(ferret_compensate_step(plan, aligned, aligned, (float *)aligned, 0.5f, 0.01f, NULL, NULL, NULL, NULL) == FERRET_EINVAL);
    CHECK(ferret_compensate_step(plan, aligned, aligned, NULL, 0.5f, 0.01f, (float *)aligned, NULL, NULL, NULL) == FERRET_EINVAL);
    CHECK(ferret_compensate_step_noalloc(NULL, aligned, aligned, NULL, 0.5f, 0.01f, NULL, NULL, NULL) == FERRET_EINVAL);
    CHECK(ferret_plan_stage_numel(plan, 3) == -1 && ferret_plan_n_stages(NULL) == -1);
    ferret_plan_destroy(plan);
    ferret_plan_destroy(NULL);

    /* a tuned bf16 plan, and a refused one */
    ferret_tuning tuning;
    memset(&tuning, 0, sizeof tuning);
    tuning.chunk_bytes = 32 * 1024;
    tuning.resident_cap = 3;
    tuning.newest_from_master = 1;
    plan = NULL;
    CHECK(ferret_plan_buckets_tuned(tensors, 5, 3, staleness, FERRET_ITERS_FULL, FERRET_RING_DEPTH_MINIMAL,
                                    FERRET_BF16_MASTER_F32, 0, &tuning, &plan) == FERRET_OK);
    CHECK(ferret_plan_stage_ring_depth(plan, 0) == 3 && ferret_plan_stage_ring_depth(plan, 2) == 1);
    CHECK(ferret_plan_master_bytes(plan) == (size_t)ferret_plan_flat_elems(plan) * 4);
    CHECK(ferret_plan_ring_bytes(plan) == (size_t)ferret_plan_ring_elems(plan) * 2);
    printf("value tuned_stage0_chunk_elems %ld\n", (long)ferret_plan_stage_chunk_elems(plan, 0));
    ferret_plan_destroy(plan);
    tuning.resident_cap = 1;
    plan = NULL;
    CHECK(ferret_plan_buckets_tuned(tensors, 5, 3, staleness, 2, 3, FERRET_BF16_MASTER_F32, 0, &tuning, &plan) == FERRET_EINVAL);
    CHECK(plan == NULL && strlen(ferret_last_error()) > 0);
    CHECK(strstr(ferret_version(), "gfx950") != NULL);

    /* ---- the pipeline planner on a tiny layer table (host only) ---- */
    const ferret_layer layers[4] = {{1.0, 2.0, 1000.0, 500.0}, {1.5, 2.5, 4000.0, 300.0},
                                    {0.5, 1.0, 2000.0, 200.0}, {1.0, 1.5, 500.0, 10.0}};
    ferret_pipeline *pipe = NULL;
    CHECK(ferret_pipeline_plan(layers, 4, 1.5, 1e9, 0.01, 1.0, &pipe) == FERRET_OK);
    CHECK(pipe != NULL && ferret_pipeline_feasible(pipe) == 1);
    const int32_t P = ferret_pipeline_n_stages(pipe);
    CHECK(P >= 1 && P <= 4 && ferret_pipeline_stage_begin(pipe, 0) == 0 && ferret_pipeline_stage_begin(pipe, P) == 4);
    CHECK(ferret_pipeline_rate(pipe) > 0.0 && ferret_pipeline_memory(pipe) > 0.0 && ferret_pipeline_memory(pipe) <= 1e9);
    printf("value pipeline_n_stages %d\nvalue pipeline_n_workers %d\nvalue pipeline_n_moves %d\n", (int)P,
           (int)ferret_pipeline_n_workers(pipe), (int)ferret_pipeline_n_moves(pipe));
    printf("value pipeline_rate_micro %ld\n", (long)(ferret_pipeline_rate(pipe) * 1e6 + 0.5));
    ferret_pipeline_destroy(pipe);
    pipe = NULL;
    CHECK(ferret_pipeline_plan(NULL, 4, 1.5, 1e9, 0.01, 1.0, &pipe) == FERRET_EINVAL);
    ferret_pipeline_destroy(NULL);

    printf("failures %d\n", failures);
    return failures ? 1 : 0;
}
