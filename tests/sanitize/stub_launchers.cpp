// Host-only stand-ins for the launchers of ferret_kernels.hip, so that the host half of the library (planning, ring
// bookkeeping, argument checks, descriptor filling, the pipeline planner) links into an ordinary executable that
// can run under AddressSanitizer, UndefinedBehaviorSanitizer or ThreadSanitizer on a machine without a GPU.
// Each stub checks what the host code hands to a launch the way the kernels rely on it.
#include <cstdio>
#include <cstdlib>

#include "ferret_internal.h"

namespace ferret {

static void require(bool ok, const char *what) {
    if (!ok) { std::fprintf(stderr, "stub launcher: %s\n", what); std::abort(); }
}

static void check_stages(const StageDesc *stage, uint32_t n_stages, uint32_t n_chunks) {
    uint32_t chunks = 0;
    for (uint32_t j = 0; j < n_stages; ++j) {
        const StageDesc &d = stage[j];
        require(d.chunk_begin == chunks, "chunk_begin is not the running count of chunks");
        require(d.chunk_elems > 0 && d.chunk_elems % 1024 == 0, "chunk size is not a multiple of one vector per lane");
        require(d.n_elems % FERRET_ALIGN_ELEMS == 0, "stage size is not padded");
        require(d.ring_depth >= 1 && d.head < d.ring_depth && d.tau < d.ring_depth && d.kp <= d.tau, "ring state out of range");
        require(d.slot_stride >= d.n_elems, "slots overlap");
        chunks += (uint32_t)((d.n_elems + d.chunk_elems - 1) / d.chunk_elems);
    }
    require(chunks == n_chunks, "n_chunks does not match the stages");
}

int launch_step(const ferret_plan &plan, const StepArgs &a, void *) {
    require(a.n_stages == plan.stages.size() && a.ring && a.grads, "step arguments incomplete");
    check_stages(a.stage, a.n_stages, a.n_chunks);
    require(a.chunk_base <= a.chunk_end && a.chunk_end <= a.n_chunks, "chunk span out of range");
    require(!a.norms_out || a.partials, "norms without partial sums");
    require(!a.fused_lambda || (a.partials && a.lambda_dev && a.v_r && a.v_a), "fused lambda block without its state");
    for (uint32_t j = 0; j < FERRET_MAX_STAGES; ++j)
        require(a.chunk_begin[j] == (j < a.n_stages ? a.stage[j].chunk_begin : UINT32_MAX), "dense chunk_begin table wrong");
    return 0;
}
int launch_lambda_update(const ferret_plan &, const StepArgs &a, void *) {
    require(a.partials && a.lambda_dev && a.v_r && a.v_a, "lambda update without its state");
    check_stages(a.stage, a.n_stages, a.n_chunks);
    return 0;
}
int launch_push(const ferret_plan &, const PushArgs &a, void *) {
    require(a.ring && a.src && a.n_stages >= 1, "push arguments incomplete");
    check_stages(a.stage, a.n_stages, a.n_chunks);
    return 0;
}
int launch_copy(void *, const void *, size_t, void *) { return 0; }
int launch_read(const void *, size_t, void *, void *) { return 0; }
int launch_mix(void *, const void *, size_t, int, size_t, int, void *) { return 0; }
const char *device_error_string(int) { return "stub"; }
int noalloc_scratch(void **ptr_out) { *ptr_out = reinterpret_cast<void *>(uintptr_t(0x7000000)); return 0; }
int profile_begin(int32_t) { return 0; }
int profile_end(float *, int32_t, int32_t *n) { *n = 0; return 0; }

}  // namespace ferret
