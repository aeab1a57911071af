// Internal declarations shared by the host planner (ferret_host.cpp) and the kernel
// launchers (ferret_kernels.hip).  Not installed; the public interface is include/ferret.h.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "ferret.h"

// Elements of bf16 storage one lane handles per vector (4 or 8); fp32 storage always 4.
// Measured on MI355X: 4 (8-byte loads, every wavefront access one contiguous run, master as one
// float4 per lane) beats 8 (16-byte loads but the master split in two half-line accesses) by ~4 %.
#ifndef FERRET_BF16_LANE_ELEMS
#define FERRET_BF16_LANE_ELEMS 4
#endif

namespace ferret {

// Bytes of the library-owned scratch array behind ferret_compensate_step_noalloc: five per-chunk series.
#define FERRET_NOALLOC_SCRATCH_BYTES ((size_t)FERRET_NOALLOC_MAX_CHUNKS * 5u * sizeof(float))

// ---- what travels to the device as a kernel argument -------------------------------------
// One entry per pipeline stage.  48 bytes; FERRET_MAX_STAGES of them stay under the 4 KiB
// kernel-argument limit.  The default step kernel (one workgroup per chunk) reads its stage's entry
// straight from the kernel-argument segment with scalar loads -- measured 5-8 % faster on MI355X than
// staging the table in LDS; only the persistent grid-stride variant (ferret_tuning.blocks_per_cu > 0)
// and the push kernel copy the live entries into LDS once per workgroup and look chunks up there.
struct StageDesc {
    uint64_t ring_base;    // element offset of the stage's arena in the ring
    uint64_t slot_stride;  // elements between consecutive slots
    uint64_t flat_off;     // element offset of the stage in slot-shaped buffers
    uint64_t n_elems;      // padded elements in the stage (multiple of FERRET_ALIGN_ELEMS)
    uint32_t chunk_begin;  // id of the stage's first chunk
    uint16_t ring_depth;   // R_j
    uint16_t head;         // slot of the newest version, V[tau]
    uint16_t tau;          // effective staleness this step
    uint16_t kp;           // K' this step (0 = no compensation)
    uint32_t chunk_elems;  // elements per chunk of this stage (the last chunk may be shorter)
};
static_assert(sizeof(StageDesc) == 48, "StageDesc layout");

struct StepArgs {
    void *ring;
    const void *grads;
    float *master;
    float *grad_out;   // nullable
    float *partials;   // float[5][n_chunks] (five series, each contiguous: 3 norms, 2 lambda inner products), nullable
    float *norms_out;  // float[n_stages][3], nullable
    float lambda;
    float lr;
    uint32_t n_stages;
    uint32_t n_chunks;
    uint32_t xcd_group;      // > 1: consecutive chunks each XCD works on (set by the launcher)
    uint32_t fused_lambda;   // 1: the step kernel also runs the "update lambda" block (series 3, 4 of partials)
    // self-tuned lambda (null / zero for the fixed-lambda step)
    float *lambda_dev;   // float[n_stages]; when set, stage j uses lambda_dev[j] instead of `lambda`
    float *v_r;
    float *v_a;
    float alpha;
    float eta_lambda;
    // gradient accumulation (null for the plain step)
    float *accum;        // fp32 flat buffer: running sum of compensated gradients
    float accum_scale;   // factor on the sum at the update
    uint32_t penalized;  // 1: step-size-penalising comparison method (pen_scale / pen_inv_c per stage)
    uint32_t masked;     // 1: mode[] selects the stages of a plain step (0 skip, 2 step)
    uint32_t chunk_base; // the launch covers chunks [chunk_base, chunk_end): all of them, or the span of the
    uint32_t chunk_end;  // stages that take part when some are left out
    uint32_t pad_;
    uint8_t mode[FERRET_MAX_STAGES];   // per stage: 0 skip, 1 accumulate only, 2 accumulate + update
    // chunk_begin of every stage again, densely packed (unused entries = UINT32_MAX), so that a
    // workgroup can find its chunk's stage with a few wide scalar loads
    uint32_t chunk_begin[FERRET_MAX_STAGES];
    float pen_scale[FERRET_MAX_STAGES];
    float pen_inv_c[FERRET_MAX_STAGES];
    StageDesc stage[FERRET_MAX_STAGES];
};
static_assert(sizeof(StepArgs) <= 4096, "StepArgs must fit the 4 KiB kernel-argument segment");

struct PushArgs {
    void *ring;
    float *master;     // nullable
    const float *src;
    uint32_t n_stages; // entries used in stage[]
    uint32_t n_chunks;
    StageDesc stage[FERRET_MAX_STAGES];   // head = slot to WRITE; chunk_begin re-based to the pushed set
};

// ---- host-side plan ------------------------------------------------------------------------
struct Stage {
    int64_t params = 0;       // |w_j|
    int64_t n_elems = 0;      // padded
    int64_t flat_off = 0;
    int64_t ring_base = 0;
    int64_t slot_stride = 0;
    int64_t chunk_begin = 0;
    int64_t n_chunks = 0;
    int64_t chunk_elems = 0;  // elements per chunk of this stage
    int32_t ring_depth = 0;
    int32_t tau = 0;          // configured staleness
    int32_t head = 0;
    int32_t valid = 0;
    mutable bool step_pending = false;  // a step wrote slot head+1 and it has not been committed
                                        // (bookkeeping that a step on a const plan may set)
};

}  // namespace ferret

struct ferret_plan {
    std::vector<ferret::Stage> stages;
    std::vector<int64_t> tensor_offset;   // inside the stage
    std::vector<int32_t> tensor_stage;
    ferret_precision prec = FERRET_F32;
    int32_t n_iters = 0;
    int64_t chunk_elems = 0;  // the caller's request: > 0 every stage uses it, 0 the plan chose per stage
    int64_t chunk_bytes = 0;  // bytes one chunk should have in flight (resolved: never 0 when chunk_elems is 0)
    int64_t n_chunks = 0;
    int64_t flat_elems = 0;
    int64_t ring_elems = 0;
    int64_t total_params = 0;
    int32_t blocks_per_cu = 0;
    int32_t resident_cap = 0;
    int32_t newest_from_master = 0;   // bf16: recompute V[tau] from the master instead of reading it
    int32_t cache_policy = 0;         // 0: by working-set size, 1: cached accesses where available, 2: non-temporal
    int32_t xcd_group = 0;            // 0: by storage type and K', 1: none, > 1: that many consecutive chunks per XCD
};

namespace ferret {

void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));

// effective staleness / iteration count / segment boundary for the plan's current state
inline int32_t effective_tau(const Stage &s) {
    int32_t have = s.valid - 1;
    return have < s.tau ? (have < 0 ? 0 : have) : s.tau;
}
inline int32_t effective_iters(int32_t n_iters, int32_t tau) {
    return n_iters < 0 ? tau : (n_iters < tau ? n_iters : tau);
}

// K' up to which the step kernel loads all K'+1 boundary versions of a vector together (its unrolled paths);
// beyond, it streams them in batches of kStreamBatch.
constexpr int32_t kUnrolledItersMax = 8;
constexpr int32_t kStreamBatch = 8;
// Bytes per element that one lane-vector of the plain step has in flight: gradient, the versions loaded
// together, the new version, and the master read and written.  Chunk sizes and the resident-workgroup cap are
// both derived from it.
inline int64_t inflight_bytes_per_elem(ferret_precision prec, int32_t kp) {
    const int64_t sb = prec == FERRET_F32 ? 4 : 2;
    const int64_t versions = kp <= kUnrolledItersMax ? kp + 1 : kStreamBatch;
    return sb * (versions + 2) + (prec == FERRET_F32 ? 0 : 8);
}

// Working sets (ring + gradient + master) up to this size stay in the 256 MB memory-side cache from one step to
// the next: every step touches the gradient and K'+2 of the R slots, and R steps touch everything.  Such plans
// are latency-bound rather than bandwidth-bound: they run the plain step with ordinary cached accesses (measured
// 5-7 % faster there than non-temporal ones) and keep one small chunk size for every stage (more workgroups).
constexpr uint64_t kCacheResidentBytes = 240ull << 20;
inline uint64_t working_set_bytes(ferret_precision prec, int64_t ring_elems, int64_t flat_elems) {
    const uint64_t sb = prec == FERRET_F32 ? 4 : 2;
    return (uint64_t)ring_elems * sb + (uint64_t)flat_elems * (sb + (prec == FERRET_F32 ? 0u : 4u));
}

// launchers implemented in ferret_kernels.hip; return hipError_t as int (0 = success)
int launch_step(const ferret_plan &plan, const StepArgs &args, void *stream);
int launch_lambda_update(const ferret_plan &plan, const StepArgs &args, void *stream);
int launch_push(const ferret_plan &plan, const PushArgs &args, void *stream);
int launch_copy(void *dst, const void *src, size_t n_bytes, void *stream);
int launch_read(const void *src, size_t n_bytes, void *sink, void *stream);
int launch_mix(void *dst, const void *src, size_t src_stride_bytes, int n_reads, size_t n_bytes, int resident_cap,
               void *stream);
const char *device_error_string(int err);
int noalloc_scratch(void **ptr_out);                        // device address of the library's own scratch on the current device
int profile_begin(int32_t capacity);                       // 0 ok, -1 bad state, >0 hipError_t
int profile_end(float *ms_out, int32_t cap, int32_t *n_out);

}  // namespace ferret
