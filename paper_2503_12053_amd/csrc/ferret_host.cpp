// Host side of libferret: the bucket planner, the ring bookkeeping and argument checks of
// the C ABI declared in include/ferret.h.  No HIP call is made in this file; device work
// goes through the launchers in ferret_kernels.hip.
//
// Paper passages behind the pieces:
//   stage = contiguous run of layers, |w_j| parameters        appendix "Notations"
//   tau_j <= P-1, stage j keeps P-j versions                  Sec. "Iterative Gradient Compensation"
//                                                             (Algorithm Design), T2
//   what a step computes                                      Alg. 1, lines "iterative approximation"
//                                                             and "model update"
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "ferret_internal.h"

namespace ferret {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

static inline int64_t vec_elems(ferret_precision p) { return p == FERRET_F32 ? 4 : FERRET_BF16_LANE_ELEMS; }
static inline int64_t storage_bytes(ferret_precision p) { return p == FERRET_F32 ? 4 : 2; }

#ifndef FERRET_THREADS
#define FERRET_THREADS 256
#endif
constexpr int64_t kThreads = FERRET_THREADS;   // workgroup size of every kernel
constexpr int64_t kStageAlign = 64;        // stage start alignment in flat buffers / ring
constexpr int64_t kDefaultSlotAlign = 64;

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Fill the per-stage device descriptors for the state the plan is in right now.
static void fill_step_descs(const ferret_plan &p, StageDesc *out) {
    for (size_t j = 0; j < p.stages.size(); ++j) {
        const Stage &s = p.stages[j];
        StageDesc &d = out[j];
        d.ring_base = (uint64_t)s.ring_base;
        d.slot_stride = (uint64_t)s.slot_stride;
        d.flat_off = (uint64_t)s.flat_off;
        d.n_elems = (uint64_t)s.n_elems;
        d.chunk_begin = (uint32_t)s.chunk_begin;
        d.chunk_elems = (uint32_t)s.chunk_elems;
        d.ring_depth = (uint16_t)s.ring_depth;
        d.head = (uint16_t)s.head;
        int32_t tau = effective_tau(s);
        d.tau = (uint16_t)tau;
        d.kp = (uint16_t)effective_iters(p.n_iters, tau);
    }
}

}  // namespace ferret

using namespace ferret;

extern "C" {

const char *ferret_last_error(void) { return g_err; }
#ifndef FERRET_SOURCE_HASH
#define FERRET_SOURCE_HASH "unknown"
#endif
const char *ferret_version(void) { return "libferret 0.2 (gfx950) src " FERRET_SOURCE_HASH; }

ferret_status ferret_plan_buckets(const ferret_tensor *tensors, int32_t n_tensors, int32_t n_stages,
                                  const int32_t *staleness, int32_t n_iters, int32_t ring_depth,
                                  ferret_precision prec, int64_t chunk_elems, ferret_plan **out_plan) {
    return ferret_plan_buckets_tuned(tensors, n_tensors, n_stages, staleness, n_iters, ring_depth,
                                     prec, chunk_elems, nullptr, out_plan);
}

ferret_status ferret_plan_buckets_tuned(const ferret_tensor *tensors, int32_t n_tensors,
                                        int32_t n_stages, const int32_t *staleness, int32_t n_iters,
                                        int32_t ring_depth, ferret_precision prec, int64_t chunk_elems,
                                        const ferret_tuning *tuning, ferret_plan **out_plan) {
    if (out_plan) *out_plan = nullptr;
    if (!tensors || !staleness || !out_plan) { set_error("plan: null argument"); return FERRET_EINVAL; }
    if (n_tensors < 1) { set_error("plan: n_tensors = %d, need >= 1", n_tensors); return FERRET_EINVAL; }
    if (n_stages < 1 || n_stages > FERRET_MAX_STAGES) {
        set_error("plan: n_stages = %d, need 1..%d", n_stages, FERRET_MAX_STAGES); return FERRET_EINVAL;
    }
    if (n_iters < 0 && n_iters != FERRET_ITERS_FULL) {
        set_error("plan: n_iters = %d, need >= 0 or FERRET_ITERS_FULL", n_iters); return FERRET_EINVAL;
    }
    if (ring_depth < 0 || ring_depth > FERRET_MAX_RING_DEPTH) {
        set_error("plan: ring_depth = %d, need 0..%d", ring_depth, FERRET_MAX_RING_DEPTH); return FERRET_EINVAL;
    }
    if (prec != FERRET_F32 && prec != FERRET_BF16_MASTER_F32) {
        set_error("plan: unknown precision %d", (int)prec); return FERRET_EINVAL;
    }
    const int64_t vec = vec_elems(prec);
    const int64_t chunk_unit = kThreads * vec;                 // one vector per thread
    constexpr int64_t kMaxChunkElems = int64_t(1) << 24;      // lanes address a chunk with 32-bit byte offsets
    if (chunk_elems < 0 || chunk_elems % chunk_unit != 0 || chunk_elems > kMaxChunkElems) {
        set_error("plan: chunk_elems = %lld, need 0 or a positive multiple of %lld up to 2^24", (long long)chunk_elems,
                  (long long)chunk_unit);
        return FERRET_EINVAL;
    }
    int64_t slot_align = kDefaultSlotAlign, slot_skew = 0, chunk_bytes = 0;
    int32_t blocks_per_cu = 0, resident_cap = 0, newest_from_master = 0, cache_policy = 0, xcd_group = 0;
    if (tuning) {
        if (tuning->reserved != 0) { set_error("plan: tuning.reserved must be 0"); return FERRET_EINVAL; }
        xcd_group = tuning->xcd_group;
        if (xcd_group < 0 || xcd_group > 4096) { set_error("plan: xcd_group = %d, need 0..4096", xcd_group); return FERRET_EINVAL; }
        chunk_bytes = tuning->chunk_bytes;
        if (chunk_bytes < 0 || chunk_bytes > (int64_t(1) << 30)) {
            set_error("plan: chunk_bytes = %lld, need 0 .. 2^30", (long long)chunk_bytes); return FERRET_EINVAL;
        }
        if (chunk_bytes > 0 && chunk_elems > 0) {
            set_error("plan: give chunk_elems or tuning.chunk_bytes, not both"); return FERRET_EINVAL;
        }
        cache_policy = tuning->cache_policy;
        if (cache_policy < 0 || cache_policy > 2) { set_error("plan: cache_policy = %d, need 0..2", cache_policy); return FERRET_EINVAL; }
        newest_from_master = tuning->newest_from_master;
        if (newest_from_master != 0 && newest_from_master != 1) {
            set_error("plan: newest_from_master = %d, need 0 or 1", newest_from_master); return FERRET_EINVAL;
        }
        if (newest_from_master && prec != FERRET_BF16_MASTER_F32) {
            set_error("plan: newest_from_master only applies to FERRET_BF16_MASTER_F32"); return FERRET_EINVAL;
        }
        resident_cap = tuning->resident_cap;
        if (resident_cap > 32 || resident_cap == 1) {      // one workgroup may reserve at most 64 KiB of the CU's 160 KiB of LDS
            set_error("plan: resident_cap = %d, need 2..32, 0 (default) or < 0 (none)", resident_cap); return FERRET_EINVAL;
        }
        if (tuning->slot_align_elems) slot_align = tuning->slot_align_elems;
        slot_skew = tuning->slot_skew_elems;
        blocks_per_cu = tuning->blocks_per_cu;
        if (slot_align < 0 || slot_align % kStageAlign != 0) {
            set_error("plan: slot_align_elems = %lld, need a multiple of %lld", (long long)slot_align,
                      (long long)kStageAlign);
            return FERRET_EINVAL;
        }
        if (slot_skew < 0 || slot_skew % FERRET_ALIGN_ELEMS != 0) {
            set_error("plan: slot_skew_elems = %lld, need a non-negative multiple of %d",
                      (long long)slot_skew, FERRET_ALIGN_ELEMS);
            return FERRET_EINVAL;
        }
        if (blocks_per_cu > 64) { set_error("plan: blocks_per_cu = %d, need <= 64", blocks_per_cu); return FERRET_EINVAL; }
        if (newest_from_master && blocks_per_cu > 0) {
            set_error("plan: newest_from_master is not available with a persistent grid (blocks_per_cu > 0)"); return FERRET_EINVAL;
        }
    }
    for (int32_t j = 0; j < n_stages; ++j) {
        if (staleness[j] < 0) { set_error("plan: staleness[%d] = %d < 0", j, staleness[j]); return FERRET_EINVAL; }
        if (ring_depth > 0 && staleness[j] >= ring_depth) {
            set_error("plan: staleness[%d] = %d needs %d stored versions but ring_depth = %d", j,
                      staleness[j], staleness[j] + 1, ring_depth);
            return FERRET_EINVAL;
        }
        if (staleness[j] >= FERRET_MAX_RING_DEPTH) {
            set_error("plan: staleness[%d] = %d too large", j, staleness[j]); return FERRET_EINVAL;
        }
    }

    ferret_plan *p = new (std::nothrow) ferret_plan();
    if (!p) { set_error("plan: out of host memory"); return FERRET_ENOMEM; }
    try {
        p->stages.resize(n_stages);
        p->tensor_offset.resize(n_tensors);
        p->tensor_stage.resize(n_tensors);
    } catch (const std::bad_alloc &) {
        delete p; set_error("plan: out of host memory"); return FERRET_ENOMEM;
    }
    p->prec = prec;
    p->n_iters = n_iters;
    p->chunk_elems = chunk_elems;
    p->cache_policy = cache_policy;
    p->xcd_group = xcd_group;
    p->blocks_per_cu = blocks_per_cu;
    p->resident_cap = resident_cap;
    p->newest_from_master = newest_from_master;

    // tensors -> stage buckets
    int32_t prev_stage = 0;
    for (int32_t i = 0; i < n_tensors; ++i) {
        const ferret_tensor &t = tensors[i];
        if (t.numel <= 0 || t.reserved != 0 || t.stage < 0 || t.stage >= n_stages) {
            set_error("plan: tensor %d: numel = %lld, stage = %d, reserved = %d", i, (long long)t.numel,
                      t.stage, t.reserved);
            delete p; return FERRET_EINVAL;
        }
        if (t.stage < prev_stage || t.stage > prev_stage + 1 || (i == 0 && t.stage != 0)) {
            set_error("plan: tensor %d is in stage %d after stage %d: stage ids must be non-decreasing "
                      "and every stage non-empty", i, t.stage, prev_stage);
            delete p; return FERRET_EINVAL;
        }
        prev_stage = t.stage;
        Stage &s = p->stages[t.stage];
        p->tensor_stage[i] = t.stage;
        p->tensor_offset[i] = s.n_elems;
        s.params += t.numel;
        s.n_elems = round_up(s.n_elems + t.numel, FERRET_ALIGN_ELEMS);
        p->total_params += t.numel;
    }
    if (prev_stage != n_stages - 1) {
        set_error("plan: stages %d..%d own no tensor", prev_stage + 1, n_stages - 1);
        delete p; return FERRET_EINVAL;
    }

    // layout
    int64_t flat = 0, ring = 0, chunks = 0;
    for (int32_t j = 0; j < n_stages; ++j) {
        Stage &s = p->stages[j];
        s.tau = staleness[j];
        s.ring_depth = ring_depth > 0 ? ring_depth : staleness[j] + 1;
        s.flat_off = flat;
        flat += round_up(s.n_elems, kStageAlign);
        s.slot_stride = round_up(s.n_elems, slot_align) + slot_skew;
        s.ring_base = ring;
        ring += round_up(s.slot_stride * s.ring_depth, kStageAlign);
    }
    // chunks.  Size per stage: the caller's; else, for plans that stream (working set beyond the memory-side
    // cache), the multiple of one-vector-per-lane nearest to chunk_bytes of traffic in flight per chunk, so that
    // every workgroup moves about the same bytes whatever its stage's K' and one resident-workgroup cap suits
    // every stage of a launch; else two vectors per lane for every stage.
    const bool by_bytes = chunk_elems == 0 && (chunk_bytes > 0 || working_set_bytes(prec, ring, flat) > kCacheResidentBytes);
    // default byte target, measured on MI355X together with the resident-workgroup cap: 48 KiB, i.e. 2048
    // elements at K' = 3 in fp32, more for stages that read fewer versions, fewer for deeper ones
    if (by_bytes && chunk_bytes == 0) chunk_bytes = 48 * 1024;
    p->chunk_bytes = by_bytes ? chunk_bytes : 0;
    for (int32_t j = 0; j < n_stages; ++j) {
        Stage &s = p->stages[j];
        s.chunk_elems = chunk_elems > 0 ? chunk_elems : 2 * chunk_unit;
        if (by_bytes) {
            const int32_t kp = effective_iters(n_iters, staleness[j]);
            // a stage that iterates nothing still reads V[0] when the weight gap is wanted (norms, gap penalty)
            const int64_t per = inflight_bytes_per_elem(prec, kp) + (kp == 0 && staleness[j] > 0 ? storage_bytes(prec) : 0);
            int64_t units = (chunk_bytes + per * chunk_unit / 2) / (per * chunk_unit);
            if (units < 1) units = 1;
            s.chunk_elems = units * chunk_unit > kMaxChunkElems ? kMaxChunkElems : units * chunk_unit;
        }
        s.chunk_begin = chunks;
        s.n_chunks = (s.n_elems + s.chunk_elems - 1) / s.chunk_elems;
        chunks += s.n_chunks;
    }
    if (chunks > 0x7fffffffLL) { set_error("plan: %lld chunks, too many; raise chunk_elems", (long long)chunks); delete p; return FERRET_EINVAL; }
    p->flat_elems = flat;
    p->ring_elems = ring;
    p->n_chunks = chunks;
    *out_plan = p;
    return FERRET_OK;
}

void ferret_plan_destroy(ferret_plan *plan) { delete plan; }

// ---- queries ----------------------------------------------------------------------------------
#define STAGE_OR(ret) \
    if (!plan || stage < 0 || stage >= (int32_t)plan->stages.size()) return ret; \
    const Stage &s = plan->stages[stage]

int32_t ferret_plan_n_stages(const ferret_plan *plan) { return plan ? (int32_t)plan->stages.size() : -1; }
int32_t ferret_plan_n_tensors(const ferret_plan *plan) { return plan ? (int32_t)plan->tensor_offset.size() : -1; }
int32_t ferret_plan_precision(const ferret_plan *plan) { return plan ? (int32_t)plan->prec : -1; }
int32_t ferret_plan_n_iters(const ferret_plan *plan) { return plan ? plan->n_iters : 0; }
int64_t ferret_plan_chunk_elems(const ferret_plan *plan) {
    if (!plan) return -1;
    int64_t largest = 0;
    for (const Stage &s : plan->stages) largest = s.chunk_elems > largest ? s.chunk_elems : largest;
    return largest;
}
int64_t ferret_plan_n_chunks(const ferret_plan *plan) { return plan ? plan->n_chunks : -1; }
int64_t ferret_plan_flat_elems(const ferret_plan *plan) { return plan ? plan->flat_elems : -1; }
int64_t ferret_plan_ring_elems(const ferret_plan *plan) { return plan ? plan->ring_elems : -1; }
size_t ferret_plan_ring_bytes(const ferret_plan *plan) { return plan ? (size_t)(plan->ring_elems * storage_bytes(plan->prec)) : 0; }
size_t ferret_plan_grad_bytes(const ferret_plan *plan) { return plan ? (size_t)(plan->flat_elems * storage_bytes(plan->prec)) : 0; }
size_t ferret_plan_master_bytes(const ferret_plan *plan) { return plan ? (size_t)(plan->flat_elems * 4) : 0; }
size_t ferret_plan_workspace_bytes(const ferret_plan *plan) {
    // five per-chunk series: three norms and the two inner products of the lambda block
    return plan ? (size_t)round_up(plan->n_chunks * 5 * (int64_t)sizeof(float), 256) : 0;
}
int64_t ferret_plan_total_params(const ferret_plan *plan) { return plan ? plan->total_params : -1; }

int64_t ferret_plan_stage_params(const ferret_plan *plan, int32_t stage) { STAGE_OR(-1); return s.params; }
int64_t ferret_plan_stage_numel(const ferret_plan *plan, int32_t stage) { STAGE_OR(-1); return s.n_elems; }
int64_t ferret_plan_stage_flat_offset(const ferret_plan *plan, int32_t stage) { STAGE_OR(-1); return s.flat_off; }
int64_t ferret_plan_stage_ring_offset(const ferret_plan *plan, int32_t stage) { STAGE_OR(-1); return s.ring_base; }
int64_t ferret_plan_stage_slot_stride(const ferret_plan *plan, int32_t stage) { STAGE_OR(-1); return s.slot_stride; }
int32_t ferret_plan_stage_ring_depth(const ferret_plan *plan, int32_t stage) { STAGE_OR(-1); return s.ring_depth; }
int32_t ferret_plan_stage_staleness(const ferret_plan *plan, int32_t stage) { STAGE_OR(-1); return s.tau; }
int64_t ferret_plan_stage_chunk_elems(const ferret_plan *plan, int32_t stage) { STAGE_OR(-1); return s.chunk_elems; }
int64_t ferret_plan_stage_n_chunks(const ferret_plan *plan, int32_t stage) { STAGE_OR(-1); return s.n_chunks; }
int64_t ferret_plan_tensor_offset(const ferret_plan *plan, int32_t tensor) {
    if (!plan || tensor < 0 || tensor >= (int32_t)plan->tensor_offset.size()) return -1;
    return plan->tensor_offset[tensor];
}

// ---- ring state -------------------------------------------------------------------------------
ferret_status ferret_plan_get_state(const ferret_plan *plan, int32_t *heads, int32_t *valid) {
    if (!plan || !heads || !valid) { set_error("get_state: null argument"); return FERRET_EINVAL; }
    for (size_t j = 0; j < plan->stages.size(); ++j) {
        heads[j] = plan->stages[j].head;
        valid[j] = plan->stages[j].valid;
    }
    return FERRET_OK;
}

ferret_status ferret_plan_set_state(ferret_plan *plan, const int32_t *heads, const int32_t *valid) {
    if (!plan || !heads || !valid) { set_error("set_state: null argument"); return FERRET_EINVAL; }
    for (size_t j = 0; j < plan->stages.size(); ++j) {
        const Stage &s = plan->stages[j];
        if (heads[j] < 0 || heads[j] >= s.ring_depth || valid[j] < 0 || valid[j] > s.ring_depth) {
            set_error("set_state: stage %zu: head = %d, valid = %d, ring depth = %d", j, heads[j], valid[j],
                      s.ring_depth);
            return FERRET_EINVAL;
        }
    }
    for (size_t j = 0; j < plan->stages.size(); ++j) {
        plan->stages[j].head = heads[j];
        plan->stages[j].valid = valid[j];
        plan->stages[j].step_pending = false;
    }
    return FERRET_OK;
}

int32_t ferret_plan_stage_effective_staleness(const ferret_plan *plan, int32_t stage) {
    STAGE_OR(-1);
    return effective_tau(s);
}
int32_t ferret_plan_stage_effective_iters(const ferret_plan *plan, int32_t stage) {
    STAGE_OR(-1);
    return effective_iters(plan->n_iters, effective_tau(s));
}
int32_t ferret_plan_stage_read_slots(const ferret_plan *plan, int32_t stage, int32_t *slots, int32_t cap) {
    STAGE_OR(-1);
    if (s.valid < 1) return 0;
    const int32_t tau = effective_tau(s), kp = effective_iters(plan->n_iters, tau), R = s.ring_depth;
    const int32_t n = kp + 1;
    for (int32_t i = 0; i < n && slots && i < cap; ++i) {
        int32_t age_from_oldest = kp == 0 ? tau : (int32_t)(((int64_t)i * tau) / kp);   // s_i
        slots[i] = ((s.head - (tau - age_from_oldest)) % R + R) % R;
    }
    return n;
}
int32_t ferret_plan_stage_write_slot(const ferret_plan *plan, int32_t stage) {
    STAGE_OR(-1);
    return s.valid == 0 ? s.head : (s.head + 1) % s.ring_depth;
}

int64_t ferret_plan_step_bytes(const ferret_plan *plan) {
    if (!plan) return -1;
    int64_t bytes = 0;
    const int64_t sb = storage_bytes(plan->prec);
    for (const Stage &s : plan->stages) {
        const int32_t kp = effective_iters(plan->n_iters, effective_tau(s));
        int64_t per = sb /*grad*/ + sb * (kp + 1) /*versions*/ + sb /*new version*/;
        if (plan->prec == FERRET_BF16_MASTER_F32) per += 8;   // master read + write
        bytes += per * s.params;
    }
    return bytes;
}

// ---- push --------------------------------------------------------------------------------------
static void advance(Stage &s) {
    if (s.valid > 0) s.head = (s.head + 1) % s.ring_depth;   // the very first version lands in slot head
    if (s.valid < s.ring_depth) ++s.valid;
    s.step_pending = false;
}

ferret_status ferret_push_version(ferret_plan *plan, void *ring, float *master, int32_t stage,
                                  const void *src, void *hip_stream) {
    if (!plan) { set_error("push_version: null plan"); return FERRET_EINVAL; }
    const int32_t P = (int32_t)plan->stages.size();
    if (stage < -1 || stage >= P) { set_error("push_version: stage = %d, need -1..%d", stage, P - 1); return FERRET_EINVAL; }
    const int32_t j0 = stage < 0 ? 0 : stage, j1 = stage < 0 ? P : stage + 1;

    if (!src) {   // commit only
        for (int32_t j = j0; j < j1; ++j)
            if (!plan->stages[j].step_pending) {
                set_error("push_version: commit of stage %d without a step since its last commit", j);
                return FERRET_ESTATE;
            }
        for (int32_t j = j0; j < j1; ++j) advance(plan->stages[j]);
        return FERRET_OK;
    }

    if (!ring) { set_error("push_version: null ring"); return FERRET_EINVAL; }
    if (!aligned16(ring) || !aligned16(src) || !aligned16(master)) {
        set_error("push_version: device pointers must be 16-byte aligned"); return FERRET_EINVAL;
    }
    if (master && plan->prec != FERRET_BF16_MASTER_F32) {
        set_error("push_version: master given but the plan is fp32"); return FERRET_EINVAL;
    }
    PushArgs a;
    memset(&a, 0, sizeof a);
    a.ring = ring;
    a.master = master;
    a.src = static_cast<const float *>(src);
    uint32_t chunks = 0, n = 0;
    for (int32_t j = j0; j < j1; ++j, ++n) {
        const Stage &s = plan->stages[j];
        StageDesc &d = a.stage[n];
        d.ring_base = (uint64_t)s.ring_base;
        d.slot_stride = (uint64_t)s.slot_stride;
        d.flat_off = (uint64_t)s.flat_off;
        d.n_elems = (uint64_t)s.n_elems;
        d.chunk_begin = chunks;
        d.chunk_elems = (uint32_t)s.chunk_elems;
        d.ring_depth = (uint16_t)s.ring_depth;
        d.head = (uint16_t)(s.valid == 0 ? s.head : (s.head + 1) % s.ring_depth);   // slot written
        chunks += (uint32_t)s.n_chunks;
    }
    a.n_stages = n;
    a.n_chunks = chunks;
    int err = launch_push(*plan, a, hip_stream);
    if (err) { set_error("push_version: launch failed: %s", device_error_string(err)); return FERRET_EDEVICE; }
    for (int32_t j = j0; j < j1; ++j) advance(plan->stages[j]);
    return FERRET_OK;
}

// ---- step --------------------------------------------------------------------------------------
// takes_part: null = every stage, else per stage non-zero = the stage is read and written by this call
static ferret_status check_step_args(const char *who, const ferret_plan *plan, void *ring, const void *grads,
                                     float *master, float *norms_out, void *grad_out, void *workspace,
                                     const int32_t *takes_part = nullptr) {
    if (!plan || !ring || !grads) { set_error("%s: null plan, ring or grads", who); return FERRET_EINVAL; }
    const bool mixed = plan->prec == FERRET_BF16_MASTER_F32;
    if (mixed && !master) { set_error("%s: bf16 plan needs the fp32 master", who); return FERRET_EINVAL; }
    if (!mixed && master) { set_error("%s: master given but the plan is fp32", who); return FERRET_EINVAL; }
    if (norms_out && !workspace) { set_error("%s: norms_out needs workspace", who); return FERRET_EINVAL; }
    if (!aligned16(ring) || !aligned16(grads) || !aligned16(master) || !aligned16(grad_out) ||
        !aligned16(workspace) || (reinterpret_cast<uintptr_t>(norms_out) & 3u)) {
        set_error("%s: device pointers must be 16-byte aligned", who); return FERRET_EINVAL;
    }
    for (size_t j = 0; j < plan->stages.size(); ++j)
        if ((!takes_part || takes_part[j] != 0) && plan->stages[j].valid < 1) {
            set_error("%s: stage %zu holds no weight version yet (push one first)", who, j);
            return FERRET_ESTATE;
        }
    return FERRET_OK;
}


// The step's scratch: five per-chunk series.
static void use_workspace(StepArgs &a, void *workspace) { a.partials = static_cast<float *>(workspace); }

static void fill_step_args(const ferret_plan *plan, StepArgs &a, void *ring, const void *grads, float *master,
                           float lambda, float lr, float *norms_out, void *grad_out, void *workspace) {
    memset(&a, 0, sizeof a);
    a.ring = ring;
    a.grads = grads;
    a.master = master;
    a.grad_out = static_cast<float *>(grad_out);
    a.norms_out = norms_out;
    if (norms_out) use_workspace(a, workspace);
    a.lambda = lambda;
    a.lr = lr;
    a.n_stages = (uint32_t)plan->stages.size();
    a.n_chunks = (uint32_t)plan->n_chunks;
    a.chunk_base = 0;
    a.chunk_end = a.n_chunks;
    fill_step_descs(*plan, a.stage);
    for (uint32_t j = 0; j < FERRET_MAX_STAGES; ++j)
        a.chunk_begin[j] = j < a.n_stages ? a.stage[j].chunk_begin : UINT32_MAX;
}

// When mode[] leaves stages out, the launch only has to cover the chunks from the first to the last stage that
// takes part (stages left out in between still get workgroups, which return at once).
static void narrow_chunk_span(const ferret_plan *plan, StepArgs &a) {
    const size_t P = plan->stages.size();
    size_t first = P, last = 0;
    for (size_t j = 0; j < P; ++j)
        if (a.mode[j] != 0) { if (first == P) first = j; last = j; }
    if (first == P) { a.chunk_base = a.chunk_end = 0; return; }
    a.chunk_base = (uint32_t)plan->stages[first].chunk_begin;
    a.chunk_end = (uint32_t)(plan->stages[last].chunk_begin + plan->stages[last].n_chunks);
}

ferret_status ferret_compensate_step(const ferret_plan *plan, void *ring, const void *grads, float *master,
                                     float lambda, float lr, float *norms_out, void *grad_out,
                                     void *workspace, void *hip_stream) {
    ferret_status rc = check_step_args("compensate_step", plan, ring, grads, master, norms_out, grad_out, workspace);
    if (rc != FERRET_OK) return rc;
    StepArgs a;
    fill_step_args(plan, a, ring, grads, master, lambda, lr, norms_out, grad_out, workspace);
    int err = launch_step(*plan, a, hip_stream);
    if (err) { set_error("compensate_step: launch failed: %s", device_error_string(err)); return FERRET_EDEVICE; }
    // bookkeeping only: remembers that slot head+1 now holds an uncommitted version
    for (const Stage &s : plan->stages) s.step_pending = true;
    return FERRET_OK;
}

ferret_status ferret_compensate_step_noalloc(const ferret_plan *plan, void *ring, const void *grads, float *master,
                                             float lambda, float lr, float *norms_out, void *grad_out,
                                             void *hip_stream) {
    const char *who = "compensate_step_noalloc";
    if (plan && plan->n_chunks > FERRET_NOALLOC_MAX_CHUNKS) {
        set_error("%s: the plan has %lld chunks, the library's own scratch holds partial sums for at most %d; "
                  "plan with a larger chunk_elems or use ferret_compensate_step with a workspace", who,
                  (long long)plan->n_chunks, FERRET_NOALLOC_MAX_CHUNKS);
        return FERRET_EINVAL;
    }
    void *scratch_ptr = nullptr;
    if (norms_out) {                    // the scratch is only touched when norms are asked for
        int err = noalloc_scratch(&scratch_ptr);
        if (err) { set_error("%s: looking up the scratch array failed: %s", who, device_error_string(err)); return FERRET_EDEVICE; }
    }
    ferret_status rc = check_step_args(who, plan, ring, grads, master, norms_out, grad_out, scratch_ptr);
    if (rc != FERRET_OK) return rc;
    StepArgs a;
    fill_step_args(plan, a, ring, grads, master, lambda, lr, norms_out, grad_out, scratch_ptr);
    int err = launch_step(*plan, a, hip_stream);
    if (err) { set_error("%s: launch failed: %s", who, device_error_string(err)); return FERRET_EDEVICE; }
    for (const Stage &s : plan->stages) s.step_pending = true;
    return FERRET_OK;
}

static ferret_status check_adaptive(const char *who, const ferret_plan *plan, const ferret_adaptive *ad,
                                    void *workspace) {
    if (!ad || !ad->lambda || !ad->v_r || !ad->v_a || !workspace) {
        set_error("%s: null adaptive state (lambda, v_r, v_a) or workspace", who); return FERRET_EINVAL;
    }
    if (!aligned16(ad->v_r) || !aligned16(ad->v_a) || (reinterpret_cast<uintptr_t>(ad->lambda) & 3u)) {
        set_error("%s: v_r and v_a must be 16-byte aligned, lambda 4-byte aligned", who); return FERRET_EINVAL;
    }
    if (!(ad->alpha >= 0.f && ad->alpha < 1.f) || !(ad->eta_lambda >= 0.f)) {
        set_error("%s: need 0 <= alpha < 1 and eta_lambda >= 0 (got %g, %g)", who, (double)ad->alpha,
                  (double)ad->eta_lambda);
        return FERRET_EINVAL;
    }
    if (plan->n_iters == 0) { set_error("%s: the plan has n_iters = 0, there is nothing for lambda to scale", who); return FERRET_EINVAL; }
    if ((ad->fused != 0 && ad->fused != 1) || ad->reserved != 0) {
        set_error("%s: fused = %d (need 0 or 1), reserved = %d (need 0)", who, ad->fused, ad->reserved); return FERRET_EINVAL;
    }
    return FERRET_OK;
}

static void set_adaptive_args(StepArgs &a, const ferret_adaptive *ad) {
    a.lambda_dev = ad->lambda;
    a.v_r = ad->v_r;
    a.v_a = ad->v_a;
    a.alpha = ad->alpha;
    a.eta_lambda = ad->eta_lambda;
}

ferret_status ferret_compensate_stages(const ferret_plan *plan, void *ring, const void *grads, float *master,
                                       const int32_t *active, float lambda, float lr, float *norms_out,
                                       void *grad_out, void *workspace, void *hip_stream) {
    const char *who = "compensate_stages";
    if (!active) { set_error("%s: null active", who); return FERRET_EINVAL; }
    ferret_status rc = check_step_args(who, plan, ring, grads, master, norms_out, grad_out, workspace, active);
    if (rc != FERRET_OK) return rc;
    StepArgs a;
    fill_step_args(plan, a, ring, grads, master, lambda, lr, norms_out, grad_out, workspace);
    a.masked = 1;
    const size_t P = plan->stages.size();
    for (size_t j = 0; j < P; ++j) a.mode[j] = active[j] ? 2 : 0;
    narrow_chunk_span(plan, a);
    int err = launch_step(*plan, a, hip_stream);
    if (err) { set_error("%s: launch failed: %s", who, device_error_string(err)); return FERRET_EDEVICE; }
    for (size_t j = 0; j < P; ++j)
        if (active[j]) plan->stages[j].step_pending = true;
    return FERRET_OK;
}

static ferret_status adaptive_impl(const char *who, const ferret_plan *plan, void *ring, const void *grads,
                                   float *master, const int32_t *active, const ferret_adaptive *ad, float lr,
                                   float *norms_out, void *grad_out, void *workspace, void *hip_stream) {
    ferret_status rc = check_step_args(who, plan, ring, grads, master, norms_out, grad_out, workspace, active);
    if (rc != FERRET_OK) return rc;
    rc = check_adaptive(who, plan, ad, workspace);
    if (rc != FERRET_OK) return rc;
    StepArgs a;
    fill_step_args(plan, a, ring, grads, master, 0.f, lr, norms_out, grad_out, workspace);
    set_adaptive_args(a, ad);
    if (active) {
        a.masked = 1;
        for (size_t j = 0; j < plan->stages.size(); ++j) a.mode[j] = active[j] ? 2 : 0;
        narrow_chunk_span(plan, a);
    }
    int err = 0;
    if (ad->eta_lambda > 0.f && ad->fused) {
        a.fused_lambda = 1;                                // one pass: the step kernel runs the lambda block too
        use_workspace(a, workspace);
    } else if (ad->eta_lambda > 0.f) {
        StepArgs state = a;                                // the state pass always goes through the workspace
        use_workspace(state, workspace);
        err = launch_lambda_update(*plan, state, hip_stream);
    }
    if (!err) err = launch_step(*plan, a, hip_stream);
    if (err) { set_error("%s: launch failed: %s", who, device_error_string(err)); return FERRET_EDEVICE; }
    for (size_t j = 0; j < plan->stages.size(); ++j)
        if (!active || active[j]) plan->stages[j].step_pending = true;
    return FERRET_OK;
}

ferret_status ferret_compensate_step_adaptive(const ferret_plan *plan, void *ring, const void *grads,
                                              float *master, const ferret_adaptive *ad, float lr,
                                              float *norms_out, void *grad_out, void *workspace,
                                              void *hip_stream) {
    return adaptive_impl("compensate_step_adaptive", plan, ring, grads, master, nullptr, ad, lr, norms_out, grad_out,
                         workspace, hip_stream);
}

ferret_status ferret_compensate_stages_adaptive(const ferret_plan *plan, void *ring, const void *grads,
                                                float *master, const int32_t *active, const ferret_adaptive *ad,
                                                float lr, float *norms_out, void *grad_out, void *workspace,
                                                void *hip_stream) {
    if (!active) { set_error("compensate_stages_adaptive: null active"); return FERRET_EINVAL; }
    return adaptive_impl("compensate_stages_adaptive", plan, ring, grads, master, active, ad, lr, norms_out, grad_out,
                         workspace, hip_stream);
}

static ferret_status accumulate_impl(const char *who, const ferret_plan *plan, void *ring, const void *grads,
                                     float *master, const ferret_accumulate *acc, const ferret_adaptive *ad,
                                     float lambda, float lr, float *norms_out, void *grad_out, void *workspace,
                                     void *hip_stream) {
    if (!acc || !acc->accum || !acc->mode) { set_error("%s: null accumulate, accum or mode", who); return FERRET_EINVAL; }
    ferret_status rc = check_step_args(who, plan, ring, grads, master, norms_out, grad_out, workspace, plan ? acc->mode : nullptr);
    if (rc != FERRET_OK) return rc;
    if (ad) {
        rc = check_adaptive(who, plan, ad, workspace);
        if (rc != FERRET_OK) return rc;
    }
    if (!aligned16(acc->accum)) { set_error("%s: accum must be 16-byte aligned", who); return FERRET_EINVAL; }
    const size_t P = plan->stages.size();
    for (size_t j = 0; j < P; ++j) {
        if (acc->mode[j] < 0 || acc->mode[j] > 2) { set_error("%s: mode[%zu] = %d, need 0..2", who, j, acc->mode[j]); return FERRET_EINVAL; }
        if (acc->staleness && (acc->staleness[j] < 0 || acc->staleness[j] > plan->stages[j].tau)) {
            set_error("%s: staleness[%zu] = %d, need 0..%d (the plan's tau)", who, j, acc->staleness[j],
                      plan->stages[j].tau);
            return FERRET_EINVAL;
        }
    }
    StepArgs a;
    fill_step_args(plan, a, ring, grads, master, lambda, lr, norms_out, grad_out, workspace);
    a.accum = acc->accum;
    a.accum_scale = acc->scale;
    for (size_t j = 0; j < P; ++j) {
        a.mode[j] = (uint8_t)acc->mode[j];
        if (acc->staleness) {
            const int32_t have = effective_tau(plan->stages[j]);
            const int32_t tau = acc->staleness[j] < have ? acc->staleness[j] : have;
            a.stage[j].tau = (uint16_t)tau;
            a.stage[j].kp = (uint16_t)effective_iters(plan->n_iters, tau);
        }
    }
    narrow_chunk_span(plan, a);
    int err = 0;
    if (ad) {
        set_adaptive_args(a, ad);
        if (ad->eta_lambda > 0.f && ad->fused) {
            a.fused_lambda = 1;          // one pass: the accumulation kernel runs the lambda block too
            use_workspace(a, workspace);
        } else if (ad->eta_lambda > 0.f) {      // lambda block of every participating stage, on this arrival's staleness
            StepArgs state = a;
            use_workspace(state, workspace);
            err = launch_lambda_update(*plan, state, hip_stream);
        }
    }
    if (!err) err = launch_step(*plan, a, hip_stream);
    if (err) { set_error("%s: launch failed: %s", who, device_error_string(err)); return FERRET_EDEVICE; }
    for (size_t j = 0; j < P; ++j)
        if (acc->mode[j] == 2) plan->stages[j].step_pending = true;
    return FERRET_OK;
}

ferret_status ferret_accumulate_step(const ferret_plan *plan, void *ring, const void *grads, float *master,
                                     const ferret_accumulate *acc, float lambda, float lr, float *norms_out,
                                     void *grad_out, void *workspace, void *hip_stream) {
    return accumulate_impl("accumulate_step", plan, ring, grads, master, acc, nullptr, lambda, lr, norms_out,
                           grad_out, workspace, hip_stream);
}

ferret_status ferret_accumulate_step_adaptive(const ferret_plan *plan, void *ring, const void *grads,
                                              float *master, const ferret_accumulate *acc,
                                              const ferret_adaptive *adaptive, float lr, float *norms_out,
                                              void *grad_out, void *workspace, void *hip_stream) {
    if (!adaptive) { set_error("accumulate_step_adaptive: null adaptive"); return FERRET_EINVAL; }
    return accumulate_impl("accumulate_step_adaptive", plan, ring, grads, master, acc, adaptive, 0.f, lr, norms_out,
                           grad_out, workspace, hip_stream);
}

ferret_status ferret_penalized_step(const ferret_plan *plan, void *ring, const void *grads, float *master,
                                    const float *scale, const float *inv_c, float lr, float *norms_out,
                                    void *grad_out, void *workspace, void *hip_stream) {
    const char *who = "penalized_step";
    ferret_status rc = check_step_args(who, plan, ring, grads, master, norms_out, grad_out, workspace);
    if (rc != FERRET_OK) return rc;
    const size_t P = plan->stages.size();
    for (size_t j = 0; j < P; ++j) {
        if (inv_c && !(inv_c[j] >= 0.f)) { set_error("%s: inv_c[%zu] = %g, need >= 0", who, j, (double)inv_c[j]); return FERRET_EINVAL; }
        if (scale && !(scale[j] == scale[j])) { set_error("%s: scale[%zu] is NaN", who, j); return FERRET_EINVAL; }
    }
    StepArgs a;
    fill_step_args(plan, a, ring, grads, master, 0.f, lr, norms_out, grad_out, workspace);
    a.penalized = 1;
    for (size_t j = 0; j < P; ++j) {
        const int32_t tau = a.stage[j].tau;
        a.stage[j].kp = 0;                                   // no iterations
        a.pen_scale[j] = scale ? scale[j] : 1.0f / (float)(tau > 1 ? tau : 1);
        a.pen_inv_c[j] = inv_c ? inv_c[j] : 0.f;
    }
    int err = launch_step(*plan, a, hip_stream);
    if (err) { set_error("%s: launch failed: %s", who, device_error_string(err)); return FERRET_EDEVICE; }
    for (const Stage &s : plan->stages) s.step_pending = true;
    return FERRET_OK;
}

ferret_status ferret_copy_bytes(void *dst, const void *src, size_t n_bytes, void *hip_stream) {
    if (!dst || !src || !aligned16(dst) || !aligned16(src) || (n_bytes & 15u)) {
        set_error("copy_bytes: need non-null 16-byte aligned pointers and a multiple of 16 bytes");
        return FERRET_EINVAL;
    }
    if (n_bytes == 0) return FERRET_OK;
    int err = launch_copy(dst, src, n_bytes, hip_stream);
    if (err) { set_error("copy_bytes: launch failed: %s", device_error_string(err)); return FERRET_EDEVICE; }
    return FERRET_OK;
}

ferret_status ferret_read_bytes(const void *src, size_t n_bytes, void *sink, void *hip_stream) {
    if (!src || !sink || !aligned16(src) || !aligned16(sink) || (n_bytes & 15u)) {
        set_error("read_bytes: need non-null 16-byte aligned pointers and a multiple of 16 bytes");
        return FERRET_EINVAL;
    }
    if (n_bytes == 0) return FERRET_OK;
    int err = launch_read(src, n_bytes, sink, hip_stream);
    if (err) { set_error("read_bytes: launch failed: %s", device_error_string(err)); return FERRET_EDEVICE; }
    return FERRET_OK;
}

ferret_status ferret_stream_mix(void *dst, const void *src, size_t src_stride_bytes, int32_t n_reads,
                                size_t n_bytes, int32_t resident_cap, void *hip_stream) {
    if (!dst || !src || !aligned16(dst) || !aligned16(src) || (n_bytes & 15u) || (src_stride_bytes & 15u)) {
        set_error("stream_mix: need non-null 16-byte aligned pointers, n_bytes and stride multiples of 16");
        return FERRET_EINVAL;
    }
    if (n_reads < 1 || n_reads > 8 || resident_cap > 32) {
        set_error("stream_mix: n_reads = %d (need 1..8), resident_cap = %d (need <= 32)", n_reads, resident_cap);
        return FERRET_EINVAL;
    }
    if (n_reads > 1 && src_stride_bytes < n_bytes) {
        set_error("stream_mix: source streams overlap (stride %zu < %zu bytes)", src_stride_bytes, n_bytes);
        return FERRET_EINVAL;
    }
    {   // dst must not overlap the sources
        const uintptr_t d0 = reinterpret_cast<uintptr_t>(dst), d1 = d0 + n_bytes;
        const uintptr_t s0 = reinterpret_cast<uintptr_t>(src), s1 = s0 + (size_t)(n_reads - 1) * src_stride_bytes + n_bytes;
        if (d0 < s1 && s0 < d1) { set_error("stream_mix: dst overlaps the sources"); return FERRET_EINVAL; }
    }
    if (n_bytes == 0) return FERRET_OK;
    int err = launch_mix(dst, src, src_stride_bytes, n_reads, n_bytes, resident_cap, hip_stream);
    if (err) { set_error("stream_mix: launch failed: %s", device_error_string(err)); return FERRET_EDEVICE; }
    return FERRET_OK;
}

ferret_status ferret_profile_begin(int32_t capacity) {
    if (capacity < 1 || capacity > (1 << 20)) { set_error("profile_begin: capacity = %d", capacity); return FERRET_EINVAL; }
    int err = profile_begin(capacity);
    if (err < 0) { set_error("profile_begin: already profiling"); return FERRET_ESTATE; }
    if (err) { set_error("profile_begin: %s", device_error_string(err)); return FERRET_EDEVICE; }
    return FERRET_OK;
}

ferret_status ferret_profile_end(float *ms_out, int32_t cap, int32_t *n_out) {
    if (!n_out || cap < 0 || (cap > 0 && !ms_out)) { set_error("profile_end: bad arguments"); return FERRET_EINVAL; }
    int err = profile_end(ms_out, cap, n_out);
    if (err == -2) { set_error("profile_end: the session belongs to the thread that called profile_begin"); return FERRET_ESTATE; }
    if (err < 0) { set_error("profile_end: profile_begin was not called"); return FERRET_ESTATE; }
    if (err) { set_error("profile_end: %s", device_error_string(err)); return FERRET_EDEVICE; }
    return FERRET_OK;
}

}  // extern "C"
