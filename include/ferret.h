/*
 * ferret.h -- C ABI of libferret: iterative gradient compensation + weight update for
 * pipelined online continual learning (Ferret), for AMD MI355X (gfx950).
 *
 * The operation (paper: Sec. "Iterative Gradient Compensation"; Alg. 1 "Iterative
 * Gradients Compensation with lambda" in the appendix "Algorithm Details"):
 * a pipeline stage j holds several versions of its parameters, because the gradient it
 * receives was computed on weights that are tau_j updates old.  Before the update the
 * stale gradient g is corrected with the weight drift accumulated since that version,
 *
 *     A_I(g, theta_new, theta_old) = g + lambda * g (.) g (.) (theta_new - theta_old)
 *                                            (Eq. "gt-taylor-expansion-approximation")
 *     g_{i+1} = A_I(g_i, V[s_{i+1}], V[s_i]),   i = 0 .. K'-1      (Alg. 1, iterative loop)
 *     theta_next = V[tau] - eta * g_{K'}                            (Alg. 1, model update)
 *
 * where V[0] is the version the gradient was computed on and V[tau] the current one.
 * Alg. 1 uses K' = tau and s_i = i.  With an iteration count K < tau the tau version
 * steps are cut into K' = min(K, tau) contiguous segments, s_i = floor(i*tau/K').
 *
 * Memory model.  Every device buffer and the stream belong to the caller; the library
 * allocates host memory only (inside the plan) and no device memory at all.  All device
 * pointers must be 16-byte aligned.  Calls enqueue work on `hip_stream` and return
 * without waiting; the returned status covers argument and launch errors only.
 * A plan is not thread-safe: use it from one thread at a time.
 *
 * Layout (all offsets in ELEMENTS, all obtainable from the plan):
 *   stage j      its tensors are laid end to end in model order, each starting at a
 *                multiple of FERRET_ALIGN_ELEMS; n_j = padded element count.  Padding
 *                elements take part in the arithmetic like any other element (keep them
 *                zero: zero gradient and zero weight stay zero).
 *   flat buffer  ("slot-shaped": grads, master, grad_out, src of push_version)
 *                stage j occupies [flat_offset_j, flat_offset_j + n_j).
 *   ring         stage-major: stage j owns an arena of ring_depth_j slots,
 *                slot s of stage j = [ring_offset_j + s*slot_stride_j, ... + n_j).
 *   storage type fp32 (FERRET_F32) or bf16 (FERRET_BF16_MASTER_F32) for ring and grads;
 *                master, grad_out, src are always fp32.
 *
 * Errors: every function returning ferret_status returns FERRET_OK or a code below and
 * leaves a message retrievable with ferret_last_error() (thread-local).  Nothing throws
 * or aborts.
 */
#ifndef FERRET_H
#define FERRET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FERRET_MAX_STAGES 64       /* stages per plan (the stage table travels as a kernel argument) */
#define FERRET_MAX_RING_DEPTH 4096
#define FERRET_ALIGN_ELEMS 8       /* tensor start alignment inside a stage, in elements */
#define FERRET_ITERS_FULL (-1)     /* n_iters: one iteration per version step (Alg. 1 literally) */
#define FERRET_RING_DEPTH_MINIMAL 0 /* ring_depth: stage j keeps tau_j + 1 versions, the paper's count
                                       (Sec. "Fine-grained Pipeline Parallelism", T2: P - j models) */

typedef enum {
    FERRET_OK = 0,
    FERRET_EINVAL = 1,   /* bad argument (null, misaligned, out of range) */
    FERRET_ESTATE = 2,   /* call not valid in the plan's current state */
    FERRET_ENOMEM = 3,   /* host allocation failed */
    FERRET_EDEVICE = 4   /* HIP reported an error on launch */
} ferret_status;

typedef enum {
    FERRET_F32 = 0,              /* fp32 versions and gradients */
    FERRET_BF16_MASTER_F32 = 1   /* bf16 versions and gradients, update applied to an fp32 master */
} ferret_precision;

/* One parameter tensor: element count and the pipeline stage that owns it.  A stage is a
 * contiguous run of layers (appendix "Notations": |w_j| = sum of |w^_i| over [L_j, L_{j+1})). */
typedef struct {
    int64_t numel;     /* > 0 */
    int32_t stage;     /* 0 .. n_stages-1, non-decreasing over the tensor list */
    int32_t reserved;  /* must be 0 */
} ferret_tensor;

/* Optional layout / launch tuning; zero in a field means "library default". */
typedef struct {
    int64_t slot_align_elems;  /* slot stride is rounded up to a multiple of this (multiple of 64) */
    int64_t slot_skew_elems;   /* then this is added (multiple of 8): de-phases the streams that
                                  read the same element of different slots */
    int64_t chunk_bytes;       /* only with chunk_elems = 0: every stage gets its own chunk size, the multiple of 1024
                                  elements nearest to chunk_bytes / (bytes one parameter of that stage has in flight
                                  in a step: gradient, the K'+1 versions -- 8 of them when K' > 8 --, new version,
                                  master read and write), so that every workgroup moves about chunk_bytes whatever
                                  the stage's K'; 0: 48 KiB for plans beyond 240 MiB, else 2048 elements throughout */
    int32_t blocks_per_cu;     /* >0: persistent grid of blocks_per_cu * (number of CUs) workgroups with
                                  the stage table staged in LDS; <0: one workgroup per chunk; 0: default */
    int32_t resident_cap;      /* >=2: at most this many workgroups resident per CU (enforced by reserving
                                  LDS that the kernel does not use; one workgroup can hold at most 64 KiB of a
                                  CU's 160 KiB, so 1 is not available); <0: no cap; 0: default */
    int32_t newest_from_master; /* FERRET_BF16_MASTER_F32 only.  1: the caller promises that in every stage the
                                  newest stored version equals the round-to-nearest-even bf16 of the master
                                  (always true when both come from ferret_push_version with a master and
                                  ferret_compensate_step); ferret_compensate_step, _noalloc and
                                  ferret_compensate_stages then recompute V[tau] from the master instead of
                                  reading it (2 bytes per parameter less).  If the promise is broken the drifts
                                  are taken against the wrong newest version.  The adaptive, accumulating and
                                  penalised steps always read V[tau] (same results, no saving); not available
                                  together with blocks_per_cu > 0.  0: read it. */
    int32_t cache_policy;      /* 0: plans whose ring, gradient and master together stay below 240 MiB (they
                                  remain in the 256 MB memory-side cache from step to step) run the plain step
                                  with ordinary cached accesses, everything else with non-temporal ones;
                                  1: cached wherever that variant exists; 2: always non-temporal.  Results are
                                  bit-identical either way. */
    int32_t xcd_group;         /* how the chunks of a launch are dealt to the GPU's 8 XCDs (workgroups go to them
                                  round-robin): 1: every XCD takes every eighth chunk; N > 1: every XCD takes runs of N
                                  consecutive chunks, i.e. a contiguous stretch of every stream; 0: 16 for fp32 plans
                                  that stream and whose median stage iterates at least three times (measured 2-3 %
                                  faster there), 1 otherwise (where grouping measured 1-3 % slower).  Results are
                                  bit-identical for any value. */
    int32_t reserved;          /* must be 0 */
} ferret_tuning;

typedef struct ferret_plan ferret_plan;   /* opaque; host memory; owned by the caller via destroy */

/* ---- planning (host only, no HIP call; Sec. "Model Partitioning and Pipeline Planning" says
 *      planning runs once, and this is the part of it that the update path consumes) ------------
 * Flattens the tensors of each stage into one bucket, fixes the layout above, cuts every
 * stage into chunks of chunk_elems elements (the unit of work of one workgroup; a chunk never
 * crosses a stage boundary) and records per stage tau_j.
 *   tensors, n_tensors  host array, model order, stage ids non-decreasing, every stage non-empty
 *   n_stages            1 .. FERRET_MAX_STAGES
 *   staleness           host int32[n_stages], 0 <= tau_j (and tau_j < ring_depth if that is > 0);
 *                       maximum staleness of stage j in a P-stage pipeline is P-1-j
 *   n_iters             K >= 0, or FERRET_ITERS_FULL
 *   ring_depth          R >= 1 versions kept per stage, or FERRET_RING_DEPTH_MINIMAL
 *   chunk_elems         0 = default: 2048 for plans whose ring, gradient and master together stay below 240 MiB
 *                       (they live in the memory-side cache); for larger plans per stage, about 48 KiB of traffic
 *                       per chunk (fp32: 2048 elements at K' = 3, 3072 at K' = 1, 1024 at K' >= 6; see
 *                       tuning->chunk_bytes); otherwise a multiple of 1024, at most 2^24, used for every stage
 *   tuning              NULL or options
 *   out_plan            receives the plan; heads start at slot 0 with no valid version
 */
ferret_status ferret_plan_buckets(const ferret_tensor *tensors, int32_t n_tensors,
                                  int32_t n_stages, const int32_t *staleness,
                                  int32_t n_iters, int32_t ring_depth,
                                  ferret_precision prec, int64_t chunk_elems,
                                  ferret_plan **out_plan);
ferret_status ferret_plan_buckets_tuned(const ferret_tensor *tensors, int32_t n_tensors,
                                        int32_t n_stages, const int32_t *staleness,
                                        int32_t n_iters, int32_t ring_depth,
                                        ferret_precision prec, int64_t chunk_elems,
                                        const ferret_tuning *tuning, ferret_plan **out_plan);
void ferret_plan_destroy(ferret_plan *plan);   /* NULL is allowed */

/* ---- plan queries (host; return -1 / 0 on a NULL plan or an index out of range) -------------- */
int32_t ferret_plan_n_stages(const ferret_plan *plan);
int32_t ferret_plan_n_tensors(const ferret_plan *plan);
int32_t ferret_plan_precision(const ferret_plan *plan);
int32_t ferret_plan_n_iters(const ferret_plan *plan);
int64_t ferret_plan_chunk_elems(const ferret_plan *plan);     /* the largest chunk size of any stage */
int64_t ferret_plan_n_chunks(const ferret_plan *plan);        /* over all stages */
int64_t ferret_plan_flat_elems(const ferret_plan *plan);      /* elements of a slot-shaped buffer */
int64_t ferret_plan_ring_elems(const ferret_plan *plan);      /* elements of the whole ring */
size_t ferret_plan_ring_bytes(const ferret_plan *plan);
size_t ferret_plan_grad_bytes(const ferret_plan *plan);       /* storage dtype */
size_t ferret_plan_master_bytes(const ferret_plan *plan);     /* fp32, flat_elems*4 (also grad_out, src) */
size_t ferret_plan_workspace_bytes(const ferret_plan *plan);  /* five floats per chunk: partial sums of the
                                                                  three norms and of the two lambda inner products */
int64_t ferret_plan_total_params(const ferret_plan *plan);    /* sum of tensor numel (no padding) */

int64_t ferret_plan_stage_params(const ferret_plan *plan, int32_t stage);      /* |w_j|, unpadded */
int64_t ferret_plan_stage_numel(const ferret_plan *plan, int32_t stage);       /* n_j, padded */
int64_t ferret_plan_stage_flat_offset(const ferret_plan *plan, int32_t stage);
int64_t ferret_plan_stage_ring_offset(const ferret_plan *plan, int32_t stage);
int64_t ferret_plan_stage_slot_stride(const ferret_plan *plan, int32_t stage);
int32_t ferret_plan_stage_ring_depth(const ferret_plan *plan, int32_t stage);
int32_t ferret_plan_stage_staleness(const ferret_plan *plan, int32_t stage);   /* configured tau_j */
int64_t ferret_plan_stage_chunk_elems(const ferret_plan *plan, int32_t stage); /* elements per chunk of this stage */
int64_t ferret_plan_stage_n_chunks(const ferret_plan *plan, int32_t stage);
int64_t ferret_plan_tensor_offset(const ferret_plan *plan, int32_t tensor);    /* inside its stage */

/* ---- ring state (host integers only) --------------------------------------------------------- */
/* head_j = slot holding the newest version; valid_j = versions held (0 .. ring_depth_j).
 * get/set let a caller checkpoint the state or adopt a ring it filled itself. */
ferret_status ferret_plan_get_state(const ferret_plan *plan, int32_t *heads, int32_t *valid);
ferret_status ferret_plan_set_state(ferret_plan *plan, const int32_t *heads, const int32_t *valid);
/* What the next step would do for `stage`: effective staleness min(tau_j, valid_j-1) (during
 * pipeline warm-up fewer than tau_j+1 versions exist), K', the K'+1 slots read oldest first
 * (returns their count, fills at most cap), and the slot written. */
int32_t ferret_plan_stage_effective_staleness(const ferret_plan *plan, int32_t stage);
int32_t ferret_plan_stage_effective_iters(const ferret_plan *plan, int32_t stage);
int32_t ferret_plan_stage_read_slots(const ferret_plan *plan, int32_t stage, int32_t *slots, int32_t cap);
int32_t ferret_plan_stage_write_slot(const ferret_plan *plan, int32_t stage);
/* Algorithmic bytes one step moves in the current state: per parameter, gradient + the K'+1
 * versions read + the new version (+ master read and write), each once. */
int64_t ferret_plan_step_bytes(const ferret_plan *plan);

/* ---- version store: push -------------------------------------------------------------------- */
/* The stage's version store (Alg. 1 inputs theta^{t-1} .. theta^{t+tau-1}; T2 in Sec.
 * "Fine-grained Pipeline Parallelism" for how many are kept) is a ring: the newest version
 * lives in slot head_j, the next one goes to (head_j+1) mod R_j and evicts the oldest.
 *   ring     device, ring_bytes, storage dtype
 *   master   device fp32 flat buffer or NULL; only with FERRET_BF16_MASTER_F32
 *   stage    0..n_stages-1, or -1 for every stage
 *   src      device fp32 flat buffer holding new weights, or NULL.
 *            src != NULL: for the chosen stage(s) write src (rounded to nearest-even bf16 when
 *              the ring is bf16) into slot (head+1) mod R, copy it to master if given, then
 *              advance head and count the version.  Use for initial weights or versions made
 *              elsewhere.
 *            src == NULL: commit only -- advance head and count the version that the preceding
 *              ferret_compensate_step wrote into that slot.  FERRET_ESTATE if no step has been
 *              issued for the stage since its last commit.
 *              A push with src != NULL while a step of the stage is still uncommitted goes to the same slot
 *              the step wrote, i.e. it replaces that step's version (the step is dropped, not committed).
 * The host state changes when the call returns; the copy itself is ordered on hip_stream.
 */
ferret_status ferret_push_version(ferret_plan *plan, void *ring, float *master, int32_t stage,
                                  const void *src, void *hip_stream);

/* ---- the step -------------------------------------------------------------------------------- */
/* One fused pass over every stage of the plan: load the stale gradient, the K'_j+1 boundary
 * versions, iterate A_I K'_j times in registers, apply the update and store the new version
 * into slot (head_j+1) mod R_j.  Does not advance heads: re-running it recomputes the same
 * slot from the same inputs, unless that slot is also the oldest version read (ring depth
 * tau_j+1), in which case the second run sees the first run's output -- commit with
 * ferret_push_version(.., src = NULL) before the next step.
 *   ring       device, storage dtype, layout above
 *   grads      device flat buffer, storage dtype: the stale gradient of every stage
 *   master     device fp32 flat buffer; required iff FERRET_BF16_MASTER_F32 (updated in place;
 *              the new version is round-to-nearest-even bf16 of the new master)
 *   lambda     compensation coefficient (a scalar, may change every call)
 *   lr         eta
 *   norms_out  device float[n_stages][3] or NULL: per stage sum g_0^2, sum g_K'^2,
 *              sum (V[tau]-V[0])^2 (deterministic: per-chunk partials summed in chunk order)
 *   grad_out   device fp32 flat buffer or NULL: the compensated gradient g_K' (for checks and
 *              for optimisers that want it)
 *   workspace  device, workspace_bytes; required iff norms_out != NULL; needs no initialisation, contents
 *              undefined after.  One workspace serves one call at a time: calls that may overlap (different
 *              streams) need separate workspaces.
 * FERRET_ESTATE if some stage holds no version yet.
 */
ferret_status ferret_compensate_step(const ferret_plan *plan, void *ring, const void *grads,
                                     float *master, float lambda, float lr, float *norms_out,
                                     void *grad_out, void *workspace, void *hip_stream);

/* ferret_compensate_step for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus
 * `workspace`, same kernels, bit-identical results; the per-chunk partial sums of the norms go through a
 * fixed array of FERRET_NOALLOC_MAX_CHUNKS * 20 bytes (5 MiB) that is part of the library's device code
 * (each GPU the library runs on holds it until the process ends).  The call allocates nothing, on the host
 * or the device, and neither does anything it calls; on its first use on a device it looks the array's
 * address up once (hipGetSymbolAddress, with that device current), so make that first call outside a
 * graph capture.  The device current on the calling thread must be the one that owns the buffers and the
 * stream.  FERRET_EINVAL if the plan has more than FERRET_NOALLOC_MAX_CHUNKS chunks (plan with a larger
 * chunk_elems, or use ferret_compensate_step).  All calls on one GPU share the one array: calls that
 * overlap in time on the same GPU (different streams or threads) race on it when norms_out is given;
 * with norms_out == NULL the array is not touched. */
#define FERRET_NOALLOC_MAX_CHUNKS 262144
ferret_status ferret_compensate_step_noalloc(const ferret_plan *plan, void *ring, const void *grads,
                                             float *master, float lambda, float lr, float *norms_out,
                                             void *grad_out, void *hip_stream);

/* The same step for some of the plan's stages only (in a pipeline the gradients of different stages
 * arrive at different times): stage j takes part iff active[j] != 0 (host int32[n_stages]).  Stages
 * left out are not read or written, their norms_out rows read 0, and they have nothing to commit.
 * For the stages that take part the result is bit-identical to ferret_compensate_step.  Only the stages that take
 * part need to hold a version (FERRET_ESTATE otherwise); the same holds for the mode array of the accumulating
 * steps and the active array of the adaptive one. */
ferret_status ferret_compensate_stages(const ferret_plan *plan, void *ring, const void *grads, float *master,
                                       const int32_t *active, float lambda, float lr, float *norms_out,
                                       void *grad_out, void *workspace, void *hip_stream);

/* ---- the step with self-tuned lambda --------------------------------------------------------- */
/* All of Alg. 1 including its "update lambda" block (Sec. "Iterative Gradient Compensation", Eq.
 * "lambda-objective-v1" and the moving averages after it).  Per stage j with effective staleness
 * >= 1, in this order and with the state as it is BEFORE the call:
 *     dv_r     = (1 - alpha) (g_0 - v_r)
 *     lambda_j = lambda_j + 2 eta_lambda ( <v_a, dv_r> - lambda_j <v_a, v_a> )
 *                (one gradient-descent step on || dv_r - lambda v_a ||^2; sums over the stage)
 *     v_r      = alpha v_r + (1 - alpha) g_0
 *     v_a      = alpha v_a + (1 - alpha) g_0 (.) g_0 (.) (V[1] - V[0])
 * and then the iterations and the update of ferret_compensate_step with the NEW lambda_j.
 * Stages whose effective staleness is 0 have nothing to compensate: their lambda_j, v_r, v_a stay
 * untouched.  The l2 term of the paper's objective is not part of Alg. 1 and is not applied.
 *   lambda       device float[n_stages], read and updated in place (one coefficient per stage:
 *                every stage runs its own instance of the algorithm)
 *   v_r, v_a     device fp32 flat buffers, updated in place; zero them before the first step
 *   alpha        moving-average coefficient, 0 <= alpha < 1
 *   eta_lambda   learning rate of lambda, >= 0 (0 leaves lambda and the averages untouched)
 * Other arguments as in ferret_compensate_step.  `workspace` is always required here (the two
 * inner products go through it before the norms do).  FERRET_EINVAL if the plan has n_iters = 0.
 * Implementation: one pass over g_0, v_r, v_a, V[0], V[1] that forms the two sums and the new
 * averages (28 bytes per fp32 parameter), a tiny kernel that steps lambda, then the same fused
 * kernel as ferret_compensate_step reading lambda_j from device memory.
 *   fused        0: the order above, which is Alg. 1's (two passes over the gradient).
 *                1: ONE pass.  The lambda block needs two sums over the whole stage before its result
 *                can scale anything, so a single pass cannot use the new lambda_j; instead the
 *                iterations of this call use lambda_j as it is BEFORE the call and lambda_j takes its
 *                step afterwards, i.e. every lambda step acts one call later than in Alg. 1.  The
 *                sequence of lambda_j, v_r, v_a for given gradients and versions is unchanged; with
 *                the paper's eta_lambda (about 1e-6) consecutive lambda_j differ in the sixth digit.
 *                Moves 16 + one stored version fewer bytes per parameter than the two passes.
 *   reserved     must be 0 */
typedef struct {
    float *lambda;
    float *v_r;
    float *v_a;
    float alpha;
    float eta_lambda;
    int32_t fused;
    int32_t reserved;
} ferret_adaptive;

ferret_status ferret_compensate_step_adaptive(const ferret_plan *plan, void *ring, const void *grads,
                                              float *master, const ferret_adaptive *adaptive, float lr,
                                              float *norms_out, void *grad_out, void *workspace,
                                              void *hip_stream);
/* The same for the stages j with active[j] != 0 only (host int32[n_stages]), as ferret_compensate_stages is to
 * ferret_compensate_step: stages left out keep their weights, lambda_j, v_r and v_a, and have nothing to commit. */
ferret_status ferret_compensate_stages_adaptive(const ferret_plan *plan, void *ring, const void *grads,
                                                float *master, const int32_t *active,
                                                const ferret_adaptive *adaptive, float lr, float *norms_out,
                                                void *grad_out, void *workspace, void *hip_stream);

/* ---- gradient accumulation (T2) -------------------------------------------------------------- */
/* Sec. "Fine-grained Pipeline Parallelism", T2: with c^a accumulation steps a stage applies one
 * update per c^a gradients and therefore keeps only 1 + ceil((P-j-1)/c^a) versions (plan the ring
 * with tau_j = ceil((P-j-1)/c^a) and FERRET_RING_DEPTH_MINIMAL).  The paper does not say how
 * compensation and accumulation compose; here every arriving gradient is compensated from the
 * version it was taken on to the stage's current version, then added to a running sum, and the
 * arrival that completes the group applies  theta_next = V[tau] - eta * scale * sum  and clears the
 * sum.  One call handles one arrival per participating stage:
 *   accum      device fp32 flat buffer, the running sums; zero it before the first arrival
 *   scale      1 for a sum of gradients, 1/c^a for their mean
 *   mode       host int32[n_stages]: 0 = stage takes no part in this call, 1 = accumulate only,
 *              2 = accumulate, update (new version into slot head+1) and clear the sum
 *   staleness  host int32[n_stages] or NULL: staleness of THIS gradient in stored versions,
 *              0 .. tau_j (it varies from arrival to arrival when c^a does not divide P-j-1);
 *              NULL = the plan's tau_j
 * Other arguments as in ferret_compensate_step; norms_out rows of skipped stages read 0.  Commit
 * the stages that were updated with ferret_push_version(.., stage, src = NULL).
 * (To step a subset of stages without accumulation use ferret_compensate_stages.) */
typedef struct {
    float *accum;
    float scale;
    const int32_t *mode;
    const int32_t *staleness;
} ferret_accumulate;

ferret_status ferret_accumulate_step(const ferret_plan *plan, void *ring, const void *grads, float *master,
                                     const ferret_accumulate *accumulate, float lambda, float lr,
                                     float *norms_out, void *grad_out, void *workspace, void *hip_stream);

/* Gradient accumulation with self-tuned lambda: Alg. 1 is run once per arriving gradient, so every
 * stage that takes part in the call (mode 1 or 2) and whose arrival has staleness >= 1 first runs the
 * "update lambda" block of ferret_compensate_step_adaptive on this gradient (V[0], V[1] counted from
 * the version THIS gradient was taken on), then compensates with the new lambda_j and accumulates as
 * ferret_accumulate_step does.  Stages with mode 0 keep lambda_j, v_r, v_a untouched.
 * adaptive->fused selects the order as in ferret_compensate_step_adaptive; `workspace` is required. */
ferret_status ferret_accumulate_step_adaptive(const ferret_plan *plan, void *ring, const void *grads,
                                              float *master, const ferret_accumulate *accumulate,
                                              const ferret_adaptive *adaptive, float lr, float *norms_out,
                                              void *grad_out, void *workspace, void *hip_stream);

/* ---- comparison methods that penalise the step size ------------------------------------------ */
/* The paper's comparison of compensation methods (Sec. "Comparisons on Gradients Compensation") names
 * "None", "Fisher", "Step-Aware", "Gap-Aware" beside its own.  "None" is n_iters = 0 and "Fisher"
 * n_iters = 1 of ferret_compensate_step.  The other two are only named there; the forms offered here
 * are this library's reading of those published methods, both instances of one update without
 * iterations,
 *     theta_next = V[tau] - eta * scale_j * g_0 / (|V[tau] - V[0]| * inv_c_j + 1):
 *   Step-Aware   scale_j = 1 / max(tau_j, 1), inv_c_j = 0   (step divided by the staleness)
 *   Gap-Aware    scale_j = 1, inv_c_j = 1 / C_j             (each element's step divided by its gap, the
 *                distance its weight moved since the stale snapshot in units of a typical step C_j)
 *   scale, inv_c  host float[n_stages], inv_c >= 0; NULL scale = the Step-Aware values for the plan's
 *                 current effective staleness, NULL inv_c = zeros
 * grad_out receives the penalised gradient; norms_out[.][1] equals norms_out[.][0] (no compensation).
 * Other arguments and the ring protocol (slot written, commit) as in ferret_compensate_step. */
ferret_status ferret_penalized_step(const ferret_plan *plan, void *ring, const void *grads, float *master,
                                    const float *scale, const float *inv_c, float lr, float *norms_out,
                                    void *grad_out, void *workspace, void *hip_stream);

/* ---- misc ------------------------------------------------------------------------------------ */
const char *ferret_last_error(void);   /* message of the calling thread's last failed call */
const char *ferret_version(void);      /* "libferret <version> (gfx950) src <hash>": hash of the sources it was built from */

/* Plain device-to-device copy through the library's own copy kernel (n_bytes multiple of 16,
 * 16-byte aligned pointers).  Measures the streaming ceiling of the machine with the same
 * launch shape as the step; not part of the method. */
ferret_status ferret_copy_bytes(void *dst, const void *src, size_t n_bytes, void *hip_stream);
/* Read-only companion: streams n_bytes from src and discards them (sink: device, >= 16 bytes, written
 * only in the practically impossible case that the data sums to a magic value; it exists so that the
 * loads cannot be optimised away).  The read ceiling of the machine for the same launch shape. */
ferret_status ferret_read_bytes(const void *src, size_t n_bytes, void *sink, void *hip_stream);
/* Mixed companion with the traffic shape of the step and none of its arithmetic: n_reads (1..8) streams
 * of n_bytes each, src_i = src + i * src_stride_bytes, are added element-wise as fp32 and written to dst
 * (n_bytes; must not overlap any source).  Non-temporal 16-byte accesses, one workgroup per 8 KiB of each
 * stream, all loads of a vector before its store, exactly like the step.  resident_cap > 0 limits the
 * workgroups resident per CU the way ferret_tuning.resident_cap does, <= 0 leaves it to the hardware.
 * n_bytes and src_stride_bytes multiples of 16, 16-byte aligned pointers.  What this kernel reaches for
 * "K'+2 reads + 1 write" is the ceiling for the step kernel on the machine at hand. */
ferret_status ferret_stream_mix(void *dst, const void *src, size_t src_stride_bytes, int32_t n_reads,
                                size_t n_bytes, int32_t resident_cap, void *hip_stream);

/* ---- measurement ------------------------------------------------------------------------------ */
/* Per-launch timing of the fused step kernel with HIP events recorded on the step's own stream,
 * immediately before and after that kernel (the norms' finalize kernel is outside the pair).
 * begin: create `capacity` event pairs; from then on every step launched by the CALLING THREAD records one
 *        pair until the capacity is used up (steps other threads launch meanwhile are not recorded).
 *        FERRET_ESTATE if a session is already open (one per process at a time).
 * end:   wait for the last recorded pair, write the durations in milliseconds (launch order) to the
 *        host array ms_out[0 .. min(cap, recorded)), store the number recorded in *n_out, destroy the
 *        events.  FERRET_ESTATE if begin was not called, or was called by another thread.
 * Safe to call from several threads (a mutex guards the session); meant for benchmarks. */
ferret_status ferret_profile_begin(int32_t capacity);
ferret_status ferret_profile_end(float *ms_out, int32_t cap, int32_t *n_out);

#ifdef __cplusplus
}
#endif
#endif /* FERRET_H */
