/*
 * CPU oracle for Ferret's iterative gradient compensation + weight update.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP
 * library's results are checked against.  It shares no code, header, table or helper
 * with the library, and nothing in the library's product path may call it.
 *
 * What it computes, for one pipeline stage (paper: Sec. "Iterative Gradient
 * Compensation", Eq. "gt-taylor-expansion-approximation", the un-numbered iteration
 * equation after it, and Alg. 1 "Iterative Gradients Compensation with lambda",
 * the "iterative approximation" loop and the "model update" line):
 *
 *   inputs   g_0            the stale gradient, taken on weight version V[0]
 *            V[0..tau]      the tau+1 stored weight versions, oldest first;
 *                           V[tau] is the current weights
 *            lambda, eta    compensation coefficient, learning rate
 *   one approximator step   A_I(g, th_new, th_old) = g + lambda * g (.) g (.) (th_new - th_old)
 *                           (elementwise: the Fisher matrix is cut to its diagonal)
 *   iteration               g_{i+1} = A_I(g_i, V[s_{i+1}], V[s_i]),  i = 0 .. K'-1
 *                           each step takes the previous step's OUTPUT as its gradient
 *   update                  theta_new = V[tau] - eta * g_{K'}
 *
 * Alg. 1 performs exactly tau iterations over adjacent versions (s_i = i).  This
 * oracle also accepts an iteration count K: K' = min(K, tau) (K < 0 means K' = tau),
 * and the tau version steps are cut into K' contiguous segments with boundaries
 * s_i = floor(i * tau / K'), so that s_0 = 0 and s_{K'} = tau.  With K >= tau this is
 * Alg. 1 literally; with K = 1 it is the single step over the whole drift.
 *
 * Arithmetic: every stored input (fp32, or bf16 widened exactly) is converted to
 * double, all arithmetic is IEEE double in the order written, and results are rounded
 * once on output.  No blocking, no reordering, no fused operations (compile without
 * -ffast-math and with -ffp-contract=off).
 *
 * Three extra sums per stage are returned (the squared norms the paper reasons with:
 * the approximation error / gradient magnitude of Sec. "Iterative Gradient
 * Compensation" and the weight gap used by gap-aware baselines):
 *   norms[0] = sum g_0^2,  norms[1] = sum g_{K'}^2,  norms[2] = sum (V[tau] - V[0])^2
 *
 * Parity status: pinned (hand-worked values, closed forms and invariants in
 * tests/test_oracle_pins.py).  The segment rule for K < tau is a reading of the
 * benchmark configurations, not of the paper; the paper itself only fixes K = tau.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ---- segment boundaries ------------------------------------------------------------ */

/* K' : number of approximator applications for staleness tau and iteration count K. */
int32_t ferret_oracle_effective_iters(int32_t K, int32_t tau)
{
    if (tau < 0) return 0;
    if (K < 0) return tau;
    return K < tau ? K : tau;
}

/* s_i = floor(i * tau / K'), i = 0..K'.  Undefined for K' = 0 (there is no loop). */
int32_t ferret_oracle_segment_boundary(int32_t i, int32_t tau, int32_t Kp)
{
    return (int32_t)(((int64_t)i * (int64_t)tau) / (int64_t)Kp);
}

/* ---- bf16 <-> fp32 ------------------------------------------------------------------ */

/* bf16 is the upper 16 bits of an IEEE binary32: widening is exact. */
float ferret_oracle_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Round an fp32 value to the nearest bf16, ties to the even mantissa; NaN stays NaN
 * (quiet bit forced so that a payload living only in the low 16 bits is not lost). */
uint16_t ferret_oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)          /* NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t keep = u >> 16;                      /* truncated result            */
    uint32_t rest = u & 0xffffu;                  /* the 16 bits being dropped   */
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u)))
        keep += 1u;                               /* may carry into exponent: that is correct (-> inf) */
    return (uint16_t)keep;
}

/* ---- one element -------------------------------------------------------------------- */

/* The iteration for a single parameter.  v[0..tau] are that parameter's stored
 * versions (already widened to double).  Returns g_{K'}. */
static double compensate_one(double g, const double *v, int32_t tau, int32_t Kp, double lambda)
{
    for (int32_t i = 0; i < Kp; ++i) {
        int32_t s_lo = ferret_oracle_segment_boundary(i, tau, Kp);
        int32_t s_hi = ferret_oracle_segment_boundary(i + 1, tau, Kp);
        double dtheta = v[s_hi] - v[s_lo];
        g = g + lambda * g * g * dtheta;
    }
    return g;
}

#define FERRET_ORACLE_MAX_VERSIONS 1024

/* ---- fp32 storage ------------------------------------------------------------------- */
/*
 * n            elements in the stage
 * n_versions   tau + 1  (>= 1)
 * V            n_versions host pointers to fp32 arrays of n elements, oldest first
 * g0           stale gradient, fp32[n]
 * K            iteration count (<0: one per version step)
 * theta_new    out fp32[n]: V[tau] - eta g_{K'}, rounded to fp32 (may alias any V[s]:
 *              every element is read before it is written)
 * g_out        out double[n] or NULL: g_{K'} unrounded
 * norms        out double[3]
 * n_threads    >1 splits the element loop with OpenMP (used only to time the oracle on
 *              all host cores); 1 gives the sequential reference
 * returns 0, or -1 on bad arguments
 */
int ferret_oracle_stage_f32(int64_t n, int32_t n_versions, const float *const *V,
                            const float *g0, int32_t K, double lambda, double eta,
                            float *theta_new, double *g_out, double *norms, int32_t n_threads)
{
    if (n < 0 || n_versions < 1 || n_versions > FERRET_ORACLE_MAX_VERSIONS) return -1;
    const int32_t tau = n_versions - 1;
    const int32_t Kp = ferret_oracle_effective_iters(K, tau);
    double sum_g0 = 0.0, sum_gk = 0.0, sum_gap = 0.0;

#pragma omp parallel for num_threads(n_threads) reduction(+ : sum_g0, sum_gk, sum_gap) if (n_threads > 1)
    for (int64_t e = 0; e < n; ++e) {
        double v[FERRET_ORACLE_MAX_VERSIONS];
        for (int32_t s = 0; s <= tau; ++s) v[s] = (double)V[s][e];
        double g_start = (double)g0[e];
        double g = compensate_one(g_start, v, tau, Kp, lambda);
        double updated = v[tau] - eta * g;
        double gap = v[tau] - v[0];
        theta_new[e] = (float)updated;
        if (g_out) g_out[e] = g;
        sum_g0 += g_start * g_start;
        sum_gk += g * g;
        sum_gap += gap * gap;
    }
    if (norms) { norms[0] = sum_g0; norms[1] = sum_gk; norms[2] = sum_gap; }
    return 0;
}

/* ---- bf16 storage with fp32 master -------------------------------------------------- */
/*
 * Mixed precision is not in the paper; the reading used: gradients and stored versions
 * are bf16 and widen exactly; the drifts are differences of the stored (bf16) versions,
 * because those are the weights the forward/backward passes really ran on; the update
 * is applied to an fp32 master copy, m_new = m - eta g_{K'}; the new stored version is
 * m_new (as fp32) rounded to bf16 with ties to even.
 *
 * V, g0, theta_new are bf16 bit patterns (uint16).  master / master_new are fp32[n]
 * and may alias each other.
 */
int ferret_oracle_stage_bf16(int64_t n, int32_t n_versions, const uint16_t *const *V,
                             const uint16_t *g0, const float *master, int32_t K,
                             double lambda, double eta, uint16_t *theta_new,
                             float *master_new, double *g_out, double *norms,
                             int32_t n_threads)
{
    if (n < 0 || n_versions < 1 || n_versions > FERRET_ORACLE_MAX_VERSIONS) return -1;
    const int32_t tau = n_versions - 1;
    const int32_t Kp = ferret_oracle_effective_iters(K, tau);
    double sum_g0 = 0.0, sum_gk = 0.0, sum_gap = 0.0;

#pragma omp parallel for num_threads(n_threads) reduction(+ : sum_g0, sum_gk, sum_gap) if (n_threads > 1)
    for (int64_t e = 0; e < n; ++e) {
        double v[FERRET_ORACLE_MAX_VERSIONS];
        for (int32_t s = 0; s <= tau; ++s) v[s] = (double)ferret_oracle_bf16_to_f32(V[s][e]);
        double g_start = (double)ferret_oracle_bf16_to_f32(g0[e]);
        double g = compensate_one(g_start, v, tau, Kp, lambda);
        double updated = (double)master[e] - eta * g;
        double gap = v[tau] - v[0];
        float m_new = (float)updated;
        master_new[e] = m_new;
        theta_new[e] = ferret_oracle_f32_to_bf16(m_new);
        if (g_out) g_out[e] = g;
        sum_g0 += g_start * g_start;
        sum_gk += g * g;
        sum_gap += gap * gap;
    }
    if (norms) { norms[0] = sum_g0; norms[1] = sum_gk; norms[2] = sum_gap; }
    return 0;
}

/* ==== adaptive lambda (Alg. 1, block "update lambda") ===================================
 *
 * Before the iterations, when eta_lambda > 0, Alg. 1 takes one gradient-descent step on
 *     || dv_r - lambda * v_a ||^2         (Eq. "lambda-objective-v1" with D - E and F
 *                                          replaced by their moving averages)
 * where, with the state BEFORE this call,
 *     dv_r = (1 - alpha) * (g_0 - v_r)                          (the "D - E" equation)
 *     d/dlambda ||dv_r - lambda v_a||^2 = -2 * < v_a, dv_r - lambda v_a >
 *     lambda <- lambda - eta_lambda * that derivative
 *             = lambda + 2 eta_lambda ( <v_a, dv_r> - lambda <v_a, v_a> )
 * and then moves the two exponential moving averages
 *     v_r <- alpha v_r + (1 - alpha) g_0
 *     v_a <- alpha v_a + (1 - alpha) g_0 (.) g_0 (.) (V[1] - V[0])
 * (V[1] - V[0] is the first version step after the snapshot the gradient was taken on).
 * The l2 term of the objective does not appear in Alg. 1 and is not applied.
 *
 * Reading for tau = 0: no later version exists, the expression V[1] - V[0] is undefined
 * and nothing is compensated, so the caller skips this block (state and lambda unchanged).
 *
 * State arrays are fp32 in storage; arithmetic is double, rounded once on output.
 * v_r_new / v_a_new may alias v_r / v_a.  Returns the new lambda (unrounded double).
 * `bf16` selects the storage type of g0 / V0 / V1 (uint16 bit patterns) versus fp32.
 */
static double widen_at(const void *p, int64_t e, int bf16)
{
    return bf16 ? (double)ferret_oracle_bf16_to_f32(((const uint16_t *)p)[e])
                : (double)((const float *)p)[e];
}

double ferret_oracle_lambda_update(int64_t n, const void *g0, const void *V0, const void *V1,
                                   int32_t bf16, double lambda, double alpha, double eta_lambda,
                                   const float *v_r, const float *v_a,
                                   float *v_r_new, float *v_a_new, double *sums /* nullable: <v_a,dv_r>, <v_a,v_a> */)
{
    double dot_a_dr = 0.0, dot_a_a = 0.0;
    for (int64_t e = 0; e < n; ++e) {
        double g = widen_at(g0, e, bf16);
        double dv_r = (1.0 - alpha) * (g - (double)v_r[e]);
        dot_a_dr += (double)v_a[e] * dv_r;
        dot_a_a += (double)v_a[e] * (double)v_a[e];
    }
    double derivative = -2.0 * (dot_a_dr - lambda * dot_a_a);
    double lambda_new = lambda - eta_lambda * derivative;
    for (int64_t e = 0; e < n; ++e) {
        double g = widen_at(g0, e, bf16);
        double first_step = widen_at(V1, e, bf16) - widen_at(V0, e, bf16);
        double r = alpha * (double)v_r[e] + (1.0 - alpha) * g;
        double a = alpha * (double)v_a[e] + (1.0 - alpha) * (g * g * first_step);
        v_r_new[e] = (float)r;
        v_a_new[e] = (float)a;
    }
    if (sums) { sums[0] = dot_a_dr; sums[1] = dot_a_a; }
    return lambda_new;
}

/* ==== gradient accumulation (T2 of Sec. "Fine-grained Pipeline Parallelism") ==============
 *
 * With c^a accumulation steps a stage applies one update per c^a gradients, which is why it
 * only has to keep 1 + ceil((P-j-1)/c^a) versions.  The paper does not say how compensation
 * and accumulation compose; the reading used here: every arriving gradient is first
 * compensated from the version it was taken on to the stage's CURRENT version (Alg. 1's
 * iterations, with that gradient's own staleness tau, counted in stored versions), then added
 * to the running sum; the arrival that completes the group applies
 *     theta_next = V[tau] - eta * scale * (sum of the compensated gradients)
 * and clears the sum.  scale is 1 for a plain sum, 1/c^a for a mean.  With c^a = 1 (sum empty
 * on entry, scale 1) this is Alg. 1 itself.
 *
 * accum_in / accum_out  fp32[n] (may alias)
 * do_update             0: accumulate only (theta_new, master_new untouched)
 *                       1: accumulate, update, clear the sum
 * bf16                  storage type of V, g0, theta_new (uint16 bit patterns) vs fp32;
 *                       with bf16 the update goes to the fp32 master (master, master_new)
 */
int ferret_oracle_accumulate(int64_t n, int32_t n_versions, const void *const *V, const void *g0,
                             int32_t bf16, const float *master, int32_t K, double lambda, double eta,
                             double scale, int32_t do_update, const float *accum_in, float *accum_out,
                             void *theta_new, float *master_new, double *g_out)
{
    if (n < 0 || n_versions < 1 || n_versions > FERRET_ORACLE_MAX_VERSIONS) return -1;
    const int32_t tau = n_versions - 1;
    const int32_t Kp = ferret_oracle_effective_iters(K, tau);
    for (int64_t e = 0; e < n; ++e) {
        double v[FERRET_ORACLE_MAX_VERSIONS];
        for (int32_t s = 0; s <= tau; ++s) v[s] = widen_at(V[s], e, bf16);
        double g = compensate_one(widen_at(g0, e, bf16), v, tau, Kp, lambda);
        double total = (double)accum_in[e] + g;
        if (g_out) g_out[e] = g;
        if (!do_update) {
            accum_out[e] = (float)total;
            continue;
        }
        double base = bf16 ? (double)master[e] : v[tau];
        float updated = (float)(base - eta * scale * total);
        if (bf16) {
            master_new[e] = updated;
            ((uint16_t *)theta_new)[e] = ferret_oracle_f32_to_bf16(updated);
        } else {
            ((float *)theta_new)[e] = updated;
        }
        accum_out[e] = 0.0f;
    }
    return 0;
}

/* ==== step-size-penalising comparison methods ============================================
 *
 * The paper's comparison of gradient-compensation methods (Sec. "Comparisons on Gradients
 * Compensation") names two methods that, in its words, mitigate staleness by penalising the
 * step size of stale gradients, "Step-Aware" and "Gap-Aware", without giving formulas.  The
 * forms used here (this repository's reading of those published methods, not the paper's):
 *   Step-Aware   the step of a gradient with staleness tau is divided by tau:
 *                  theta_next = V[tau] - (eta / max(tau, 1)) * g_0
 *   Gap-Aware    every element's step is divided by its gap, the distance the weight has moved
 *                since the stale snapshot measured in units of a typical step size C:
 *                  G = |V[tau] - V[0]| / C + 1,   theta_next = V[tau] - eta * g_0 / G
 * Both are the one update
 *     theta_next = V[tau] - eta * scale * g_0 / (|V[tau] - V[0]| * inv_c + 1)
 * with (scale, inv_c) = (1/max(tau,1), 0) and (1, 1/C).  No iteration takes place; g_out is the
 * penalised gradient scale * g_0 / G.  bf16 storage: update on the fp32 master as elsewhere.
 * Parity status: pinned against closed forms and a hand-worked example; unpinned against the
 * paper, which prints no formula for these methods.
 */
int ferret_oracle_penalized(int64_t n, const void *V0, const void *Vtau, const void *g0, int32_t bf16,
                            const float *master, double eta, double scale, double inv_c,
                            void *theta_new, float *master_new, double *g_out)
{
    if (n < 0) return -1;
    for (int64_t e = 0; e < n; ++e) {
        double newest = widen_at(Vtau, e, bf16);
        double gap = fabs(newest - widen_at(V0, e, bf16)) * inv_c + 1.0;
        double g = scale * widen_at(g0, e, bf16) / gap;
        double base = bf16 ? (double)master[e] : newest;
        float updated = (float)(base - eta * g);
        if (g_out) g_out[e] = g;
        if (bf16) {
            master_new[e] = updated;
            ((uint16_t *)theta_new)[e] = ferret_oracle_f32_to_bf16(updated);
        } else {
            ((float *)theta_new)[e] = updated;
        }
    }
    return 0;
}
