// Pipeline planner of libferret (host only): cost model, Alg. 2 "Iterative Configuration Search" and
// Alg. 3 "Brute-force planning" of the paper, behind the C ABI of include/ferret_planner.h.
//
// The search keeps each worker's rate and memory share cached: a move touches one worker, so one
// round of the while-loop costs O(moves * P * c^a) instead of re-evaluating every worker.
#pragma STDC FP_CONTRACT OFF   // plain IEEE double operations: decisions between near-equal merits must not
                               // depend on whether the compiler fused a multiply-add
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <limits>
#include <new>
#include <numeric>
#include <thread>
#include <vector>

#include "ferret_internal.h"
#include "ferret_planner.h"

namespace {

using ferret::set_error;

struct StageAgg {
    std::vector<double> w, a, inner;   // |w_j|, |a_j|, activations T1 frees in stage j
    double t_f = 0, t_b = 0, total_w = 0;
    int P() const { return (int)w.size(); }
};

struct Worker {
    int delay = 0;
    int recompute = 0;
    std::vector<int> accum, omit;
};

struct Move { int worker, kind, stage; };

bool aggregate(const ferret_layer *layers, int n_layers, const int32_t *L, int P, StageAgg &S) {
    if (P < 1 || L[0] != 0 || L[P] != n_layers) return false;
    S.w.assign(P, 0); S.a.assign(P, 0); S.inner.assign(P, 0);
    S.t_f = S.t_b = 0;
    for (int j = 0; j < P; ++j) {
        if (L[j + 1] <= L[j]) return false;
        double tf = 0, tb = 0;
        for (int l = L[j]; l < L[j + 1]; ++l) {
            S.w[j] += layers[l].n_params;
            S.a[j] += layers[l].n_acts;
            if (l > L[j]) S.inner[j] += layers[l].n_acts;
            tf += layers[l].t_f;
            tb += layers[l].t_b;
        }
        S.t_f = std::max(S.t_f, tf);
        S.t_b = std::max(S.t_b, tb);
    }
    S.total_w = std::accumulate(S.w.begin(), S.w.end(), 0.0);
    return true;
}

inline long long lcm_ll(long long x, long long y) { return x / std::gcd(x, y) * y; }

// rate share of one live worker: sum_i w_i/W * 1/c^a_i * sum_{j<c^a_i} A_{i,j}
double worker_rate(const StageAgg &S, const Worker &wk, double c, double v_d) {
    const int P = S.P();
    const double r = wk.recompute;
    const double period = S.t_f + S.t_b + r * S.t_f;
    // suffix LCM of (c^o_k + 1), k = i..P-1
    std::vector<long long> suffix(P + 1, 1);
    for (int k = P - 1; k >= 0; --k) suffix[k] = lcm_ll(suffix[k + 1], wk.omit[k] + 1);
    double rate = 0;
    for (int i = 0; i < P; ++i) {
        const int ca = wk.accum[i];
        double s = 0;
        for (int j = 0; j < ca; ++j) {
            const double expo = -c * ((P + j) * S.t_f + (P - i + j) * S.t_b + r * (P - i + j) * S.t_f);
            s += std::exp(expo) * v_d / ((double)suffix[i] * period);
        }
        rate += S.w[i] / S.total_w * (1.0 / ca) * s;
    }
    return rate;
}

inline int ceil_div(int x, int y) { return (x + y - 1) / y; }

double worker_memory(const StageAgg &S, const Worker &wk) {
    const int P = S.P();
    double m = 0;
    for (int i = 0; i < P; ++i) {
        const int versions = 1 + ceil_div(P - i - 1, wk.accum[i]) - wk.omit[i];
        m += versions * (S.w[i] + S.a[i] - wk.recompute * S.inner[i]);
    }
    return m;
}

// S2: smallest c^a' that lowers ceil((P-j-1)/c^a); 0 if none.
int next_accum(int P, int j, int ca) {
    const int d = P - j - 1;
    const int cur = d > 0 ? ceil_div(d, ca) : 0;
    return cur < 2 ? 0 : ceil_div(d, cur - 1);
}

struct SearchResult {
    bool feasible = false;
    std::vector<Worker> workers;
    std::vector<Move> trace;
    double rate = 0, memory = 0;
};

// Alg. 2 for one value of c^r.  Everything a candidate move needs is cached so that a round of the
// while-loop costs O(N P (P + N)) additions and no exponentials:
//   numer[i][k]   exp(-c((P+k) t^f + (P-i+k) t^b + c^r (P-i+k) t^f)) V_D, shared by all workers
//   term[n][i]    stage i's share of worker n's rate, |w_i|/W * 1/c^a * sum_k numer[i][k]/(lcm_i * period)
// and every sum is formed in the same order as a plain evaluation of the cost model would form it
// (stage terms left to right, A_{i,k} for k = 0, 1, ..., workers in index order), so the decisions
// do not depend on the caching.
SearchResult itersearch(const StageAgg &S, double t_d, int c_r, double M, double c, double v_d) {
    const int P = S.P();
    SearchResult out;
    const int N = (int)std::ceil((S.t_f + S.t_b + c_r * S.t_f) / t_d);
    const double r = c_r, period = S.t_f + S.t_b + r * S.t_f;

    std::vector<std::vector<double>> numer(P);
    auto numerator = [&](int i, int k) -> double {
        std::vector<double> &row = numer[i];
        while ((int)row.size() <= k) {
            const int j = (int)row.size();
            const double expo = -c * ((P + j) * S.t_f + (P - i + j) * S.t_b + r * (P - i + j) * S.t_f);
            row.push_back(std::exp(expo) * v_d);
        }
        return row[k];
    };
    // stage i's term for accumulation steps ca and LCM denominator lcm
    auto stage_term = [&](int i, int ca, long long lcm) {
        double sum = 0;
        for (int k = 0; k < ca; ++k) sum += numerator(i, k) / ((double)lcm * period);
        return S.w[i] / S.total_w * (1.0 / ca) * sum;
    };
    auto suffix_lcm = [&](const Worker &wk, std::vector<long long> &suf) {
        suf.assign(P + 1, 1);
        for (int k = P - 1; k >= 0; --k) suf[k] = lcm_ll(suf[k + 1], wk.omit[k] + 1);
    };
    auto stage_mem = [&](const Worker &wk, int i) {
        const int versions = 1 + ceil_div(P - i - 1, wk.accum[i]) - wk.omit[i];
        return versions * (S.w[i] + S.a[i] - wk.recompute * S.inner[i]);
    };

    out.workers.resize(N);
    std::vector<std::vector<double>> term(N, std::vector<double>(P)), memt(N, std::vector<double>(P));
    std::vector<double> rate(N), mem(N);
    std::vector<long long> suf;
    auto refresh = [&](int n) {          // recompute worker n's cached terms and sums from its configuration
        const Worker &wk = out.workers[n];
        suffix_lcm(wk, suf);
        double rr = 0, mm = 0;
        for (int i = 0; i < P; ++i) {
            term[n][i] = stage_term(i, wk.accum[i], suf[i]);
            memt[n][i] = stage_mem(wk, i);
            rr += term[n][i];
            mm += memt[n][i];
        }
        rate[n] = rr; mem[n] = mm;
    };
    for (int n = 0; n < N; ++n) {
        Worker &wk = out.workers[n];
        wk.delay = n; wk.recompute = c_r;
        wk.accum.assign(P, 1); wk.omit.assign(P, 0);
        refresh(n);
    }
    auto total = [&](const std::vector<double> &x) {
        double t = 0;
        for (int n = 0; n < N; ++n) if (out.workers[n].delay >= 0) t += x[n];
        return t;
    };
    double R = total(rate), Mem = total(mem);
    std::vector<double> cand_term(P), cand_mem(P);
    while (Mem > M) {
        bool found = false;
        double best_merit = -1;
        Move best{};
        // totals with worker n replaced by (r2, m2), or dropped
        auto consider = [&](int n, int kind, int j, double r2, double m2, bool removed) {
            double R2 = 0, M2 = 0;
            for (int k = 0; k < N; ++k) {
                if (out.workers[k].delay < 0) continue;
                if (k == n) { if (!removed) { R2 += r2; M2 += m2; } }
                else { R2 += rate[k]; M2 += mem[k]; }
            }
            const double dR = R2 - R, dM = M2 - Mem;
            if (dM >= 0) return;
            const double merit = dR >= 0 ? std::numeric_limits<double>::infinity() : dM / dR;
            if (merit > best_merit) { found = true; best_merit = merit; best = Move{n, kind, j}; }
        };
        for (int n = 0; n < N; ++n) {
            const Worker &wk = out.workers[n];
            if (wk.delay < 0) continue;
            suffix_lcm(wk, suf);
            for (int j = 0; j + 1 < P; ++j) {           // S2: only stage j's term and memory change
                const int nxt = next_accum(P, j, wk.accum[j]);
                if (wk.omit[j] != 0 || nxt == 0) continue;
                const double tj = stage_term(j, nxt, suf[j]);
                const double mj = (1 + ceil_div(P - j - 1, nxt)) * (S.w[j] + S.a[j] - wk.recompute * S.inner[j]);
                double r2 = 0, m2 = 0;
                for (int i = 0; i < P; ++i) { r2 += i == j ? tj : term[n][i]; m2 += i == j ? mj : memt[n][i]; }
                consider(n, 2, j, r2, m2, false);
            }
            for (int j = 0; j + 1 < P; ++j) {           // S3: the LCM of every stage i <= j changes
                if (wk.omit[j] != 0 || ceil_div(P - j - 1, wk.accum[j]) != 1) continue;
                long long lcm = lcm_ll(suf[j + 1], (long long)(P - 1 - j) + 1);
                double r2 = 0, m2 = 0;
                for (int i = j; i >= 0; --i) {
                    if (i < j) lcm = lcm_ll(lcm, wk.omit[i] + 1);
                    cand_term[i] = stage_term(i, i == j ? 1 : wk.accum[i], lcm);
                }
                const double mj = (1 + ceil_div(P - j - 1, 1) - (P - 1 - j)) * (S.w[j] + S.a[j] - wk.recompute * S.inner[j]);
                for (int i = 0; i < P; ++i) { r2 += i <= j ? cand_term[i] : term[n][i]; m2 += i == j ? mj : memt[n][i]; }
                consider(n, 3, j, r2, m2, false);
            }
            bool all_omitted = true;
            for (int j = 0; j + 1 < P; ++j) all_omitted &= wk.omit[j] != 0;
            if (all_omitted) consider(n, 4, -1, 0.0, 0.0, true);
        }
        if (!found) { out.feasible = false; out.rate = 0; out.memory = Mem; return out; }
        Worker &wk = out.workers[best.worker];
        if (best.kind == 2) wk.accum[best.stage] = next_accum(P, best.stage, wk.accum[best.stage]);
        else if (best.kind == 3) { wk.accum[best.stage] = 1; wk.omit[best.stage] = P - 1 - best.stage; }
        else wk.delay = -1;
        if (wk.delay >= 0) refresh(best.worker);
        out.trace.push_back(best);
        R = total(rate);
        Mem = total(mem);
    }
    out.feasible = true; out.rate = R; out.memory = Mem;
    return out;
}

SearchResult search(const StageAgg &S, double t_d, double M, double c, double v_d) {
    SearchResult r0 = itersearch(S, t_d, 0, M, c, v_d), r1 = itersearch(S, t_d, 1, M, c, v_d);
    return r1.rate > r0.rate ? r1 : r0;
}

bool check_layers(const char *who, const ferret_layer *layers, int32_t n_layers) {
    if (!layers || n_layers < 1) { set_error("%s: need at least one layer", who); return false; }
    for (int i = 0; i < n_layers; ++i)
        if (!(layers[i].t_f > 0) || !(layers[i].t_b > 0) || !(layers[i].n_params >= 0) || !(layers[i].n_acts >= 0)) {
            set_error("%s: layer %d needs t_f > 0, t_b > 0, n_params >= 0, n_acts >= 0", who, i);
            return false;
        }
    return true;
}

}  // namespace

struct ferret_pipeline {
    std::vector<int32_t> L;
    SearchResult res;
    double t_c = 0;
};

extern "C" {

ferret_status ferret_pipeline_evaluate(const ferret_layer *layers, int32_t n_layers, const int32_t *L,
                                       int32_t n_stages, int32_t n_workers, const int32_t *delay,
                                       const int32_t *recompute, const int32_t *accum, const int32_t *omit,
                                       double c, double v_d, double *rate_out, double *memory_out) {
    const char *who = "pipeline_evaluate";
    if (!check_layers(who, layers, n_layers)) return FERRET_EINVAL;
    if (!L || !delay || !recompute || !accum || !omit || !rate_out || !memory_out || n_workers < 0) {
        set_error("%s: null argument", who); return FERRET_EINVAL;
    }
    StageAgg S;
    if (n_stages < 1 || !aggregate(layers, n_layers, L, n_stages, S)) {
        set_error("%s: L must run 0 = L[0] < ... < L[P] = n_layers", who); return FERRET_EINVAL;
    }
    if (!(S.total_w > 0)) { set_error("%s: the model has no parameters", who); return FERRET_EINVAL; }
    double R = 0, M = 0;
    for (int n = 0; n < n_workers; ++n) {
        if (delay[n] < 0) continue;
        Worker wk;
        wk.delay = delay[n]; wk.recompute = recompute[n] ? 1 : 0;
        wk.accum.assign(accum + (size_t)n * n_stages, accum + (size_t)(n + 1) * n_stages);
        wk.omit.assign(omit + (size_t)n * n_stages, omit + (size_t)(n + 1) * n_stages);
        for (int j = 0; j < n_stages; ++j)
            if (wk.accum[j] < 1 || wk.omit[j] < 0) {
                set_error("%s: worker %d stage %d: c^a = %d, c^o = %d", who, n, j, wk.accum[j], wk.omit[j]);
                return FERRET_EINVAL;
            }
        R += worker_rate(S, wk, c, v_d);
        M += worker_memory(S, wk);
    }
    *rate_out = R; *memory_out = M;
    return FERRET_OK;
}

ferret_status ferret_pipeline_search(const ferret_layer *layers, int32_t n_layers, const int32_t *L,
                                     int32_t n_stages, double t_d, double memory_budget, double c, double v_d,
                                     ferret_pipeline **out) {
    const char *who = "pipeline_search";
    if (out) *out = nullptr;
    if (!check_layers(who, layers, n_layers)) return FERRET_EINVAL;
    if (!L || !out || !(t_d > 0)) { set_error("%s: null argument or t_d <= 0", who); return FERRET_EINVAL; }
    StageAgg S;
    if (n_stages < 1 || !aggregate(layers, n_layers, L, n_stages, S) || !(S.total_w > 0)) {
        set_error("%s: bad partition or a model without parameters", who); return FERRET_EINVAL;
    }
    if ((S.t_f + S.t_b + S.t_f) / t_d > 4096) { set_error("%s: more than 4096 workers needed", who); return FERRET_EINVAL; }
    ferret_pipeline *p = new (std::nothrow) ferret_pipeline();
    if (!p) { set_error("%s: out of host memory", who); return FERRET_ENOMEM; }
    p->L.assign(L, L + n_stages + 1);
    p->res = search(S, t_d, memory_budget, c, v_d);
    *out = p;
    return FERRET_OK;
}

ferret_status ferret_pipeline_plan(const ferret_layer *layers, int32_t n_layers, double t_d,
                                   double memory_budget, double c, double v_d, ferret_pipeline **out) {
    const char *who = "pipeline_plan";
    if (out) *out = nullptr;
    if (!check_layers(who, layers, n_layers)) return FERRET_EINVAL;
    if (!out || !(t_d > 0)) { set_error("%s: null argument or t_d <= 0", who); return FERRET_EINVAL; }
    std::vector<double> per(n_layers);
    double largest = 0, total_w = 0;
    for (int i = 0; i < n_layers; ++i) {
        per[i] = layers[i].t_f + layers[i].t_b;
        largest = std::max(largest, per[i]);
        total_w += layers[i].n_params;
    }
    if (!(total_w > 0)) { set_error("%s: the model has no parameters", who); return FERRET_EINVAL; }
    // candidate bounds: every run of consecutive layers, summed left to right
    std::vector<double> bounds;
    for (int k = 0; k < n_layers; ++k)
        for (int i = 0; i + k < n_layers; ++i) {
            double t = 0;
            for (int l = i; l <= i + k; ++l) t += per[l];
            if (t >= largest) bounds.push_back(t);
        }
    std::sort(bounds.begin(), bounds.end());
    bounds.erase(std::unique(bounds.begin(), bounds.end()), bounds.end());

    ferret_pipeline *best = new (std::nothrow) ferret_pipeline();
    if (!best) { set_error("%s: out of host memory", who); return FERRET_ENOMEM; }
    // the distinct partitions, in the order of their bounds (consecutive bounds often give the same one)
    struct Candidate { std::vector<int32_t> L; double t_c; StageAgg S; SearchResult res; };
    std::vector<Candidate> cands;
    for (double t_c : bounds) {
        std::vector<int32_t> L{0};
        double t_sum = 0;
        for (int i = 0; i < n_layers; ++i) {
            t_sum += per[i];
            if (t_sum > t_c) { L.push_back(i); t_sum = per[i]; }
        }
        L.push_back(n_layers);
        if (!cands.empty() && L == cands.back().L) continue;      // same partition as the smaller bound before it
        Candidate cd;
        aggregate(layers, n_layers, L.data(), (int)L.size() - 1, cd.S);
        if ((cd.S.t_f + cd.S.t_b + cd.S.t_f) / t_d > 4096) continue;
        cd.L = std::move(L);
        cd.t_c = t_c;
        cands.push_back(std::move(cd));
    }
    // every partition is searched on its own; the searches share nothing, so they run on several threads and
    // the winner is then picked in bound order with a strict comparison, exactly as a serial loop would
    unsigned n_threads = std::thread::hardware_concurrency();
    if (const char *env = std::getenv("FERRET_PLANNER_THREADS")) n_threads = (unsigned)std::max(1, std::atoi(env));
    n_threads = std::max(1u, std::min({n_threads, 16u, (unsigned)cands.size()}));
    std::atomic<size_t> next{0};
    std::atomic<bool> failed{false};
    auto work = [&]() {
        try {
            for (size_t i = next++; i < cands.size(); i = next++)
                cands[i].res = search(cands[i].S, t_d, memory_budget, c, v_d);
        } catch (...) { failed = true; }
    };
    {
        std::vector<std::thread> pool;
        try {
            for (unsigned t = 1; t < n_threads; ++t) pool.emplace_back(work);
        } catch (...) { /* fewer threads than asked for: the calling thread does the rest */ }
        work();
        for (std::thread &t : pool) t.join();
    }
    if (failed) { delete best; set_error("%s: out of host memory", who); return FERRET_ENOMEM; }
    for (Candidate &cd : cands)
        if (cd.res.rate > best->res.rate) { best->res = std::move(cd.res); best->L = std::move(cd.L); best->t_c = cd.t_c; }
    *out = best;
    return FERRET_OK;
}

void ferret_pipeline_destroy(ferret_pipeline *p) { delete p; }

int32_t ferret_pipeline_feasible(const ferret_pipeline *p) { return p && p->res.feasible ? 1 : 0; }
int32_t ferret_pipeline_n_stages(const ferret_pipeline *p) { return p && !p->L.empty() ? (int32_t)p->L.size() - 1 : 0; }
int32_t ferret_pipeline_n_workers(const ferret_pipeline *p) { return p ? (int32_t)p->res.workers.size() : 0; }
int32_t ferret_pipeline_stage_begin(const ferret_pipeline *p, int32_t j) {
    return p && j >= 0 && j < (int32_t)p->L.size() ? p->L[j] : -1;
}
double ferret_pipeline_rate(const ferret_pipeline *p) { return p ? p->res.rate : 0.0; }
double ferret_pipeline_memory(const ferret_pipeline *p) { return p ? p->res.memory : 0.0; }
double ferret_pipeline_stage_bound(const ferret_pipeline *p) { return p ? p->t_c : 0.0; }

#define WORKER_OR(ret) \
    if (!p || n < 0 || n >= (int32_t)p->res.workers.size()) return ret; \
    const Worker &wk = p->res.workers[n]
int32_t ferret_pipeline_worker_delay(const ferret_pipeline *p, int32_t n) { WORKER_OR(-1); return wk.delay; }
int32_t ferret_pipeline_worker_recompute(const ferret_pipeline *p, int32_t n) { WORKER_OR(-1); return wk.recompute; }
int32_t ferret_pipeline_worker_accum(const ferret_pipeline *p, int32_t n, int32_t j) {
    WORKER_OR(-1); return j >= 0 && j < (int32_t)wk.accum.size() ? wk.accum[j] : -1;
}
int32_t ferret_pipeline_worker_omit(const ferret_pipeline *p, int32_t n, int32_t j) {
    WORKER_OR(-1); return j >= 0 && j < (int32_t)wk.omit.size() ? wk.omit[j] : -1;
}
int32_t ferret_pipeline_stage_versions(const ferret_pipeline *p, int32_t n, int32_t j) {
    WORKER_OR(-1);
    const int P = (int)wk.accum.size();
    if (j < 0 || j >= P) return -1;
    return 1 + ceil_div(P - j - 1, wk.accum[j]) - wk.omit[j];
}
int32_t ferret_pipeline_n_moves(const ferret_pipeline *p) { return p ? (int32_t)p->res.trace.size() : 0; }
ferret_status ferret_pipeline_move(const ferret_pipeline *p, int32_t k, int32_t *worker, int32_t *kind,
                                   int32_t *stage) {
    if (!p || !worker || !kind || !stage || k < 0 || k >= (int32_t)p->res.trace.size()) {
        set_error("pipeline_move: bad arguments"); return FERRET_EINVAL;
    }
    *worker = p->res.trace[k].worker; *kind = p->res.trace[k].kind; *stage = p->res.trace[k].stage;
    return FERRET_OK;
}

}  // extern "C"
