// HIP kernels of libferret for gfx950 (MI355X, CDNA4) and their launchers.
//
// The step kernel is one fused, memory-bound pass (Alg. 1 of the paper, loop "iterative
// approximation" + line "model update"; one approximator step is Eq.
// "gt-taylor-expansion-approximation"):
//
//   per element:  g   <- stale gradient
//                 g   <- g + lambda * g * g * (V[s_{i+1}] - V[s_i])     i = 0 .. K'-1
//                 new <- V[tau] - eta * g        (bf16 storage: on the fp32 master, then
//                                                 round-to-nearest-even to bf16)
//
// Design for the machine (every choice below was measured on MI355X):
//   * every operand is touched exactly once, with 128-bit (fp32) / 64-bit (bf16) accesses --
//     non-temporal for plans that stream, ordinary cached ones for plans small enough to stay in
//     the memory-side cache from step to step; consecutive lanes of a 64-wide wavefront touch
//     consecutive vectors, so every access of a wavefront is one contiguous run of memory;
//   * one workgroup of 256 lanes per chunk, vectors one after the other: all loads of a vector
//     (gradient + K'+1 versions) are issued before the first arithmetic, and the hardware
//     dispatcher balances the load.  A stage's chunk size is chosen by the plan so that every
//     workgroup moves about the same bytes whatever its stage's K' (2048 elements at K' = 3 in
//     fp32, more for shallower stages, fewer for deeper ones); a cap on resident workgroups per CU
//     (unused LDS) then keeps the traffic in flight at the measured optimum for large steps;
//   * a stage's tensors are one flat bucket; the stage table (48 B per stage) arrives as a kernel
//     argument; the chunk id is the block index, so the stage is found with scalar loads and all
//     stream base addresses live in SGPRs (lanes add a 32-bit offset).  A persistent grid-stride
//     variant that stages the table in LDS once per workgroup is kept as an option;
//   * the three per-stage sums are reduced inside the wavefront with cross-lane shuffles, across
//     the four wavefronts through LDS, written as one partial per chunk and summed in a fixed
//     order (fp64) by a second tiny kernel, so results do not depend on the launch shape;
//   * no matrix cores: there is no contraction anywhere on this path.
#include <hip/hip_runtime.h>

#include <mutex>
#include <thread>
#include <vector>

#include "ferret_internal.h"

// The file builds as one translation unit (FERRET_TU undefined) or, to compile in parallel, three times:
// FERRET_TU = 1 holds the step and state kernels for fp32 storage, 2 those for bf16 storage, 0 everything
// else (the small kernels, the launch logic, the profiler).
#ifndef FERRET_TU
#define FERRET_TU_COMMON 1
#define FERRET_TU_F32 1
#define FERRET_TU_BF16 1
#else
#define FERRET_TU_COMMON (FERRET_TU == 0)
#define FERRET_TU_F32 (FERRET_TU == 1)
#define FERRET_TU_BF16 (FERRET_TU == 2)
#endif

namespace ferret {

#ifndef FERRET_THREADS
#define FERRET_THREADS 256
#endif
constexpr int kThreads = FERRET_THREADS;
constexpr int kWaves = kThreads / 64;
#ifndef FERRET_UNROLL
#define FERRET_UNROLL 1
#endif
constexpr int kUnroll = FERRET_UNROLL;   // vectors per lane per stream loaded together when a chunk spans several groups
[[maybe_unused]] constexpr int kUnrolledItersSmall = 4;    // LEVEL 0 kernels: every stage has K' <= 4
[[maybe_unused]] constexpr int kUnrolledItersMid = kUnrolledItersMax;   // LEVEL 1 kernels: K' <= 8; LEVEL 2 adds the streamed path (batches of kStreamBatch boundaries) for any K'
[[maybe_unused]] constexpr uint64_t kCapThresholdBytes = 512ull << 20;

// 16-byte vectors as clang vector types (so that the non-temporal builtins accept them)
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

// ---- small device helpers ---------------------------------------------------------------------
// NT = true: non-temporal access (the data is not used again before it would be evicted anyway: steps that
// stream far more than the caches hold); NT = false: ordinary cached access (steps whose whole working set
// stays in the 256 MB memory-side cache from one step to the next).
template <bool NT, typename T>
__device__ __forceinline__ T ld(const T *p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, typename T>
__device__ __forceinline__ void st(T *p, const T &v) {
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}
__device__ __forceinline__ v4f make_v4f(float a, float b, float c, float d) {
    v4f r; r.x = a; r.y = b; r.z = c; r.w = d; return r;
}
__device__ __forceinline__ uint32_t uniform(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ uint64_t uniform(uint64_t x) {
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest, ties to even; NaN keeps its sign and becomes quiet.
__device__ __forceinline__ uint32_t bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    uint32_t nan = (u >> 16) | 0x40u;
    return ((u & 0x7fffffffu) > 0x7f800000u) ? nan : rounded;
}
__device__ __forceinline__ uint32_t bf16_pack(float lo, float hi) { return bf16_rne(lo) | (bf16_rne(hi) << 16); }

// Storage traits: the lane-vector of the ring / gradient storage type.
//   kElems      elements one lane handles per vector        kStoreBytes  bytes per stored element
//   Raw         register type of one load of that vector    kRawBytes    bytes of that vector
//   kMaster     the update goes to an fp32 master copy (kF4 = kElems/4 float4s per lane-vector)
template <bool NT_>
struct F32StoreT {
    using Raw = v4f;
    static constexpr int kElems = 4, kStoreBytes = 4, kRawBytes = 16, kF4 = 1;
    static constexpr bool kMaster = false, kNT = NT_;
    __device__ static __forceinline__ void widen(const Raw &r, float (&x)[kElems]) {
        x[0] = r.x; x[1] = r.y; x[2] = r.z; x[3] = r.w;
    }
    __device__ static __forceinline__ Raw narrow(const float (&x)[kElems]) { return make_v4f(x[0], x[1], x[2], x[3]); }
};
template <bool NT_>
struct Bf16Store8T {     // eight bf16 (16 bytes) per lane: widest loads, master as two float4 32 bytes apart
    using Raw = v4u;
    static constexpr int kElems = 8, kStoreBytes = 2, kRawBytes = 16, kF4 = 2;
    static constexpr bool kMaster = true, kNT = NT_;
    __device__ static __forceinline__ void widen(const Raw &r, float (&x)[kElems]) {
        x[0] = bf16_lo(r.x); x[1] = bf16_hi(r.x); x[2] = bf16_lo(r.y); x[3] = bf16_hi(r.y);
        x[4] = bf16_lo(r.z); x[5] = bf16_hi(r.z); x[6] = bf16_lo(r.w); x[7] = bf16_hi(r.w);
    }
    __device__ static __forceinline__ Raw narrow(const float (&x)[kElems]) {
        Raw o;
        o.x = bf16_pack(x[0], x[1]); o.y = bf16_pack(x[2], x[3]);
        o.z = bf16_pack(x[4], x[5]); o.w = bf16_pack(x[6], x[7]);
        return o;
    }
};
template <bool NT_>
struct Bf16Store4T {     // four bf16 (8 bytes) per lane: every access of a wavefront is one contiguous run
    using Raw = v2u;
    static constexpr int kElems = 4, kStoreBytes = 2, kRawBytes = 8, kF4 = 1;
    static constexpr bool kMaster = true, kNT = NT_;
    __device__ static __forceinline__ void widen(const Raw &r, float (&x)[kElems]) {
        x[0] = bf16_lo(r.x); x[1] = bf16_hi(r.x); x[2] = bf16_lo(r.y); x[3] = bf16_hi(r.y);
    }
    __device__ static __forceinline__ Raw narrow(const float (&x)[kElems]) {
        Raw o;
        o.x = bf16_pack(x[0], x[1]); o.y = bf16_pack(x[2], x[3]);
        return o;
    }
};
#if FERRET_BF16_LANE_ELEMS == 8
template <bool NT_> using Bf16StoreT = Bf16Store8T<NT_>;
#else
template <bool NT_> using Bf16StoreT = Bf16Store4T<NT_>;
#endif
using F32Store = F32StoreT<true>;
using Bf16Store = Bf16StoreT<true>;
using F32StoreCached = F32StoreT<false>;
using Bf16StoreCached = Bf16StoreT<false>;

// Per-chunk partial sums a step can produce: series 0..2 are the three norms, series 3..4 the two inner
// products of the "update lambda" block when that block is fused into the step (OUT & 16).
constexpr int kSeries = 5;

// A_I applied in place: g <- g + lambda * g * g * (v_new - v_old)
__device__ __forceinline__ float approximator(float g, float lambda, float v_new, float v_old) {
    return fmaf(lambda * g * g, v_new - v_old, g);
}

// Ring slot arithmetic without divisions (all values wave-uniform; the host guarantees head < R and tau < R):
// x mod R for x < 2R, and the slot of the oldest version read, (head - tau) mod R.
__device__ __forceinline__ uint32_t wrap(uint32_t x, uint32_t R) { return x >= R ? x - R : x; }
__device__ __forceinline__ uint32_t oldest_slot(uint32_t head, uint32_t tau, uint32_t R) {
    return head >= tau ? head - tau : head + R - tau;
}

// Everything a lane needs to know about the chunk it works on.  All pointers are wave-uniform
// (they live in scalar registers); lanes add a 32-bit byte offset, which is the addressing form
// the global load/store instructions take directly.
template <int NV>
struct ChunkPtrs {
    const char *g;                  // gradient, storage type
    const char *v[NV];              // boundary versions, oldest first; v[NV-1] = V[tau]
    char *out;                      // slot of the new version
    char *master;                   // fp32 master (bf16 storage only)
    char *g_out;                    // fp32 compensated gradient, nullable
    char *accum;                    // fp32 running sum of compensated gradients (accumulation kernels)
    float acc_scale;                // factor applied to the sum at the update
    bool acc_update;                // this arrival completes the group: update and clear the sum
    float pen_scale, pen_inv_c;     // step-size penalty of the comparison methods (OUT & 8)
    const char *v1;                 // V[1], the version one step after V[0] (fused lambda block, OUT & 16)
    char *v_r, *v_a;                // fp32 moving averages of the lambda block
    float alpha;
};

template <bool NT, typename T>
__device__ __forceinline__ T ld_off(const char *base, uint32_t byte_off) {
    return ld<NT>(reinterpret_cast<const T *>(base + byte_off));
}
template <bool NT, typename T>
__device__ __forceinline__ void st_off(char *base, uint32_t byte_off, const T &v) {
    st<NT>(reinterpret_cast<T *>(base + byte_off), v);
}

template <typename S>
__device__ __forceinline__ void load_master(const char *master, uint32_t vec, v4f (&m)[S::kF4], bool needed = true) {
    if (S::kMaster && needed) {
#pragma unroll
        for (int q = 0; q < S::kF4; ++q) m[q] = ld_off<S::kNT, v4f>(master, vec * (uint32_t)(S::kElems * 4) + 16u * q);
    }
}

// With bf16 storage and the caller's promise that the newest stored version is exactly the
// round-to-nearest-even bf16 of the master (true whenever both were produced by this library), the
// newest version need not be read: it is recomputed from the master that is loaded anyway.
template <typename S>
__device__ __forceinline__ typename S::Raw newest_from_master(const v4f (&m)[S::kF4]) {
    float w[S::kElems];
#pragma unroll
    for (int q = 0; q < S::kF4; ++q) { w[4 * q] = m[q].x; w[4 * q + 1] = m[q].y; w[4 * q + 2] = m[q].z; w[4 * q + 3] = m[q].w; }
    return S::narrow(w);
}

template <typename S, int OUT>
__device__ __forceinline__ void load_accum(const char *accum, uint32_t vec, v4f (&ac)[S::kF4]) {
    if (OUT & 2) {
#pragma unroll
        for (int q = 0; q < S::kF4; ++q) ac[q] = ld_off<S::kNT, v4f>(accum, vec * (uint32_t)(S::kElems * 4) + 16u * q);
    }
}

// theta_next = V[tau] - eta * g (fp32 storage), or master - eta * g with the stored version its
// round-to-nearest-even bf16; then the stores of one lane-vector.
template <typename S, int NV, int OUT>
__device__ __forceinline__ void update_and_store(const ChunkPtrs<NV> &p, uint32_t vec, float (&g)[S::kElems],
                                                 const float (&newest)[S::kElems], const float (&first)[S::kElems],
                                                 const v4f (&m_in)[S::kF4], const v4f (&ac_in)[S::kF4], float lr) {
    constexpr int E = S::kElems;
    constexpr uint32_t kF32Bytes = E * 4;
    if (OUT & 8) {          // comparison methods: shrink the step by scale / (|V[tau]-V[0]| / C + 1)
#pragma unroll
        for (int e = 0; e < E; ++e) g[e] = p.pen_scale * g[e] / fmaf(fabsf(newest[e] - first[e]), p.pen_inv_c, 1.0f);
    }
    if (OUT & 1) {
#pragma unroll
        for (int q = 0; q < S::kF4; ++q)
            st_off<S::kNT>(p.g_out, vec * kF32Bytes + 16u * q, make_v4f(g[4 * q], g[4 * q + 1], g[4 * q + 2], g[4 * q + 3]));
    }
    float step[E];          // what the update subtracts eta times: g, or scale * (running sum + g)
#pragma unroll
    for (int e = 0; e < E; ++e) step[e] = g[e];
    if (OUT & 2) {          // gradient accumulation: add this compensated gradient to the running sum
#pragma unroll
        for (int q = 0; q < S::kF4; ++q) {
            step[4 * q + 0] += ac_in[q].x; step[4 * q + 1] += ac_in[q].y;
            step[4 * q + 2] += ac_in[q].z; step[4 * q + 3] += ac_in[q].w;
        }
        if (!p.acc_update) {        // uniform: not the last arrival of the group, only the sum moves
#pragma unroll
            for (int q = 0; q < S::kF4; ++q)
                st_off<S::kNT>(p.accum, vec * kF32Bytes + 16u * q,
                       make_v4f(step[4 * q], step[4 * q + 1], step[4 * q + 2], step[4 * q + 3]));
            return;
        }
#pragma unroll
        for (int q = 0; q < S::kF4; ++q) st_off<S::kNT>(p.accum, vec * kF32Bytes + 16u * q, make_v4f(0.f, 0.f, 0.f, 0.f));
#pragma unroll
        for (int e = 0; e < E; ++e) step[e] *= p.acc_scale;
    }
    float w[E];
    if (S::kMaster) {
#pragma unroll
        for (int q = 0; q < S::kF4; ++q) {
            w[4 * q + 0] = fmaf(-lr, step[4 * q + 0], m_in[q].x); w[4 * q + 1] = fmaf(-lr, step[4 * q + 1], m_in[q].y);
            w[4 * q + 2] = fmaf(-lr, step[4 * q + 2], m_in[q].z); w[4 * q + 3] = fmaf(-lr, step[4 * q + 3], m_in[q].w);
            st_off<S::kNT>(p.master, vec * kF32Bytes + 16u * q, make_v4f(w[4 * q], w[4 * q + 1], w[4 * q + 2], w[4 * q + 3]));
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) w[e] = fmaf(-lr, step[e], newest[e]);
    }
    st_off<S::kNT>(p.out, vec * (uint32_t)S::kRawBytes, S::narrow(w));
}

// What the fused lambda block loads per lane-vector besides the step's own inputs.
template <typename S>
struct LambdaIn {
    typename S::Raw v1;
    v4f vr[S::kF4], va[S::kF4];
};

template <typename S, int OUT, int NV>
__device__ __forceinline__ void load_lambda_in(const ChunkPtrs<NV> &p, uint32_t vec, LambdaIn<S> &in) {
    if (OUT & 16) {
        in.v1 = ld_off<S::kNT, typename S::Raw>(p.v1, vec * (uint32_t)S::kRawBytes);
#pragma unroll
        for (int q = 0; q < S::kF4; ++q) {
            in.vr[q] = ld_off<S::kNT, v4f>(p.v_r, vec * (uint32_t)(S::kElems * 4) + 16u * q);
            in.va[q] = ld_off<S::kNT, v4f>(p.v_a, vec * (uint32_t)(S::kElems * 4) + 16u * q);
        }
    }
}

// Alg. 1, block "update lambda", on one lane-vector: its share of <v_a, g_0 - v_r> and <v_a, v_a> on
// the OLD averages, then v_r <- alpha v_r + (1-alpha) g_0 and v_a <- alpha v_a + (1-alpha) g_0 g_0 (V[1]-V[0]).
template <typename S, int NV>
__device__ __forceinline__ void lambda_state_vector(const ChunkPtrs<NV> &p, uint32_t vec, const float (&g)[S::kElems],
                                                    const float (&w0)[S::kElems], const LambdaIn<S> &in,
                                                    float (&acc)[kSeries]) {
    constexpr uint32_t FB = S::kElems * 4;
    float w1[S::kElems];
    S::widen(in.v1, w1);
    const float alpha = p.alpha, beta = 1.0f - p.alpha;
#pragma unroll
    for (int q = 0; q < S::kF4; ++q) {
        float r[4] = {in.vr[q].x, in.vr[q].y, in.vr[q].z, in.vr[q].w};
        float s4[4] = {in.va[q].x, in.va[q].y, in.va[q].z, in.va[q].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float gi = g[4 * q + i];
            acc[3] = fmaf(s4[i], gi - r[i], acc[3]);
            acc[4] = fmaf(s4[i], s4[i], acc[4]);
            r[i] = fmaf(alpha, r[i], beta * gi);
            s4[i] = fmaf(alpha, s4[i], beta * (gi * gi * (w1[4 * q + i] - w0[4 * q + i])));
        }
        st_off<S::kNT>(p.v_r, vec * FB + 16u * q, make_v4f(r[0], r[1], r[2], r[3]));
        st_off<S::kNT>(p.v_a, vec * FB + 16u * q, make_v4f(s4[0], s4[1], s4[2], s4[3]));
    }
}

// Finish one vector: iterate, update, store.  raw_g / raw_v hold the loaded inputs.
template <typename S, int NV, bool COMP, bool NORMS, int OUT>
__device__ __forceinline__ void finish_vector(const ChunkPtrs<NV> &p, uint32_t vec,
                                              const typename S::Raw &raw_g,
                                              const typename S::Raw (&raw_v)[NV], const v4f (&m_in)[S::kF4],
                                              const v4f (&ac_in)[S::kF4], const LambdaIn<S> &lin, float lambda,
                                              float lr, float (&acc)[kSeries]) {
    constexpr int E = S::kElems;
    float g[E], prev[E], cur[E], first[E];
    S::widen(raw_g, g);
    S::widen(raw_v[0], prev);
#pragma unroll
    for (int e = 0; e < E; ++e) first[e] = prev[e];
    if (OUT & 16) lambda_state_vector<S, NV>(p, vec, g, first, lin, acc);
    if (NORMS) {
#pragma unroll
        for (int e = 0; e < E; ++e) acc[0] = fmaf(g[e], g[e], acc[0]);
    }
#pragma unroll
    for (int s = 1; s < NV; ++s) {
        S::widen(raw_v[s], cur);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if (COMP) g[e] = approximator(g[e], lambda, cur[e], prev[e]);
            prev[e] = cur[e];
        }
    }
    if (NORMS) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            acc[1] = fmaf(g[e], g[e], acc[1]);
            float gap = prev[e] - first[e];
            acc[2] = fmaf(gap, gap, acc[2]);
        }
    }
    update_and_store<S, NV, OUT>(p, vec, g, prev, first, m_in, ac_in, lr);
}

// A chunk with a compile-time number NV of versions to read.  Groups of kThreads*kUnroll vectors
// run without bounds checks; what is left (< one group, or a ragged last chunk) runs one
// predicated vector at a time.  Within a group all loads come first and all stores last, which
// is also what makes the in-place case (new version written over the oldest one read) safe:
// each vector is read and written by the same lane.
template <typename S, int NV, bool COMP, bool NORMS, int OUT>
__device__ __forceinline__ void run_chunk(const ChunkPtrs<NV> &p, uint32_t n_vecs, float lambda,
                                          float lr, float (&acc)[kSeries]) {
    using Raw = typename S::Raw;
    constexpr uint32_t RB = S::kRawBytes;
    const uint32_t tid = threadIdx.x;
    const uint32_t group = kThreads * kUnroll;
    const uint32_t n_grouped = n_vecs / group * group;

    for (uint32_t base = 0; base < n_grouped; base += group) {
        Raw rg[kUnroll], rv[kUnroll][NV];
        v4f m[kUnroll][S::kF4], ac[kUnroll][S::kF4];
        LambdaIn<S> lin[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) rg[u] = ld_off<S::kNT, Raw>(p.g, (base + u * kThreads + tid) * RB);
#pragma unroll
        for (int s = 0; s < NV - ((OUT & 4) ? 1 : 0); ++s)
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) rv[u][s] = ld_off<S::kNT, Raw>(p.v[s], (base + u * kThreads + tid) * RB);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            load_master<S>(p.master, base + u * kThreads + tid, m[u], !(OUT & 2) || p.acc_update);
            load_accum<S, OUT>(p.accum, base + u * kThreads + tid, ac[u]);
            load_lambda_in<S, OUT>(p, base + u * kThreads + tid, lin[u]);
            if constexpr ((OUT & 4) != 0 && S::kMaster) rv[u][NV - 1] = newest_from_master<S>(m[u]);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            finish_vector<S, NV, COMP, NORMS, OUT>(p, base + u * kThreads + tid, rg[u], rv[u], m[u], ac[u], lin[u],
                                                   lambda, lr, acc);
    }
    for (uint32_t vec = n_grouped + tid; vec < n_vecs; vec += kThreads) {
        Raw rg = ld_off<S::kNT, Raw>(p.g, vec * RB), rv[NV];
        v4f m[S::kF4], ac[S::kF4];
        LambdaIn<S> lin;
#pragma unroll
        for (int s = 0; s < NV - ((OUT & 4) ? 1 : 0); ++s) rv[s] = ld_off<S::kNT, Raw>(p.v[s], vec * RB);
        load_master<S>(p.master, vec, m, !(OUT & 2) || p.acc_update);
        load_accum<S, OUT>(p.accum, vec, ac);
        load_lambda_in<S, OUT>(p, vec, lin);
        if constexpr ((OUT & 4) != 0 && S::kMaster) rv[NV - 1] = newest_from_master<S>(m);
        finish_vector<S, NV, COMP, NORMS, OUT>(p, vec, rg, rv, m, ac, lin, lambda, lr, acc);
    }
}

// Any number of versions (K' > 8): stream them, kStreamBatch boundaries at a time.  `arena` points at this
// chunk's first element in slot 0 of the stage; slots are slot_bytes apart.
template <typename S, bool NORMS, int OUT>
__device__ __forceinline__ void run_chunk_streamed(const ChunkPtrs<1> &p, const char *arena, uint64_t slot_bytes,
                                                   uint32_t R, uint32_t head, uint32_t tau, uint32_t kp,
                                                   uint32_t n_vecs, float lambda, float lr, float (&acc)[kSeries]) {
    using Raw = typename S::Raw;
    constexpr int E = S::kElems;
    constexpr uint32_t RB = S::kRawBytes;
    const uint32_t oldest = oldest_slot(head, tau, R);
    // boundary s_i = floor(i tau / K') advances by tau div K' per iteration plus a carry from the remainders:
    // one division per chunk instead of one per boundary
    const uint32_t step_q = tau / kp, step_r = tau - step_q * kp;
    for (uint32_t vec = threadIdx.x; vec < n_vecs; vec += kThreads) {
        float g[E], prev[E], cur[E], first[E];
        v4f m[S::kF4], ac[S::kF4];
        Raw rg = ld_off<S::kNT, Raw>(p.g, vec * RB);
        Raw r0 = ld_off<S::kNT, Raw>(arena + (uint64_t)oldest * slot_bytes, vec * RB);      // kp >= 1 here: V[0] is not V[tau]
        load_master<S>(p.master, vec, m, !(OUT & 2) || p.acc_update);
        load_accum<S, OUT>(p.accum, vec, ac);
        LambdaIn<S> lin;
        load_lambda_in<S, OUT>(p, vec, lin);
        S::widen(rg, g);
        S::widen(r0, prev);
#pragma unroll
        for (int e = 0; e < E; ++e) first[e] = prev[e];
        if (OUT & 16) lambda_state_vector<S, 1>(p, vec, g, first, lin, acc);
        if (NORMS) {
#pragma unroll
            for (int e = 0; e < E; ++e) acc[0] = fmaf(g[e], g[e], acc[0]);
        }
        // Batches of kStreamBatch boundaries, two register sets used in turn: the loads of the next batch are
        // issued before the iterations of the current one, so memory latency overlaps across batches.
        // batches are loaded in the order of their boundaries, so the running boundary (its slot and the
        // remainder of i tau / K') is carried from one batch to the next
        uint32_t slot = oldest, rem = 0;
        auto load_batch = [&](uint32_t i, Raw (&r)[kStreamBatch]) {
            const uint32_t count = kp - i + 1 < (uint32_t)kStreamBatch ? kp - i + 1 : (uint32_t)kStreamBatch;   // uniform
#pragma unroll
            for (int b = 0; b < kStreamBatch; ++b) {
                if ((uint32_t)b >= count) break;
                rem += step_r;                                        // boundary i + b from boundary i + b - 1
                const uint32_t carry = rem >= kp ? 1u : 0u;
                rem -= carry ? kp : 0u;
                slot = wrap(slot + step_q + carry, R);
                if ((OUT & 4) != 0 && S::kMaster && i + b == kp) r[b] = newest_from_master<S>(m);
                else r[b] = ld_off<S::kNT, Raw>(arena + (uint64_t)slot * slot_bytes, vec * RB);
            }
        };
        auto iterate_batch = [&](uint32_t i, const Raw (&r)[kStreamBatch]) {
            const uint32_t count = kp - i + 1 < (uint32_t)kStreamBatch ? kp - i + 1 : (uint32_t)kStreamBatch;
#pragma unroll
            for (int b = 0; b < kStreamBatch; ++b) {
                if ((uint32_t)b >= count) break;
                S::widen(r[b], cur);
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    g[e] = approximator(g[e], lambda, cur[e], prev[e]);
                    prev[e] = cur[e];
                }
            }
        };
        Raw ra[kStreamBatch], rb[kStreamBatch];
        load_batch(1, ra);
        for (uint32_t i = 1; i <= kp; i += 2 * kStreamBatch) {
            const bool second = i + kStreamBatch <= kp;             // uniform
            if (second) load_batch(i + kStreamBatch, rb);
            iterate_batch(i, ra);
            if (second) {
                if (i + 2 * kStreamBatch <= kp) load_batch(i + 2 * kStreamBatch, ra);
                iterate_batch(i + kStreamBatch, rb);
            }
        }
        if (NORMS) {
#pragma unroll
            for (int e = 0; e < E; ++e) {
                acc[1] = fmaf(g[e], g[e], acc[1]);
                float gap = prev[e] - first[e];
                acc[2] = fmaf(gap, gap, acc[2]);
            }
        }
        update_and_store<S, 1, OUT>(p, vec, g, prev, first, m, ac, lr);
    }
}

// Sum over the 64 lanes of a wavefront; every lane ends with the total.
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// ---- ordered sums of per-chunk partials ------------------------------------------------------------
// The library's one summation order for a stage's series of per-chunk partials, so that sums do not depend
// on which kernel forms them or how the step was launched: 1024 "virtual lanes"; lane v adds the partials of
// chunks c0+v, c0+v+1024, ... in that order in fp64; the 64 lanes of each of the 16 virtual wavefronts are
// combined by an xor-shuffle tree; the 16 wavefront sums are added in wavefront order.  A workgroup of
// THREADS < 1024 real lanes plays 1024/THREADS virtual lanes per real lane, v = t + THREADS*q: the same lane
// position in virtual wavefront t/64 + (THREADS/64)*q, so every addition pairs the same operands.
// Must be called by all THREADS lanes of the workgroup; total[] is valid in every lane afterwards.
constexpr int kSumLanes = 1024;
constexpr int kSumWaves = kSumLanes / 64;

template <int NS, int THREADS>
__device__ __forceinline__ void ordered_sums(const float *series0, size_t series_stride, uint32_t c0, uint32_t c1,
                                             double (&red)[kSeries][kSumWaves], double (&total)[NS]) {
    constexpr int Q = kSumLanes / THREADS, WAVES = THREADS / 64;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
#pragma unroll 1
    for (int q = 0; q < Q; ++q) {
        double s[NS];
#pragma unroll
        for (int k = 0; k < NS; ++k) s[k] = 0.0;
        uint32_t c = c0 + t + (uint32_t)(THREADS * q);
        for (; c + 3u * kSumLanes < c1; c += 4u * kSumLanes) {          // four independent loads per series in flight
            float x[NS][4];
#pragma unroll
            for (int k = 0; k < NS; ++k)
#pragma unroll
                for (int u = 0; u < 4; ++u) x[k][u] = series0[(size_t)k * series_stride + c + (uint32_t)(u * kSumLanes)];
#pragma unroll
            for (int k = 0; k < NS; ++k)
#pragma unroll
                for (int u = 0; u < 4; ++u) s[k] += (double)x[k][u];
        }
        for (; c < c1; c += kSumLanes)
#pragma unroll
            for (int k = 0; k < NS; ++k) s[k] += (double)series0[(size_t)k * series_stride + c];
#pragma unroll
        for (int k = 0; k < NS; ++k) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) s[k] += __shfl_xor(s[k], off, 64);
            if (lane == 0) red[k][wave + WAVES * q] = s[k];
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < NS; ++k) {
        double sum = 0.0;
#pragma unroll
        for (int w = 0; w < kSumWaves; ++w) sum += red[k][w];
        total[k] = sum;
    }
}

// Alg. 1, "update lambda": one gradient-descent step on || (1-alpha)(g_0 - v_r) - lambda v_a ||^2 given the two
// inner products over the stage,  lambda <- lambda + 2 eta_lambda ((1-alpha) <v_a, g_0 - v_r> - lambda <v_a, v_a>).
__device__ __forceinline__ float lambda_descent_step(float lambda_f, double dot_a_dr, double dot_a_a, float alpha,
                                                     float eta_lambda) {
    dot_a_dr *= (double)(1.0f - alpha);
    const double lambda = (double)lambda_f;
    return (float)(lambda + 2.0 * (double)eta_lambda * (dot_a_dr - lambda * dot_a_a));
}

// The wave-uniform facts about one chunk, taken from its stage's table entry.
struct ChunkInfo {
    const char *arena;       // this chunk's first element in slot 0 of the stage's ring arena
    uint64_t slot_bytes;     // distance between slots
    uint64_t flat_elem0;     // this chunk's first element in slot-shaped buffers
    uint32_t n_vecs;         // 16-byte storage vectors in the chunk
    uint32_t R, head, tau, kp;
    uint32_t stage;
    bool acc_update;         // accumulation kernels: this call updates the stage
    bool skip;               // accumulation kernels: the stage takes no part in this call
};

template <typename S>
__device__ __forceinline__ ChunkInfo chunk_info(const StepArgs &a, const StageDesc &d, uint32_t chunk,
                                                uint32_t stage) {
    constexpr uint64_t kStoreBytes = S::kStoreBytes;
    ChunkInfo c;
    const uint32_t chunk_elems = uniform(d.chunk_elems);
    const uint64_t e0 = (uint64_t)(chunk - uniform(d.chunk_begin)) * chunk_elems;
    const uint64_t left = uniform(d.n_elems) - e0;
    const uint32_t n_here = left < chunk_elems ? (uint32_t)left : chunk_elems;
    c.n_vecs = n_here / S::kElems;
    c.R = uniform((uint32_t)d.ring_depth);
    c.head = uniform((uint32_t)d.head);
    c.tau = uniform((uint32_t)d.tau);
    c.kp = uniform((uint32_t)d.kp);
    c.slot_bytes = uniform(d.slot_stride) * kStoreBytes;
    c.arena = static_cast<const char *>(a.ring) + (uniform(d.ring_base) + e0) * kStoreBytes;
    c.flat_elem0 = uniform(d.flat_off) + e0;
    c.stage = stage;
    const uint32_t mode = (a.accum || a.masked) ? a.mode[stage] : 2u;     // 0 skip, 1 accumulate, 2 (accumulate +) update
    c.acc_update = mode == 2u;
    c.skip = mode == 0u;
    return c;
}

// Fixed-NV dispatch target: builds the chunk's pointers.
template <typename S, int NV, bool COMP, bool NORMS, int OUT>
__device__ __forceinline__ void do_chunk(const StepArgs &a, const ChunkInfo &c, float lambda, float (&acc)[kSeries]) {
    constexpr uint64_t kStoreBytes = S::kStoreBytes;
    ChunkPtrs<NV> p;
    p.g = static_cast<const char *>(a.grads) + c.flat_elem0 * kStoreBytes;
    const uint32_t oldest = oldest_slot(c.head, c.tau, c.R);
    constexpr uint32_t kp = NV - 1;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        // NV == 1: only V[tau].  Otherwise boundary s_i = floor(i*tau/K') of the K' = NV-1 segments (a division by
        // a compile-time constant; i*tau stays far below 2^32).
        const uint32_t s_i = NV == 1 ? c.tau : ((uint32_t)i * c.tau) / (kp ? kp : 1u);
        p.v[i] = c.arena + (uint64_t)wrap(oldest + s_i, c.R) * c.slot_bytes;
    }
    p.out = const_cast<char *>(c.arena) + (uint64_t)wrap(c.head + 1u, c.R) * c.slot_bytes;
    p.master = a.master ? reinterpret_cast<char *>(a.master) + c.flat_elem0 * 4 : nullptr;
    p.g_out = (OUT & 1) ? reinterpret_cast<char *>(a.grad_out) + c.flat_elem0 * 4 : nullptr;
    p.accum = (OUT & 2) ? reinterpret_cast<char *>(a.accum) + c.flat_elem0 * 4 : nullptr;
    p.acc_scale = a.accum_scale;
    p.acc_update = c.acc_update;
    p.pen_scale = (OUT & 8) ? a.pen_scale[c.stage] : 1.f;
    p.pen_inv_c = (OUT & 8) ? a.pen_inv_c[c.stage] : 0.f;
    p.v1 = (OUT & 16) ? c.arena + (uint64_t)wrap(oldest + 1u, c.R) * c.slot_bytes : nullptr;
    p.v_r = (OUT & 16) ? reinterpret_cast<char *>(a.v_r) + c.flat_elem0 * 4 : nullptr;
    p.v_a = (OUT & 16) ? reinterpret_cast<char *>(a.v_a) + c.flat_elem0 * 4 : nullptr;
    p.alpha = a.alpha;
    run_chunk<S, NV, COMP, NORMS, OUT>(p, c.n_vecs, lambda, a.lr, acc);
}

// LDS of a step workgroup: cross-wavefront reduction of the chunk's partial sums.
struct StepLds {
    float red[kSeries][kWaves];
};

// One chunk, whatever its K': picks the unrolled variant (K' <= 4 or <= 8) or the streamed one, then
// reduces the three partial sums of the workgroup and writes the chunk's partial.
template <typename S, int LEVEL, bool NORMS, int OUT>
__device__ __forceinline__ void process_chunk(const StepArgs &a, const ChunkInfo &c, uint32_t chunk, StepLds &lds) {
    float acc[kSeries] = {0.f, 0.f, 0.f, 0.f, 0.f};
    constexpr int PLAIN = OUT & ~16;      // a stage without staleness has no lambda block
    if (c.skip) return;  // uniform: this stage is not part of the call (its norms are reported as zero elsewhere)
    // the coefficient: one scalar for the call, or this stage's self-tuned one from device memory
    // (read through the constant address space: a scalar load; the array was last written by an
    // earlier kernel of the same stream)
    typedef const float __attribute__((address_space(4))) *const_f32_ptr;
    const float lambda = a.lambda_dev ? *reinterpret_cast<const_f32_ptr>(reinterpret_cast<uintptr_t>(a.lambda_dev + c.stage))
                                      : a.lambda;
    // versions to read: the K'+1 boundaries; with K' = 0 only V[tau], plus V[0] when the weight
    // gap is wanted for the norms
    if (c.kp == 0) {
        if ((NORMS || (OUT & 8)) && c.tau > 0) do_chunk<S, 2, false, NORMS, PLAIN>(a, c, lambda, acc);
        else do_chunk<S, 1, false, NORMS, PLAIN>(a, c, lambda, acc);
    } else if (c.kp == 1) {
        do_chunk<S, 2, true, NORMS, OUT>(a, c, lambda, acc);
    } else if (c.kp == 2) {
        do_chunk<S, 3, true, NORMS, OUT>(a, c, lambda, acc);
    } else if (c.kp == 3) {
        do_chunk<S, 4, true, NORMS, OUT>(a, c, lambda, acc);
    } else if (c.kp == 4) {
        do_chunk<S, 5, true, NORMS, OUT>(a, c, lambda, acc);
    } else if (LEVEL >= 1 && c.kp == 5) {
        do_chunk<S, 6, true, NORMS, OUT>(a, c, lambda, acc);
    } else if (LEVEL >= 1 && c.kp == 6) {
        do_chunk<S, 7, true, NORMS, OUT>(a, c, lambda, acc);
    } else if (LEVEL >= 1 && c.kp == 7) {
        do_chunk<S, 8, true, NORMS, OUT>(a, c, lambda, acc);
    } else if (LEVEL >= 1 && c.kp == 8) {
        do_chunk<S, 9, true, NORMS, OUT>(a, c, lambda, acc);
    } else if (LEVEL >= 2) {
        constexpr uint64_t kStoreBytes = S::kStoreBytes;
        ChunkPtrs<1> p;
        p.g = static_cast<const char *>(a.grads) + c.flat_elem0 * kStoreBytes;
        p.v[0] = nullptr;
        p.out = const_cast<char *>(c.arena) + (uint64_t)wrap(c.head + 1u, c.R) * c.slot_bytes;
        p.master = a.master ? reinterpret_cast<char *>(a.master) + c.flat_elem0 * 4 : nullptr;
        p.g_out = (OUT & 1) ? reinterpret_cast<char *>(a.grad_out) + c.flat_elem0 * 4 : nullptr;
        p.accum = (OUT & 2) ? reinterpret_cast<char *>(a.accum) + c.flat_elem0 * 4 : nullptr;
        p.acc_scale = a.accum_scale;
        p.acc_update = c.acc_update;
        p.pen_scale = 1.f;
        p.pen_inv_c = 0.f;
        p.v1 = (OUT & 16) ? c.arena + (uint64_t)wrap(oldest_slot(c.head, c.tau, c.R) + 1u, c.R) * c.slot_bytes : nullptr;
        p.v_r = (OUT & 16) ? reinterpret_cast<char *>(a.v_r) + c.flat_elem0 * 4 : nullptr;
        p.v_a = (OUT & 16) ? reinterpret_cast<char *>(a.v_a) + c.flat_elem0 * 4 : nullptr;
        p.alpha = a.alpha;
        run_chunk_streamed<S, NORMS, OUT>(p, c.arena, c.slot_bytes, c.R, c.head, c.tau, c.kp, c.n_vecs,
                                           lambda, a.lr, acc);
    }
    constexpr bool FUSED = (OUT & 16) != 0;
    if constexpr (NORMS || FUSED) {
        constexpr int k0 = NORMS ? 0 : 3, k1 = FUSED ? kSeries : 3;      // the series this kernel produces
        const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
#pragma unroll
        for (int k = k0; k < k1; ++k) {
            float s = wave_sum(acc[k]);
            if (lane == 0) lds.red[k][wave] = s;
        }
        __syncthreads();
        if (threadIdx.x >= (uint32_t)k0 && threadIdx.x < (uint32_t)k1) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) s += lds.red[threadIdx.x][w];
            a.partials[(size_t)threadIdx.x * a.n_chunks + chunk] = s;     // each series contiguous
        }
    }
}

// ---- the step kernel ----------------------------------------------------------------------------
// PERSISTENT = true : a fixed grid strides over the chunks; the stage table is staged in LDS once
//                     per workgroup and each chunk's stage is looked up there.
// PERSISTENT = false: one workgroup per chunk, scheduled by the hardware dispatcher; the table is
//                     read straight from the kernel-argument segment with scalar loads (the
//                     block index is uniform, so nothing needs LDS or a barrier).
// LEVEL 0 / 1 / 2   : largest K' of any stage is <= 4 / <= 8 / anything; paths a launch cannot
//                     need are not compiled in, which keeps the register footprint small.
template <typename S, bool PERSISTENT, int LEVEL, bool NORMS, int OUT>
__global__ void __launch_bounds__(kThreads) step_kernel(const StepArgs a) {
    __shared__ StepLds lds;
    if constexpr (PERSISTENT) {
        __shared__ StageDesc tab[FERRET_MAX_STAGES];
        {   // stage table: kernel-argument segment -> LDS, 12 dwords per stage
            const uint32_t *src = reinterpret_cast<const uint32_t *>(a.stage);
            uint32_t *dst = reinterpret_cast<uint32_t *>(tab);
            const uint32_t n_words = a.n_stages * (sizeof(StageDesc) / 4);
            for (uint32_t i = threadIdx.x; i < n_words; i += kThreads) dst[i] = src[i];
        }
        __syncthreads();
        uint32_t stage = 0;
        for (uint32_t chunk = a.chunk_base + blockIdx.x; chunk < a.chunk_end; chunk += gridDim.x) {
            while (stage + 1 < a.n_stages && chunk >= tab[stage + 1].chunk_begin) ++stage;
            stage = uniform(stage);
            const ChunkInfo c = chunk_info<S>(a, tab[stage], chunk, stage);
            process_chunk<S, LEVEL, NORMS, OUT>(a, c, chunk, lds);
            if (NORMS) __syncthreads();     // lds.red is reused by the next chunk
        }
    } else {
        // Workgroups are dealt to the 8 XCDs round-robin in the order of their ids.  With xcd_group = G > 1 the
        // block index is permuted inside every full run of 8 G chunks so that each XCD works on G consecutive
        // chunks (a contiguous run of every stream) instead of every eighth chunk; a last partial run keeps the
        // identity.  A bijection on the launch's chunks, so results cannot depend on it.
        uint32_t chunk = a.chunk_base + blockIdx.x;
        if (a.xcd_group > 1u) {
            const uint32_t G = a.xcd_group, span = 8u * G, n = a.chunk_end - a.chunk_base, b = blockIdx.x;
            const uint32_t g = b / span, within = b - g * span;
            if ((g + 1u) * span <= n) chunk = a.chunk_base + g * span + (within & 7u) * G + (within >> 3);
        }
        // stage = number of stages (beyond the first) that begin at or before this chunk;
        // unused table entries hold UINT32_MAX and never count
        uint32_t stage = 0;
#pragma unroll
        for (uint32_t j = 1; j < 16; ++j) stage += chunk >= a.chunk_begin[j] ? 1u : 0u;
        if (a.n_stages > 16) {
#pragma unroll
            for (uint32_t j = 16; j < FERRET_MAX_STAGES; ++j) stage += chunk >= a.chunk_begin[j] ? 1u : 0u;
        }
        const ChunkInfo c = chunk_info<S>(a, a.stage[stage], chunk, stage);
        process_chunk<S, LEVEL, NORMS, OUT>(a, c, chunk, lds);
    }
}

// ---- self-tuned lambda: state pass + lambda step ---------------------------------------------------
// Alg. 1, block "update lambda", for every stage with staleness >= 1, one workgroup per chunk:
// forms the chunk's share of <v_a, g_0 - v_r> and <v_a, v_a> on the OLD averages and writes the new
// ones, v_r <- alpha v_r + (1-alpha) g_0 and v_a <- alpha v_a + (1-alpha) g_0 g_0 (V[1]-V[0]).
// Reads g_0, V[0], V[1] (storage type) and v_r, v_a (fp32) once each: 28 bytes per fp32 parameter.
// stage_sums_kernel sums the stage's two series afterwards and takes the lambda step.
template <typename S>
__global__ void __launch_bounds__(kThreads) lambda_state_kernel(const StepArgs a) {
    using Raw = typename S::Raw;
    constexpr int E = S::kElems;
    constexpr uint32_t RB = S::kRawBytes, FB = E * 4;
    __shared__ StepLds lds;
    const uint32_t chunk = a.chunk_base + blockIdx.x;
    uint32_t stage = 0;
#pragma unroll
    for (uint32_t j = 1; j < 16; ++j) stage += chunk >= a.chunk_begin[j] ? 1u : 0u;
    if (a.n_stages > 16) {
#pragma unroll
        for (uint32_t j = 16; j < FERRET_MAX_STAGES; ++j) stage += chunk >= a.chunk_begin[j] ? 1u : 0u;
    }
    const ChunkInfo c = chunk_info<S>(a, a.stage[stage], chunk, stage);
    if (c.tau == 0 || c.skip) return;       // uniform over the workgroup: nothing to tune, or no gradient arrived
    float acc0 = 0.f, acc1 = 0.f;
    {
        const uint32_t oldest = oldest_slot(c.head, c.tau, c.R);
        const char *g_ptr = static_cast<const char *>(a.grads) + c.flat_elem0 * S::kStoreBytes;
        const char *v0 = c.arena + (uint64_t)oldest * c.slot_bytes;
        const char *v1 = c.arena + (uint64_t)wrap(oldest + 1u, c.R) * c.slot_bytes;
        char *vr_ptr = reinterpret_cast<char *>(a.v_r) + c.flat_elem0 * 4;
        char *va_ptr = reinterpret_cast<char *>(a.v_a) + c.flat_elem0 * 4;
        const float alpha = a.alpha, beta = 1.0f - a.alpha;
        for (uint32_t vec = threadIdx.x; vec < c.n_vecs; vec += kThreads) {
            const Raw rg = ld_off<S::kNT, Raw>(g_ptr, vec * RB), r0 = ld_off<S::kNT, Raw>(v0, vec * RB),
                      r1 = ld_off<S::kNT, Raw>(v1, vec * RB);
            v4f vr[S::kF4], va[S::kF4];
#pragma unroll
            for (int q = 0; q < S::kF4; ++q) {
                vr[q] = ld_off<S::kNT, v4f>(vr_ptr, vec * FB + 16u * q);
                va[q] = ld_off<S::kNT, v4f>(va_ptr, vec * FB + 16u * q);
            }
            float g[E], w0[E], w1[E];
            S::widen(rg, g);
            S::widen(r0, w0);
            S::widen(r1, w1);
#pragma unroll
            for (int q = 0; q < S::kF4; ++q) {
                float r[4] = {vr[q].x, vr[q].y, vr[q].z, vr[q].w}, s4[4] = {va[q].x, va[q].y, va[q].z, va[q].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float gi = g[4 * q + i];
                    acc0 = fmaf(s4[i], gi - r[i], acc0);
                    acc1 = fmaf(s4[i], s4[i], acc1);
                    r[i] = fmaf(alpha, r[i], beta * gi);
                    s4[i] = fmaf(alpha, s4[i], beta * (gi * gi * (w1[4 * q + i] - w0[4 * q + i])));
                }
                st_off<S::kNT>(vr_ptr, vec * FB + 16u * q, make_v4f(r[0], r[1], r[2], r[3]));
                st_off<S::kNT>(va_ptr, vec * FB + 16u * q, make_v4f(s4[0], s4[1], s4[2], s4[3]));
            }
        }
    }
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const float s0 = wave_sum(acc0), s1 = wave_sum(acc1);
    if (lane == 0) { lds.red[0][wave] = s0; lds.red[1][wave] = s1; }
    __syncthreads();
    if (threadIdx.x < 2) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += lds.red[threadIdx.x][w];
        a.partials[(size_t)threadIdx.x * a.n_chunks + chunk] = s;
    }
}

#if FERRET_TU_COMMON
// The per-stage reductions, one small kernel after the pass that wrote the partials: one workgroup of 1024 lanes
// per stage and job.  (Forming the sums inside the step kernel instead, by the last of a
// stage's workgroups to arrive, was measured on MI355X and is slower: the arrival count needs one device-scope
// atomic per workgroup, and 42 000 of those on one address take 545 us; spread over 16 counters per stage on
// separate cache lines they still cost, together with the wait for the partial's store to be acknowledged,
// 12 us of a 306 us kernel, more than the 7 us that the second launch and its gap cost.)
// Grid = (stage, job), job = first_job + blockIdx.y: jobs 0..2 add up one of the three norm series of the stage, job 3
// sums the stage's two lambda series and takes the lambda step.  A launch covers the jobs that are wanted: norms
// only (0..2), norms and lambda step after a one-pass adaptive step (0..3), or the lambda step alone (3).
constexpr uint32_t kJobLambda = 3;
__global__ void __launch_bounds__(kSumLanes) stage_sums_kernel(const StepArgs a, uint32_t first_job) {
    __shared__ double red[kSeries][kSumWaves];
    const uint32_t j = blockIdx.x, job = first_job + blockIdx.y;
    const bool absent = (a.accum || a.masked) && a.mode[j] == 0;     // the stage took no part: nothing was written for it
    const uint32_t c0 = a.stage[j].chunk_begin;
    const uint32_t c1 = j + 1 < a.n_stages ? a.stage[j + 1].chunk_begin : a.n_chunks;
    if (job == kJobLambda) {
        if (a.stage[j].tau == 0 || absent) return;      // nothing to tune, or no gradient arrived
        // the two series: 0 and 1 when the state pass produced them, 3 and 4 when the one-pass step did
        double total[2];
        ordered_sums<2, kSumLanes>(a.partials + (size_t)(a.fused_lambda ? 3u : 0u) * a.n_chunks, a.n_chunks, c0, c1, red, total);
        if (threadIdx.x == 0)
            a.lambda_dev[j] = lambda_descent_step(a.lambda_dev[j], total[0], total[1], a.alpha, a.eta_lambda);
        return;
    }
    if (absent) {
        if (threadIdx.x == 0) a.norms_out[j * 3 + job] = 0.f;
        return;
    }
    double total[1];
    ordered_sums<1, kSumLanes>(a.partials + (size_t)job * a.n_chunks, a.n_chunks, c0, c1, red, total);
    if (threadIdx.x == 0) a.norms_out[j * 3 + job] = (float)total[0];
}

// ---- push: fp32 source -> ring slot (+ master) ----------------------------------------------------
template <bool BF16>
__global__ void __launch_bounds__(kThreads) push_kernel(const PushArgs a) {
    __shared__ StageDesc tab[FERRET_MAX_STAGES];
    {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(a.stage);
        uint32_t *dst = reinterpret_cast<uint32_t *>(tab);
        const uint32_t n_words = a.n_stages * (sizeof(StageDesc) / 4);
        for (uint32_t i = threadIdx.x; i < n_words; i += kThreads) dst[i] = src[i];
    }
    __syncthreads();
    uint32_t stage = 0;
    for (uint32_t chunk = blockIdx.x; chunk < a.n_chunks; chunk += gridDim.x) {
        while (stage + 1 < a.n_stages && chunk >= tab[stage + 1].chunk_begin) ++stage;
        stage = uniform(stage);
        const StageDesc &d = tab[stage];
        const uint32_t chunk_elems = uniform(d.chunk_elems);
        const uint64_t e0 = (uint64_t)(chunk - uniform(d.chunk_begin)) * chunk_elems;
        const uint64_t left = uniform(d.n_elems) - e0;
        const uint32_t n_here = left < chunk_elems ? (uint32_t)left : chunk_elems;
        const uint64_t flat0 = uniform(d.flat_off) + e0;
        const uint64_t ring0 = uniform(d.ring_base) + (uint64_t)uniform((uint32_t)d.head) * uniform(d.slot_stride) + e0;
        const float4 *src = reinterpret_cast<const float4 *>(a.src + flat0);
        float4 *mst = a.master ? reinterpret_cast<float4 *>(a.master + flat0) : nullptr;
        if (BF16) {
            uint4 *dst = reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(a.ring) + ring0);
            for (uint32_t v = threadIdx.x; v < n_here / 8; v += kThreads) {
                float4 x0 = src[2 * (size_t)v], x1 = src[2 * (size_t)v + 1];
                uint4 o;
                o.x = bf16_pack(x0.x, x0.y); o.y = bf16_pack(x0.z, x0.w);
                o.z = bf16_pack(x1.x, x1.y); o.w = bf16_pack(x1.z, x1.w);
                dst[v] = o;
                if (mst) { mst[2 * (size_t)v] = x0; mst[2 * (size_t)v + 1] = x1; }
            }
        } else {
            float4 *dst = reinterpret_cast<float4 *>(reinterpret_cast<float *>(a.ring) + ring0);
            for (uint32_t v = threadIdx.x; v < n_here / 4; v += kThreads) dst[v] = src[v];
        }
    }
}

// Plain streaming copy: one workgroup per 16 KiB, four 16-byte vectors per lane, loads before stores.
constexpr int kCopyVecsPerLane = 4;
__global__ void __launch_bounds__(kThreads) copy_kernel(v4u *dst, const v4u *src, size_t n_vecs) {
    const size_t base = (size_t)blockIdx.x * kThreads * kCopyVecsPerLane + threadIdx.x;
    v4u x[kCopyVecsPerLane];
#pragma unroll
    for (int u = 0; u < kCopyVecsPerLane; ++u)
        if (base + (size_t)u * kThreads < n_vecs) x[u] = ld<true>(&src[base + (size_t)u * kThreads]);
#pragma unroll
    for (int u = 0; u < kCopyVecsPerLane; ++u)
        if (base + (size_t)u * kThreads < n_vecs) st<true>(&dst[base + (size_t)u * kThreads], x[u]);
}

// Plain streaming read with the same shape; the data is summed and compared with a value it never has.
__global__ void __launch_bounds__(kThreads) read_kernel(const v4u *src, size_t n_vecs, v4u *sink) {
    const size_t base = (size_t)blockIdx.x * kThreads * kCopyVecsPerLane + threadIdx.x;
    v4u x[kCopyVecsPerLane];
#pragma unroll
    for (int u = 0; u < kCopyVecsPerLane; ++u) {
        x[u] = v4u{0u, 0u, 0u, 0u};
        if (base + (size_t)u * kThreads < n_vecs) x[u] = ld<true>(&src[base + (size_t)u * kThreads]);
    }
    v4u s = x[0];
#pragma unroll
    for (int u = 1; u < kCopyVecsPerLane; ++u) s += x[u];
    if (s.x == 0x9e3779b9u && s.y == 0x7f4a7c15u && s.z == 0xf39cc060u && s.w == 0x5cedc834u) sink[0] = s;
}

// Streaming kernel with the step's traffic shape and none of its arithmetic: NR read streams added
// element-wise into one write stream.  One workgroup per kMixVecsPerLane vectors per lane (8 KiB of each
// stream), processed one vector at a time: all NR loads, the sum, the store.
constexpr int kMixVecsPerLane = 2;
template <int NR>
__global__ void __launch_bounds__(kThreads) mix_kernel(char *dst, const char *src, size_t stride, size_t n_vecs) {
    const size_t base = (size_t)blockIdx.x * kThreads * kMixVecsPerLane;
    const size_t left = n_vecs - base;                                 // > 0 by the launch's grid
    const uint32_t here = left < (size_t)(kThreads * kMixVecsPerLane) ? (uint32_t)left : (uint32_t)(kThreads * kMixVecsPerLane);
    const char *s0 = src + base * 16;
    char *d0 = dst + base * 16;
    for (uint32_t vec = threadIdx.x; vec < here; vec += kThreads) {
        v4f x[NR];
#pragma unroll
        for (int i = 0; i < NR; ++i) x[i] = ld_off<true, v4f>(s0 + (size_t)i * stride, vec * 16u);
        v4f sum = x[0];
#pragma unroll
        for (int i = 1; i < NR; ++i) sum += x[i];
        st_off<true>(d0, vec * 16u, sum);
    }
}

// ---- per-launch event timing of the step kernel ---------------------------------------------------
// One profiling session per process at a time, owned by the thread that began it: only that thread's launches
// are recorded (another thread stepping another plan meanwhile is left alone), and begin/end from two threads
// cannot interleave.
struct Profiler {
    std::mutex mutex;
    std::vector<hipEvent_t> start, stop;
    int32_t used = 0;
    bool on = false;
    std::thread::id owner;
};
static Profiler g_prof;

static void profile_destroy_events() {
    for (size_t i = 0; i < g_prof.start.size(); ++i) {
        if (g_prof.start[i]) (void)hipEventDestroy(g_prof.start[i]);
        if (g_prof.stop[i]) (void)hipEventDestroy(g_prof.stop[i]);
    }
    g_prof.start.clear();
    g_prof.stop.clear();
}

int profile_begin(int32_t capacity) {
    std::lock_guard<std::mutex> lock(g_prof.mutex);
    if (g_prof.on) return -1;
    g_prof.start.assign(capacity, nullptr);
    g_prof.stop.assign(capacity, nullptr);
    for (int32_t i = 0; i < capacity; ++i) {
        hipError_t e = hipEventCreate(&g_prof.start[i]);
        if (e == hipSuccess) e = hipEventCreate(&g_prof.stop[i]);
        if (e != hipSuccess) { profile_destroy_events(); return (int)e; }      // nothing is left behind
    }
    g_prof.used = 0;
    g_prof.owner = std::this_thread::get_id();
    g_prof.on = true;
    return 0;
}

int profile_end(float *ms_out, int32_t cap, int32_t *n_out) {
    std::lock_guard<std::mutex> lock(g_prof.mutex);
    if (!g_prof.on) return -1;
    if (g_prof.owner != std::this_thread::get_id()) return -2;
    hipError_t e = hipSuccess;
    if (g_prof.used > 0) e = hipEventSynchronize(g_prof.stop[g_prof.used - 1]);
    for (int32_t i = 0; i < g_prof.used && i < cap && e == hipSuccess; ++i)
        e = hipEventElapsedTime(&ms_out[i], g_prof.start[i], g_prof.stop[i]);
    *n_out = g_prof.used;
    profile_destroy_events();
    g_prof.on = false;
    return (int)e;
}

// The event pair for the launch the calling thread is about to make, or -1 if none is to be recorded.
static int32_t profile_claim() {
    std::lock_guard<std::mutex> lock(g_prof.mutex);
    if (!g_prof.on || g_prof.owner != std::this_thread::get_id() || g_prof.used >= (int32_t)g_prof.start.size()) return -1;
    return g_prof.used++;
}

// ---- launchers ------------------------------------------------------------------------------------
static int g_cu_count[64];   // per device ordinal, 0 = not queried yet

static int cu_count(int *err) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { *err = (int)e; return 0; }
    if (dev < 0 || dev >= 64) return 256;
    if (g_cu_count[dev] == 0) {
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) { *err = (int)e; return 0; }
        g_cu_count[dev] = n > 0 ? n : 256;
    }
    return g_cu_count[dev];
}

static uint32_t grid_for(const ferret_plan &plan, uint32_t n_chunks, int *err) {
    int bpc = plan.blocks_per_cu;
    if (bpc <= 0) return n_chunks;                // default: one workgroup per chunk
    int cus = cu_count(err);
    if (*err) return 0;
    uint64_t g = (uint64_t)cus * (uint64_t)bpc;
    return g < n_chunks ? (uint32_t)g : n_chunks;
}

// Resident-workgroup cap.  Measured on MI355X: for steps that stream far more than the 256 MB
// memory-side cache holds, throughput depends on how many workgroups a CU holds at once, with a sharp
// optimum that moves with the traffic of one chunk: with 2048-element chunks of fp32 in every stage the best
// count is 5 for K' = 0 (4 when the weight gap is read as well), 4 for K' = 1, 3 for K' = 2..4, 2 beyond
// (and 3 for bf16 at K' = 4); one too few costs 5-10 %, one too many 2-5 %.  ceil(120 KiB / bytes one
// chunk moves) reproduces those counts.  The launch enforces the count by reserving LDS the kernel never
// touches: with 160 KiB of LDS per CU, a workgroup that holds floor(160 KiB / cap) bytes lets exactly
// `cap` of them be resident.
constexpr uint32_t kLdsPerCu = 160u * 1024u;
constexpr uint32_t kLdsPerBlockMax = 64u * 1024u;
// LDS is granted in granules; measured on MI355X: a workgroup asking for 53,744 bytes fits three times
// into a CU and one asking for 53,776 does not, which is what a 1280-byte granule (160 KiB / 128) gives
// and a 512- or 1024-byte one would not.  Totals below are multiples of 1280 with every partial granule
// counted against the workgroup, so they also hold if the granule is 256 or 512 bytes.
constexpr uint32_t kLdsGranule = 1280u;

// Dynamic LDS bytes that make exactly `cap` workgroups fit a CU, for a kernel with `static_bytes` of its own.
static uint32_t dyn_lds_for_cap(int32_t cap, uint32_t static_bytes) {
    if (cap <= 0) return 0;
    uint32_t total = kLdsPerCu / (uint32_t)cap / kLdsGranule * kLdsGranule;
    if (total > kLdsPerBlockMax) total = kLdsPerBlockMax;
    return total > static_bytes ? total - static_bytes : 0u;
}
constexpr uint64_t kInFlightTargetBytes = 120u * 1024u;
constexpr uint64_t kStateTargetBytes = 100u * 1024u;     // the same for lambda_state_kernel

// Also reports, for launches that stream (traffic far beyond the memory-side cache), the K' of the stage at the
// traffic-weighted median (-1 for launches that do not stream).
static uint32_t reserve_lds_for_cap(const ferret_plan &plan, const StepArgs &a, bool persistent, int32_t *median_kp) {
    int32_t cap = plan.resident_cap;
    *median_kp = -1;
    {
        // default: cap only steps whose traffic is far beyond the memory-side cache; steps that run out
        // of that cache are latency-bound instead and want every wave they can get
        // Bytes one chunk of each stage moves; the cap is taken from the stage at the traffic-weighted median,
        // because workgroups are dispatched in chunk order and mostly one stage's chunks are resident at a time.
        const uint64_t sb = plan.prec == FERRET_F32 ? 4 : 2;
        uint64_t total = 0;
        uint64_t block[FERRET_MAX_STAGES], traffic[FERRET_MAX_STAGES];
        uint32_t order[FERRET_MAX_STAGES], kps[FERRET_MAX_STAGES], n = 0;
        for (uint32_t j = 0; j < a.n_stages; ++j) {
            if ((a.accum || a.masked) && a.mode[j] == 0) continue;
            const uint32_t kp = a.stage[j].kp;
            // versions loaded together: all K'+1 on the unrolled paths; on the streamed one a batch counts (measured
            // with its two register sets used in turn: best cap 3-4 for bf16, 2-3 for fp32, which this reproduces)
            uint64_t per = (uint64_t)inflight_bytes_per_elem(plan.prec, (int32_t)kp);
            if (kp == 0 && a.stage[j].tau > 0 && (a.partials || a.penalized)) per += sb;   // V[0] for the gap
            if (a.fused_lambda && a.stage[j].tau > 0) per += sb + 8;   // V[1], v_r, v_a
            if (a.accum) {
                if (a.mode[j] == 2) {
                    per += 8 - sb;          // an arrival that updates: the running sum read and cleared as well
                } else {
                    // an arrival that only adds writes no version and touches no master; what it loads together is the
                    // gradient, the versions and the running sum (measured: 350 M parameters in bf16, K = 4, 1190 us at
                    // 3 resident workgroups, 1101 at the 4 this gives; fp32 K = 1 and K = 3 stay at their optimum, 3)
                    const uint64_t versions = kp <= (uint32_t)kUnrolledItersMax ? kp + 1u : (uint32_t)kStreamBatch;
                    per = sb * (versions + 1u) + 4u;
                }
            }
            block[n] = per * a.stage[j].chunk_elems;
            traffic[n] = a.stage[j].n_elems * (sb * (kp + 3u) + (plan.prec == FERRET_F32 ? 0u : 8u) +
                                               (a.fused_lambda && a.stage[j].tau > 0 ? sb + 16u : 0u));
            total += traffic[n];
            kps[n] = kp;
            order[n] = n;
            ++n;
        }
        if (total <= kCapThresholdBytes || n == 0) return cap > 0 ? dyn_lds_for_cap(cap, (persistent ? (uint32_t)sizeof(StageDesc) * FERRET_MAX_STAGES : 0u) + (uint32_t)sizeof(StepLds)) : 0;
        for (uint32_t i = 1; i < n; ++i)                      // insertion sort by bytes per chunk
            for (uint32_t k = i; k > 0 && block[order[k]] < block[order[k - 1]]; --k) {
                const uint32_t t = order[k]; order[k] = order[k - 1]; order[k - 1] = t;
            }
        // With the lambda block fused in, the stage at the 40 % point instead: a cap too low for the lighter chunks
        // costs more than one too high for the heavier ones (measured at the ViT-B-sized workload with one iteration
        // per version step, where 45 % of the traffic is in chunks of <= 52 KiB and the rest in 64-88 KiB: cap 3
        // 605 us, cap 2 643 us; with K <= 5 all heavy stages share one chunk size and either point gives cap 2).
        const uint64_t point = a.fused_lambda ? 4u : 5u;      // tenths of the traffic
        uint64_t seen = 0, block_bytes = block[order[n - 1]];
        for (uint32_t i = 0; i < n; ++i) {
            seen += traffic[order[i]];
            if (10 * seen >= point * total) { block_bytes = block[order[i]]; break; }
        }
        // the traffic-weighted median of K' itself: the smallest k with at least half the traffic in stages of K' <= k
        for (uint32_t k = 0; *median_kp < 0; ++k) {
            uint64_t upto = 0;
            for (uint32_t i = 0; i < n; ++i) upto += kps[i] <= k ? traffic[i] : 0u;
            if (2 * upto >= total) *median_kp = (int32_t)k;
        }
        if (cap == 0) {
            cap = (int32_t)((kInFlightTargetBytes + block_bytes - 1) / block_bytes);
            // Two resident workgroups are the optimum only with the lambda block fused in (its three write streams);
            // wherever the rule above says 2 for another launch, 3 measured the same or better: fp32 K = 5 383 -> 380 us,
            // accumulation at K = 1 294 -> 275 (arrivals that only add) and 340 -> 335 (arrivals that update), bf16
            // K = 8 1556 -> 1487, bf16 accumulation with one iteration per version step 2063 -> 1692 and 2456 -> 2141.
            const int32_t floor_cap = a.fused_lambda ? 2 : 3;
            if (cap < floor_cap) cap = floor_cap;
            if (cap >= 8) return 0;                           // 8 fit anyway
        }
    }
    if (cap <= 0) return 0;
    // what step_kernel declares itself: the reduction buffers, and the stage table of the persistent variant
    const uint32_t used = (persistent ? (uint32_t)sizeof(StageDesc) * FERRET_MAX_STAGES : 0u) + (uint32_t)sizeof(StepLds);
    return dyn_lds_for_cap(cap, used);
}

#endif  // FERRET_TU_COMMON

template <typename S, bool PERSISTENT, int LEVEL>
static hipError_t launch_step_level(const StepArgs &a, bool norms, bool gout, bool elide, uint32_t grid,
                                    uint32_t dyn_lds, hipStream_t st) {
#define FERRET_LAUNCH(NO, OUT) \
    hipLaunchKernelGGL((step_kernel<S, PERSISTENT, LEVEL, NO, OUT>), dim3(grid), dim3(kThreads), dyn_lds, st, a)
    if constexpr (S::kMaster && !PERSISTENT) {
        if (elide) {       // newest version recomputed from the master instead of read
            if (norms) { if (gout) FERRET_LAUNCH(true, 5); else FERRET_LAUNCH(true, 4); }
            else       { if (gout) FERRET_LAUNCH(false, 5); else FERRET_LAUNCH(false, 4); }
            return hipGetLastError();
        }
    }
    if (norms) { if (gout) FERRET_LAUNCH(true, 1); else FERRET_LAUNCH(true, 0); }
    else       { if (gout) FERRET_LAUNCH(false, 1); else FERRET_LAUNCH(false, 0); }
#undef FERRET_LAUNCH
    return hipGetLastError();
}

// Launches of the step-size-penalising comparison methods: no iterations, so the smallest kernel level.
template <typename S>
static hipError_t launch_step_penalized(const StepArgs &a, bool norms, bool gout, uint32_t grid, uint32_t dyn_lds,
                                        hipStream_t st) {
#define FERRET_LAUNCH(NO, OUT) \
    hipLaunchKernelGGL((step_kernel<S, false, 0, NO, OUT>), dim3(grid), dim3(kThreads), dyn_lds, st, a)
    if (norms) { if (gout) FERRET_LAUNCH(true, 9); else FERRET_LAUNCH(true, 8); }
    else       { if (gout) FERRET_LAUNCH(false, 9); else FERRET_LAUNCH(false, 8); }
#undef FERRET_LAUNCH
    return hipGetLastError();
}

// Launches with the "update lambda" block fused in (one pass; the iterations use lambda as it was before
// this call's lambda step).
template <typename S, int LEVEL>
static hipError_t launch_step_fused_level(const StepArgs &a, bool norms, bool gout, uint32_t grid, uint32_t dyn_lds,
                                          hipStream_t st) {
#define FERRET_LAUNCH(NO, OUT) \
    hipLaunchKernelGGL((step_kernel<S, false, LEVEL, NO, OUT>), dim3(grid), dim3(kThreads), dyn_lds, st, a)
    if (norms) { if (gout) FERRET_LAUNCH(true, 17); else FERRET_LAUNCH(true, 16); }
    else       { if (gout) FERRET_LAUNCH(false, 17); else FERRET_LAUNCH(false, 16); }
#undef FERRET_LAUNCH
    return hipGetLastError();
}
template <typename S>
static hipError_t launch_step_fused(const StepArgs &a, int level, bool norms, bool gout, uint32_t grid,
                                    uint32_t dyn_lds, hipStream_t st) {
    if (level == 0) return launch_step_fused_level<S, 0>(a, norms, gout, grid, dyn_lds, st);
    if (level == 1) return launch_step_fused_level<S, 1>(a, norms, gout, grid, dyn_lds, st);
    return launch_step_fused_level<S, 2>(a, norms, gout, grid, dyn_lds, st);
}

// Gradient-accumulation launches: one workgroup per chunk, every K' covered by one kernel.
template <typename S>
static hipError_t launch_step_accum(const StepArgs &a, bool norms, bool gout, uint32_t grid, uint32_t dyn_lds,
                                    hipStream_t st) {
#define FERRET_LAUNCH(NO, OUT) \
    hipLaunchKernelGGL((step_kernel<S, false, 2, NO, OUT>), dim3(grid), dim3(kThreads), dyn_lds, st, a)
    if (norms) { if (gout) FERRET_LAUNCH(true, 3); else FERRET_LAUNCH(true, 2); }
    else       { if (gout) FERRET_LAUNCH(false, 3); else FERRET_LAUNCH(false, 2); }
#undef FERRET_LAUNCH
    return hipGetLastError();
}

// Accumulation with the "update lambda" block fused in.
template <typename S>
static hipError_t launch_step_accum_fused(const StepArgs &a, bool norms, bool gout, uint32_t grid, uint32_t dyn_lds,
                                          hipStream_t st) {
#define FERRET_LAUNCH(NO, OUT) \
    hipLaunchKernelGGL((step_kernel<S, false, 2, NO, OUT>), dim3(grid), dim3(kThreads), dyn_lds, st, a)
    if (norms) { if (gout) FERRET_LAUNCH(true, 19); else FERRET_LAUNCH(true, 18); }
    else       { if (gout) FERRET_LAUNCH(false, 19); else FERRET_LAUNCH(false, 18); }
#undef FERRET_LAUNCH
    return hipGetLastError();
}

template <typename S, bool PERSISTENT>
static hipError_t launch_step_typed(const StepArgs &a, int level, bool norms, bool gout, bool elide, uint32_t grid,
                                    uint32_t dyn_lds, hipStream_t st) {
    if (level == 0) return launch_step_level<S, PERSISTENT, 0>(a, norms, gout, elide, grid, dyn_lds, st);
    if (level == 1) return launch_step_level<S, PERSISTENT, 1>(a, norms, gout, elide, grid, dyn_lds, st);
    return launch_step_level<S, PERSISTENT, 2>(a, norms, gout, elide, grid, dyn_lds, st);
}

// What launch_step has decided; the per-type halves below turn it into the kernel launch.
struct StepLaunch {
    bool persistent, norms, gout, elide;
    bool cached;         // ordinary cached accesses instead of non-temporal ones (plain step at the smallest level only)
    int level;
    uint32_t chunks;     // chunks the launch covers (one workgroup each unless persistent)
    uint32_t grid, lds;
};

template <typename S, typename SCached>
static hipError_t launch_step_for(const StepArgs &a, const StepLaunch &l, hipStream_t st) {
    if (l.cached) return launch_step_level<SCached, false, 0>(a, l.norms, l.gout, false, l.grid, l.lds, st);
    if (a.fused_lambda && a.accum) return launch_step_accum_fused<S>(a, l.norms, l.gout, l.chunks, l.lds, st);
    if (a.fused_lambda) return launch_step_fused<S>(a, l.level, l.norms, l.gout, l.chunks, l.lds, st);
    if (a.penalized) return launch_step_penalized<S>(a, l.norms, l.gout, l.chunks, l.lds, st);
    if (a.accum) return launch_step_accum<S>(a, l.norms, l.gout, l.chunks, l.lds, st);
    return l.persistent ? launch_step_typed<S, true>(a, l.level, l.norms, l.gout, false, l.grid, l.lds, st)
                        : launch_step_typed<S, false>(a, l.level, l.norms, l.gout, l.elide, l.grid, l.lds, st);
}
template <typename S>
static hipError_t launch_state_for(const StepArgs &a, uint32_t lds, hipStream_t st) {
    hipLaunchKernelGGL(lambda_state_kernel<S>, dim3(a.chunk_end - a.chunk_base), dim3(kThreads), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_step_f32(const StepArgs &a, const StepLaunch &l, hipStream_t st);
hipError_t launch_step_bf16(const StepArgs &a, const StepLaunch &l, hipStream_t st);
hipError_t launch_state_f32(const StepArgs &a, uint32_t lds, hipStream_t st);
hipError_t launch_state_bf16(const StepArgs &a, uint32_t lds, hipStream_t st);
#if FERRET_TU_F32
hipError_t launch_step_f32(const StepArgs &a, const StepLaunch &l, hipStream_t st) { return launch_step_for<F32Store, F32StoreCached>(a, l, st); }
hipError_t launch_state_f32(const StepArgs &a, uint32_t lds, hipStream_t st) { return launch_state_for<F32Store>(a, lds, st); }
#endif
#if FERRET_TU_BF16
hipError_t launch_step_bf16(const StepArgs &a, const StepLaunch &l, hipStream_t st) { return launch_step_for<Bf16Store, Bf16StoreCached>(a, l, st); }
hipError_t launch_state_bf16(const StepArgs &a, uint32_t lds, hipStream_t st) { return launch_state_for<Bf16Store>(a, lds, st); }
#endif

#if FERRET_TU_COMMON
int launch_step(const ferret_plan &plan, const StepArgs &args, void *stream) {
    if (args.n_chunks == 0) return 0;
    int err = 0;
    const uint32_t n_launch = args.chunk_end - args.chunk_base;     // 0: no stage takes part, only the norms are cleared
    const uint32_t grid = grid_for(plan, n_launch, &err);
    if (err) return err;
    hipStream_t st = static_cast<hipStream_t>(stream);
    StepArgs a = args;
    int streamed = 0;    // kernel level: which K' the launch has to cover
    for (uint32_t j = 0; j < a.n_stages; ++j) {
        const int need = a.stage[j].kp <= kUnrolledItersSmall ? 0 : (a.stage[j].kp <= kUnrolledItersMid ? 1 : 2);
        streamed = need > streamed ? need : streamed;
    }
    const bool norms = a.norms_out != nullptr, gout = a.grad_out != nullptr;
    const int32_t timed = profile_claim();
    if (timed >= 0) (void)hipEventRecord(g_prof.start[timed], st);
    StepLaunch l;
    l.persistent = grid < n_launch && !a.accum && !a.penalized && !a.fused_lambda;
    l.chunks = n_launch;
    l.norms = norms;
    l.gout = gout;
    l.elide = plan.newest_from_master != 0;
    l.level = streamed;
    l.grid = l.persistent ? grid : n_launch;
    int32_t median_kp = -1;
    l.lds = reserve_lds_for_cap(plan, a, l.persistent, &median_kp);
    // XCD grouping (measured on MI355X at the resident caps above, step_kernel us without -> with 16 chunks per XCD):
    // fp32, K' = 3: 306 -> 299; K' = 4: 355 -> 347; one iteration per version step (K' 7..0): 400 -> 395; accumulation
    // 396 -> 388; 350 M parameters as fp32, K' = 4: 1528 -> 1487; but K' <= 2: 256 -> 257, 213 -> 214; with the lambda block
    // fused in 530 -> 534; bf16 storage 1132 -> 1166.  Group sizes of 14..24 are equivalent, 2..8 and beyond 32 lose.
    // So: fp32 launches that stream and whose median stage has K' >= 3 group 16 chunks per XCD, everything else none.
    a.xcd_group = l.persistent ? 1u
                  : plan.xcd_group > 0 ? (uint32_t)plan.xcd_group
                  : (plan.prec == FERRET_F32 && median_kp >= 3 && !a.fused_lambda) ? 16u : 1u;
    const uint64_t working_set = working_set_bytes(plan.prec, plan.ring_elems, plan.flat_elems);
    l.cached = !l.persistent && streamed == 0 && !a.accum && !a.penalized && !a.fused_lambda && !a.lambda_dev && !l.elide &&
               plan.cache_policy != 2 && (plan.cache_policy == 1 || working_set <= kCacheResidentBytes);
    hipError_t e = hipSuccess;
    if (n_launch > 0) e = plan.prec == FERRET_F32 ? launch_step_f32(a, l, st) : launch_step_bf16(a, l, st);
    if (timed >= 0) (void)hipEventRecord(g_prof.stop[timed], st);
    if (e != hipSuccess) return (int)e;
    // the stages' sums: the three norms, and after a one-pass adaptive step lambda's step for the next call
    const uint32_t first_job = norms ? 0u : kJobLambda, n_jobs = (norms ? 3u : 0u) + (a.fused_lambda ? 1u : 0u);
    if (n_jobs > 0) {
        hipLaunchKernelGGL(stage_sums_kernel, dim3(a.n_stages, n_jobs), dim3(kSumLanes), 0, st, a, first_job);
        e = hipGetLastError();
    }
    return (int)e;
}

int launch_lambda_update(const ferret_plan &plan, const StepArgs &args, void *stream) {
    if (args.n_chunks == 0 || args.chunk_end == args.chunk_base) return 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // same kind of resident-workgroup rule as the step (measured optimum for this pass: 2 workgroups per
    // CU at fp32, 352 us against 381 us uncapped at the ViT-B-sized workload); it moves 3 storage elements +
    // 4 fp32 per parameter
    uint32_t lds = 0;
    {
        const uint64_t per = (plan.prec == FERRET_F32 ? 4u : 2u) * 3u + 16u;
        uint64_t bytes = 0, elems = 0, weighted = 0;
        for (uint32_t j = 0; j < args.n_stages; ++j)
            if (args.stage[j].tau >= 1 && !((args.accum || args.masked) && args.mode[j] == 0)) {
                bytes += args.stage[j].n_elems * per;
                elems += args.stage[j].n_elems;
                weighted += args.stage[j].n_elems * args.stage[j].chunk_elems;
            }
        const uint64_t chunk_elems = elems ? weighted / elems : 1;     // size-weighted mean over the stages that take part
        const int32_t env = plan.resident_cap;
        int32_t cap = env != 0 ? env : (bytes > kCapThresholdBytes
                                            ? (int32_t)((kStateTargetBytes + chunk_elems * per - 1) / (chunk_elems * per)) : -1);
        if (cap > 0 && cap < 8) {
            if (cap < 2) cap = 2;
            lds = dyn_lds_for_cap(cap, (uint32_t)sizeof(StepLds));
        }
    }
    hipError_t e = plan.prec == FERRET_F32 ? launch_state_f32(args, lds, st) : launch_state_bf16(args, lds, st);
    if (e != hipSuccess) return (int)e;
    hipLaunchKernelGGL(stage_sums_kernel, dim3(args.n_stages, 1), dim3(kSumLanes), 0, st, args, kJobLambda);
    return (int)hipGetLastError();
}

int launch_push(const ferret_plan &plan, const PushArgs &a, void *stream) {
    if (a.n_chunks == 0) return 0;
    int err = 0;
    const uint32_t grid = grid_for(plan, a.n_chunks, &err);
    if (err) return err;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (plan.prec == FERRET_F32)
        hipLaunchKernelGGL(push_kernel<false>, dim3(grid), dim3(kThreads), 0, st, a);
    else
        hipLaunchKernelGGL(push_kernel<true>, dim3(grid), dim3(kThreads), 0, st, a);
    return (int)hipGetLastError();
}

int launch_copy(void *dst, const void *src, size_t n_bytes, void *stream) {
    const size_t n_vecs = n_bytes / 16;
    const size_t per_block = (size_t)kThreads * kCopyVecsPerLane;
    const size_t blocks = (n_vecs + per_block - 1) / per_block;
    if (blocks > 0x7fffffffull) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(copy_kernel, dim3((uint32_t)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<v4u *>(dst), static_cast<const v4u *>(src), n_vecs);
    return (int)hipGetLastError();
}

int launch_read(const void *src, size_t n_bytes, void *sink, void *stream) {
    const size_t n_vecs = n_bytes / 16;
    const size_t per_block = (size_t)kThreads * kCopyVecsPerLane;
    const size_t blocks = (n_vecs + per_block - 1) / per_block;
    if (blocks > 0x7fffffffull) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(read_kernel, dim3((uint32_t)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const v4u *>(src), n_vecs, static_cast<v4u *>(sink));
    return (int)hipGetLastError();
}

int launch_mix(void *dst, const void *src, size_t src_stride_bytes, int n_reads, size_t n_bytes, int resident_cap,
               void *stream) {
    const size_t n_vecs = n_bytes / 16;
    const size_t per_block = (size_t)kThreads * kMixVecsPerLane;
    const size_t blocks = (n_vecs + per_block - 1) / per_block;
    if (blocks > 0x7fffffffull) return (int)hipErrorInvalidValue;
    const uint32_t lds = dyn_lds_for_cap(resident_cap, 0u);
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *d = static_cast<char *>(dst);
    const char *s = static_cast<const char *>(src);
#define FERRET_MIX(NR) \
    case NR: hipLaunchKernelGGL(mix_kernel<NR>, dim3((uint32_t)blocks), dim3(kThreads), lds, st, d, s, src_stride_bytes, n_vecs); break
    switch (n_reads) {
        FERRET_MIX(1); FERRET_MIX(2); FERRET_MIX(3); FERRET_MIX(4);
        FERRET_MIX(5); FERRET_MIX(6); FERRET_MIX(7); FERRET_MIX(8);
        default: return (int)hipErrorInvalidValue;
    }
#undef FERRET_MIX
    return (int)hipGetLastError();
}

const char *device_error_string(int err) { return hipGetErrorString(static_cast<hipError_t>(err)); }

// ---- library-owned scratch of the entry point that allocates nothing ---------------------------------
// The per-chunk partial sums of ferret_compensate_step_noalloc live in this array instead of a caller's
// workspace.  Every GPU the library runs on holds its own copy at its own address; in host code the
// array's name is only a handle for hipGetSymbolAddress, never an address to pass to a kernel.
static __device__ __align__(256) unsigned char scratch[FERRET_NOALLOC_SCRATCH_BYTES];
static void *g_scratch_ptr[64];          // per device ordinal: device address of `scratch`, null = not looked up yet
static std::mutex g_scratch_mutex;

int noalloc_scratch(void **ptr_out) {
    *ptr_out = nullptr;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= 64) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {           // once per device, with that device current
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr_out = g_scratch_ptr[dev];
    return 0;
}
#endif  // FERRET_TU_COMMON

}  // namespace ferret
