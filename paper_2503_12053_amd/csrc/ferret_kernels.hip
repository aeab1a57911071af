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
// Design for the machine:
//   * every operand is touched exactly once, with 128-bit loads/stores; consecutive lanes of a
//     64-wide wavefront touch consecutive 16-byte vectors, so a wavefront moves 1 KiB per
//     instruction per stream;
//   * all loads of a group (gradient + K'+1 versions, kUnroll vectors each) are issued before
//     the first arithmetic, so each lane keeps (K'+2)*kUnroll 16-byte requests in flight;
//   * a stage's tensors are one flat bucket; the stage table (48 B per stage) arrives as a
//     kernel argument, is copied to LDS once per workgroup, and a persistent grid strides over
//     fixed-size chunks, looking up the chunk's stage in LDS;
//   * the three per-stage sums are reduced inside the wavefront with cross-lane shuffles, across
//     the four wavefronts through LDS, written as one partial per chunk and summed in chunk
//     order (fp64) by a second tiny kernel, so results do not depend on the grid;
//   * no matrix cores: there is no contraction anywhere on this path.
#include <hip/hip_runtime.h>

#include <vector>

#include "ferret_internal.h"

namespace ferret {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kUnroll = 2;          // 16-byte vectors per lane per stream in flight
constexpr int kMaxUnrolledVersions = 5;   // K' <= 4 runs fully unrolled

// ---- small device helpers ---------------------------------------------------------------------
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

// One 16-byte vector of the storage type, widened to fp32 lanes.
struct F32Store {
    using Raw = float4;
    static constexpr int kElems = 4;
    __device__ static __forceinline__ void widen(const Raw &r, float (&x)[kElems]) {
        x[0] = r.x; x[1] = r.y; x[2] = r.z; x[3] = r.w;
    }
};
struct Bf16Store {
    using Raw = uint4;
    static constexpr int kElems = 8;
    __device__ static __forceinline__ void widen(const Raw &r, float (&x)[kElems]) {
        x[0] = bf16_lo(r.x); x[1] = bf16_hi(r.x); x[2] = bf16_lo(r.y); x[3] = bf16_hi(r.y);
        x[4] = bf16_lo(r.z); x[5] = bf16_hi(r.z); x[6] = bf16_lo(r.w); x[7] = bf16_hi(r.w);
    }
};

// A_I applied in place: g <- g + lambda * g * g * (v_new - v_old)
__device__ __forceinline__ float approximator(float g, float lambda, float v_new, float v_old) {
    return fmaf(lambda * g * g, v_new - v_old, g);
}

// Everything a lane needs to know about the chunk it works on (all wave-uniform).
template <typename S, int NV>
struct ChunkPtrs {
    const typename S::Raw *g;                 // gradient
    const typename S::Raw *v[NV];             // boundary versions, oldest first; v[NV-1] = V[tau]
    typename S::Raw *out;                     // slot of the new version
    float4 *master;                           // bf16 storage only
    float4 *g_out;                            // nullable
};

// Finish one vector: iterate, update, store.  x_g and x_v hold the widened inputs.
template <typename S, int NV, bool COMP, bool NORMS, bool GOUT>
__device__ __forceinline__ void finish_vector(const ChunkPtrs<S, NV> &p, uint32_t vec,
                                              const typename S::Raw &raw_g,
                                              const typename S::Raw (&raw_v)[NV], const float4 (&m_in)[2],
                                              float lambda, float lr, float (&acc)[3]) {
    constexpr int E = S::kElems;
    float g[E], prev[E], cur[E], first[E];
    S::widen(raw_g, g);
    S::widen(raw_v[0], prev);
#pragma unroll
    for (int e = 0; e < E; ++e) first[e] = prev[e];
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
    if constexpr (E == 4) {           // fp32 storage: update the newest version directly
        float4 o;
        o.x = fmaf(-lr, g[0], prev[0]); o.y = fmaf(-lr, g[1], prev[1]);
        o.z = fmaf(-lr, g[2], prev[2]); o.w = fmaf(-lr, g[3], prev[3]);
        p.out[vec] = o;
        if (GOUT) p.g_out[vec] = make_float4(g[0], g[1], g[2], g[3]);
    } else {                          // bf16 storage: update the master, store its rounding
        float4 m0 = m_in[0], m1 = m_in[1];
        m0.x = fmaf(-lr, g[0], m0.x); m0.y = fmaf(-lr, g[1], m0.y);
        m0.z = fmaf(-lr, g[2], m0.z); m0.w = fmaf(-lr, g[3], m0.w);
        m1.x = fmaf(-lr, g[4], m1.x); m1.y = fmaf(-lr, g[5], m1.y);
        m1.z = fmaf(-lr, g[6], m1.z); m1.w = fmaf(-lr, g[7], m1.w);
        p.master[2 * (size_t)vec] = m0;
        p.master[2 * (size_t)vec + 1] = m1;
        uint4 o;
        o.x = bf16_pack(m0.x, m0.y); o.y = bf16_pack(m0.z, m0.w);
        o.z = bf16_pack(m1.x, m1.y); o.w = bf16_pack(m1.z, m1.w);
        p.out[vec] = o;
        if (GOUT) {
            p.g_out[2 * (size_t)vec] = make_float4(g[0], g[1], g[2], g[3]);
            p.g_out[2 * (size_t)vec + 1] = make_float4(g[4], g[5], g[6], g[7]);
        }
    }
}

// A chunk with a compile-time number NV of versions to read.  Groups of kThreads*kUnroll vectors
// run without bounds checks; what is left (< one group, or a ragged last chunk) runs one
// predicated vector at a time.  Within a group all loads come first and all stores last, which
// is also what makes the in-place case (new version written over the oldest one read) safe:
// each vector is read and written by the same lane.
template <typename S, int NV, bool COMP, bool NORMS, bool GOUT>
__device__ __forceinline__ void run_chunk(const ChunkPtrs<S, NV> &p, uint32_t n_vecs, float lambda,
                                          float lr, float (&acc)[3]) {
    using Raw = typename S::Raw;
    constexpr bool kMaster = S::kElems == 8;
    const uint32_t tid = threadIdx.x;
    const uint32_t group = kThreads * kUnroll;
    const uint32_t n_grouped = n_vecs / group * group;

    for (uint32_t base = 0; base < n_grouped; base += group) {
        Raw rg[kUnroll], rv[kUnroll][NV];
        float4 m[kUnroll][2];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) rg[u] = p.g[base + u * kThreads + tid];
#pragma unroll
        for (int s = 0; s < NV; ++s)
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) rv[u][s] = p.v[s][base + u * kThreads + tid];
        if (kMaster) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                size_t vec = base + u * kThreads + tid;
                m[u][0] = p.master[2 * vec];
                m[u][1] = p.master[2 * vec + 1];
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            finish_vector<S, NV, COMP, NORMS, GOUT>(p, base + u * kThreads + tid, rg[u], rv[u], m[u], lambda,
                                                    lr, acc);
    }
    for (uint32_t vec = n_grouped + tid; vec < n_vecs; vec += kThreads) {
        Raw rg = p.g[vec], rv[NV];
        float4 m[2];
#pragma unroll
        for (int s = 0; s < NV; ++s) rv[s] = p.v[s][vec];
        if (kMaster) { m[0] = p.master[2 * (size_t)vec]; m[1] = p.master[2 * (size_t)vec + 1]; }
        finish_vector<S, NV, COMP, NORMS, GOUT>(p, vec, rg, rv, m, lambda, lr, acc);
    }
}

// Any number of versions (K' > 4): stream them one boundary at a time.
template <typename S, bool NORMS, bool GOUT>
__device__ __forceinline__ void run_chunk_streamed(const typename S::Raw *g_ptr, const typename S::Raw *arena,
                                                   uint64_t slot_stride_vecs, uint32_t R, uint32_t head,
                                                   uint32_t tau, uint32_t kp, typename S::Raw *out,
                                                   float4 *master, float4 *g_out, uint32_t n_vecs,
                                                   float lambda, float lr, float (&acc)[3]) {
    using Raw = typename S::Raw;
    constexpr int E = S::kElems;
    const uint32_t oldest = (head + R - tau) % R;
    for (uint32_t vec = threadIdx.x; vec < n_vecs; vec += kThreads) {
        float g[E], prev[E], cur[E], first[E];
        Raw rg = g_ptr[vec];
        Raw r0 = arena[(uint64_t)oldest * slot_stride_vecs + vec];
        S::widen(rg, g);
        S::widen(r0, prev);
#pragma unroll
        for (int e = 0; e < E; ++e) first[e] = prev[e];
        if (NORMS) {
#pragma unroll
            for (int e = 0; e < E; ++e) acc[0] = fmaf(g[e], g[e], acc[0]);
        }
        for (uint32_t i = 1; i <= kp; ++i) {
            uint32_t s_i = (uint32_t)(((uint64_t)i * tau) / kp);
            uint32_t slot = (oldest + s_i) % R;
            Raw r = arena[(uint64_t)slot * slot_stride_vecs + vec];
            S::widen(r, cur);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                g[e] = approximator(g[e], lambda, cur[e], prev[e]);
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
        if constexpr (E == 4) {
            float4 o;
            o.x = fmaf(-lr, g[0], prev[0]); o.y = fmaf(-lr, g[1], prev[1]);
            o.z = fmaf(-lr, g[2], prev[2]); o.w = fmaf(-lr, g[3], prev[3]);
            out[vec] = o;
            if (GOUT) g_out[vec] = make_float4(g[0], g[1], g[2], g[3]);
        } else {
            float4 m0 = master[2 * (size_t)vec], m1 = master[2 * (size_t)vec + 1];
            m0.x = fmaf(-lr, g[0], m0.x); m0.y = fmaf(-lr, g[1], m0.y);
            m0.z = fmaf(-lr, g[2], m0.z); m0.w = fmaf(-lr, g[3], m0.w);
            m1.x = fmaf(-lr, g[4], m1.x); m1.y = fmaf(-lr, g[5], m1.y);
            m1.z = fmaf(-lr, g[6], m1.z); m1.w = fmaf(-lr, g[7], m1.w);
            master[2 * (size_t)vec] = m0;
            master[2 * (size_t)vec + 1] = m1;
            uint4 o;
            o.x = bf16_pack(m0.x, m0.y); o.y = bf16_pack(m0.z, m0.w);
            o.z = bf16_pack(m1.x, m1.y); o.w = bf16_pack(m1.z, m1.w);
            out[vec] = o;
            if (GOUT) {
                g_out[2 * (size_t)vec] = make_float4(g[0], g[1], g[2], g[3]);
                g_out[2 * (size_t)vec + 1] = make_float4(g[4], g[5], g[6], g[7]);
            }
        }
    }
}

// Sum over the 64 lanes of a wavefront; every lane ends with the total.
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// Fixed-NV dispatch target: builds the chunk's pointers from the stage entry.
template <typename S, int NV, bool COMP, bool NORMS, bool GOUT>
__device__ __forceinline__ void do_chunk(const StepArgs &a, const typename S::Raw *arena, uint64_t stride_vecs,
                                         uint64_t flat_vec0, uint32_t R, uint32_t head, uint32_t tau,
                                         uint32_t n_vecs, float (&acc)[3]) {
    using Raw = typename S::Raw;
    ChunkPtrs<S, NV> p;
    p.g = reinterpret_cast<const Raw *>(a.grads) + flat_vec0;
    const uint32_t oldest = (head + R - tau) % R;
    constexpr uint32_t kp = NV - 1;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        // NV == 1: only V[tau].  Otherwise boundary s_i = floor(i*tau/K') of the K' = NV-1 segments.
        uint32_t s_i = NV == 1 ? tau : (uint32_t)(((uint64_t)i * tau) / (kp ? kp : 1));
        p.v[i] = arena + (uint64_t)((oldest + s_i) % R) * stride_vecs;
    }
    p.out = const_cast<Raw *>(arena) + (uint64_t)((head + 1) % R) * stride_vecs;
    constexpr uint64_t f4_per_vec = S::kElems / 4;
    p.master = a.master ? reinterpret_cast<float4 *>(a.master) + flat_vec0 * f4_per_vec : nullptr;
    p.g_out = GOUT ? reinterpret_cast<float4 *>(a.grad_out) + flat_vec0 * f4_per_vec : nullptr;
    run_chunk<S, NV, COMP, NORMS, GOUT>(p, n_vecs, a.lambda, a.lr, acc);
}

// ---- the step kernel ----------------------------------------------------------------------------
// STREAMED = false: every stage has K' <= 4 (the common case); the generic path is not even
// compiled in, which keeps the register footprint small.
template <typename S, bool STREAMED, bool NORMS, bool GOUT>
__global__ void __launch_bounds__(kThreads) step_kernel(const StepArgs a) {
    using Raw = typename S::Raw;
    __shared__ StageDesc tab[FERRET_MAX_STAGES];
    __shared__ float red[3][kWaves];

    {   // stage table: kernel-argument segment -> LDS, 12 dwords per stage
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
        const uint64_t e0 = (uint64_t)(chunk - uniform(d.chunk_begin)) * a.chunk_elems;
        const uint64_t n_stage = uniform(d.n_elems);
        const uint64_t left = n_stage - e0;
        const uint32_t n_here = left < a.chunk_elems ? (uint32_t)left : a.chunk_elems;
        const uint32_t n_vecs = n_here / S::kElems;
        const uint32_t R = uniform((uint32_t)d.ring_depth), head = uniform((uint32_t)d.head);
        const uint32_t tau = uniform((uint32_t)d.tau), kp = uniform((uint32_t)d.kp);
        const uint64_t stride_vecs = uniform(d.slot_stride) / S::kElems;
        const Raw *arena = reinterpret_cast<const Raw *>(a.ring) + (uniform(d.ring_base) + e0) / S::kElems;
        const uint64_t flat_vec0 = (uniform(d.flat_off) + e0) / S::kElems;

        float acc[3] = {0.f, 0.f, 0.f};
        // versions to read: the K'+1 boundaries; with K' = 0 only V[tau], plus V[0] when the
        // weight gap is wanted for the norms
        if (kp == 0) {
            if (NORMS && tau > 0)
                do_chunk<S, 2, false, NORMS, GOUT>(a, arena, stride_vecs, flat_vec0, R, head, tau, n_vecs, acc);
            else
                do_chunk<S, 1, false, NORMS, GOUT>(a, arena, stride_vecs, flat_vec0, R, head, tau, n_vecs, acc);
        } else if (kp == 1) {
            do_chunk<S, 2, true, NORMS, GOUT>(a, arena, stride_vecs, flat_vec0, R, head, tau, n_vecs, acc);
        } else if (kp == 2) {
            do_chunk<S, 3, true, NORMS, GOUT>(a, arena, stride_vecs, flat_vec0, R, head, tau, n_vecs, acc);
        } else if (kp == 3) {
            do_chunk<S, 4, true, NORMS, GOUT>(a, arena, stride_vecs, flat_vec0, R, head, tau, n_vecs, acc);
        } else if (kp == 4) {
            do_chunk<S, 5, true, NORMS, GOUT>(a, arena, stride_vecs, flat_vec0, R, head, tau, n_vecs, acc);
        } else if (STREAMED) {
            constexpr uint64_t f4_per_vec = S::kElems / 4;
            run_chunk_streamed<S, NORMS, GOUT>(
                reinterpret_cast<const Raw *>(a.grads) + flat_vec0, arena, stride_vecs, R, head, tau, kp,
                const_cast<Raw *>(arena) + (uint64_t)((head + 1) % R) * stride_vecs,
                a.master ? reinterpret_cast<float4 *>(a.master) + flat_vec0 * f4_per_vec : nullptr,
                GOUT ? reinterpret_cast<float4 *>(a.grad_out) + flat_vec0 * f4_per_vec : nullptr, n_vecs,
                a.lambda, a.lr, acc);
        }

        if (NORMS) {
            const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                float s = wave_sum(acc[k]);
                if (lane == 0) red[k][wave] = s;
            }
            __syncthreads();
            if (threadIdx.x < 3) {
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) s += red[threadIdx.x][w];
                a.partials[(size_t)chunk * 3 + threadIdx.x] = s;
            }
            __syncthreads();
        }
    }
}

// Sum the per-chunk partials of each stage in chunk order, in fp64.  One workgroup per stage.
__global__ void __launch_bounds__(kThreads) norms_finalize_kernel(const StepArgs a, float *norms_out) {
    __shared__ double red[3][kThreads];
    const uint32_t j = blockIdx.x;
    const uint32_t c0 = a.stage[j].chunk_begin;
    const uint32_t c1 = j + 1 < a.n_stages ? a.stage[j + 1].chunk_begin : a.n_chunks;
    double s[3] = {0.0, 0.0, 0.0};
    for (uint32_t c = c0 + threadIdx.x; c < c1; c += kThreads) {
        s[0] += (double)a.partials[(size_t)c * 3 + 0];
        s[1] += (double)a.partials[(size_t)c * 3 + 1];
        s[2] += (double)a.partials[(size_t)c * 3 + 2];
    }
    for (int k = 0; k < 3; ++k) red[k][threadIdx.x] = s[k];
    __syncthreads();
    for (int width = kThreads / 2; width >= 1; width >>= 1) {
        if ((int)threadIdx.x < width)
            for (int k = 0; k < 3; ++k) red[k][threadIdx.x] += red[k][threadIdx.x + width];
        __syncthreads();
    }
    if (threadIdx.x < 3) norms_out[j * 3 + threadIdx.x] = (float)red[threadIdx.x][0];
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
        const uint64_t e0 = (uint64_t)(chunk - uniform(d.chunk_begin)) * a.chunk_elems;
        const uint64_t left = uniform(d.n_elems) - e0;
        const uint32_t n_here = left < a.chunk_elems ? (uint32_t)left : a.chunk_elems;
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

__global__ void __launch_bounds__(kThreads) copy_kernel(uint4 *dst, const uint4 *src, size_t n_vecs) {
    const size_t stride = (size_t)gridDim.x * kThreads * kUnroll;
    size_t i = (size_t)blockIdx.x * kThreads * kUnroll + threadIdx.x;
    for (; i + kThreads < n_vecs; i += stride) {
        uint4 x = src[i], y = src[i + kThreads];
        dst[i] = x;
        dst[i + kThreads] = y;
    }
    if (i < n_vecs) dst[i] = src[i];
}

// ---- per-launch event timing of the step kernel ---------------------------------------------------
struct Profiler {
    std::vector<hipEvent_t> start, stop;
    int32_t used = 0;
    bool on = false;
};
static Profiler g_prof;

int profile_begin(int32_t capacity) {
    if (g_prof.on) return -1;
    g_prof.start.assign(capacity, nullptr);
    g_prof.stop.assign(capacity, nullptr);
    for (int32_t i = 0; i < capacity; ++i) {
        hipError_t e = hipEventCreate(&g_prof.start[i]);
        if (e == hipSuccess) e = hipEventCreate(&g_prof.stop[i]);
        if (e != hipSuccess) return (int)e;
    }
    g_prof.used = 0;
    g_prof.on = true;
    return 0;
}

int profile_end(float *ms_out, int32_t cap, int32_t *n_out) {
    if (!g_prof.on) return -1;
    hipError_t e = hipSuccess;
    if (g_prof.used > 0) e = hipEventSynchronize(g_prof.stop[g_prof.used - 1]);
    for (int32_t i = 0; i < g_prof.used && i < cap && e == hipSuccess; ++i)
        e = hipEventElapsedTime(&ms_out[i], g_prof.start[i], g_prof.stop[i]);
    *n_out = g_prof.used;
    for (size_t i = 0; i < g_prof.start.size(); ++i) {
        if (g_prof.start[i]) (void)hipEventDestroy(g_prof.start[i]);
        if (g_prof.stop[i]) (void)hipEventDestroy(g_prof.stop[i]);
    }
    g_prof.start.clear();
    g_prof.stop.clear();
    g_prof.on = false;
    return (int)e;
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
    if (bpc < 0) return n_chunks;                 // one workgroup per chunk
    if (bpc == 0) bpc = 8;
    int cus = cu_count(err);
    if (*err) return 0;
    uint64_t g = (uint64_t)cus * (uint64_t)bpc;
    return g < n_chunks ? (uint32_t)g : n_chunks;
}

template <typename S>
static hipError_t launch_step_typed(const StepArgs &a, bool streamed, bool norms, bool gout, uint32_t grid,
                                    hipStream_t st) {
#define FERRET_LAUNCH(ST, NO, GO) \
    hipLaunchKernelGGL((step_kernel<S, ST, NO, GO>), dim3(grid), dim3(kThreads), 0, st, a)
    if (streamed) {
        if (norms) { if (gout) FERRET_LAUNCH(true, true, true); else FERRET_LAUNCH(true, true, false); }
        else       { if (gout) FERRET_LAUNCH(true, false, true); else FERRET_LAUNCH(true, false, false); }
    } else {
        if (norms) { if (gout) FERRET_LAUNCH(false, true, true); else FERRET_LAUNCH(false, true, false); }
        else       { if (gout) FERRET_LAUNCH(false, false, true); else FERRET_LAUNCH(false, false, false); }
    }
#undef FERRET_LAUNCH
    return hipGetLastError();
}

int launch_step(const ferret_plan &plan, const StepArgs &a, float *norms_out, void *stream) {
    if (a.n_chunks == 0) return 0;
    int err = 0;
    const uint32_t grid = grid_for(plan, a.n_chunks, &err);
    if (err) return err;
    hipStream_t st = static_cast<hipStream_t>(stream);
    bool streamed = false;
    for (uint32_t j = 0; j < a.n_stages; ++j) streamed |= a.stage[j].kp + 1 > kMaxUnrolledVersions;
    const bool norms = norms_out != nullptr, gout = a.grad_out != nullptr;
    const bool timed = g_prof.on && g_prof.used < (int32_t)g_prof.start.size();
    if (timed) (void)hipEventRecord(g_prof.start[g_prof.used], st);
    hipError_t e = plan.prec == FERRET_F32 ? launch_step_typed<F32Store>(a, streamed, norms, gout, grid, st)
                                           : launch_step_typed<Bf16Store>(a, streamed, norms, gout, grid, st);
    if (timed) (void)hipEventRecord(g_prof.stop[g_prof.used++], st);
    if (e != hipSuccess) return (int)e;
    if (norms) {
        hipLaunchKernelGGL(norms_finalize_kernel, dim3(a.n_stages), dim3(kThreads), 0, st, a, norms_out);
        e = hipGetLastError();
    }
    return (int)e;
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
    int err = 0;
    int cus = cu_count(&err);
    if (err) return err;
    const size_t n_vecs = n_bytes / 16;
    size_t want = (n_vecs + kThreads * kUnroll - 1) / (kThreads * kUnroll);
    size_t cap = (size_t)cus * 8;
    uint32_t grid = (uint32_t)(want < cap ? want : cap);
    hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), n_vecs);
    return (int)hipGetLastError();
}

const char *device_error_string(int err) { return hipGetErrorString(static_cast<hipError_t>(err)); }

}  // namespace ferret
