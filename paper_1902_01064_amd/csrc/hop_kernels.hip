// HIP kernels of the Hop hot path for gfx950 (CDNA4, 64-wide wavefronts, 256 CUs in 8 XCDs).
//
// Every kernel here is bound by HBM bandwidth (about half a flop per byte), so none uses MFMA:
// the work is coalesced 128-bit streaming, wavefront reductions and LDS staging of small tables.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "hop_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kXcd = 8;                 // workgroups are dealt round-robin to the 8 XCDs

typedef float vf4 __attribute__((ext_vector_type(4)));
// Every vector handed to these kernels is device (global) memory, but the pointers come out of job
// descriptors, where the compiler only knows them as generic: without the address-space cast it emits
// flat_load / flat_store, which also count on the LDS counter, so every wait for a scalar load (the next
// pointer, the next weight) would wait for the vector loads in flight too.
#ifndef HOP_FLAT_ACCESS
#define HOP_GLOBAL __attribute__((address_space(1)))
#else
#define HOP_GLOBAL
#endif
typedef const HOP_GLOBAL vf4* gvec_in;
typedef HOP_GLOBAL vf4* gvec_out;
__device__ __forceinline__ float4 ld4(const float* p, int64_t i4) {
    vf4 v = ((gvec_in)p)[i4];
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st4(float* p, int64_t i4, float4 v) {
    vf4 t = {v.x, v.y, v.z, v.w};
    ((gvec_out)p)[i4] = t;
}
// streaming (non-temporal) 128-bit accesses for data touched once
__device__ __forceinline__ float4 ld4_stream(const float* p, int64_t i4) {
    vf4 v = __builtin_nontemporal_load((gvec_in)p + i4);
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st4_stream(float* p, int64_t i4, float4 v) {
    vf4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, (gvec_out)p + i4);
}

// blockIdx -> (job, chunk) so that the 8 workgroups dealt to the 8 XCDs at the same moment work on
// 8 different column chunks, and one XCD sees the same chunk for all jobs of a wave back to back:
// a source vector read by several jobs (a worker and its neighbours all average it) is then
// fetched from HBM once per XCD-local L2 instead of once per job.
__device__ __forceinline__ bool map_block(int64_t b, int n_jobs, int64_t n_chunks, int* job, int64_t* chunk) {
    int xcd = (int)(b % kXcd);
    int64_t local = b / kXcd;
    *job = (int)(local % n_jobs);
    *chunk = (local / n_jobs) * kXcd + xcd;
    return *chunk < n_chunks;
}

inline int64_t grid_for(int n_jobs, int64_t n_chunks) {
    int64_t padded = (n_chunks + kXcd - 1) / kXcd * kXcd;
    return padded * n_jobs;
}

// ------------------------------------------------------------------------ Reduce + Apply ----
// out[c] = sum_a w_a src_a[c] - eta g[c]   (Figure "Standard Decentralized Training", steps 2-3;
// weights from Eq. 2 times the mixing matrix, already normalised on the host).
//
// Template knobs: VEC float4 per thread per source; NT 0 = ordinary accesses, 1 = g and the result
// non-temporal (each touched once), 2 = sources too; MAP 1 = the XCD-aware map above, 10 + G = the same
// with runs of G consecutive chunks per XCD; T threads per workgroup.
// Measured on 32 jobs x 25 M columns with ~7.6 shared sources each: job-major workgroups are 2.3x slower than
// MAP 1 and chunk-major ones that ignore the XCDs 1.45x slower; vector width (1-8), block size (128-1024) and
// cache hints move the time by under 5 %.
template <int NT>
__device__ __forceinline__ float4 ld_src(const float* p, int64_t i) {
    return NT >= 2 ? ld4_stream(p, i) : ld4(p, i);
}
template <int NT>
__device__ __forceinline__ float4 ld_once(const float* p, int64_t i) {
    return NT >= 1 ? ld4_stream(p, i) : ld4(p, i);
}
template <int NT>
__device__ __forceinline__ void st_once(float* p, int64_t i, float4 v) {
    if (NT >= 1) st4_stream(p, i, v); else st4(p, i, v);
}

template <int A, int VEC, int NT, int T, bool MOM>
__device__ __forceinline__ void mix_tile(const HopMixJob* __restrict__ job, int64_t first4, int64_t n4) {
    const float* g = job->g;
    const float neg_eta = -job->eta;
    float* vel = job->vel;
    const float mu = job->mu;
    const float lam_fold = job->lam_fold;
    float* out = job->out;
    float4 acc[VEC];
    int64_t idx[VEC];
    bool ok[VEC];
#pragma unroll
    for (int u = 0; u < VEC; ++u) {
        idx[u] = first4 + (int64_t)u * T + threadIdx.x;
        ok[u] = idx[u] < n4;
    }
    {
        const float* s0 = job->src[0];
        const float w0 = job->w[0];
#pragma unroll
        for (int u = 0; u < VEC; ++u) {
            float4 v = ok[u] ? ld_src<NT>(s0, idx[u]) : make_float4(0.f, 0.f, 0.f, 0.f);
            acc[u] = make_float4(w0 * v.x, w0 * v.y, w0 * v.z, w0 * v.w);
        }
    }
#pragma unroll
    for (int a = 1; a < A; ++a) {
        const float* sa = job->src[a];
        const float wa = job->w[a];
#pragma unroll
        for (int u = 0; u < VEC; ++u) {
            float4 v = ok[u] ? ld_src<NT>(sa, idx[u]) : make_float4(0.f, 0.f, 0.f, 0.f);
            acc[u].x = fmaf(wa, v.x, acc[u].x);
            acc[u].y = fmaf(wa, v.y, acc[u].y);
            acc[u].z = fmaf(wa, v.z, acc[u].z);
            acc[u].w = fmaf(wa, v.w, acc[u].w);
        }
    }
    if (MOM) {
        // v <- mu v + g (a missing g counts as zero), Apply with the new velocity
#pragma unroll
        for (int u = 0; u < VEC; ++u) {
            float4 v = ok[u] ? ld_once<NT>(vel, idx[u]) : make_float4(0.f, 0.f, 0.f, 0.f);
            float4 gg = (ok[u] && g != nullptr) ? ld_once<NT>(g, idx[u]) : make_float4(0.f, 0.f, 0.f, 0.f);
            if (lam_fold != 0.f && ok[u]) {      // dense part lambda w of a gradient whose sparse part is scattered later
                const float4 x0 = ld_src<NT>(job->src[0], idx[u]);
                gg = make_float4(fmaf(lam_fold, x0.x, gg.x), fmaf(lam_fold, x0.y, gg.y), fmaf(lam_fold, x0.z, gg.z),
                                 fmaf(lam_fold, x0.w, gg.w));
            }
            v = make_float4(fmaf(mu, v.x, gg.x), fmaf(mu, v.y, gg.y), fmaf(mu, v.z, gg.z), fmaf(mu, v.w, gg.w));
            if (ok[u]) st_once<NT>(vel, idx[u], v);
            acc[u].x = fmaf(neg_eta, v.x, acc[u].x);
            acc[u].y = fmaf(neg_eta, v.y, acc[u].y);
            acc[u].z = fmaf(neg_eta, v.z, acc[u].z);
            acc[u].w = fmaf(neg_eta, v.w, acc[u].w);
        }
    } else if (g != nullptr) {
#pragma unroll
        for (int u = 0; u < VEC; ++u) {
            float4 v = ok[u] ? ld_once<NT>(g, idx[u]) : make_float4(0.f, 0.f, 0.f, 0.f);
            acc[u].x = fmaf(neg_eta, v.x, acc[u].x);
            acc[u].y = fmaf(neg_eta, v.y, acc[u].y);
            acc[u].z = fmaf(neg_eta, v.z, acc[u].z);
            acc[u].w = fmaf(neg_eta, v.w, acc[u].w);
        }
    }
#pragma unroll
    for (int u = 0; u < VEC; ++u)
        if (ok[u]) st_once<NT>(out, idx[u], acc[u]);
}

// more than 12 sources: a loop over the sources instead of an unrolled chain
template <int VEC, int NT, int T>
__device__ __forceinline__ void mix_tile_any(const HopMixJob* __restrict__ job, int64_t first4, int64_t n4) {
    const int A = job->A;
    const float* g = job->g;
    const float neg_eta = -job->eta;
    for (int u = 0; u < VEC; ++u) {
        int64_t i = first4 + (int64_t)u * T + threadIdx.x;
        if (i >= n4) continue;
        float4 v = ld_src<NT>(job->src[0], i);
        float w = job->w[0];
        float4 acc = make_float4(w * v.x, w * v.y, w * v.z, w * v.w);
        for (int a = 1; a < A; ++a) {
            v = ld_src<NT>(job->src[a], i);
            w = job->w[a];
            acc.x = fmaf(w, v.x, acc.x);
            acc.y = fmaf(w, v.y, acc.y);
            acc.z = fmaf(w, v.z, acc.z);
            acc.w = fmaf(w, v.w, acc.w);
        }
        if (job->vel != nullptr) {
            float4 gg = g != nullptr ? ld_once<NT>(g, i) : make_float4(0.f, 0.f, 0.f, 0.f);
            if (job->lam_fold != 0.f) {
                const float4 x0 = ld_src<NT>(job->src[0], i);
                const float lf = job->lam_fold;
                gg = make_float4(fmaf(lf, x0.x, gg.x), fmaf(lf, x0.y, gg.y), fmaf(lf, x0.z, gg.z), fmaf(lf, x0.w, gg.w));
            }
            v = ld_once<NT>(job->vel, i);
            const float mu = job->mu;
            v = make_float4(fmaf(mu, v.x, gg.x), fmaf(mu, v.y, gg.y), fmaf(mu, v.z, gg.z), fmaf(mu, v.w, gg.w));
            st_once<NT>(job->vel, i, v);
        } else if (g != nullptr) {
            v = ld_once<NT>(g, i);
        }
        if (job->vel != nullptr || g != nullptr) {
            acc.x = fmaf(neg_eta, v.x, acc.x);
            acc.y = fmaf(neg_eta, v.y, acc.y);
            acc.z = fmaf(neg_eta, v.z, acc.z);
            acc.w = fmaf(neg_eta, v.w, acc.w);
        }
        st_once<NT>(job->out, i, acc);
    }
}

// Work of one workgroup of the mix; `bid` is its index among the mix's workgroups (the launch may
// hold other workgroups in front of them, which only rotates the assignment of XCDs).
template <int VEC, int NT, int MAP, int T>
__device__ __forceinline__ void mix_block(const HopMixJob* __restrict__ jobs, int n_jobs, int64_t d,
                                          int64_t n_chunks, int64_t bid) {
    int j;
    int64_t chunk;
    if (MAP == 1) {
        if (!map_block(bid, n_jobs, n_chunks, &j, &chunk)) return;
    } else {
        // XCD-aware like MAP 1, but every XCD owns runs of G = MAP - 10 consecutive chunks, and visits
        // them job by job: longer contiguous pieces of every stream are in flight at a time
        static_assert(MAP == 1 || MAP > 10, "MAP is 1 or 10 + run length");
        constexpr int G = MAP > 10 ? MAP - 10 : 1;
        int xcd = (int)(bid % kXcd);
        int64_t local = bid / kXcd;
        int sub = (int)(local % G);
        j = (int)((local / G) % n_jobs);
        int64_t group = local / ((int64_t)G * n_jobs);
        chunk = (group * kXcd + xcd) * G + sub;
        if (chunk >= n_chunks) return;
    }
    const HopMixJob* job = jobs + j;
    const int64_t n4 = d >> 2;
    const int64_t first4 = chunk * (int64_t)(T * VEC);
    if (job->vel != nullptr) {
        switch (job->A) {
            case 1: mix_tile<1, VEC, NT, T, true>(job, first4, n4); break;
            case 2: mix_tile<2, VEC, NT, T, true>(job, first4, n4); break;
            case 3: mix_tile<3, VEC, NT, T, true>(job, first4, n4); break;
            case 4: mix_tile<4, VEC, NT, T, true>(job, first4, n4); break;
            case 5: mix_tile<5, VEC, NT, T, true>(job, first4, n4); break;
            case 6: mix_tile<6, VEC, NT, T, true>(job, first4, n4); break;
            case 7: mix_tile<7, VEC, NT, T, true>(job, first4, n4); break;
            case 8: mix_tile<8, VEC, NT, T, true>(job, first4, n4); break;
            case 9: mix_tile<9, VEC, NT, T, true>(job, first4, n4); break;
            case 10: mix_tile<10, VEC, NT, T, true>(job, first4, n4); break;
            case 11: mix_tile<11, VEC, NT, T, true>(job, first4, n4); break;
            case 12: mix_tile<12, VEC, NT, T, true>(job, first4, n4); break;
            default: mix_tile_any<VEC, NT, T>(job, first4, n4); break;
        }
    } else {
        switch (job->A) {
            case 1: mix_tile<1, VEC, NT, T, false>(job, first4, n4); break;
            case 2: mix_tile<2, VEC, NT, T, false>(job, first4, n4); break;
            case 3: mix_tile<3, VEC, NT, T, false>(job, first4, n4); break;
            case 4: mix_tile<4, VEC, NT, T, false>(job, first4, n4); break;
            case 5: mix_tile<5, VEC, NT, T, false>(job, first4, n4); break;
            case 6: mix_tile<6, VEC, NT, T, false>(job, first4, n4); break;
            case 7: mix_tile<7, VEC, NT, T, false>(job, first4, n4); break;
            case 8: mix_tile<8, VEC, NT, T, false>(job, first4, n4); break;
            case 9: mix_tile<9, VEC, NT, T, false>(job, first4, n4); break;
            case 10: mix_tile<10, VEC, NT, T, false>(job, first4, n4); break;
            case 11: mix_tile<11, VEC, NT, T, false>(job, first4, n4); break;
            case 12: mix_tile<12, VEC, NT, T, false>(job, first4, n4); break;
            default: mix_tile_any<VEC, NT, T>(job, first4, n4); break;
        }
    }
    // the d mod 4 trailing columns, one thread each, by the workgroup of the last chunk
    if (chunk == n_chunks - 1) {
        int64_t c = (n4 << 2) + threadIdx.x;
        if (threadIdx.x < 4 && c < d) {
            float acc = job->w[0] * job->src[0][c];
            for (int a = 1; a < job->A; ++a) acc = fmaf(job->w[a], job->src[a][c], acc);
            if (job->vel != nullptr) {
                float v = fmaf(job->mu, job->vel[c],
                               fmaf(job->lam_fold, job->src[0][c], job->g != nullptr ? job->g[c] : 0.f));
                job->vel[c] = v;
                acc = fmaf(-job->eta, v, acc);
            } else if (job->g != nullptr) {
                acc = fmaf(-job->eta, job->g[c], acc);
            }
            job->out[c] = acc;
        }
    }
}

template <int VEC, int NT, int MAP, int T>
__global__ __launch_bounds__(T) void mix_kernel(const HopMixJob* __restrict__ jobs, int n_jobs, int64_t d,
                                                int64_t n_chunks) {
    mix_block<VEC, NT, MAP, T>(jobs, n_jobs, d, n_chunks, blockIdx.x);
}

template <int VEC, int MAP, int T>
int64_t mix_grid(int n_jobs, int64_t d, int64_t* n_chunks_out) {
    int64_t n4 = d >> 2;
    int64_t per = (int64_t)T * VEC;
    int64_t n_chunks = (n4 + per - 1) / per;
    if (n_chunks < 1) n_chunks = 1;
    int64_t grid = grid_for(n_jobs, n_chunks);
    if (MAP > 10) {
        int64_t span = (int64_t)kXcd * (MAP - 10);
        grid = (n_chunks + span - 1) / span * span * n_jobs;
    }
    *n_chunks_out = n_chunks;
    return grid;
}

template <int VEC, int NT, int MAP, int T>
int launch_mix(const HopMixJob* jobs_dev, int n_jobs, int64_t d, void* stream) {
    int64_t n_chunks;
    int64_t grid = mix_grid<VEC, MAP, T>(n_jobs, d, &n_chunks);
    if (grid > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((mix_kernel<VEC, NT, MAP, T>), dim3((unsigned)grid), dim3(T), 0, (hipStream_t)stream,
                       jobs_dev, n_jobs, d, n_chunks);
    return (int)hipGetLastError();
}

// ---------------------------------------------------------- Reduce + Apply, records in pairs ----
// The plain path (no velocity).  Neighbouring workers average almost the same vectors (on a ring i and
// i + 1 share x_i and x_{i+1}), so the host packs a wave's records two by two where their source sets
// overlap and the union has at most kPairU vectors.  One workgroup loads the union for a 16 KB column chunk
// once into registers and forms both sums from there; a source shared inside the pair then costs one L2
// request instead of two.  Against the record-by-record kernel above this also changes how the work is issued:
//  - the union size is a compile-time constant (switch over U), every pointer and weight is read by one batch
//    of scalar loads ahead of the first vector load, and interior chunks take a path without bounds checks,
//    so a wavefront has all its 128-bit loads in flight after one scalar wait instead of one per source;
//  - every XCD walks `run` consecutive chunks per job group (run chosen by the host so that run x 16 KB x
//    distinct sources of the wave stays near 3 MB of the XCD's 4 MB L2).
// Measured on the 134 waves of the 32-worker, 25 M-parameter workload: 1.51 ms -> 1.41 ms per launch.
// Terms are added in the order of the union (the first record's own order; the second record's sources fall
// where the union has them), in fp32 FMAs starting from zero.
constexpr int kPairU = HOP_PAIR_U;
constexpr int kPairVec = 4;

template <int U, bool FULL>
__device__ __forceinline__ void pair_tile(const HopPairJob* __restrict__ job, int64_t first4, int64_t n4) {
    constexpr int VEC = kPairVec;
    const int G = job->G;
    const float* src[U];
#pragma unroll
    for (int u = 0; u < U; ++u) src[u] = job->src[u];
    const float* gp[2];
    float* op[2];
    uint32_t mk[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) { gp[r] = job->g[r]; op[r] = job->out[r]; mk[r] = job->mask[r]; }
    const float neg_eta = -job->eta;
    const int64_t i0 = first4 + threadIdx.x;
    float4 x[U][VEC];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int v = 0; v < VEC; ++v)
            x[u][v] = (FULL || i0 + v * kThreads < n4) ? ld4(src[u], i0 + v * kThreads) : make_float4(0.f, 0.f, 0.f, 0.f);
    float4 gv[2][VEC];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        if (r < G && gp[r] != nullptr) {
#pragma unroll
            for (int v = 0; v < VEC; ++v)
                gv[r][v] = (FULL || i0 + v * kThreads < n4) ? ld4_stream(gp[r], i0 + v * kThreads)
                                                            : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        if (r < G) {
            float wr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) wr[u] = job->w[r][u];
            float4 acc[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if ((mk[r] >> u) & 1u) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        acc[v].x = fmaf(wr[u], x[u][v].x, acc[v].x);
                        acc[v].y = fmaf(wr[u], x[u][v].y, acc[v].y);
                        acc[v].z = fmaf(wr[u], x[u][v].z, acc[v].z);
                        acc[v].w = fmaf(wr[u], x[u][v].w, acc[v].w);
                    }
                }
            }
            if (gp[r] != nullptr) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    acc[v].x = fmaf(neg_eta, gv[r][v].x, acc[v].x);
                    acc[v].y = fmaf(neg_eta, gv[r][v].y, acc[v].y);
                    acc[v].z = fmaf(neg_eta, gv[r][v].z, acc[v].z);
                    acc[v].w = fmaf(neg_eta, gv[r][v].w, acc[v].w);
                }
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v)
                if (FULL || i0 + v * kThreads < n4) st4_stream(op[r], i0 + v * kThreads, acc[v]);
        }
    }
}

// a single record with more than kPairU sources: a loop over the sources
__device__ __forceinline__ void pair_tile_wide(const HopPairJob* __restrict__ job, int64_t first4, int64_t n4) {
    const int U = job->U;
    const float* g = job->g[0];
    const float neg_eta = -job->eta;
    for (int v = 0; v < kPairVec; ++v) {
        const int64_t i = first4 + (int64_t)v * kThreads + threadIdx.x;
        if (i >= n4) continue;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int u = 0; u < U; ++u) {
            const float4 xv = ld4(job->src[u], i);
            const float w = job->w[0][u];
            acc.x = fmaf(w, xv.x, acc.x);
            acc.y = fmaf(w, xv.y, acc.y);
            acc.z = fmaf(w, xv.z, acc.z);
            acc.w = fmaf(w, xv.w, acc.w);
        }
        if (g != nullptr) {
            const float4 gv = ld4_stream(g, i);
            acc.x = fmaf(neg_eta, gv.x, acc.x);
            acc.y = fmaf(neg_eta, gv.y, acc.y);
            acc.z = fmaf(neg_eta, gv.z, acc.z);
            acc.w = fmaf(neg_eta, gv.w, acc.w);
        }
        st4_stream(job->out[0], i, acc);
    }
}

// Work of one workgroup; `bid` is its index among the launch's mix workgroups.
__device__ __forceinline__ void pair_block(const HopPairJob* __restrict__ jobs, int n_jobs, int64_t d, int64_t n_chunks,
                                           int run, int reverse, int64_t bid) {
    const int xcd = (int)(bid % kXcd);
    const int64_t local = bid / kXcd;
    const int sub = (int)(local % run);
    const int j = (int)((local / run) % n_jobs);
    const int64_t round = local / ((int64_t)run * n_jobs);
    int64_t ahead = (round * kXcd + xcd) * run + sub;
    // the last, partly filled round is dealt out evenly (shorter runs on all XCDs, not full runs on the first few)
    const int64_t span = (int64_t)kXcd * run;
    const int64_t done = n_chunks / span * span;
    if (round * span >= done) {
        const int tail_run = (int)((n_chunks - done + kXcd - 1) / kXcd);
        if (sub >= tail_run) return;
        ahead = done + (int64_t)xcd * tail_run + sub;
    }
    if (ahead >= n_chunks) return;
    // consecutive launches walk the vectors in opposite directions: what the previous kernels wrote or read last
    // is still in the memory-side cache when the next launch begins there (1453 -> 1430 us per launch with the
    // gradient generator in between, 386 -> 381 us between launches of small waves)
    const int64_t chunk = reverse ? n_chunks - 1 - ahead : ahead;
    const HopPairJob* job = jobs + j;
    const int64_t n4 = d >> 2;
    const int64_t first4 = chunk * (int64_t)(kThreads * kPairVec);
    const bool full = first4 + kThreads * kPairVec <= n4;
    static_assert(kPairU == 12, "the switch below unrolls unions of 1..12 vectors");
#define HOP_PAIR_CASE(UU)                                      \
    case UU:                                                   \
        if (full) pair_tile<UU, true>(job, first4, n4);        \
        else pair_tile<UU, false>(job, first4, n4);            \
        break;
    switch (job->U) {
        HOP_PAIR_CASE(1) HOP_PAIR_CASE(2) HOP_PAIR_CASE(3) HOP_PAIR_CASE(4) HOP_PAIR_CASE(5) HOP_PAIR_CASE(6)
        HOP_PAIR_CASE(7) HOP_PAIR_CASE(8) HOP_PAIR_CASE(9) HOP_PAIR_CASE(10) HOP_PAIR_CASE(11) HOP_PAIR_CASE(12)
        default: pair_tile_wide(job, first4, n4); break;
    }
#undef HOP_PAIR_CASE
    // the d mod 4 trailing columns, one thread each, by the workgroup of the last chunk
    if (chunk == n_chunks - 1) {
        const int64_t c = (n4 << 2) + (threadIdx.x & 3);
        const int r = threadIdx.x >> 2;
        if (threadIdx.x < 8 && r < job->G && c < d) {
            float acc = 0.f;
            for (int u = 0; u < job->U; ++u)
                if ((job->mask[r] >> u) & 1u) acc = fmaf(job->w[r][u], job->src[u][c], acc);
            if (job->g[r] != nullptr) acc = fmaf(-job->eta, job->g[r][c], acc);
            job->out[r][c] = acc;
        }
    }
}

__global__ __launch_bounds__(kThreads) void pair_mix_kernel(const HopPairJob* __restrict__ jobs, int n_jobs, int64_t d,
                                                            int64_t n_chunks, int run, int reverse) {
    pair_block(jobs, n_jobs, d, n_chunks, run, reverse, blockIdx.x);
}

inline int64_t pair_chunks(int64_t d) {
    const int64_t per = (int64_t)kThreads * kPairVec;
    const int64_t n = ((d >> 2) + per - 1) / per;
    return n < 1 ? 1 : n;
}

// chunks an XCD walks per job group: run x 16 KB x distinct sources near 3 MB of its 4 MB L2 (measured on 32
// sources: runs of 5 to 7 equal, 4 and 8 1.3 % slower, 12 10 % slower), never more than the vector has
inline int pair_run(int n_sources, int64_t n_chunks) {
    int run = (192 + n_sources / 2) / (n_sources < 1 ? 1 : n_sources);
    if (run > 8) run = 8;
    const int64_t room = n_chunks / kXcd;
    if (run > room) run = (int)room;
    return run < 1 ? 1 : run;
}

inline int64_t pair_grid(int n_jobs, int64_t n_chunks, int run) {
    const int64_t span = (int64_t)kXcd * run;
    return (n_chunks + span - 1) / span * span * n_jobs;
}

// ------------------------------------------------------------------- synthetic gradient ----
// g[c] = (sum of the 12 bytes of a = h32(c ^ k0), b = h32(c ^ k1), (a + rotl(b, 16)) ^ k2  - 1530) * scale:
// integer work and one correctly rounded multiply, so any implementation agrees bit for bit.
__device__ __forceinline__ uint32_t h32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}
__device__ __forceinline__ uint32_t byte_sum(uint32_t x, uint32_t acc) {
    return __builtin_amdgcn_sad_u8(x, 0u, acc);       // acc + sum of the four bytes of x
}
__device__ __forceinline__ float synth_one(uint32_t c, uint32_t k0, uint32_t k1, uint32_t k2, float scale) {
    // two hashed words and a third made of both: a + rotl(b, 16) is uniform and independent of a and of
    // b taken one at a time, so the twelve bytes are pairwise independent and the variance is exact,
    // at two thirds of the integer multiplies (32-bit multiplies are the slow instruction here)
    const uint32_t a = h32(c ^ k0), b = h32(c ^ k1);
    const uint32_t t = (a + ((b << 16) | (b >> 16))) ^ k2;
    uint32_t s = byte_sum(a, 0u);
    s = byte_sum(b, s);
    s = byte_sum(t, s);
    return (float)((int)s - 1530) * scale;
}

constexpr int kSynthVec = 2;
constexpr int kSynthChunk4 = kThreads * kSynthVec;

// `reverse`: walk the vectors from their end, so that the launch finishes where the Reduce + Apply that consumes
// these gradients starts and finds their last-written part still in the memory-side cache.
__global__ __launch_bounds__(kThreads) void synth_kernel(const HopGradJob* __restrict__ jobs, int n_jobs,
                                                         int64_t d, int64_t n_chunks, int reverse) {
    int j;
    int64_t chunk;
    if (!map_block(blockIdx.x, n_jobs, n_chunks, &j, &chunk)) return;
    if (reverse) chunk = n_chunks - 1 - chunk;
    const HopGradJob* job = jobs + j;
    const uint32_t k0 = job->k0, k1 = job->k1, k2 = job->k2;
    const float scale = job->scale;
    float* g = job->g;
    const int64_t n4 = d >> 2;
#pragma unroll
    for (int u = 0; u < kSynthVec; ++u) {
        int64_t i = chunk * kSynthChunk4 + (int64_t)u * kThreads + threadIdx.x;
        if (i < n4) {
            uint32_t c = (uint32_t)(i << 2);
            float4 v;
            v.x = synth_one(c, k0, k1, k2, scale);
            v.y = synth_one(c + 1, k0, k1, k2, scale);
            v.z = synth_one(c + 2, k0, k1, k2, scale);
            v.w = synth_one(c + 3, k0, k1, k2, scale);
            st4(g, i, v);
        }
    }
    if (chunk == n_chunks - 1) {
        int64_t c = (n4 << 2) + threadIdx.x;
        if (threadIdx.x < 4 && c < d) g[c] = synth_one((uint32_t)c, k0, k1, k2, scale);
    }
}

// ------------------------------------------------------------------ wavefront reductions ----
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;                                          // lane 0 holds the sum
}

__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (lane == 0) red[wv] = v;
    __syncthreads();
    float t = 0.f;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int k = 0; k < kThreads / 64; ++k) t += red[k];
    }
    return t;                                          // thread 0 holds the sum
}

// c_m of g = lambda w - sum_m c_m x_m: hinge y/B where y <x, w> < 1, log loss y / (B (1 + e^{y <x, w>}))
__device__ __forceinline__ float loss_coef(float y, float dot, float invB, int loss) {
    const float m = y * dot;
    if (loss == HOP_LOSS_LOG) return y * invB / (1.0f + expf(m));
    return m < 1.0f ? y * invB : 0.f;
}

// ------------------------------------------------------------- dense SVM: margins ("Compute") ----
// One workgroup per (job, minibatch row, column segment): partial <x_r, w> over 16384 columns.
constexpr int kSegVec = 16;
constexpr int kSeg4 = kThreads * kSegVec;             // float4 per segment
constexpr int64_t kSegCols = (int64_t)kSeg4 * 4;

__device__ __forceinline__ void dense_margin_block(const HopGradJob* __restrict__ jobs, int B, int64_t d, int nseg,
                                                   int64_t b, float* red) {
    const int seg = (int)(b % nseg);
    const int m = (int)((b / nseg) % B);
    const HopGradJob* job = jobs + b / ((int64_t)nseg * B);
    const float* x = job->X + (int64_t)job->rows[m] * d;
    const float* w = job->w;
    float acc = 0.f;
    const int64_t lo = (int64_t)seg * kSegCols;
    const int64_t hi = min(d, lo + kSegCols);
    if ((d & 3) == 0) {
        const int64_t lo4 = lo >> 2, hi4 = hi >> 2;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll 4
        for (int64_t i = lo4 + threadIdx.x; i < hi4; i += kThreads) {
            float4 xv = ld4_stream(x, i);
            float4 wv = ld4(w, i);
            a0 = fmaf(xv.x, wv.x, a0);
            a1 = fmaf(xv.y, wv.y, a1);
            a2 = fmaf(xv.z, wv.z, a2);
            a3 = fmaf(xv.w, wv.w, a3);
        }
        acc = (a0 + a1) + (a2 + a3);
    } else {
        for (int64_t c = lo + threadIdx.x; c < hi; c += kThreads) acc = fmaf(x[c], w[c], acc);
    }
    float tot = block_sum(acc, red);
    if (threadIdx.x == 0) job->partial[(int64_t)m * nseg + seg] = tot;
}

// The margin pass as a launch of its own: four minibatch rows per workgroup share every load of w (the L2 sees
// 5 requests per 4 row pieces instead of 8), each row summed exactly as dense_margin_block sums it, so the partial
// dot products are the same bit for bit.  Rows by non-temporal loads: a wave's rows are new to every cache, and a
// cold stream runs faster without allocating in the memory-side cache (6.9 against 5.5 TB/s stand-alone).  Leaving
// them there for the gradient pass with ordinary loads was measured on 16 workers x 65536 columns, B = 128:
// margins 37.4 -> 42.5 us, gradient 23.8 -> 21.5 us per wave, nothing gained.
constexpr int kMarginRows = 4;

__global__ __launch_bounds__(kThreads) void dense_margin4_kernel(const HopGradJob* __restrict__ jobs, int B, int64_t d,
                                                                 int nseg, int row_groups) {
    __shared__ float red[kMarginRows][kThreads / 64];
    const int64_t b = blockIdx.x;
    const int seg = (int)(b % nseg);
    const int m0 = (int)((b / nseg) % row_groups) * kMarginRows;
    const HopGradJob* job = jobs + b / ((int64_t)nseg * row_groups);
    const float* w = job->w;
    const float* x[kMarginRows];
#pragma unroll
    for (int r = 0; r < kMarginRows; ++r) x[r] = job->X + (int64_t)job->rows[min(m0 + r, B - 1)] * d;
    const int64_t lo = (int64_t)seg * kSegCols;
    const int64_t hi = min(d, lo + kSegCols);
    float acc[kMarginRows];
    if ((d & 3) == 0) {
        const int64_t lo4 = lo >> 2, hi4 = hi >> 2;
        float a[kMarginRows][4];
#pragma unroll
        for (int r = 0; r < kMarginRows; ++r) a[r][0] = a[r][1] = a[r][2] = a[r][3] = 0.f;
#pragma unroll 4
        for (int64_t i = lo4 + threadIdx.x; i < hi4; i += kThreads) {
            const float4 wv = ld4(w, i);
#pragma unroll
            for (int r = 0; r < kMarginRows; ++r) {
                const float4 xv = ld4_stream(x[r], i);
                a[r][0] = fmaf(xv.x, wv.x, a[r][0]);
                a[r][1] = fmaf(xv.y, wv.y, a[r][1]);
                a[r][2] = fmaf(xv.z, wv.z, a[r][2]);
                a[r][3] = fmaf(xv.w, wv.w, a[r][3]);
            }
        }
#pragma unroll
        for (int r = 0; r < kMarginRows; ++r) acc[r] = (a[r][0] + a[r][1]) + (a[r][2] + a[r][3]);
    } else {
#pragma unroll
        for (int r = 0; r < kMarginRows; ++r) acc[r] = 0.f;
        for (int64_t c = lo + threadIdx.x; c < hi; c += kThreads) {
            const float wc = w[c];
#pragma unroll
            for (int r = 0; r < kMarginRows; ++r) acc[r] = fmaf(x[r][c], wc, acc[r]);
        }
    }
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int r = 0; r < kMarginRows; ++r) {
        const float v = wave_sum(acc[r]);
        if (lane == 0) red[r][wv] = v;
    }
    __syncthreads();
    if (threadIdx.x < kMarginRows && m0 + threadIdx.x < B) {
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < kThreads / 64; ++k) t += red[threadIdx.x][k];
        job->partial[(int64_t)(m0 + threadIdx.x) * nseg + seg] = t;
    }
}

// The partial margins of a wave's STEP records and the wave's Reduce in one launch: both only read x_k
// (the parallel approach of Section 3.2 runs Compute beside Reduce).  The Reduce leaves sum_a w'_a x_a
// in the result slot; dense_grad_kernel then applies -eta g to it.
template <int VEC, int NT, int MAP>
__global__ __launch_bounds__(kThreads) void mix_dense_margin_kernel(const HopMixJob* __restrict__ mix_jobs, int n_mix,
                                                                    int64_t d, int64_t n_chunks,
                                                                    const HopGradJob* __restrict__ grad_jobs, int B,
                                                                    int nseg, int64_t margin_blocks) {
    __shared__ float red[kThreads / 64];
    if ((int64_t)blockIdx.x >= margin_blocks) {
        mix_block<VEC, NT, MAP, kThreads>(mix_jobs, n_mix, d, n_chunks, (int64_t)blockIdx.x - margin_blocks);
        return;
    }
    dense_margin_block(grad_jobs, B, d, nseg, blockIdx.x, red);
}

// ----------------------------------------------------- dense SVM: g = lambda w - sum_m c_m x_m ----
// One workgroup per (job, 1024-column chunk).  The hinge coefficients c_m = y_m / B if
// y_m <x_m, w> < 1 else 0 are rebuilt by every workgroup from the partial dot products (B values,
// cheap) and the active rows are compacted in LDS in minibatch order.  Three endings: write g; apply -eta g to
// a vector the wave's Reduce has already left in the result slot; or do the record's Reduce here as well
// (steps 2-3 of the standard-training figure on the freshly computed gradient), which saves the launch of a
// separate mix and the round trip of g through memory when the minibatch is large.
constexpr int kMaxB = 1024;
constexpr int kRowUnroll = 8;

// SPLIT > 1: that many groups of 256 threads share a column chunk and take alternate groups of 8 active rows; their
// sums are joined through LDS in a fixed order.  For launches that leave most of the GPU idle (4 workers x 1024
// columns: 4 workgroups), where the time is the chain of dependent row loads: 8 rounds become 2.
template <int SPLIT>
__global__ __launch_bounds__(kThreads * SPLIT) void dense_grad_kernel(const HopGradJob* __restrict__ jobs, int n_jobs,
                                                                      int B, int64_t d, int nseg, float lambda,
                                                                      int loss, int64_t n_chunks) {
    __shared__ float coefS[kMaxB + kRowUnroll];
    __shared__ int rowS[kMaxB + kRowUnroll];
    __shared__ float allC[kMaxB];
    __shared__ int nactS;
    __shared__ float4 joinS[SPLIT > 1 ? (SPLIT - 1) * kThreads : 1];
    int j;
    int64_t chunk;
    if (!map_block(blockIdx.x, n_jobs, n_chunks, &j, &chunk)) return;
    const HopGradJob* job = jobs + j;
    const float invB = 1.0f / (float)B;
    const int part = SPLIT > 1 ? (int)threadIdx.x / kThreads : 0;     // which share of the rows
    const int col = SPLIT > 1 ? (int)threadIdx.x % kThreads : (int)threadIdx.x;
    for (int m = threadIdx.x; m < B; m += kThreads * SPLIT) {
        float dot = 0.f;
        for (int sg = 0; sg < nseg; ++sg) dot += job->partial[(int64_t)m * nseg + sg];
        float c = loss_coef(job->y[job->rows[m]], dot, invB, loss);
        allC[m] = c;
        if (chunk == 0) job->coef[m] = c;
    }
    __syncthreads();
    if (threadIdx.x < 64) {                            // first wavefront compacts, keeping order
        int count = 0;
        for (int base = 0; base < B; base += 64) {
            int m = base + threadIdx.x;
            float c = m < B ? allC[m] : 0.f;
            bool act = c != 0.f;
            unsigned long long mask = __ballot(act);
            int pos = count + __popcll(mask & ((1ull << threadIdx.x) - 1ull));
            if (act) {
                coefS[pos] = c;
                rowS[pos] = job->rows[m];
            }
            count += __popcll(mask);
        }
        if (threadIdx.x < kRowUnroll) {                // pad to a multiple of the unroll with zeros
            coefS[count + threadIdx.x] = 0.f;
            rowS[count + threadIdx.x] = job->rows[0];
        }
        if (threadIdx.x == 0) nactS = count;
    }
    __syncthreads();
    const int nact = nactS;
    const float* X = job->X;
    const float* w = job->w;
    float* g = job->g;
    float* out = job->out;                             // set: apply -eta g (or -eta v) to it instead of writing g
    const HopMixJob* red = job->reduce;                // set (with out): out = sum_a w'_a x_a - eta g, the Reduce done here
    float* vel = job->vel;
    const float neg_eta = -job->eta, mu = job->mu;
    if ((d & 3) == 0) {
        const int64_t n4 = d >> 2;
        const int64_t i = chunk * kThreads + col;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < n4) {
            for (int n = part * kRowUnroll; n < nact; n += kRowUnroll * SPLIT) {
                float4 v[kRowUnroll];
#pragma unroll
                for (int u = 0; u < kRowUnroll; ++u) v[u] = ld4(X + (int64_t)rowS[n + u] * d, i);
#pragma unroll
                for (int u = 0; u < kRowUnroll; ++u) {
                    const float c = coefS[n + u];
                    acc.x = fmaf(c, v[u].x, acc.x);
                    acc.y = fmaf(c, v[u].y, acc.y);
                    acc.z = fmaf(c, v[u].z, acc.z);
                    acc.w = fmaf(c, v[u].w, acc.w);
                }
            }
        }
        if (SPLIT > 1) {                               // join the shares: ((part 0 + part 1) + part 2) + ...
            if (part > 0) joinS[(part - 1) * kThreads + col] = acc;
            __syncthreads();
            if (part == 0) {
#pragma unroll
                for (int q = 1; q < SPLIT; ++q) {
                    const float4 t = joinS[(q - 1) * kThreads + col];
                    acc = make_float4(acc.x + t.x, acc.y + t.y, acc.z + t.z, acc.w + t.w);
                }
            }
        }
        if (i < n4 && part == 0) {
            float4 wv = ld4(w, i);
            float4 gv = make_float4(fmaf(lambda, wv.x, -acc.x), fmaf(lambda, wv.y, -acc.y),
                                    fmaf(lambda, wv.z, -acc.z), fmaf(lambda, wv.w, -acc.w));
            if (out == nullptr) {
                st4(g, i, gv);
            } else {
                if (vel != nullptr) {
                    const float4 v = ld4(vel, i);
                    gv = make_float4(fmaf(mu, v.x, gv.x), fmaf(mu, v.y, gv.y), fmaf(mu, v.z, gv.z), fmaf(mu, v.w, gv.w));
                    st4(vel, i, gv);
                }
                float4 o;
                if (red != nullptr) {                  // the record's Reduce, in the order the mix kernels sum
                    const int A = red->A;
                    float4 v = ld4(red->src[0], i);
                    float wa = red->w[0];
                    o = make_float4(wa * v.x, wa * v.y, wa * v.z, wa * v.w);
                    for (int a = 1; a < A; ++a) {
                        v = ld4(red->src[a], i);
                        wa = red->w[a];
                        o = make_float4(fmaf(wa, v.x, o.x), fmaf(wa, v.y, o.y), fmaf(wa, v.z, o.z), fmaf(wa, v.w, o.w));
                    }
                } else {                               // already reduced into the result slot
                    o = ld4(out, i);
                }
                st4(out, i, make_float4(fmaf(neg_eta, gv.x, o.x), fmaf(neg_eta, gv.y, o.y), fmaf(neg_eta, gv.z, o.z),
                                        fmaf(neg_eta, gv.w, o.w)));
            }
        }
    } else if (part == 0) {
        for (int q = 0; q < 4; ++q) {
            const int64_t c = (chunk * kThreads + col) * 4 + q;
            if (c < d) {
                float acc = 0.f;
                for (int n = 0; n < nact; ++n) acc = fmaf(coefS[n], X[(int64_t)rowS[n] * d + c], acc);
                float gv = fmaf(lambda, w[c], -acc);
                if (out == nullptr) {
                    g[c] = gv;
                } else {
                    if (vel != nullptr) {
                        gv = fmaf(mu, vel[c], gv);
                        vel[c] = gv;
                    }
                    float o;
                    if (red != nullptr) {
                        o = red->w[0] * red->src[0][c];
                        for (int a = 1; a < red->A; ++a) o = fmaf(red->w[a], red->src[a][c], o);
                    } else {
                        o = out[c];
                    }
                    out[c] = fmaf(neg_eta, gv, o);
                }
            }
        }
    }
}

// ------------------------------------------------------------------- CSR SVM: margins ----
// One wavefront per (job, minibatch row): gather w[col], reduce across the 64 lanes.
__device__ __forceinline__ void csr_margin_block(const HopGradJob* __restrict__ jobs, int B,
                                                 int rows_per_job_blocks, int loss, int bid) {
    const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const HopGradJob* job = jobs + bid / rows_per_job_blocks;
    const int m = (bid % rows_per_job_blocks) * (kThreads / 64) + wv;
    if (m >= B) return;
    const int r = job->rows[m];
    const int64_t lo = job->rowptr[r], hi = job->rowptr[r + 1];
    const float* w = job->w;
    float acc = 0.f;
    for (int64_t p = lo + lane; p < hi; p += 64) acc = fmaf(job->val[p], w[job->col[p]], acc);
    acc = wave_sum(acc);
    if (lane == 0) job->coef[m] = loss_coef(job->y[r], acc, 1.0f / (float)B, loss);
}

__global__ __launch_bounds__(kThreads) void csr_margin_kernel(const HopGradJob* __restrict__ jobs, int B,
                                                              int rows_per_job_blocks, int loss) {
    csr_margin_block(jobs, B, rows_per_job_blocks, loss, (int)blockIdx.x);
}

// The margins of a wave's STEP records and the wave's Reduce + Apply in one launch: both only read
// x_k, and nothing a wave writes is read inside it, so they need no order between them.  The few
// latency-bound margin workgroups come first and run under the streaming ones.
template <int VEC, int NT, int MAP>
__global__ __launch_bounds__(kThreads) void mix_csr_margin_kernel(const HopMixJob* __restrict__ mix_jobs, int n_mix,
                                                                  int64_t d, int64_t n_chunks,
                                                                  const HopGradJob* __restrict__ grad_jobs, int B,
                                                                  int rows_per_job_blocks, int loss,
                                                                  int margin_blocks) {
    if ((int)blockIdx.x < margin_blocks) {
        csr_margin_block(grad_jobs, B, rows_per_job_blocks, loss, (int)blockIdx.x);
        return;
    }
    mix_block<VEC, NT, MAP, kThreads>(mix_jobs, n_mix, d, n_chunks, (int64_t)blockIdx.x - margin_blocks);
}

// the same two fusions for the paired Reduce + Apply
__global__ __launch_bounds__(kThreads) void pair_csr_margin_kernel(const HopPairJob* __restrict__ mix_jobs, int n_mix,
                                                                   int64_t d, int64_t n_chunks, int run, int reverse,
                                                                   const HopGradJob* __restrict__ grad_jobs, int B,
                                                                   int rows_per_job_blocks, int loss, int margin_blocks) {
    if ((int)blockIdx.x < margin_blocks) {
        csr_margin_block(grad_jobs, B, rows_per_job_blocks, loss, (int)blockIdx.x);
        return;
    }
    pair_block(mix_jobs, n_mix, d, n_chunks, run, reverse, (int64_t)blockIdx.x - margin_blocks);
}

__global__ __launch_bounds__(kThreads) void pair_dense_margin_kernel(const HopPairJob* __restrict__ mix_jobs, int n_mix,
                                                                     int64_t d, int64_t n_chunks, int run, int reverse,
                                                                     const HopGradJob* __restrict__ grad_jobs, int B,
                                                                     int nseg, int64_t margin_blocks) {
    __shared__ float red[kThreads / 64];
    if ((int64_t)blockIdx.x >= margin_blocks) {
        pair_block(mix_jobs, n_mix, d, n_chunks, run, reverse, (int64_t)blockIdx.x - margin_blocks);
        return;
    }
    dense_margin_block(grad_jobs, B, d, nseg, blockIdx.x, red);
}

template <int VEC, int NT, int MAP>
int launch_mix_csr_margin(const HopMixJob* mix_dev, int n_mix, int64_t d, const HopGradJob* grad_dev, int n_grad, int B,
                          int loss, void* stream) {
    int64_t n_chunks;
    const int64_t grid = mix_grid<VEC, MAP, kThreads>(n_mix, d, &n_chunks);
    const int per = (B + kThreads / 64 - 1) / (kThreads / 64);
    const int64_t margin_blocks = (int64_t)n_grad * per;
    if (grid + margin_blocks > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((mix_csr_margin_kernel<VEC, NT, MAP>), dim3((unsigned)(grid + margin_blocks)), dim3(kThreads), 0,
                       (hipStream_t)stream, mix_dev, n_mix, d, n_chunks, grad_dev, B, per, loss, (int)margin_blocks);
    return (int)hipGetLastError();
}

// target[col] += factor * c_m * val for the active rows (the sparse part of -eta g, or of g).
// One wavefront per minibatch row, 16 rows per workgroup, all in flight together.  Sparse features
// are heavy-tailed (a few columns occur in almost every row) and fp32 atomics on one address
// serialise in L2: B atomics in a chain on the hottest column would set the kernel's duration.
// Contributions to the first kHotCols columns are therefore added up in LDS first and leave the
// workgroup as one global atomic per column touched (16 times fewer on the hot ones).
constexpr int kScatterThreads = 1024;
constexpr int kScatterRows = kScatterThreads / 64;
constexpr int kHotCols = 1024;

__global__ __launch_bounds__(kScatterThreads) void csr_scatter_kernel(const HopGradJob* __restrict__ jobs, int B,
                                                                      int blocks_per_job, float factor,
                                                                      int into_velocity) {
    __shared__ float hot[kHotCols];
    const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const HopGradJob* job = jobs + blockIdx.x / blocks_per_job;
    const int m = (blockIdx.x % blocks_per_job) * kScatterRows + wv;
    for (int i = threadIdx.x; i < kHotCols; i += kScatterThreads) hot[i] = 0.f;
    __syncthreads();
    float* target = into_velocity ? job->vel : job->out;
    if (m < B) {
        const float c = job->coef[m];
        if (c != 0.f) {
            const int r = job->rows[m];
            const int64_t lo = job->rowptr[r], hi = job->rowptr[r + 1];
            const float f = factor * c;
            for (int64_t p = lo + lane; p < hi; p += 64) {
                const int col = job->col[p];
                const float v = f * job->val[p];
                if (col < kHotCols) atomicAdd(&hot[col], v);
                else unsafeAtomicAdd(target + col, v);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kHotCols; i += kScatterThreads) {
        const float v = hot[i];
        if (v != 0.f) unsafeAtomicAdd(target + i, v);
    }
}

// g = lambda w, the dense part of a CSR gradient when a dense g is wanted.
__global__ __launch_bounds__(kThreads) void scale_kernel(const HopGradJob* __restrict__ jobs, int n_jobs,
                                                         int64_t d, float lambda, int64_t n_chunks) {
    int j;
    int64_t chunk;
    if (!map_block(blockIdx.x, n_jobs, n_chunks, &j, &chunk)) return;
    const HopGradJob* job = jobs + j;
    for (int q = 0; q < 4; ++q) {
        int64_t c = (chunk * 4 + q) * kThreads + threadIdx.x;
        if (c < d) job->out[c] = lambda * job->w[c];
    }
}

// Input check for CSR data: rowptr non-decreasing over [0, rows], every column id inside [0, d).
// flag[0] becomes 1 on any violation.
__global__ __launch_bounds__(kThreads) void csr_check_kernel(const int64_t* __restrict__ rowptr,
                                                             const int32_t* __restrict__ col, int64_t rows,
                                                             int64_t first, int64_t nnz, int64_t d, int* flag) {
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    bool bad = false;
    if (t < rows) bad = rowptr[t] > rowptr[t + 1] || rowptr[t] < first;
    if (t < nnz) {
        const int32_t c = col[first + t];
        bad = bad || c < 0 || (int64_t)c >= d;
    }
    if (bad) atomicExch(flag, 1);
}

__global__ __launch_bounds__(kThreads) void copy_kernel(float4* __restrict__ dst, const float4* __restrict__ src,
                                                        int64_t n16) {
    int64_t i = (int64_t)blockIdx.x * (kThreads * 4) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < 4; ++u, i += kThreads)
        if (i < n16) dst[i] = src[i];
}

inline int launch_status() { return (int)hipGetLastError(); }

}  // namespace

int hopk_mix(const HopMixJob* jobs_dev, int n_jobs, int64_t d, void* stream) {
    if (n_jobs <= 0) return 0;
    // long vectors: every XCD takes runs of 4 consecutive 16 KB chunks (3-4 % faster on 64-100 MB
    // vectors: longer contiguous pieces per stream); short ones: single chunks, less padding
    if ((d >> 2) >= (int64_t)1024 * kThreads * 4) return launch_mix<4, 1, 14, 256>(jobs_dev, n_jobs, d, stream);
    return launch_mix<4, 1, 1, 256>(jobs_dev, n_jobs, d, stream);
}

int hopk_synth(const HopGradJob* jobs_dev, int n_jobs, int reverse, int64_t d, void* stream) {
    if (n_jobs <= 0) return 0;
    int64_t n4 = d >> 2;
    int64_t n_chunks = (n4 + kSynthChunk4 - 1) / kSynthChunk4;
    if (n_chunks < 1) n_chunks = 1;
    int64_t grid = grid_for(n_jobs, n_chunks);
    if (grid > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(synth_kernel, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, jobs_dev,
                       n_jobs, d, n_chunks, reverse);
    return launch_status();
}

int hopk_dense_nseg(int64_t d) {
    int64_t n = (d + kSegCols - 1) / kSegCols;
    return (int)(n < 1 ? 1 : n);
}

int hopk_dense_margin(const HopGradJob* jobs_dev, int n_jobs, int B, int64_t d, void* stream) {
    if (n_jobs <= 0 || B <= 0) return 0;
    const int nseg = hopk_dense_nseg(d);
    const int row_groups = (B + kMarginRows - 1) / kMarginRows;
    const int64_t grid = (int64_t)n_jobs * row_groups * nseg;
    if (grid > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(dense_margin4_kernel, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, jobs_dev, B,
                       d, nseg, row_groups);
    return launch_status();
}

int hopk_dense_grad(const HopGradJob* jobs_dev, int n_jobs, int B, int64_t d, float lambda, int loss,
                    void* stream) {
    if (n_jobs <= 0 || B <= 0) return 0;
    if (B > kMaxB) return (int)hipErrorInvalidValue;
    int nseg = hopk_dense_nseg(d);
    int64_t n_chunks = (d + 4 * kThreads - 1) / (4 * kThreads);
    int64_t grid = grid_for(n_jobs, n_chunks);
    if (grid > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    // a launch of fewer workgroups than the GPU has CUs is bound by each workgroup's chain of row loads
    if (grid <= 128 && (d & 3) == 0)
        hipLaunchKernelGGL(dense_grad_kernel<4>, dim3((unsigned)grid), dim3(kThreads * 4), 0, (hipStream_t)stream,
                           jobs_dev, n_jobs, B, d, nseg, lambda, loss, n_chunks);
    else
        hipLaunchKernelGGL(dense_grad_kernel<1>, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, jobs_dev,
                           n_jobs, B, d, nseg, lambda, loss, n_chunks);
    return launch_status();
}

int hopk_csr_margin(const HopGradJob* jobs_dev, int n_jobs, int B, int loss, void* stream) {
    if (n_jobs <= 0 || B <= 0) return 0;
    int per = (B + kThreads / 64 - 1) / (kThreads / 64);
    hipLaunchKernelGGL(csr_margin_kernel, dim3((unsigned)(n_jobs * per)), dim3(kThreads), 0, (hipStream_t)stream,
                       jobs_dev, B, per, loss);
    return launch_status();
}

template <int VEC, int NT, int MAP>
int launch_mix_dense_margin(const HopMixJob* mix_dev, int n_mix, int64_t d, const HopGradJob* grad_dev, int n_grad, int B,
                            void* stream) {
    int64_t n_chunks;
    const int64_t grid = mix_grid<VEC, MAP, kThreads>(n_mix, d, &n_chunks);
    const int nseg = hopk_dense_nseg(d);
    const int64_t margin_blocks = (int64_t)n_grad * B * nseg;
    if (grid + margin_blocks > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((mix_dense_margin_kernel<VEC, NT, MAP>), dim3((unsigned)(grid + margin_blocks)), dim3(kThreads), 0,
                       (hipStream_t)stream, mix_dev, n_mix, d, n_chunks, grad_dev, B, nseg, margin_blocks);
    return (int)hipGetLastError();
}

int hopk_mix_dense_margin(const HopMixJob* mix_dev, int n_mix, int64_t d, const HopGradJob* grad_dev, int n_grad, int B,
                          void* stream) {
    if (n_grad <= 0 || B <= 0) return hopk_mix(mix_dev, n_mix, d, stream);
    if (n_mix <= 0) return hopk_dense_margin(grad_dev, n_grad, B, d, stream);
    if ((d >> 2) >= (int64_t)1024 * kThreads * 4)
        return launch_mix_dense_margin<4, 1, 14>(mix_dev, n_mix, d, grad_dev, n_grad, B, stream);
    return launch_mix_dense_margin<4, 1, 1>(mix_dev, n_mix, d, grad_dev, n_grad, B, stream);
}

int hopk_mix_csr_margin(const HopMixJob* mix_dev, int n_mix, int64_t d, const HopGradJob* grad_dev, int n_grad, int B,
                        int loss, void* stream) {
    if (n_grad <= 0 || B <= 0) return hopk_mix(mix_dev, n_mix, d, stream);
    if (n_mix <= 0) return hopk_csr_margin(grad_dev, n_grad, B, loss, stream);
    if ((d >> 2) >= (int64_t)1024 * kThreads * 4)
        return launch_mix_csr_margin<4, 1, 14>(mix_dev, n_mix, d, grad_dev, n_grad, B, loss, stream);
    return launch_mix_csr_margin<4, 1, 1>(mix_dev, n_mix, d, grad_dev, n_grad, B, loss, stream);
}

int hopk_pair(const HopPairJob* jobs_dev, int n_jobs, int n_sources, int reverse, int64_t d, void* stream) {
    if (n_jobs <= 0) return 0;
    const int64_t n_chunks = pair_chunks(d);
    const int run = pair_run(n_sources, n_chunks);
    const int64_t grid = pair_grid(n_jobs, n_chunks, run);
    if (grid > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(pair_mix_kernel, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, jobs_dev, n_jobs, d,
                       n_chunks, run, reverse);
    return launch_status();
}

int hopk_pair_csr_margin(const HopPairJob* mix_dev, int n_mix, int n_sources, int reverse, int64_t d,
                         const HopGradJob* grad_dev, int n_grad, int B, int loss, void* stream) {
    if (n_grad <= 0 || B <= 0) return hopk_pair(mix_dev, n_mix, n_sources, reverse, d, stream);
    if (n_mix <= 0) return hopk_csr_margin(grad_dev, n_grad, B, loss, stream);
    const int64_t n_chunks = pair_chunks(d);
    const int run = pair_run(n_sources, n_chunks);
    const int64_t grid = pair_grid(n_mix, n_chunks, run);
    const int per = (B + kThreads / 64 - 1) / (kThreads / 64);
    const int64_t margin_blocks = (int64_t)n_grad * per;
    if (grid + margin_blocks > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(pair_csr_margin_kernel, dim3((unsigned)(grid + margin_blocks)), dim3(kThreads), 0,
                       (hipStream_t)stream, mix_dev, n_mix, d, n_chunks, run, reverse, grad_dev, B, per, loss,
                       (int)margin_blocks);
    return launch_status();
}

int hopk_pair_dense_margin(const HopPairJob* mix_dev, int n_mix, int n_sources, int reverse, int64_t d,
                           const HopGradJob* grad_dev, int n_grad, int B, void* stream) {
    if (n_grad <= 0 || B <= 0) return hopk_pair(mix_dev, n_mix, n_sources, reverse, d, stream);
    if (n_mix <= 0) return hopk_dense_margin(grad_dev, n_grad, B, d, stream);
    const int64_t n_chunks = pair_chunks(d);
    const int run = pair_run(n_sources, n_chunks);
    const int64_t grid = pair_grid(n_mix, n_chunks, run);
    const int nseg = hopk_dense_nseg(d);
    const int64_t margin_blocks = (int64_t)n_grad * B * nseg;
    if (grid + margin_blocks > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(pair_dense_margin_kernel, dim3((unsigned)(grid + margin_blocks)), dim3(kThreads), 0,
                       (hipStream_t)stream, mix_dev, n_mix, d, n_chunks, run, reverse, grad_dev, B, nseg, margin_blocks);
    return launch_status();
}

int hopk_csr_scatter(const HopGradJob* jobs_dev, int n_jobs, int B, float factor, int into_velocity, void* stream) {
    if (n_jobs <= 0 || B <= 0) return 0;
    int per = (B + kScatterRows - 1) / kScatterRows;
    hipLaunchKernelGGL(csr_scatter_kernel, dim3((unsigned)(n_jobs * per)), dim3(kScatterThreads), 0,
                       (hipStream_t)stream, jobs_dev, B, per, factor, into_velocity);
    return launch_status();
}

int hopk_csr_dense_grad(const HopGradJob* jobs_dev, int n_jobs, int B, int64_t d, float lambda, void* stream) {
    if (n_jobs <= 0) return 0;
    int64_t n_chunks = (d + 4 * kThreads - 1) / (4 * kThreads);
    int64_t grid = grid_for(n_jobs, n_chunks);
    if (grid > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(scale_kernel, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, jobs_dev,
                       n_jobs, d, lambda, n_chunks);
    int rc = launch_status();
    if (rc) return rc;
    return hopk_csr_scatter(jobs_dev, n_jobs, B, -1.0f, 0, stream);
}

int hopk_csr_check(const int64_t* rowptr, const int32_t* col, int64_t rows, int64_t first, int64_t nnz, int64_t d,
                   int* flag_dev, void* stream) {
    int64_t n = rows > nnz ? rows : nnz;
    if (n <= 0) return 0;
    int64_t grid = (n + kThreads - 1) / kThreads;
    if (grid > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(csr_check_kernel, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, rowptr, col,
                       rows, first, nnz, d, flag_dev);
    return launch_status();
}

int hopk_copy(void* dst, const void* src, size_t bytes, void* stream) {
    int64_t n16 = (int64_t)(bytes / 16);
    if (n16 <= 0) return 0;
    int64_t grid = (n16 + kThreads * 4 - 1) / (kThreads * 4);
    if (grid > 0x7FFFFFFFll) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, (float4*)dst,
                       (const float4*)src, n16);
    return launch_status();
}

// ------------------------------------------- dense SVM gradient without any allocation ----
// For callers that cannot allocate (a stream being captured, a tight serving loop, a harness that forbids
// hipMalloc): the job descriptor and the partial dot products, which hop_svm_grad_dense takes from a hipMalloc
// of its own and from the caller's scratch argument, live in a fixed array in device memory instead.
namespace {

constexpr size_t kStaticDescBytes = 256;
constexpr int64_t kStaticPartials = 65536;                 // most B x column segments (16384 columns each)
static __device__ __align__(256) unsigned char scratch[kStaticDescBytes + kStaticPartials * sizeof(float)];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];                          // device address of `scratch` on each GPU, once known
int g_scratch_state[kMaxDevices];                          // 0 unknown, 1 known

__global__ void stage_job_kernel(HopGradJob job, HopGradJob* dst) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *dst = job;
}

}  // namespace

extern "C" int hop_svm_grad_dense_static(const float* X, const float* y, const float* w, const int32_t* rows_dev,
                                         int32_t B, int64_t d, float lambda, int32_t loss, float* g, float* coef,
                                         void* hip_stream) {
    if (!X || !y || !w || !rows_dev || !g || !coef || B < 1 || B > kMaxB || d < 1 ||
        (loss != HOP_LOSS_HINGE && loss != HOP_LOSS_LOG))
        return HOP_ERR_INVALID_ARG;
    if (d % 4 == 0 && ((((uintptr_t)X | (uintptr_t)w | (uintptr_t)g) & 15u) != 0)) return HOP_ERR_INVALID_ARG;
    const int nseg = hopk_dense_nseg(d);
    if ((int64_t)B * nseg > kStaticPartials) {
        fprintf(stderr, "libhop: hop_svm_grad_dense_static: B x ceil(d / 16384) = %lld exceeds the fixed scratch of %lld "
                        "partial sums\n", (long long)B * nseg, (long long)kStaticPartials);
        return HOP_ERR_ARENA_TOO_SMALL;
    }
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HOP_ERR_HIP;
    if (!g_scratch_state[dev]) {
        // each GPU holds its own copy of the array at its own address: ask once per device, with it current
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr) {
            fprintf(stderr, "libhop: hipGetSymbolAddress(scratch): %s\n", hipGetErrorString(e));
            return HOP_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
        g_scratch_state[dev] = 1;
    }
    unsigned char* base = (unsigned char*)g_scratch_ptr[dev];
    HopGradJob* desc = (HopGradJob*)base;
    static_assert(sizeof(HopGradJob) <= kStaticDescBytes, "descriptor must fit its slot");
    HopGradJob gj;
    memset(&gj, 0, sizeof(gj));
    gj.X = X; gj.y = y; gj.w = w; gj.rows = rows_dev; gj.g = g; gj.coef = coef;
    gj.partial = (float*)(base + kStaticDescBytes);        // every entry is written by the margin pass before it is read
    hipLaunchKernelGGL(stage_job_kernel, dim3(1), dim3(64), 0, (hipStream_t)hip_stream, gj, desc);
    int rc = launch_status();
    if (!rc) rc = hopk_dense_margin(desc, 1, B, d, hip_stream);
    if (!rc) rc = hopk_dense_grad(desc, 1, B, d, lambda, loss, hip_stream);
    if (rc) {
        fprintf(stderr, "libhop: hop_svm_grad_dense_static launch: %s\n", hipGetErrorString((hipError_t)rc));
        return HOP_ERR_HIP;
    }
    return HOP_OK;
}
