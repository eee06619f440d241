// C ABI of the Hop hot path: contexts, layout of the parameter rings in the caller's arena,
// translation of a schedule into device job descriptors, and the per-wave kernel launches.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <new>

#include "hop_internal.h"

namespace {

constexpr int64_t kAlignFloats = 64;       // 256 bytes
constexpr int kMaxBatch = 1024;
constexpr size_t kMaxPendingEvents = 1 << 15;
constexpr int64_t kDenseInPlaceBytes = 2 << 20;

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

int effective_max_ig(int s, const hop_opts* o) {
    if (o && o->notify_ack) return 2;      // a sender is never more than 2 iterations ahead of a receiver
    int ig = o ? o->max_ig : 0;
    return ig > 0 ? ig : std::max(s, 1);
}

// Versions a ring must hold: the paper's #queues = max_ig + 1 when updates arrive in order (the tag
// taken is the sender's last Send); with reordering a reader in iteration k may take tag k - s while
// the sender, at most max_ig ahead, has produced version k + max_ig + 1.  Exact-tag mode (s = 0) reads
// tag k while versions up to k + max_ig + 1 exist.
int ring_depth(int s, int max_ig, uint32_t max_latency) {
    if (s >= 1) return max_latency > 1 ? s + max_ig + 2 : max_ig + 1;
    return max_ig + 2;
}

// Every slot starts on a 256-byte boundary; the extra 256 bytes keep the slots of a power-of-two d
// from all mapping to the same HBM channel phase.
int64_t slot_stride(int64_t d) {
    return round_up(d, kAlignFloats) + kAlignFloats;
}

int64_t partial_floats(int64_t d, int batch) {
    return round_up((int64_t)std::max(batch, 1) * hopk_dense_nseg(d), kAlignFloats);
}

int hip_fail(hop_ctx* ctx, hipError_t e, const char* what) {
    if (ctx) ctx->last_error = std::string(what) + ": " + hipGetErrorString(e);
    std::fprintf(stderr, "libhop: %s: %s\n", what, hipGetErrorString(e));
    return HOP_ERR_HIP;
}

#define HOP_HIP(ctx, call)                                          \
    do {                                                            \
        hipError_t e_ = (call);                                     \
        if (e_ != hipSuccess) return hip_fail((ctx), e_, #call);    \
    } while (0)

#define HOP_LAUNCH(ctx, call)                                                        \
    do {                                                                             \
        int e_ = (call);                                                             \
        if (e_ != 0) return hip_fail((ctx), (hipError_t)e_, "kernel launch " #call); \
    } while (0)

// Forget the descriptors laid out in the schedule's workspace (the memory is the caller's).
void free_device_side(hop_schedule* s) {
    s->mix_dev = nullptr;
    s->pair_dev = nullptr;
    s->grad_dev = nullptr;
    s->rows_dev = nullptr;
    s->coef_dev = nullptr;
    s->built_mode = -1;
    if (s->graph_exec) (void)hipGraphExecDestroy((hipGraphExec_t)s->graph_exec);
    s->graph_exec = nullptr;
}

constexpr size_t kWsAlign = 256;
inline size_t ws_round(size_t v) { return (v + kWsAlign - 1) / kWsAlign * kWsAlign; }

// Device bytes the descriptors of R records with minibatches of B need: sample ids, coefficients, one
// Reduce descriptor per record in both forms, one gradient descriptor per record.
size_t workspace_need(size_t R, size_t B) {
    return 2 * ws_round(R * B * sizeof(float)) + ws_round(R * sizeof(HopMixJob)) + ws_round(R * sizeof(HopPairJob)) +
           ws_round(R * sizeof(HopGradJob)) + kWsAlign;
}

}  // namespace

// Pack the Reduce jobs of one wave two by two: a record is joined with the later record (among the next 64 still
// single) that shares the most sources with it, provided the union stays within HOP_PAIR_U vectors.  Union order:
// the first record's sources in its own order, then what the second adds.  Only waves whose records read every
// distinct vector at least twice on average are paired: there a shared load in registers saves an L2 request that
// matters (32 workers, 23 records of ~7 sources per wave: 1472 -> 1434 us per launch); where records share little
// (64 workers, 9 records of ~5 sources per wave) single records run 3 % faster than pairs, which halve the number
// of workgroups per column chunk without saving many loads.  Returns the distinct vectors of the wave.
int hop_pack_pairs(const HopMixJob* jobs, int n, std::vector<HopPairJob>& out) {
    std::vector<char> used((size_t)n, 0);
    std::vector<const float*> all;
    for (int i = 0; i < n; ++i) all.insert(all.end(), jobs[i].src, jobs[i].src + jobs[i].A);
    const size_t reads = all.size();
    std::sort(all.begin(), all.end());
    const int distinct = (int)(std::unique(all.begin(), all.end()) - all.begin());
    const bool pairing = reads >= 2 * (size_t)distinct;
    for (int i = 0; i < n; ++i) {
        if (used[i]) continue;
        used[i] = 1;
        const HopMixJob& a = jobs[i];
        int best = -1, best_overlap = 0;
        if (pairing && a.A <= HOP_PAIR_U) {
            int seen = 0;
            for (int k = i + 1; k < n && seen < 64; ++k) {
                if (used[k]) continue;
                ++seen;
                const HopMixJob& b = jobs[k];
                int overlap = 0;
                for (int q = 0; q < b.A; ++q)
                    if (std::find(a.src, a.src + a.A, b.src[q]) != a.src + a.A) ++overlap;
                if (overlap > best_overlap && a.A + b.A - overlap <= HOP_PAIR_U) {
                    best = k;
                    best_overlap = overlap;
                }
            }
        }
        HopPairJob pj;
        std::memset(&pj, 0, sizeof(pj));
        pj.eta = a.eta;
        pj.G = 1;
        pj.U = a.A;
        pj.out[0] = a.out;
        pj.g[0] = a.g;
        for (int q = 0; q < a.A; ++q) {
            pj.src[q] = a.src[q];
            pj.w[0][q] = a.w[q];
            if (q < 32) pj.mask[0] |= 1u << q;
        }
        if (best >= 0) {
            used[best] = 1;
            const HopMixJob& b = jobs[best];
            pj.G = 2;
            pj.out[1] = b.out;
            pj.g[1] = b.g;
            for (int q = 0; q < b.A; ++q) {
                int u = (int)(std::find(pj.src, pj.src + pj.U, b.src[q]) - pj.src);
                if (u == pj.U) pj.src[pj.U++] = b.src[q];
                pj.w[1][u] += b.w[q];      // a record that lists one vector twice keeps the sum of its weights
                pj.mask[1] |= 1u << u;
            }
        }
        out.push_back(pj);
    }
    return distinct;
}

namespace {

float* slot_ptr(const hop_ctx* c, int worker, int slot) {
    return c->ring + ((int64_t)worker * c->slots + slot) * c->stride;
}

// Translate the schedule into device descriptors for the context's current gradient source.
int build_jobs(hop_ctx* c, hop_schedule* s) {
    free_device_side(s);
    const int R = (int)s->kind.size();
    const int mode = c->grad_mode;
    const int B = s->batch;
    if ((mode == HOP_GRAD_SVM_DENSE || mode == HOP_GRAD_SVM_CSR) && B <= 0) return HOP_ERR_STATE;
    // the minibatch ids were drawn modulo the data-set sizes known to hop_simulate: a data set
    // attached since then must have the same number of rows, or the ids could point past its end
    if (mode == HOP_GRAD_SVM_DENSE || mode == HOP_GRAD_SVM_CSR)
        for (int i = 0; i < c->N; ++i)
            if ((size_t)i >= s->rows_at_sim.size() || s->rows_at_sim[i] != c->data[i].rows) return HOP_ERR_STATE;
    if (!s->workspace || s->workspace_bytes < workspace_need((size_t)R, (size_t)std::max(B, 0)))
        return HOP_ERR_ARENA_TOO_SMALL;       // hop_schedule_bind first
    char* ws = s->workspace;
    auto carve = [&ws](size_t bytes) {
        char* p = ws;
        ws += ws_round(bytes);
        return p;
    };
    if (B > 0) {
        s->rows_dev = (int32_t*)carve((size_t)R * B * sizeof(int32_t));
        s->coef_dev = (float*)carve((size_t)R * B * sizeof(float));
        HOP_HIP(c, hipMemcpy(s->rows_dev, s->batch_rows.data(), (size_t)R * B * sizeof(int32_t),
                             hipMemcpyHostToDevice));
        HOP_HIP(c, hipMemset(s->coef_dev, 0, (size_t)R * B * sizeof(float)));
    }
    // dense minibatches of up to 2 MB per record take the margins-beside-the-Reduce path of launch_waves (measured:
    // 0.65 -> 0.51 ms per pass at 256 KB per record; at 32 MB the margin pass wants a launch of its own for occupancy)
    s->dense_in_place = mode == HOP_GRAD_SVM_DENSE && (int64_t)B * c->d * 4 <= kDenseInPlaceBytes;
    // Larger dense minibatches: margins, then a gradient kernel that also does the Reduce + Apply of its record
    // (the time is the rows'; a separate mix launch of a few hundred KB per record would only add its start-up,
    // measured 4 us + gap per wave at 16 workers x 65536 columns).  The wave's mix then only holds the records
    // without a gradient (jumps).  Their descriptors come first in the wave's range, so both lists are contiguous.
    const bool dense_fused = mode == HOP_GRAD_SVM_DENSE && !s->dense_in_place;
    std::vector<HopMixJob> mix((size_t)std::max(R, 1));
    std::vector<HopGradJob> grad;
    s->grad_begin.assign(s->n_waves + 1, 0);
    s->wave_mix_jobs.assign(s->n_waves, 0);
    s->wave_mix_bytes.assign(s->n_waves, 0.0);
    s->wave_grad_bytes.assign(s->n_waves, 0.0);
    const float eta = c->opts.lr;
    std::vector<int> grad_seen((size_t)c->N, 0);
    if (R > 0) s->mix_dev = (HopMixJob*)carve((size_t)R * sizeof(HopMixJob));
    auto has_gradient = [&](int e) {
        return (s->kind[e] == HOP_STEP || s->kind[e] == HOP_APPLY) && mode != HOP_GRAD_ZERO;
    };
    for (int w = 0; w < s->n_waves; ++w) {
        const int jb = s->wave_begin[w], je = s->wave_begin[w + 1];
        int n_plain = je - jb;                         // records whose Reduce stays in the wave's mix launch
        if (dense_fused) {
            n_plain = 0;
            for (int p = jb; p < je; ++p) n_plain += has_gradient(s->wave_order[p]) ? 0 : 1;
        }
        s->wave_mix_jobs[w] = n_plain;
        int next_plain = jb, next_fused = jb + n_plain;
        for (int p = jb; p < je; ++p) {
            const int e = s->wave_order[p];
            const int i = s->worker[e];
            const bool fused = dense_fused && has_gradient(e);
            const int pos = !dense_fused ? p : (fused ? next_fused++ : next_plain++);
            HopMixJob& mj = mix[pos];
            std::memset(&mj, 0, sizeof(mj));
            mj.out = slot_ptr(c, i, s->out_slot[e]);
            mj.eta = eta;
            mj.A = s->src_begin[e + 1] - s->src_begin[e];
            for (int a = 0; a < mj.A; ++a) {
                int q = s->src_begin[e] + a;
                mj.src[a] = slot_ptr(c, s->src_worker[q], s->src_slot[q]);
                mj.w[a] = s->src_weight[q];
            }
            if (has_gradient(e)) {                     // STEP and APPLY records
                HopGradJob gj;
                std::memset(&gj, 0, sizeof(gj));
                gj.w = mj.src[0];
                // a worker's successive gradient records rotate through its buffers, so the gradients of
                // grad_ahead consecutive waves (at most one record per worker and wave) can exist side by side
                gj.g = c->gbuf + ((int64_t)i * c->grad_ahead + grad_seen[i]++ % c->grad_ahead) * c->stride;
                if (B > 0) {
                    gj.rows = s->rows_dev + (size_t)e * B;
                    gj.coef = s->coef_dev + (size_t)e * B;
                }
                const HopData& dd = c->data[i];
                bool want_job = true;
                if (mode == HOP_GRAD_SVM_DENSE) {
                    if (!dd.X || !dd.y) return HOP_ERR_STATE;
                    gj.X = dd.X;
                    gj.y = dd.y;
                    gj.partial = c->partial + (int64_t)i * partial_floats(c->d, c->opts.batch);
                    // the gradient kernel applies -eta g (through the velocity, if any) itself, so no dense g is
                    // written and read back: in place on the vector the mix has reduced (small minibatches), or on
                    // its own Reduce of the record's sources (large ones)
                    gj.out = mj.out;
                    gj.eta = eta;
                    if (fused) gj.reduce = s->mix_dev + pos;
                    if (c->vel) {
                        gj.vel = c->vel + (int64_t)i * c->stride;
                        gj.mu = c->opts.momentum;
                    }
                    s->wave_grad_bytes[w] += 4.0 * (c->vel ? 2.0 * c->d : 0.0) + 4.0 * c->d;
                    if (fused) s->wave_grad_bytes[w] += 4.0 * (double)c->d * mj.A;
                    s->wave_grad_bytes[w] += 4.0 * ((double)B * c->d + 2.0 * c->d) + 8.0 * B;
                } else if (mode == HOP_GRAD_SVM_CSR) {
                    if (!dd.rowptr || !dd.col || !dd.val || !dd.y) return HOP_ERR_STATE;
                    gj.rowptr = dd.rowptr;
                    gj.col = dd.col;
                    gj.val = dd.val;
                    gj.y = dd.y;
                    gj.out = mj.out;                   // where the sparse part of -eta g is scattered
                    if (c->vel) {
                        // with a velocity, lambda w goes into it inside the mix (v <- mu v + lambda x_self) and the
                        // sparse part is scattered into both the velocity (-c x) and the result (+eta c x)
                        mj.vel = c->vel + (int64_t)i * c->stride;
                        mj.mu = c->opts.momentum;
                        mj.lam_fold = c->opts.lambda;
                        gj.vel = mj.vel;
                    } else {
                        // lambda w folds into the self term: sum_a w'_a x_a - eta lambda x_self - eta (sparse part)
                        mj.w[0] = mj.w[0] - eta * c->opts.lambda;
                    }
                } else if (mode == HOP_GRAD_SYNTH) {
                    hoprng::synth_keys(c->opts.seed, i, s->iter[e], &gj.k0, &gj.k1, &gj.k2);
                    gj.scale = hoprng::synth_scale(c->synth_variance);
                    mj.g = gj.g;
                    s->wave_grad_bytes[w] += 4.0 * c->d;
                } else {  // external
                    mj.g = c->external + (int64_t)i * c->d;
                    want_job = false;
                }
                if (want_job) grad.push_back(gj);
                if (c->vel && mj.g && !mj.vel) {
                    mj.vel = c->vel + (int64_t)i * c->stride;
                    mj.mu = c->opts.momentum;
                }
            }
            if (!fused) s->wave_mix_bytes[w] += 4.0 * (double)c->d * (mj.A + 1 + (mj.g ? 1 : 0) + (mj.vel ? 2 : 0));
        }
        s->grad_begin[w + 1] = (int32_t)grad.size();
    }
    if (R > 0) HOP_HIP(c, hipMemcpy(s->mix_dev, mix.data(), (size_t)R * sizeof(HopMixJob), hipMemcpyHostToDevice));
    // without velocities the Reduce runs on records packed in pairs
    s->pair_begin.assign(s->n_waves + 1, 0);
    s->wave_sources.assign(s->n_waves, 0);
    if (!c->vel && R > 0) {
        std::vector<HopPairJob> pairs;
        pairs.reserve((size_t)R);
        for (int w = 0; w < s->n_waves; ++w) {
            s->wave_sources[w] = hop_pack_pairs(mix.data() + s->wave_begin[w], s->wave_mix_jobs[w], pairs);
            s->pair_begin[w + 1] = (int32_t)pairs.size();
        }
        s->pair_dev = (HopPairJob*)carve((size_t)R * sizeof(HopPairJob));
        HOP_HIP(c, hipMemcpy(s->pair_dev, pairs.data(), pairs.size() * sizeof(HopPairJob), hipMemcpyHostToDevice));
    }
    if (!grad.empty()) {
        s->grad_dev = (HopGradJob*)carve((size_t)R * sizeof(HopGradJob));
        HOP_HIP(c, hipMemcpy(s->grad_dev, grad.data(), grad.size() * sizeof(HopGradJob), hipMemcpyHostToDevice));
    }
    s->built_mode = mode;
    s->built_epoch = c->epoch;
    return HOP_OK;
}

// ---- profiling with HIP events on the context's stream ----
int prof_flush(hop_ctx* c) {
    HopProfile& p = c->prof;
    if (p.pending_kernel.empty()) return HOP_OK;
    HOP_HIP(c, hipStreamSynchronize((hipStream_t)c->stream));
    for (size_t n = 0; n < p.pending_kernel.size(); ++n) {
        float ms = 0.f;
        HOP_HIP(c, hipEventElapsedTime(&ms, (hipEvent_t)p.ev[2 * n], (hipEvent_t)p.ev[2 * n + 1]));
        int k = p.pending_kernel[n];
        p.ms[k] += ms;
        p.launches[k] += 1;
        p.bytes[k] += p.pending_bytes[n];
    }
    p.pending_kernel.clear();
    p.pending_bytes.clear();
    return HOP_OK;
}

int prof_begin(hop_ctx* c, int kernel, double bytes) {
    if (!c->profiling) return HOP_OK;
    HopProfile& p = c->prof;
    if (p.pending_kernel.size() >= kMaxPendingEvents) {
        int rc = prof_flush(c);
        if (rc) return rc;
    }
    size_t n = p.pending_kernel.size();
    while (p.ev.size() < 2 * (n + 1)) {
        hipEvent_t e;
        HOP_HIP(c, hipEventCreate(&e));
        p.ev.push_back((void*)e);
    }
    p.pending_kernel.push_back(kernel);
    p.pending_bytes.push_back(bytes);
    HOP_HIP(c, hipEventRecord((hipEvent_t)p.ev[2 * n], (hipStream_t)c->stream));
    return HOP_OK;
}

int prof_end(hop_ctx* c) {
    if (!c->profiling) return HOP_OK;
    size_t n = c->prof.pending_kernel.size() - 1;
    HOP_HIP(c, hipEventRecord((hipEvent_t)c->prof.ev[2 * n + 1], (hipStream_t)c->stream));
    return HOP_OK;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

extern "C" {

const char* hop_strerror(int code) {
    switch (code) {
        case HOP_OK: return "ok";
        case HOP_ERR_INVALID_ARG: return "invalid argument";
        case HOP_ERR_BAD_GRAPH: return "bad communication graph";
        case HOP_ERR_BAD_WEIGHTS: return "bad mixing weights";
        case HOP_ERR_BAD_BACKUP: return "backup workers not below the in-degree";
        case HOP_ERR_ARENA_TOO_SMALL: return "device arena too small";
        case HOP_ERR_DEADLOCK: return "protocol stalled with unfinished workers";
        case HOP_ERR_SLOT_DEAD: return "accepted version already overwritten in its ring";
        case HOP_ERR_HIP: return "HIP runtime error";
        case HOP_ERR_NO_DEVICE: return "context has no device memory";
        case HOP_ERR_STATE: return "call out of order";
        case HOP_ERR_NOMEM: return "out of host memory";
        default: return "unknown error";
    }
}

int hop_version(void) { return 1; }

int hop_opts_default(hop_opts* o) {
    if (!o) return HOP_ERR_INVALID_ARG;
    std::memset(o, 0, sizeof(*o));
    o->max_ig = 0;
    o->skip_on = 0;
    o->max_skip = 10;
    o->trigger = 1;
    o->lr = 0.01f;
    o->lambda = 1e-4f;
    o->batch = 0;
    o->loss = HOP_LOSS_HINGE;
    o->seed = 0;
    o->momentum = 0.f;
    o->max_latency = 0;
    o->serial = 0;
    o->notify_ack = 0;
    o->grad_ahead = 1;
    return HOP_OK;
}

int hop_layout(int64_t d, int32_t s, const hop_opts* o, int32_t* depth, int64_t* stride) {
    if (d < 1 || s < 0) return HOP_ERR_INVALID_ARG;
    int ig = effective_max_ig(s, o);
    if (depth) *depth = ring_depth(s, ig, o ? o->max_latency : 0) + ((o && o->serial) ? 1 : 0);
    if (stride) *stride = slot_stride(d);
    return HOP_OK;
}

size_t hop_arena_bytes(int32_t N, int64_t d, int32_t s, int32_t b, const hop_opts* o) {
    int32_t D = 0;
    int64_t stride = 0;
    if (N < 1 || b < 0 || hop_layout(d, s, o, &D, &stride) != HOP_OK) return 0;
    int batch = o ? o->batch : 0;
    if (o && (o->grad_ahead < 0 || o->grad_ahead > kMaxGradAhead)) return 0;
    const int ahead = o && o->grad_ahead > 1 ? o->grad_ahead : 1;
    int64_t floats = (int64_t)N * D * stride + (int64_t)N * ahead * stride + (int64_t)N * partial_floats(d, batch);
    if (o && o->momentum > 0.f) floats += (int64_t)N * stride;
    return (size_t)floats * sizeof(float);
}

static int init_ctx(hop_ctx** out, const hop_graph* g, const float* W, int32_t N, int64_t d, int32_t s, int32_t b,
                    const hop_opts* opts, const hop_device* dev);

int hop_init(hop_ctx** out, const hop_graph* g, const float* W, int32_t N, int64_t d, int32_t s, int32_t b,
             const hop_opts* opts, const hop_device* dev) {
    try {
        return init_ctx(out, g, W, N, d, s, b, opts, dev);
    } catch (const std::bad_alloc&) {
        return HOP_ERR_NOMEM;
    }
}

static int init_ctx(hop_ctx** out, const hop_graph* g, const float* W, int32_t N, int64_t d, int32_t s, int32_t b,
                    const hop_opts* opts, const hop_device* dev) {
    if (!out) return HOP_ERR_INVALID_ARG;
    *out = nullptr;
    if (!g || !W || !g->row_ptr || N < 1 || d < 1 || d > 0xFFFFFFFFll || s < 0 || b < 0 || g->N != N)
        return HOP_ERR_INVALID_ARG;
    if (N > 1 && !g->col) return HOP_ERR_INVALID_ARG;
    hop_opts o;
    hop_opts_default(&o);
    if (opts) o = *opts;
    if (o.max_ig < 0 || o.max_skip < 1 || o.trigger < 0 || o.batch < 0 || o.batch > kMaxBatch ||
        (o.loss != HOP_LOSS_HINGE && o.loss != HOP_LOSS_LOG) || !(o.momentum >= 0.f && o.momentum < 1.f) ||
        o.grad_ahead < 0 || o.grad_ahead > kMaxGradAhead)
        return HOP_ERR_INVALID_ARG;
    // NOTIFY-ACK supports neither backup workers nor staleness (Section 3.3); it is built for standard training
    if (o.notify_ack && (s != 0 || b != 0 || o.skip_on || o.serial || o.max_latency > 1)) return HOP_ERR_INVALID_ARG;
    std::unique_ptr<hop_ctx> holder(new (std::nothrow) hop_ctx());
    hop_ctx* c = holder.get();
    if (!c) return HOP_ERR_NOMEM;
    c->N = N; c->d = d; c->s = s; c->b = b; c->opts = o;
    c->max_ig = effective_max_ig(s, &o);
    c->D = ring_depth(s, c->max_ig, o.max_latency);
    c->slots = c->D + (o.serial ? 1 : 0);
    c->stride = slot_stride(d);
    c->grad_ahead = o.grad_ahead > 1 ? o.grad_ahead : 1;
    int rc = HOP_OK;
    c->in_nbrs.assign(N, {});
    c->out_nbrs.assign(N, {});
    if (g->row_ptr[0] != 0) rc = HOP_ERR_BAD_GRAPH;
    for (int i = 0; i < N && rc == HOP_OK; ++i) {
        int lo = g->row_ptr[i], hi = g->row_ptr[i + 1];
        if (hi < lo || hi - lo + 1 > HOP_MAX_A) { rc = HOP_ERR_BAD_GRAPH; break; }
        for (int p = lo; p < hi; ++p) {
            int j = g->col[p];
            if (j < 0 || j >= N || j == i || (p > lo && j <= g->col[p - 1])) { rc = HOP_ERR_BAD_GRAPH; break; }
            c->in_nbrs[i].push_back(j);
        }
    }
    if (rc == HOP_OK) {
        for (int i = 0; i < N; ++i)
            for (int j : c->in_nbrs[i]) c->out_nbrs[j].push_back(i);   // ascending by construction
        for (int i = 0; i < N; ++i)
            if (b > 0 && b >= (int)c->in_nbrs[i].size()) rc = HOP_ERR_BAD_BACKUP;
        // the bounds of Theorems 1 and 2 need a path from every node to every other one: everything must be
        // reachable from node 0 along the edges and against them
        for (int dir = 0; dir < 2 && rc == HOP_OK; ++dir) {
            const auto& adj = dir == 0 ? c->out_nbrs : c->in_nbrs;
            std::vector<char> seen((size_t)N, 0);
            std::vector<int> stack{0};
            seen[0] = 1;
            int reached = 1;
            while (!stack.empty()) {
                int u = stack.back();
                stack.pop_back();
                for (int v : adj[u])
                    if (!seen[v]) { seen[v] = 1; ++reached; stack.push_back(v); }
            }
            if (reached != N) rc = HOP_ERR_BAD_GRAPH;
        }
    }
    if (rc == HOP_OK) {
        c->W.assign(W, W + (size_t)N * N);
        for (int i = 0; i < N && rc == HOP_OK; ++i) {
            double col_sum = 0.0;
            for (int j = 0; j < N; ++j) {
                float v = W[(size_t)j * N + i];
                if (!(v >= 0.f)) rc = HOP_ERR_BAD_WEIGHTS;
                bool edge = j == i || std::binary_search(c->in_nbrs[i].begin(), c->in_nbrs[i].end(), j);
                if (!edge && v != 0.f) rc = HOP_ERR_BAD_WEIGHTS;
                col_sum += v;
            }
            if (!(W[(size_t)i * N + i] > 0.f) || std::fabs(col_sum - 1.0) > 1e-6) rc = HOP_ERR_BAD_WEIGHTS;
        }
    }
    if (rc == HOP_OK && dev) {
        size_t need = hop_arena_bytes(N, d, s, b, &o);
        if (!dev->arena || ((uintptr_t)dev->arena & 255u)) rc = HOP_ERR_INVALID_ARG;
        else if (dev->arena_bytes < need) rc = HOP_ERR_ARENA_TOO_SMALL;
        else {
            c->has_device = true;
            c->arena = (char*)dev->arena;
            c->arena_bytes = dev->arena_bytes;
            c->stream = dev->hip_stream;
            c->ring = (float*)dev->arena;
            c->gbuf = c->ring + (int64_t)N * c->slots * c->stride;
            c->partial = c->gbuf + (int64_t)N * c->grad_ahead * c->stride;
            c->vel = o.momentum > 0.f ? c->partial + (int64_t)N * partial_floats(d, o.batch) : nullptr;
        }
    }
    if (rc != HOP_OK) return rc;
    c->data.assign(N, HopData{});
    c->version.assign(N, 0);
    *out = holder.release();
    return HOP_OK;
}

int hop_destroy(hop_ctx* c) {
    if (!c) return HOP_ERR_INVALID_ARG;
    for (hop_schedule* s : c->schedules) s->owner = nullptr;   // they outlive the context as host data only
    for (void* e : c->prof.ev) (void)hipEventDestroy((hipEvent_t)e);
    if (c->capture_stream) (void)hipStreamDestroy((hipStream_t)c->capture_stream);
    delete c;
    return HOP_OK;
}

int hop_set_params(hop_ctx* c, const float* p0, int per_worker, int on_device) {
    if (!c || !p0) return HOP_ERR_INVALID_ARG;
    if (!c->has_device) return HOP_ERR_NO_DEVICE;
    hipStream_t st = (hipStream_t)c->stream;
    for (int i = 0; i < c->N; ++i) {
        const float* src = per_worker ? p0 + (int64_t)i * c->d : p0;
        // x_0: ring slot 0, or the current-parameter slot of the serial approach
        HOP_HIP(c, hipMemcpyAsync(slot_ptr(c, i, c->opts.serial ? c->D : 0), src, (size_t)c->d * sizeof(float),
                                  on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, st));
    }
    if (c->vel) HOP_HIP(c, hipMemsetAsync(c->vel, 0, (size_t)c->N * c->stride * sizeof(float), st));
    if (!on_device) HOP_HIP(c, hipStreamSynchronize(st));   // p0 is only borrowed for the call
    std::fill(c->version.begin(), c->version.end(), 0);
    c->running = nullptr;
    c->next_wave = 0;
    return HOP_OK;
}

int hop_set_rows(hop_ctx* c, int32_t worker, int64_t rows) {
    if (!c || worker < 0 || worker >= c->N || rows < 0 || rows > 0x7FFFFFFFll) return HOP_ERR_INVALID_ARG;
    c->data[worker] = HopData{};
    c->data[worker].rows = rows;
    c->epoch++;
    return HOP_OK;
}

int hop_set_data_dense(hop_ctx* c, int32_t worker, const float* X, const float* y, int64_t rows) {
    if (!c || worker < 0 || worker >= c->N || !X || !y || rows < 1 || rows > 0x7FFFFFFFll)
        return HOP_ERR_INVALID_ARG;
    if (!c->has_device) return HOP_ERR_NO_DEVICE;
    if ((c->d % 4 == 0) && !aligned16(X)) return HOP_ERR_INVALID_ARG;
    HopData dd;
    dd.rows = rows;
    dd.X = X;
    dd.y = y;
    c->data[worker] = dd;
    c->epoch++;
    return HOP_OK;
}

int hop_set_data_csr(hop_ctx* c, int32_t worker, const int64_t* rowptr, const int32_t* col, const float* val,
                     const float* y, int64_t rows) {
    if (!c || worker < 0 || worker >= c->N || !rowptr || !col || !val || !y || rows < 1 || rows > 0x7FFFFFFFll)
        return HOP_ERR_INVALID_ARG;
    if (!c->has_device) return HOP_ERR_NO_DEVICE;
    {
        // The gather and scatter kernels index parameter vectors with these column ids: check on the
        // device, once, that the row pointers are ordered and every id lies in [0, d).
        hipStream_t st = (hipStream_t)c->stream;
        int64_t ends[2] = {0, 0};
        HOP_HIP(c, hipStreamSynchronize(st));
        HOP_HIP(c, hipMemcpy(&ends[0], rowptr, sizeof(int64_t), hipMemcpyDeviceToHost));
        HOP_HIP(c, hipMemcpy(&ends[1], rowptr + rows, sizeof(int64_t), hipMemcpyDeviceToHost));
        if (ends[0] < 0 || ends[1] < ends[0]) return HOP_ERR_INVALID_ARG;
        int* flag = reinterpret_cast<int*>(c->partial);       // scratch of the context, idle between passes
        HOP_HIP(c, hipMemsetAsync(flag, 0, sizeof(int), st));
        HOP_LAUNCH(c, hopk_csr_check(rowptr, col, rows, ends[0], ends[1] - ends[0], c->d, flag, c->stream));
        int bad = 0;
        HOP_HIP(c, hipMemcpyAsync(&bad, flag, sizeof(int), hipMemcpyDeviceToHost, st));
        HOP_HIP(c, hipStreamSynchronize(st));
        if (bad) return HOP_ERR_INVALID_ARG;
    }
    HopData dd;
    dd.rows = rows;
    dd.rowptr = rowptr;
    dd.col = col;
    dd.val = val;
    dd.y = y;
    c->data[worker] = dd;
    c->epoch++;
    return HOP_OK;
}

int hop_set_grad_source(hop_ctx* c, int mode, float variance, const float* external) {
    if (!c || mode < HOP_GRAD_ZERO || mode > HOP_GRAD_EXTERNAL) return HOP_ERR_INVALID_ARG;
    if (mode == HOP_GRAD_SYNTH && !(variance >= 0.f)) return HOP_ERR_INVALID_ARG;
    if (mode == HOP_GRAD_EXTERNAL && (!external || !aligned16(external) || (c->d % 4 != 0 && c->N > 1)))
        return HOP_ERR_INVALID_ARG;
    c->grad_mode = mode;
    c->synth_variance = variance;
    c->external = external;
    c->epoch++;
    return HOP_OK;
}

int hop_simulate(hop_ctx* c, const hop_delay_model* dm, int32_t max_iter, hop_schedule** out) {
    if (!c || !out || max_iter < 0) return HOP_ERR_INVALID_ARG;
    *out = nullptr;
    if (dm) {
        if (dm->kind < HOP_DELAY_NONE || dm->kind > HOP_DELAY_TABLE) return HOP_ERR_INVALID_ARG;
        if (dm->kind == HOP_DELAY_TABLE && (!dm->table || dm->table_iters < max_iter)) return HOP_ERR_INVALID_ARG;
    }
    hop_schedule* s = new (std::nothrow) hop_schedule();
    if (!s) return HOP_ERR_NOMEM;
    int rc;
    try {
        rc = hop_run_protocol(c, dm, max_iter, s);
    } catch (const std::bad_alloc&) {
        rc = HOP_ERR_NOMEM;
    }
    if (rc != HOP_OK && rc != HOP_ERR_DEADLOCK) {
        delete s;
        return rc;
    }
    try {
        c->schedules.push_back(s);
    } catch (const std::bad_alloc&) {
        delete s;
        return HOP_ERR_NOMEM;
    }
    s->owner = c;
    *out = s;
    return rc;
}

int hop_schedule_view(const hop_schedule* s, hop_schedule_arrays* v) {
    if (!s || !v) return HOP_ERR_INVALID_ARG;
    std::memset(v, 0, sizeof(*v));
    v->n_records = (int32_t)s->kind.size();
    v->n_sources = (int32_t)s->src_worker.size();
    v->n_waves = s->n_waves;
    v->n_workers = s->N;
    v->depth = s->D;
    v->batch = s->batch;
    v->stalled = s->stalled;
    v->n_jumps = s->n_jumps;
    v->late_sends = s->late_sends;
    v->kind = s->kind.data();
    v->worker = s->worker.data();
    v->iter = s->iter.data();
    v->time = s->time.data();
    v->wave = s->wave.data();
    v->out_slot = s->out_slot.data();
    v->src_begin = s->src_begin.data();
    v->src_worker = s->src_worker.data();
    v->src_tag = s->src_tag.data();
    v->src_slot = s->src_slot.data();
    v->src_weight = s->src_weight.data();
    v->batch_rows = s->batch > 0 ? s->batch_rows.data() : nullptr;
    v->final_iter = s->final_iter.data();
    v->finish_time = s->finish_time.data();
    v->wave_begin = s->wave_begin.data();
    v->wave_order = s->wave_order.data();
    return HOP_OK;
}

int hop_schedule_free(hop_schedule* s) {
    if (!s) return HOP_ERR_INVALID_ARG;
    if (hop_ctx* c = s->owner) {
        if (c->running == s) {
            c->running = nullptr;
            c->next_wave = 0;
        }
        c->schedules.erase(std::remove(c->schedules.begin(), c->schedules.end(), s), c->schedules.end());
    }
    free_device_side(s);
    delete s;
    return HOP_OK;
}

size_t hop_schedule_bytes(const hop_schedule* s) {
    if (!s) return 0;
    return workspace_need(s->kind.size(), (size_t)std::max(s->batch, 0));
}

int hop_schedule_bind(hop_ctx* c, hop_schedule* s, void* workspace, size_t bytes) {
    if (!c || !s || !workspace || ((uintptr_t)workspace & (kWsAlign - 1))) return HOP_ERR_INVALID_ARG;
    if (!c->has_device) return HOP_ERR_NO_DEVICE;
    if (s->owner != c) return HOP_ERR_INVALID_ARG;
    if (bytes < hop_schedule_bytes(s)) return HOP_ERR_ARENA_TOO_SMALL;
    if (c->running == s) {
        c->running = nullptr;
        c->next_wave = 0;
    }
    free_device_side(s);                   // descriptors are laid out again by the next hop_step
    s->workspace = (char*)workspace;
    s->workspace_bytes = bytes;
    return HOP_OK;
}

// Enqueue the kernels of waves [wb, we) on `stream`.  `timed` brackets every kernel group with
// profiling events (never while a stream is being captured into a graph).
static int launch_waves(hop_ctx* c, hop_schedule* s, int wb, int we, void* stream, bool timed) {
    const int B = s->batch;
    const int mode = c->grad_mode;
    for (int w = wb; w < we; ++w) {
        const int jb = s->wave_begin[w], nj = s->wave_mix_jobs[w];
        const int gb = s->grad_begin[w], ng = s->grad_begin[w + 1] - gb;
        const HopGradJob* gj = s->grad_dev ? s->grad_dev + gb : nullptr;
        const HopPairJob* pj = s->pair_dev ? s->pair_dev + s->pair_begin[w] : nullptr;   // null: contexts with a velocity
        const int np = s->pair_dev ? s->pair_begin[w + 1] - s->pair_begin[w] : 0;
        int rc;
        if (mode == HOP_GRAD_SYNTH && c->grad_ahead > 1) {
            // the generator launches of the waves up to the next multiple of grad_ahead back to back, this wave's
            // last (it ends where the wave's Reduce + Apply starts); a call that starts inside such a group
            // generates the rest of it (the values depend on seed, worker and iteration only).  One launch per
            // wave, not one for all: ~23 write streams side by side run at 6.0 TB/s, ~90 at 5.4
            if (w == wb || w % c->grad_ahead == 0) {
                const int last = std::min((w / c->grad_ahead + 1) * c->grad_ahead, s->n_waves);
                for (int q = last - 1; q >= w; --q) {
                    const int nq = s->grad_begin[q + 1] - s->grad_begin[q];
                    if (nq <= 0) continue;
                    if (timed && (rc = prof_begin(c, HOP_KERNEL_SYNTH, s->wave_grad_bytes[q]))) return rc;
                    HOP_LAUNCH(c, hopk_synth(s->grad_dev + s->grad_begin[q], nq, (q & 1) ^ 1, c->d, stream));
                    if (timed && (rc = prof_end(c))) return rc;
                }
            }
        } else if (ng > 0 && mode == HOP_GRAD_SYNTH) {
            if (timed && (rc = prof_begin(c, HOP_KERNEL_SYNTH, s->wave_grad_bytes[w]))) return rc;
            // the generator ends where this wave's Reduce + Apply starts (it walks odd waves from the end), so the
            // last-written part of the gradients is still in the memory-side cache: 1441 -> 1430 us per mix launch on
            // 32 workers x 25 M columns; ending at the far side instead costs 12 us
            HOP_LAUNCH(c, hopk_synth(gj, ng, (w & 1) ^ 1, c->d, stream));
            if (timed && (rc = prof_end(c))) return rc;
        } else if (ng > 0 && mode == HOP_GRAD_SVM_DENSE && s->dense_in_place) {
            // Small minibatches are bound by launches, not bytes.  Compute beside Reduce (Section 3.2): partial
            // margins and the wave's Reduce in one launch, then the gradient kernel, which applies -eta g to the
            // reduced vectors in place: two dependent launches per wave, not three.  Timed as gradient work.
            if (timed && (rc = prof_begin(c, HOP_KERNEL_GRAD, s->wave_grad_bytes[w] + s->wave_mix_bytes[w]))) return rc;
            if (pj)
                HOP_LAUNCH(c, hopk_pair_dense_margin(pj, np, s->wave_sources[w], w & 1, c->d, gj, ng, B, stream));
            else
                HOP_LAUNCH(c, hopk_mix_dense_margin(s->mix_dev + jb, nj, c->d, gj, ng, B, stream));
            HOP_LAUNCH(c, hopk_dense_grad(gj, ng, B, c->d, c->opts.lambda, c->opts.loss, stream));
            if (timed && (rc = prof_end(c))) return rc;
            continue;
        } else if (ng > 0 && mode == HOP_GRAD_SVM_DENSE) {
            // Large minibatches: margins, then gradient + Reduce + Apply of the same records in one kernel.
            if (timed && (rc = prof_begin(c, HOP_KERNEL_GRAD, s->wave_grad_bytes[w]))) return rc;
            HOP_LAUNCH(c, hopk_dense_margin(gj, ng, B, c->d, stream));
            HOP_LAUNCH(c, hopk_dense_grad(gj, ng, B, c->d, c->opts.lambda, c->opts.loss, stream));
            if (timed && (rc = prof_end(c))) return rc;
        }
        if (nj == 0) continue;                         // every record of the wave was finished by its gradient kernel
        const bool csr = ng > 0 && mode == HOP_GRAD_SVM_CSR;
        if (timed && (rc = prof_begin(c, HOP_KERNEL_MIX, s->wave_mix_bytes[w]))) return rc;
        if (csr && pj)   // margins and Reduce + Apply both only read x_k: one launch
            HOP_LAUNCH(c, hopk_pair_csr_margin(pj, np, s->wave_sources[w], w & 1, c->d, gj, ng, B, c->opts.loss, stream));
        else if (csr)
            HOP_LAUNCH(c, hopk_mix_csr_margin(s->mix_dev + jb, nj, c->d, gj, ng, B, c->opts.loss, stream));
        else if (pj)
            HOP_LAUNCH(c, hopk_pair(pj, np, s->wave_sources[w], w & 1, c->d, stream));
        else
            HOP_LAUNCH(c, hopk_mix(s->mix_dev + jb, nj, c->d, stream));
        if (timed && (rc = prof_end(c))) return rc;
        if (csr) {
            if (timed && (rc = prof_begin(c, HOP_KERNEL_GRAD, s->wave_grad_bytes[w]))) return rc;
            HOP_LAUNCH(c, hopk_csr_scatter(gj, ng, B, c->opts.lr, 0, stream));
            if (c->vel) HOP_LAUNCH(c, hopk_csr_scatter(gj, ng, B, -1.0f, 1, stream));
            if (timed && (rc = prof_end(c))) return rc;
        }
    }
    return HOP_OK;
}

// Record waves [0, n_waves) once into a HIP graph (captured on a stream of the library's own, default
// priority; the caller's may be the null stream, which cannot be captured) and keep the executable.
static int capture_graph(hop_ctx* c, hop_schedule* s) {
    if (s->graph_exec) {
        (void)hipGraphExecDestroy((hipGraphExec_t)s->graph_exec);
        s->graph_exec = nullptr;
    }
    if (!c->capture_stream) {
        hipStream_t st;
        HOP_HIP(c, hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
        c->capture_stream = (void*)st;
    }
    hipStream_t cs = (hipStream_t)c->capture_stream;
    HOP_HIP(c, hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal));
    int rc = launch_waves(c, s, 0, s->n_waves, c->capture_stream, false);
    hipGraph_t graph = nullptr;
    hipError_t e = hipStreamEndCapture(cs, &graph);
    if (rc != HOP_OK) {
        if (graph) (void)hipGraphDestroy(graph);
        return rc;
    }
    if (e != hipSuccess) return hip_fail(c, e, "hipStreamEndCapture");
    hipGraphExec_t exec = nullptr;
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) return hip_fail(c, e, "hipGraphInstantiate");
    s->graph_exec = (void*)exec;
    s->graph_epoch = c->epoch;
    s->graph_mode = c->grad_mode;
    return HOP_OK;
}

int hop_step(hop_ctx* c, const hop_schedule* sched, int32_t wave_begin, int32_t wave_end) {
    if (!c || !sched) return HOP_ERR_INVALID_ARG;
    if (!c->has_device) return HOP_ERR_NO_DEVICE;
    hop_schedule* s = const_cast<hop_schedule*>(sched);
    if (s->owner != c) return HOP_ERR_INVALID_ARG;
    if (wave_end < 0) wave_end = s->n_waves;
    if (wave_begin < 0 || wave_begin > wave_end || wave_end > s->n_waves) return HOP_ERR_INVALID_ARG;
    if (wave_begin != 0 && (c->running != s || wave_begin != c->next_wave)) return HOP_ERR_STATE;
    if (s->built_mode != c->grad_mode || s->built_epoch != c->epoch) {
        int rc;
        try {
            rc = build_jobs(c, s);
        } catch (const std::bad_alloc&) {
            rc = HOP_ERR_NOMEM;
        }
        if (rc != HOP_OK) return rc;
    }
    c->running = s;
    int rc;
    if (c->use_graph && !c->profiling && wave_begin == 0 && wave_end == s->n_waves && s->n_waves > 0) {
        if (!s->graph_exec || s->graph_epoch != c->epoch || s->graph_mode != c->grad_mode)
            if ((rc = capture_graph(c, s)) != HOP_OK) return rc;
        HOP_HIP(c, hipGraphLaunch((hipGraphExec_t)s->graph_exec, (hipStream_t)c->stream));
    } else if ((rc = launch_waves(c, s, wave_begin, wave_end, c->stream, c->profiling)) != HOP_OK) {
        return rc;
    }
    for (int p = s->wave_begin[wave_begin]; p < s->wave_begin[wave_end]; ++p) {
        int e = s->wave_order[p];
        const int kind = s->kind[e];
        if (kind == HOP_STEP || kind == HOP_REDUCE) c->version[s->worker[e]] = s->iter[e] + 1;
        else if (kind == HOP_JUMP) c->version[s->worker[e]] = s->iter[e];
    }
    c->next_wave = wave_end;
    return HOP_OK;
}

int hop_use_graph(hop_ctx* c, int enable) {
    if (!c) return HOP_ERR_INVALID_ARG;
    if (!c->has_device) return HOP_ERR_NO_DEVICE;
    c->use_graph = enable != 0;
    return HOP_OK;
}

int hop_params(hop_ctx* c, int32_t worker, const float** dev_ptr, int32_t* iter) {
    if (!c || worker < 0 || worker >= c->N) return HOP_ERR_INVALID_ARG;
    if (!c->has_device) return HOP_ERR_NO_DEVICE;
    if (dev_ptr) *dev_ptr = slot_ptr(c, worker, c->opts.serial ? c->D : c->version[worker] % c->D);
    if (iter) *iter = c->version[worker];
    return HOP_OK;
}

int hop_slot(hop_ctx* c, int32_t worker, int32_t slot, float** dev_ptr) {
    if (!c || !dev_ptr || worker < 0 || worker >= c->N || slot < 0 || slot >= c->slots) return HOP_ERR_INVALID_ARG;
    if (!c->has_device) return HOP_ERR_NO_DEVICE;
    *dev_ptr = slot_ptr(c, worker, slot);
    return HOP_OK;
}

int hop_coef(hop_ctx* c, const hop_schedule* s, int32_t record, const float** dev_ptr) {
    if (!c || !s || !dev_ptr || record < 0 || record >= (int)s->kind.size()) return HOP_ERR_INVALID_ARG;
    if (!s->coef_dev || s->batch <= 0) return HOP_ERR_STATE;
    *dev_ptr = s->coef_dev + (size_t)record * s->batch;
    return HOP_OK;
}

int hop_profile(hop_ctx* c, int enable) {
    if (!c) return HOP_ERR_INVALID_ARG;
    if (!c->has_device) return HOP_ERR_NO_DEVICE;
    if (!enable && c->profiling) {
        int rc = prof_flush(c);
        if (rc) return rc;
    }
    c->profiling = enable != 0;
    return HOP_OK;
}

int hop_profile_read(hop_ctx* c, int kernel, double* ms, int64_t* launches, double* bytes) {
    if (!c || kernel < 0 || kernel >= HOP_KERNEL_COUNT) return HOP_ERR_INVALID_ARG;
    if (!c->has_device) return HOP_ERR_NO_DEVICE;
    int rc = prof_flush(c);
    if (rc) return rc;
    if (ms) *ms = c->prof.ms[kernel];
    if (launches) *launches = c->prof.launches[kernel];
    if (bytes) *bytes = c->prof.bytes[kernel];
    c->prof.ms[kernel] = 0;
    c->prof.launches[kernel] = 0;
    c->prof.bytes[kernel] = 0;
    return HOP_OK;
}

// ---- stand-alone kernels: upload one descriptor set, launch, wait, release ----
int hop_mix(const hop_mix_job* jobs, int32_t n_jobs, int64_t d, void* stream) {
    if (!jobs || n_jobs < 0 || d < 1) return HOP_ERR_INVALID_ARG;
    if (n_jobs == 0) return HOP_OK;
    std::vector<HopMixJob> host((size_t)n_jobs);
    for (int j = 0; j < n_jobs; ++j) {
        const hop_mix_job& in = jobs[j];
        if (in.A < 1 || in.A > HOP_MAX_A || !in.out || !aligned16(in.out) || (in.g && !aligned16(in.g)))
            return HOP_ERR_INVALID_ARG;
        HopMixJob& mj = host[j];
        std::memset(&mj, 0, sizeof(mj));
        if (in.vel && (!aligned16(in.vel) || !(in.mu >= 0.f))) return HOP_ERR_INVALID_ARG;
        mj.out = in.out;
        mj.g = in.g;
        mj.vel = in.vel;
        mj.mu = in.mu;
        mj.eta = in.eta;
        mj.A = in.A;
        for (int a = 0; a < in.A; ++a) {
            if (!in.src[a] || !aligned16(in.src[a])) return HOP_ERR_INVALID_ARG;
            mj.src[a] = in.src[a];
            mj.w[a] = in.w[a];
        }
    }
    bool any_vel = false;
    for (const HopMixJob& mj : host) any_vel = any_vel || mj.vel != nullptr;
    std::vector<HopPairJob> pairs;
    int n_sources = 0;
    if (!any_vel) n_sources = hop_pack_pairs(host.data(), n_jobs, pairs);    // the path hop_step takes without velocities
    const size_t bytes = any_vel ? host.size() * sizeof(HopMixJob) : pairs.size() * sizeof(HopPairJob);
    void* dev = nullptr;
    HOP_HIP(nullptr, hipMalloc(&dev, bytes));
    hipError_t e = hipMemcpy(dev, any_vel ? (const void*)host.data() : (const void*)pairs.data(), bytes,
                             hipMemcpyHostToDevice);
    int rc = 0;
    if (e == hipSuccess)
        rc = any_vel ? hopk_mix((const HopMixJob*)dev, n_jobs, d, stream)
                     : hopk_pair((const HopPairJob*)dev, (int)pairs.size(), n_sources, 0, d, stream);
    hipError_t e2 = hipStreamSynchronize((hipStream_t)stream);
    (void)hipFree(dev);
    if (e != hipSuccess) return hip_fail(nullptr, e, "hipMemcpy");
    if (rc) return hip_fail(nullptr, (hipError_t)rc, "mix launch");
    if (e2 != hipSuccess) return hip_fail(nullptr, e2, "hipStreamSynchronize");
    return HOP_OK;
}

int64_t hop_grad_scratch_floats(int64_t d, int32_t B) {
    if (d < 1 || B < 1) return 0;
    return partial_floats(d, B);
}

static int run_one_grad(const HopGradJob& gj, int kind, int B, int64_t d, float lambda, int loss, void* stream) {
    HopGradJob* dev = nullptr;
    HOP_HIP(nullptr, hipMalloc((void**)&dev, sizeof(HopGradJob)));
    hipError_t e = hipMemcpy(dev, &gj, sizeof(HopGradJob), hipMemcpyHostToDevice);
    int rc = 0;
    if (e == hipSuccess) {
        if (kind == HOP_GRAD_SVM_DENSE) {
            rc = hopk_dense_margin(dev, 1, B, d, stream);
            if (!rc) rc = hopk_dense_grad(dev, 1, B, d, lambda, loss, stream);
        } else if (kind == HOP_GRAD_SVM_CSR) {
            rc = hopk_csr_margin(dev, 1, B, loss, stream);
            if (!rc) rc = hopk_csr_dense_grad(dev, 1, B, d, lambda, stream);
        } else {
            rc = hopk_synth(dev, 1, 0, d, stream);
        }
    }
    hipError_t e2 = hipStreamSynchronize((hipStream_t)stream);
    (void)hipFree(dev);
    if (e != hipSuccess) return hip_fail(nullptr, e, "hipMemcpy");
    if (rc) return hip_fail(nullptr, (hipError_t)rc, "gradient launch");
    if (e2 != hipSuccess) return hip_fail(nullptr, e2, "hipStreamSynchronize");
    return HOP_OK;
}

int hop_svm_grad_dense(const float* X, const float* y, const float* w, const int32_t* rows_dev, int32_t B,
                       int64_t d, float lambda, int32_t loss, float* g, float* coef, float* scratch,
                       void* stream) {
    if (!X || !y || !w || !rows_dev || !g || !coef || !scratch || B < 1 || B > kMaxBatch || d < 1 ||
        (loss != HOP_LOSS_HINGE && loss != HOP_LOSS_LOG))
        return HOP_ERR_INVALID_ARG;
    if (d % 4 == 0 && (!aligned16(X) || !aligned16(w) || !aligned16(g))) return HOP_ERR_INVALID_ARG;
    HopGradJob gj;
    std::memset(&gj, 0, sizeof(gj));
    gj.X = X; gj.y = y; gj.w = w; gj.rows = rows_dev; gj.g = g; gj.coef = coef; gj.partial = scratch;
    return run_one_grad(gj, HOP_GRAD_SVM_DENSE, B, d, lambda, loss, stream);
}

int hop_svm_grad_csr(const int64_t* rowptr, const int32_t* col, const float* val, const float* y, const float* w,
                     const int32_t* rows_dev, int32_t B, int64_t d, float lambda, int32_t loss, float* g,
                     float* coef, void* stream) {
    if (!rowptr || !col || !val || !y || !w || !rows_dev || !g || !coef || B < 1 || B > kMaxBatch || d < 1 ||
        (loss != HOP_LOSS_HINGE && loss != HOP_LOSS_LOG))
        return HOP_ERR_INVALID_ARG;
    HopGradJob gj;
    std::memset(&gj, 0, sizeof(gj));
    gj.rowptr = rowptr; gj.col = col; gj.val = val; gj.y = y; gj.w = w; gj.rows = rows_dev;
    gj.g = g; gj.out = g; gj.coef = coef;
    return run_one_grad(gj, HOP_GRAD_SVM_CSR, B, d, lambda, loss, stream);
}

int hop_synth_grad(uint64_t seed, int32_t worker, int32_t iter, float variance, float* g, int64_t d, void* stream) {
    if (!g || d < 1 || d > 0xFFFFFFFFll || !(variance >= 0.f) || !aligned16(g)) return HOP_ERR_INVALID_ARG;
    HopGradJob gj;
    std::memset(&gj, 0, sizeof(gj));
    gj.g = g;
    hoprng::synth_keys(seed, worker, iter, &gj.k0, &gj.k1, &gj.k2);
    gj.scale = hoprng::synth_scale(variance);
    return run_one_grad(gj, HOP_GRAD_SYNTH, 0, d, 0.f, HOP_LOSS_HINGE, stream);
}

int hop_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || (bytes & 15u) || !aligned16(dst) || !aligned16(src)) return HOP_ERR_INVALID_ARG;
    int rc = hopk_copy(dst, src, bytes, stream);
    if (rc) return hip_fail(nullptr, (hipError_t)rc, "copy launch");
    return HOP_OK;
}

int hop_download(void* host_dst, const void* dev_src, size_t bytes, void* stream) {
    if (!host_dst || !dev_src) return HOP_ERR_INVALID_ARG;
    if (bytes == 0) return HOP_OK;
    HOP_HIP(nullptr, hipMemcpyAsync(host_dst, dev_src, bytes, hipMemcpyDeviceToHost, (hipStream_t)stream));
    HOP_HIP(nullptr, hipStreamSynchronize((hipStream_t)stream));
    return HOP_OK;
}

}  // extern "C"
