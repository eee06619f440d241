// Internal declarations shared by the host side (hop_api.cpp, hop_sim.cpp) and the
// kernels (hop_kernels.hip).  Nothing here is part of the public ABI.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "hop.h"

// ---- device-side job descriptors (plain data, uploaded once per schedule) ----------
struct alignas(16) HopMixJob {
    float* out;
    const float* g;            // null: no gradient term
    float* vel;                // null: no momentum; else v <- mu v + g in place, Apply uses v
    float eta;
    int32_t A;
    float mu;
    float lam_fold;            // with vel: v <- mu v + g + lam_fold * src[0] (the dense part of a sparse gradient)
    const float* src[HOP_MAX_A];
    float w[HOP_MAX_A];
};

constexpr int kMaxGradAhead = 16;
constexpr int HOP_PAIR_U = 12;   // most vectors in the union of a pair of records (the kernel unrolls up to this)

// One or two records of a wave whose source sets overlap, run by one workgroup per column chunk: the union of
// their sources (each loaded once), and per record a membership mask over the union with its weights.  A single
// record may have up to HOP_MAX_A sources; a pair at most 12 in the union.  Records with a velocity keep HopMixJob.
struct alignas(16) HopPairJob {
    int32_t U, G;              // vectors in the union, records (1 or 2)
    float eta;
    int32_t reserved;
    float* out[2];
    const float* g[2];         // null: no gradient term
    uint32_t mask[2];          // bit u: the record averages src[u]
    const float* src[HOP_MAX_A];
    float w[2][HOP_MAX_A];     // weight of src[u] in record r (0 where the record does not read it)
};

struct alignas(16) HopGradJob {
    // dense: X row-major rows x d; csr: rowptr/col/val
    const float* X;
    const int64_t* rowptr;
    const int32_t* col;
    const float* val;
    const float* y;
    const float* w;            // x_{k,i}: the version the gradient is taken at
    const int32_t* rows;       // B sample ids
    float* g;                  // dense gradient buffer of the worker (dense / synth modes)
    float* coef;               // B hinge coefficients of this record
    float* partial;            // dense: B x nseg partial dot products
    float* out;                // csr: the vector the sparse part is scattered into; dense: if set, the gradient is
                               // applied to it in place (out -= eta g) instead of being written to g
    float* vel;                // with momentum: csr, the velocity the sparse part is scattered into as well;
                               // dense with out set, v <- mu v + g in place and out -= eta v
    const HopMixJob* reduce;   // dense with out set: if set, out = sum_a w'_a x_a - eta g (the gradient kernel does the
                               // record's Reduce too); if null, out already holds the reduced vector
    float eta, mu;             // dense with out set
    uint32_t k0, k1, k2;       // synth: hash keys of (seed, worker, iteration)
    float scale;               // synth: fp32 factor
};

// Packs the Reduce jobs of one wave for pair_mix_kernel (appends to `out`; see its definition for the rule); returns the
// number of distinct vectors the jobs read.  Host only.
int hop_pack_pairs(const HopMixJob* jobs, int n, std::vector<HopPairJob>& out);

// ---- kernel launchers (hop_kernels.hip); all return a hipError_t as int ------------
int hopk_mix(const HopMixJob* jobs_dev, int n_jobs, int64_t d, void* stream);
int hopk_synth(const HopGradJob* jobs_dev, int n_jobs, int reverse, int64_t d, void* stream);
int hopk_dense_margin(const HopGradJob* jobs_dev, int n_jobs, int B, int64_t d, void* stream);
int hopk_dense_grad(const HopGradJob* jobs_dev, int n_jobs, int B, int64_t d, float lambda, int loss, void* stream);
int hopk_csr_margin(const HopGradJob* jobs_dev, int n_jobs, int B, int loss, void* stream);
int hopk_mix_dense_margin(const HopMixJob* mix_dev, int n_mix, int64_t d, const HopGradJob* grad_dev, int n_grad, int B,
                          void* stream);
int hopk_mix_csr_margin(const HopMixJob* mix_dev, int n_mix, int64_t d, const HopGradJob* grad_dev, int n_grad, int B,
                        int loss, void* stream);
// n_sources: distinct vectors the jobs read (sizes the XCD runs); reverse: walk the vectors from their end
int hopk_pair(const HopPairJob* jobs_dev, int n_jobs, int n_sources, int reverse, int64_t d, void* stream);
int hopk_pair_csr_margin(const HopPairJob* mix_dev, int n_mix, int n_sources, int reverse, int64_t d,
                         const HopGradJob* grad_dev, int n_grad, int B, int loss, void* stream);
int hopk_pair_dense_margin(const HopPairJob* mix_dev, int n_mix, int n_sources, int reverse, int64_t d,
                           const HopGradJob* grad_dev, int n_grad, int B, void* stream);
int hopk_csr_scatter(const HopGradJob* jobs_dev, int n_jobs, int B, float factor, int into_velocity, void* stream);
int hopk_csr_dense_grad(const HopGradJob* jobs_dev, int n_jobs, int B, int64_t d, float lambda, void* stream);
int hopk_csr_check(const int64_t* rowptr, const int32_t* col, int64_t rows, int64_t first, int64_t nnz, int64_t d,
                   int* flag_dev, void* stream);
int hopk_copy(void* dst, const void* src, size_t bytes, void* stream);
int hopk_dense_nseg(int64_t d);                 // column segments per row in the margin pass

// ---- host-side random numbers (hop_sim.cpp) ---------------------------------------
namespace hoprng {
enum : uint64_t { STREAM_DELAY = 1, STREAM_BATCH = 2, STREAM_SYNTHGRAD = 6, STREAM_LATENCY = 7 };
uint64_t mix(uint64_t seed, uint64_t stream, uint64_t a, uint64_t b, uint64_t c);
void synth_keys(uint64_t seed, int worker, int iter, uint32_t* k0, uint32_t* k1, uint32_t* k2);
float synth_scale(float variance);
}  // namespace hoprng

// ---- schedule ----------------------------------------------------------------------
struct hop_schedule {
    int N = 0, D = 0, K = 0, batch = 0, stalled = 0, n_jumps = 0, n_waves = 0, late_sends = 0;   // D: slots per worker in memory
    std::vector<int32_t> kind, worker, iter, wave, out_slot, src_begin, src_worker, src_tag, src_slot;
    std::vector<uint64_t> time;
    std::vector<float> src_weight;
    std::vector<int32_t> batch_rows, final_iter, wave_begin, wave_order;
    std::vector<uint64_t> finish_time;
    std::vector<int64_t> rows_at_sim;   // data-set sizes the minibatch ids were drawn for

    // device side: descriptors laid out by hop_step, for the context's current gradient mode, inside the
    // workspace the caller lent with hop_schedule_bind (the library allocates no device memory for a schedule)
    hop_ctx* owner = nullptr;
    char* workspace = nullptr;
    size_t workspace_bytes = 0;
    int built_mode = -1;
    uint64_t built_epoch = 0;
    HopMixJob* mix_dev = nullptr;       // n_records, in wave order
    HopPairJob* pair_dev = nullptr;     // the same records packed in pairs, wave by wave (null with a velocity)
    HopGradJob* grad_dev = nullptr;     // STEP records only, in wave order
    int32_t* rows_dev = nullptr;        // n_records x batch
    float* coef_dev = nullptr;          // n_records x batch
    bool dense_in_place = false;        // dense SVM: margins beside the Reduce, gradient applied in place
    std::vector<int32_t> grad_begin;    // n_waves + 1 offsets into grad_dev
    std::vector<int32_t> pair_begin;    // n_waves + 1 offsets into pair_dev
    std::vector<int32_t> wave_sources;  // distinct vectors each wave reads
    std::vector<int32_t> wave_mix_jobs; // records in each wave's mix launch (its first descriptors; the rest, if any,
                                        // are reduced by their gradient kernel)
    std::vector<double> wave_mix_bytes; // algorithmic bytes of each wave's mix launch
    std::vector<double> wave_grad_bytes;
    void* graph_exec = nullptr;         // hipGraphExec_t of waves [0, n_waves), see hop_use_graph()
    uint64_t graph_epoch = 0;
    int graph_mode = -1;
};

// ---- context -----------------------------------------------------------------------
struct HopData {
    int64_t rows = 0;
    const float* X = nullptr;
    const int64_t* rowptr = nullptr;
    const int32_t* col = nullptr;
    const float* val = nullptr;
    const float* y = nullptr;
};

struct HopProfile {
    std::vector<void*> ev;              // pairs of hipEvent_t, recycled
    std::vector<int> pending_kernel;    // kernel id of each recorded pair
    std::vector<double> pending_bytes;
    double ms[HOP_KERNEL_COUNT] = {0, 0, 0};
    int64_t launches[HOP_KERNEL_COUNT] = {0, 0, 0};
    double bytes[HOP_KERNEL_COUNT] = {0, 0, 0};
};

struct hop_ctx {
    int N = 0, s = 0, b = 0, D = 0, max_ig = 0;
    int slots = 0;                      // slots per worker in memory: D, plus the current-parameter slot D when serial
    int64_t d = 0, stride = 0;
    hop_opts opts{};
    std::vector<std::vector<int>> in_nbrs, out_nbrs;
    std::vector<float> W;               // N x N, W[j*N+i]
    // device
    bool has_device = false;
    char* arena = nullptr;
    size_t arena_bytes = 0;
    void* stream = nullptr;
    float* ring = nullptr;              // N x D x stride
    float* gbuf = nullptr;              // N x grad_ahead x stride
    int grad_ahead = 1;                 // gradient buffers per worker (hop_opts.grad_ahead, at least 1)
    float* partial = nullptr;           // N x batch x nseg
    float* vel = nullptr;               // N x stride velocities, only with momentum
    std::vector<HopData> data;
    int grad_mode = HOP_GRAD_ZERO;
    float synth_variance = 0.f;
    const float* external = nullptr;
    uint64_t epoch = 0;                 // bumped whenever job descriptors would change
    std::vector<int32_t> version;       // newest iteration held per worker
    std::vector<hop_schedule*> schedules;   // live schedules of this context (hop_simulate .. hop_schedule_free)
    const hop_schedule* running = nullptr;
    int next_wave = 0;
    bool profiling = false;
    bool use_graph = false;
    void* capture_stream = nullptr;     // library-owned stream used only to record graphs
    HopProfile prof;
    std::string last_error;
};

int hop_run_protocol(const hop_ctx* ctx, const hop_delay_model* dm, int K, hop_schedule* out);
