/*
 * hop.h - C ABI of the MI355X-native hot path of Hop, the heterogeneity-aware
 * decentralized training protocol (arXiv 1902.01064).
 *
 * N simulated workers are kept as fp32 parameter replicas in one GPU's HBM.
 * Every worker owns a ring of D versions of its parameter vector; a "Send" of
 * the paper is a reference (worker, iteration tag) into that ring (Section 6.1:
 * one queue per iteration, index iter mod #queues).  A host discrete-event
 * simulator applies the queue protocol of Sections 4 and 5 to seeded compute
 * delays and emits a schedule: one record per worker iteration saying which
 * (neighbour, tag) updates its Recv accepted and with which weights.  HIP
 * kernels then run the records: the hinge-loss SVM minibatch gradient
 * ("Compute") and the fused Reduce + Apply
 *        x_{k+1,i} = sum_a w'_a x_{(j_a, t_a)} - eta g_{k,i}
 * (Figure "Standard Decentralized Training", steps 2 and 3).
 *
 * Conventions
 *  - Every function returns HOP_OK (0) or a negative HOP_ERR_* code; nothing
 *    throws or aborts across this boundary.  hop_strerror() names a code.
 *  - "host" pointers are ordinary memory, read during the call only.  "device"
 *    pointers are HIP device memory of the current device; those handed in
 *    (arena, data sets, external gradients) are borrowed for the life of the
 *    context and never freed by the library.  Pointers handed out are borrowed
 *    from the library and stay valid until the object they belong to is freed.
 *  - Kernel launches are enqueued on the caller's stream and return at once;
 *    the caller synchronises.  One context per thread.
 *  - All vectors are contiguous fp32.  Worker i's version v lives in ring slot
 *    v mod D at arena + ((i * D + slot) * stride) floats, stride from
 *    hop_layout().
 */
#ifndef HOP_H
#define HOP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HOP_MAX_A 32   /* most vectors one Reduce can average: |N_in(i)| + 1 */

enum {
    HOP_OK = 0,
    HOP_ERR_INVALID_ARG = -1,     /* null pointer, negative size, unknown enum value */
    HOP_ERR_BAD_GRAPH = -2,       /* index out of range, self edge, unsorted or duplicate neighbour,
                                     degree + 1 > HOP_MAX_A, or not strongly connected (Theorems 1 and 2) */
    HOP_ERR_BAD_WEIGHTS = -3,     /* negative weight, weight on a non-edge, zero self weight, or a
                                     receiver's column not summing to 1 within 1e-6 (Section 3.1) */
    HOP_ERR_BAD_BACKUP = -4,      /* b >= |N_in(i)| for some i (backup-worker figure: N_buw < |N_in|) */
    HOP_ERR_ARENA_TOO_SMALL = -5,
    HOP_ERR_DEADLOCK = -6,        /* events ran out with unfinished workers; the schedule of what
                                     did happen is still returned */
    HOP_ERR_SLOT_DEAD = -7,       /* an accepted version was already overwritten in its ring */
    HOP_ERR_HIP = -8,             /* a HIP runtime call failed */
    HOP_ERR_NO_DEVICE = -9,       /* context was created without device memory (host-only) */
    HOP_ERR_STATE = -10,          /* call out of order (no data set, waves out of sequence, ...) */
    HOP_ERR_NOMEM = -11
};

/* Compute-delay models (Section 7.3.1 / 7.3.5 slow-downs).  One time unit is 2^20 ticks. */
enum {
    HOP_DELAY_NONE = 0,           /* 1 unit                                                   */
    HOP_DELAY_EXP1 = 1,           /* Exp(1) units                                             */
    HOP_DELAY_BERNOULLI6 = 2,     /* 6 units with probability 1/N, else 1 (Section 7.3.1)     */
    HOP_DELAY_TABLE = 3           /* ticks given per (worker, iteration)                      */
};
#define HOP_TICKS_NEVER (1ull << 62)   /* a duration at or above this never completes */

enum {
    HOP_GRAD_ZERO = 0,            /* g = 0 (pure averaging)                                   */
    HOP_GRAD_SVM_DENSE = 1,       /* hinge SVM on dense rows                                  */
    HOP_GRAD_SVM_CSR = 2,         /* hinge SVM on CSR rows                                    */
    HOP_GRAD_SYNTH = 3,           /* seeded synthetic gradient, variance given                */
    HOP_GRAD_EXTERNAL = 4         /* caller's device buffer, N x d floats, read at every STEP */
};

/* Kinds of schedule records.  STEP: Reduce + Apply of one iteration (parallel approach, Section 3.2).  JUMP: the
 * Reduce without gradient of a skipped stretch (Section 5).  With the serial approach an iteration is two records:
 * APPLY (y_k = x_k - eta g(x_k), into the ring slot that is sent) and REDUCE (x_{k+1} = sum_a w'_a y_a, into the
 * worker's current parameters). */
enum { HOP_STEP = 0, HOP_JUMP = 1, HOP_APPLY = 2, HOP_REDUCE = 3 };

/* Loss of the linear SVM: hinge, or the log loss the paper's own runs use (Section 7.2). */
enum { HOP_LOSS_HINGE = 0, HOP_LOSS_LOG = 1 };

enum { HOP_KERNEL_MIX = 0, HOP_KERNEL_GRAD = 1, HOP_KERNEL_SYNTH = 2, HOP_KERNEL_COUNT = 3 };

typedef struct hop_ctx hop_ctx;             /* opaque, owned by the library */
typedef struct hop_schedule hop_schedule;   /* opaque, owned by the library until hop_schedule_free */

/* Communication graph G = (V, E) of Section 3.1 as CSR over receivers: the non-self in-coming
 * neighbours of node i are col[row_ptr[i] .. row_ptr[i+1]), ascending.  The self-loop is implied. */
typedef struct {
    int32_t N;
    const int32_t* row_ptr;       /* host, N + 1 */
    const int32_t* col;           /* host, row_ptr[N] */
} hop_graph;

/* Device memory and stream lent by the caller. */
typedef struct {
    void* arena;                  /* device, at least hop_arena_bytes(), 256-byte aligned */
    size_t arena_bytes;
    void* hip_stream;             /* hipStream_t, 0 = the null stream */
} hop_device;

typedef struct {
    int32_t max_ig;               /* token-queue bound of Section 4.2; 0 = max(s, 1) */
    int32_t skip_on;              /* Section 5 skipping iterations */
    int32_t max_skip;             /* most iterations per jump (default 10) */
    int32_t trigger;              /* jump only if more than this many iterations behind (default 1) */
    float lr;                     /* eta */
    float lambda;                 /* L2 coefficient of the SVM */
    int32_t batch;                /* minibatch size B, 0 = no data */
    int32_t loss;                 /* HOP_LOSS_* */
    uint64_t seed;
    float momentum;               /* mu in [0, 1): v <- mu v + g, x <- reduce - eta v per worker (Section 7.2
                                     uses 0.9); 0 = plain SGD, no velocity buffers */
    uint32_t max_latency;         /* ticks; 0 or 1: every update arrives one tick after its Send, in order;
                                     larger: seeded uniform 1..max_latency per update, so updates on an edge
                                     can overtake each other (Section 6.1) and the ring gets s + max_ig + 2 slots */
    int32_t serial;               /* 1: the serial approach of Section 3.2 (Compute and Apply on x_k, Send the
                                     result, then Recv and Reduce) instead of the parallel one; every worker then
                                     has one more slot, index D, for its current parameters */
    int32_t notify_ack;           /* 1: NOTIFY-ACK (Section 3.3) instead of token queues: Send(k) waits until every
                                     out-going neighbour has acknowledged update k - 1, sent right after its Reduce;
                                     standard training only (s = 0, b = 0, no skipping, not serial, latency 1),
                                     anything else is HOP_ERR_INVALID_ARG; ring as for max_ig = 2 */
    int32_t grad_ahead;           /* HOP_GRAD_SYNTH: gradients of this many consecutive waves are generated in
                                     front of the first of them (0 or 1: wave by wave; at most 16); every
                                     worker then has that many gradient buffers in the arena.  Same values either
                                     way; fewer switches between the arithmetic-bound generator and the
                                     memory-bound Reduce + Apply, which runs slower right after one */
} hop_opts;

typedef struct {
    int32_t kind;                 /* HOP_DELAY_* */
    int32_t table_iters;          /* HOP_DELAY_TABLE: columns of table */
    const double* mult;           /* host, N per-worker factors, NULL = all 1; >= 2^62 freezes a worker */
    const uint64_t* table;        /* host, N x table_iters ticks, HOP_DELAY_TABLE only */
} hop_delay_model;

/* Flat view of a schedule; all arrays are host memory owned by the schedule.  Record e averages the
 * vectors src_*[src_begin[e] .. src_begin[e+1]) (self term first, then accepted neighbours by
 * ascending id) and writes ring slot out_slot[e] of worker[e]. */
typedef struct {
    int32_t n_records, n_sources, n_waves, n_workers;
    int32_t depth;                /* slots per worker (hop_layout) */
    int32_t batch;                /* row ids per STEP record, 0 if none */
    int32_t stalled;              /* 1 if the run ended in HOP_ERR_DEADLOCK */
    int32_t n_jumps;
    int32_t late_sends;           /* updates sent to a receiver already past their tag (Section 6.2 b) */
    int32_t reserved;
    const int32_t* kind;          /* HOP_STEP / HOP_JUMP */
    const int32_t* worker;
    const int32_t* iter;          /* STEP, APPLY, REDUCE: the iteration k; JUMP: the iteration jumped to */
    const uint64_t* time;         /* simulated tick of the Reduce */
    const int32_t* wave;          /* level in the slot-dependence order, see hop_step */
    const int32_t* out_slot;
    const int32_t* src_begin;     /* n_records + 1 */
    const int32_t* src_worker;
    const int32_t* src_tag;       /* iteration tag of the version read */
    const int32_t* src_slot;
    const float* src_weight;      /* w'_a, sums to 1 per record */
    const int32_t* batch_rows;    /* n_records x batch sample ids (zeros for JUMP), or NULL */
    const int32_t* final_iter;    /* n_workers: Iter(i) when the run ended */
    const uint64_t* finish_time;  /* n_workers: tick at which K was reached (0 if never) */
    const int32_t* wave_begin;    /* n_waves + 1 offsets into wave_order */
    const int32_t* wave_order;    /* record ids grouped by wave, ascending id inside a wave */
} hop_schedule_arrays;

/* One fused Reduce + Apply:  out[c] = sum_{a<A} w[a] * src[a][c] - eta * g[c]  for c < d.
 * g may be NULL (a jump's Reduce, Section 5).  out may alias none of src.  With vel != NULL the
 * velocity is updated in place first, vel[c] = mu * vel[c] + g[c], and takes g's place in Apply. */
typedef struct {
    float* out;                   /* device */
    const float* g;               /* device or NULL */
    float eta;
    int32_t A;                    /* 1 .. HOP_MAX_A */
    const float* src[HOP_MAX_A];  /* device */
    float w[HOP_MAX_A];
    float* vel;                   /* device or NULL */
    float mu;
} hop_mix_job;

/* Static text for a HOP_* result code (never NULL); the version of this interface (1). */
const char* hop_strerror(int code);
int hop_version(void);

/* Fills *o with the defaults (max_ig 0, skip off, max_skip 10, trigger 1, lr 0.01, lambda 1e-4,
 * batch 0, hinge loss, seed 0, momentum 0, latency 1, parallel approach, token queues). */
int hop_opts_default(hop_opts* o);

/* Slots per worker and slot stride (in floats) for d parameters under staleness bound s.  The ring has
 * D = max_ig + 1 versions for s >= 1 (Section 6.1's #queues; s + max_ig + 2 when max_latency > 1),
 * max_ig + 2 for s = 0; version v lives in slot v mod D.  depth = D, or D + 1 with the serial approach
 * (slot D: the worker's current parameters, never sent). */
int hop_layout(int64_t d, int32_t s, const hop_opts* o, int32_t* depth, int64_t* stride);

/* Bytes of device memory hop_init needs for rings, gradient buffers and scratch, for the same N, d, s, b and
 * options as hop_init will be given (backup workers change which updates are averaged, not how many versions
 * are kept, so b only has to be valid: 0 is returned for b < 0, as for any other argument hop_init would
 * refuse on sight). */
size_t hop_arena_bytes(int32_t N, int64_t d, int32_t s, int32_t b, const hop_opts* o);

/* Creates a context.  W is host, N x N row-major, W[j*N + i] = weight of sender j at receiver i
 * (Section 3.1; every receiver's column sums to 1).  s = staleness bound (Section 4.4), b = backup
 * workers N_buw per node (Section 4.3).  opts NULL = defaults.  dev NULL = host-only context: the
 * simulator works, anything touching the GPU returns HOP_ERR_NO_DEVICE. */
int hop_init(hop_ctx** out, const hop_graph* g, const float* W, int32_t N, int64_t d, int32_t s,
             int32_t b, const hop_opts* opts, const hop_device* dev);
/* Frees the context; waits for nothing: synchronise the stream first if kernels may still be running. */
int hop_destroy(hop_ctx* ctx);

/* x_{0,i} = p_0 (update-queue figure, line "Initialize local model parameters").  per_worker 0: p0
 * holds d floats for everyone; 1: N x d.  on_device says where p0 lives.  Resets every worker to
 * iteration 0. */
int hop_set_params(hop_ctx* ctx, const float* p0, int per_worker, int on_device);

/* Sample count of a worker's data set when no data is attached (host-only contexts): minibatch row
 * ids are drawn modulo this. */
int hop_set_rows(hop_ctx* ctx, int32_t worker, int64_t rows);
/* Dense rows-by-d fp32 row-major features and +-1 labels, device memory.  Attach data before
 * hop_simulate: the minibatch ids of a schedule are drawn for the row counts known then, and hop_step
 * returns HOP_ERR_STATE if a worker's row count has changed since. */
int hop_set_data_dense(hop_ctx* ctx, int32_t worker, const float* X, const float* y, int64_t rows);
/* CSR features: rowptr int64 [rows+1], col int32 ascending per row, val fp32; labels y; device.
 * The call checks on the device that rowptr is non-decreasing and every column id lies in [0, d)
 * (the kernels index parameter vectors with them) and returns HOP_ERR_INVALID_ARG otherwise; it
 * synchronises the stream. */
int hop_set_data_csr(hop_ctx* ctx, int32_t worker, const int64_t* rowptr, const int32_t* col,
                     const float* val, const float* y, int64_t rows);
/* Where STEP records take their gradient from.  variance: HOP_GRAD_SYNTH only.  external:
 * HOP_GRAD_EXTERNAL only, device, N x d floats (worker-major), read whenever a STEP runs. */
int hop_set_grad_source(hop_ctx* ctx, int mode, float variance, const float* external);

/* Runs the queue protocol (update and token queues, backup workers, bounded staleness, skipping:
 * Sections 4.1 - 4.4 and 5) for max_iter iterations per worker on the host, on the compute delays of
 * `delays` (NULL: one time unit each), and returns the schedule (also when the result is
 * HOP_ERR_DEADLOCK).  Touches no device memory. */
int hop_simulate(hop_ctx* ctx, const hop_delay_model* delays, int32_t max_iter, hop_schedule** out);
/* Fills `out` with borrowed pointers to the schedule's host arrays (see hop_schedule_arrays), valid until
 * hop_schedule_free; HOP_ERR_INVALID_ARG for a NULL argument. */
int hop_schedule_view(const hop_schedule* s, hop_schedule_arrays* out);
/* Frees a schedule (host memory only: its device-side descriptors live in the caller's workspace).  A
 * schedule may outlive its context (its host arrays stay valid), but hop_step refuses it once the
 * context is gone. */
int hop_schedule_free(hop_schedule* s);

/* Device memory hop_step needs for the descriptors of this schedule (per record: the sources, weights and
 * result of its Reduce, the inputs of its Compute, its minibatch sample ids and loss coefficients), and
 * the call that lends it: `workspace` is device memory of at least hop_schedule_bytes(s) bytes, 256-byte
 * aligned, borrowed until the schedule is freed or bound again; the library allocates no device memory
 * for a schedule.  hop_step returns HOP_ERR_ARENA_TOO_SMALL for a schedule without workspace.  Binding
 * again (other memory) is allowed between passes; the descriptors are then laid out anew. */
size_t hop_schedule_bytes(const hop_schedule* s);
int hop_schedule_bind(hop_ctx* ctx, hop_schedule* s, void* workspace, size_t bytes);

/* Enqueues waves [wave_begin, wave_end) of the schedule: per wave the gradient kernels of its STEP
 * records (Compute on x_k, Section 3.2), then one fused Reduce + Apply launch over all its records.
 * Variations by gradient source: with CSR data, and with dense minibatches of up to 2 MB per record, the
 * margins ride in the Reduce launch and the gradient is applied to the results right after it (scattered,
 * or in place); with larger dense minibatches the gradient kernel itself reduces and applies its record,
 * and the Reduce launch only holds the records without a gradient; synthetic gradients of up to
 * hop_opts.grad_ahead consecutive waves are generated in front of the first of them.  The results are the
 * same in every arrangement up to the rounding of the sums.  The first call for a schedule (and the first after the gradient
 * source or a data set changed) copies the descriptors into the schedule's workspace with synchronous
 * host-to-device copies; after that the call only launches.  Records of one wave touch no
 * ring slot in a conflicting way, so the result equals running the records one by one in schedule
 * order.  Waves must be run in order starting from 0 after hop_set_params (or continue where the last
 * call stopped); wave_end = -1 means "to the end".  A finished schedule may be started again from
 * wave 0 without resetting parameters (it then continues from whatever the rings hold). */
int hop_step(hop_ctx* ctx, const hop_schedule* s, int32_t wave_begin, int32_t wave_end);

/* With enable != 0, a hop_step call that covers the whole schedule (wave_begin 0, wave_end -1 or
 * n_waves) and is not being profiled records its launches once into a HIP graph and replays that
 * graph from then on: one launch call per pass instead of up to four per wave, which is what
 * matters for schedules of many small waves (Exp(1) delays de-synchronise the workers).  Partial
 * ranges and profiled passes always run kernel by kernel.  Off by default. */
int hop_use_graph(hop_ctx* ctx, int enable);

/* Newest parameter vector of a worker (device, d floats) and its iteration number. */
int hop_params(hop_ctx* ctx, int32_t worker, const float** dev_ptr, int32_t* iter);
/* Address of one ring slot (device, d floats). */
int hop_slot(hop_ctx* ctx, int32_t worker, int32_t slot, float** dev_ptr);
/* Loss coefficients c_m of a STEP record (hinge: y_m / B where active, else 0; log loss: see
 * hop_svm_grad_dense) as the gradient kernel computed them (device, batch floats); valid after that
 * record's wave has run and until the schedule is freed or its descriptors are rebuilt. */
int hop_coef(hop_ctx* ctx, const hop_schedule* s, int32_t record, const float** dev_ptr);

/* Per-kernel timing with HIP events on the context's stream.  hop_profile_read synchronises the
 * stream and returns, for launches since the last read: total milliseconds, number of launches and
 * the algorithmic bytes those launches had to move (for HOP_KERNEL_MIX: 4 d (A + 2) per STEP,
 * 4 d (A + 1) per JUMP or gradient-free STEP, 8 d more where a velocity is read and written). */
int hop_profile(hop_ctx* ctx, int enable);
int hop_profile_read(hop_ctx* ctx, int kernel, double* ms, int64_t* launches, double* bytes);

/* Stand-alone kernels on caller-supplied device memory (same code the schedule runs).  Unlike
 * hop_step these calls are synchronous: they upload a small descriptor (hipMalloc / hipFree inside),
 * launch on the given stream and wait for it.  All vectors must be 16-byte aligned (when d is a
 * multiple of 4 this includes every row of X); a misaligned or NULL pointer, A outside 1..HOP_MAX_A
 * or B outside 1..1024 gives HOP_ERR_INVALID_ARG and nothing is launched.  The contents of device
 * index arrays (sample ids in rows_dev, CSR row pointers and column ids) are NOT checked here: the
 * caller guarantees ids in range, as hop_set_data_csr does for a context's data. */
/* Fused Reduce + Apply for n_jobs independent jobs (host array), each over d columns. */
int hop_mix(const hop_mix_job* jobs, int32_t n_jobs, int64_t d, void* hip_stream);
/* Linear-SVM minibatch (sub)gradient g = lambda w - sum_m c_m x_{r_m}; hinge: c_m = y/B if
 * y <x, w> < 1 else 0; log loss: c_m = y / (B (1 + exp(y <x, w>))).  rows_dev holds B sample ids
 * (device int32).  coef (device, B floats) receives c_m.  scratch: device,
 * hop_grad_scratch_floats(d, B) floats. */
int64_t hop_grad_scratch_floats(int64_t d, int32_t B);
int hop_svm_grad_dense(const float* X, const float* y, const float* w, const int32_t* rows_dev,
                       int32_t B, int64_t d, float lambda, int32_t loss, float* g, float* coef,
                       float* scratch, void* hip_stream);
/* The same gradient for callers that cannot allocate device memory - a stream under graph capture, a tight
 * serving loop, a harness that forbids hipMalloc.  Same arguments and results as hop_svm_grad_dense without
 * the scratch argument: the descriptor and the partial dot products live in a fixed array of device memory
 * inside the library (256 KB + 256 B per GPU, held until the process ends), and the call only enqueues three
 * kernels on the stream and returns (no allocation, no copy, no wait: the caller synchronises).  Limit:
 * B x ceil(d / 16384) <= 65536, else HOP_ERR_ARENA_TOO_SMALL and nothing is launched.  All calls on one GPU
 * share that array: calls whose kernels could overlap (different streams, or a captured graph replayed
 * beside another call) race and must be ordered by the caller.  Nothing in the array needs clearing between
 * calls: every partial sum a call reads was written by the same call. */
int hop_svm_grad_dense_static(const float* X, const float* y, const float* w, const int32_t* rows_dev,
                              int32_t B, int64_t d, float lambda, int32_t loss, float* g, float* coef,
                              void* hip_stream);
/* Same on CSR features; g (device, d floats) receives the dense gradient. */
int hop_svm_grad_csr(const int64_t* rowptr, const int32_t* col, const float* val, const float* y,
                     const float* w, const int32_t* rows_dev, int32_t B, int64_t d, float lambda,
                     int32_t loss, float* g, float* coef, void* hip_stream);
/* Synthetic gradient of (seed, worker, iteration): centred sum of 12 pairwise independent hashed bytes per element times
 * sqrt(variance / 65535). */
int hop_synth_grad(uint64_t seed, int32_t worker, int32_t iter, float variance, float* g, int64_t d,
                   void* hip_stream);
/* Plain device-to-device copy kernel (bytes multiple of 16); used to calibrate traffic counters. */
int hop_copy(void* dst, const void* src, size_t bytes, void* hip_stream);
/* Copies bytes from device memory (for instance a pointer handed out by hop_coef) to host memory
 * and waits for the stream. */
int hop_download(void* host_dst, const void* dev_src, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* HOP_H */
