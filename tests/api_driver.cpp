// Host-only walk through the C ABI for the sanitizer build (no GPU, no kernels): argument checking,
// schedule views read to their full lengths, object lifetimes in awkward orders.
#include <cstdio>
#include <cstring>
#include <vector>

#include "hop_internal.h"

// The kernel launchers live in the HIP translation unit; a context without device memory never
// reaches them, so the sanitizer build only needs the symbols.
int hopk_mix(const HopMixJob*, int, int64_t, void*) { return 1; }
int hopk_synth(const HopGradJob*, int, int, int64_t, void*) { return 1; }
int hopk_dense_margin(const HopGradJob*, int, int, int64_t, void*) { return 1; }
int hopk_dense_grad(const HopGradJob*, int, int, int64_t, float, int, void*) { return 1; }
int hopk_csr_margin(const HopGradJob*, int, int, int, void*) { return 1; }
int hopk_mix_dense_margin(const HopMixJob*, int, int64_t, const HopGradJob*, int, int, void*) { return 1; }
int hopk_mix_csr_margin(const HopMixJob*, int, int64_t, const HopGradJob*, int, int, int, void*) { return 1; }
int hopk_pair(const HopPairJob*, int, int, int, int64_t, void*) { return 1; }
int hopk_pair_csr_margin(const HopPairJob*, int, int, int, int64_t, const HopGradJob*, int, int, int, void*) { return 1; }
int hopk_pair_dense_margin(const HopPairJob*, int, int, int, int64_t, const HopGradJob*, int, int, void*) { return 1; }
int hopk_csr_scatter(const HopGradJob*, int, int, float, int, void*) { return 1; }
int hopk_csr_dense_grad(const HopGradJob*, int, int, int64_t, float, void*) { return 1; }
int hopk_csr_check(const int64_t*, const int32_t*, int64_t, int64_t, int64_t, int64_t, int*, void*) { return 1; }
int hopk_copy(void*, const void*, size_t, void*) { return 1; }
int hopk_dense_nseg(int64_t d) { return (int)((d + 16383) / 16384); }

#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            std::printf("FAIL line %d: %s\n", __LINE__, #cond);             \
            return 1;                                                       \
        }                                                                   \
    } while (0)

struct Graph {
    std::vector<int32_t> row_ptr, col;
    std::vector<float> W;
    int N;
};

static Graph ring(int n) {
    Graph g;
    g.N = n;
    g.row_ptr.push_back(0);
    for (int i = 0; i < n; ++i) {
        std::vector<int> nb;
        if (n > 1) nb.push_back((i + n - 1) % n);
        if (n > 2) nb.push_back((i + 1) % n);
        if (nb.size() == 2 && nb[0] > nb[1]) std::swap(nb[0], nb[1]);
        for (int j : nb) g.col.push_back(j);
        g.row_ptr.push_back((int32_t)g.col.size());
    }
    g.W.assign((size_t)n * n, 0.f);
    for (int i = 0; i < n; ++i) {
        int deg = g.row_ptr[i + 1] - g.row_ptr[i];
        g.W[(size_t)i * n + i] = 1.0f / (float)(deg + 1);
        for (int p = g.row_ptr[i]; p < g.row_ptr[i + 1]; ++p) g.W[(size_t)g.col[p] * n + i] = 1.0f / (float)(deg + 1);
    }
    return g;
}

static long touch(const hop_schedule_arrays& v) {
    long sum = 0;
    for (int e = 0; e < v.n_records; ++e) {
        sum += v.kind[e] + v.worker[e] + v.iter[e] + v.wave[e] + v.out_slot[e] + (long)(v.time[e] & 1);
        for (int a = v.src_begin[e]; a < v.src_begin[e + 1]; ++a)
            sum += v.src_worker[a] + v.src_tag[a] + v.src_slot[a] + (v.src_weight[a] > 0.f);
        if (v.batch_rows)
            for (int m = 0; m < v.batch; ++m) sum += v.batch_rows[(size_t)e * v.batch + m];
    }
    sum += v.src_begin[v.n_records] == v.n_sources;
    for (int i = 0; i < v.n_workers; ++i) sum += v.final_iter[i] + (long)(v.finish_time[i] & 1);
    for (int w = 0; w < v.n_waves; ++w)
        for (int p = v.wave_begin[w]; p < v.wave_begin[w + 1]; ++p) sum += v.wave_order[p];
    return sum;
}

// Pairing of a wave's Reduce jobs: every record once, unions within the kernel's limit, weights and sources kept.
static int test_pack_pairs() {
    std::vector<float> pool(64);
    unsigned z = 12345;
    auto rnd = [&z](int n) { z = z * 1664525u + 1013904223u; return (int)((z >> 8) % (unsigned)n); };
    for (int trial = 0; trial < 200; ++trial) {
        const int n = 1 + rnd(40), n_src = 2 + rnd(40), max_a = 1 + rnd(trial % 7 == 0 ? HOP_MAX_A : 9);
        std::vector<HopMixJob> jobs((size_t)n);
        std::vector<float> outs((size_t)n);
        size_t reads = 0;
        std::vector<char> seen((size_t)n_src, 0);
        for (int i = 0; i < n; ++i) {
            HopMixJob& j = jobs[(size_t)i];
            std::memset(&j, 0, sizeof(j));
            j.out = &outs[(size_t)i];
            j.eta = 0.5f;
            j.g = rnd(3) ? &pool[0] : nullptr;
            j.A = 1 + rnd(max_a);
            for (int a = 0; a < j.A; ++a) {
                const int sidx = rnd(n_src);                        // duplicates inside one record may happen
                j.src[a] = &pool[(size_t)sidx];
                j.w[a] = 0.125f * (float)(1 + rnd(8));
                seen[(size_t)sidx] = 1;
            }
            reads += (size_t)j.A;
        }
        int distinct = 0;
        for (char c : seen) distinct += c;
        std::vector<HopPairJob> out;
        EXPECT(hop_pack_pairs(jobs.data(), n, out) == distinct);
        std::vector<int> times((size_t)n, 0);
        bool any_pair = false;
        for (const HopPairJob& pj : out) {
            EXPECT(pj.G == 1 || pj.G == 2);
            EXPECT(pj.U >= 1 && pj.U <= HOP_MAX_A && (pj.G == 1 || pj.U <= HOP_PAIR_U));
            any_pair = any_pair || pj.G == 2;
            for (int r = 0; r < pj.G; ++r) {
                const int i = (int)(pj.out[r] - outs.data());
                EXPECT(i >= 0 && i < n);
                ++times[(size_t)i];
                const HopMixJob& j = jobs[(size_t)i];
                EXPECT(pj.g[r] == j.g && pj.eta == j.eta);
                // per distinct vector: what the pair holds for this record (entries switched on) adds up to the
                // record's own weights on it (a record may list a vector twice), and nothing else is switched on
                for (size_t v = 0; v < pool.size(); ++v) {
                    float have = 0.f, want = 0.f;
                    for (int u = 0; u < pj.U; ++u)
                        if (pj.src[u] == &pool[v] && (u >= 32 || ((pj.mask[r] >> u) & 1u))) have += pj.w[r][u];
                    for (int a = 0; a < j.A; ++a)
                        if (j.src[a] == &pool[v]) want += j.w[a];
                    EXPECT(have == want);
                }
            }
        }
        for (int t : times) EXPECT(t == 1);
        if (reads < 2 * (size_t)distinct) EXPECT(!any_pair);      // records that share little stay single
    }
    return 0;
}

int main() {
    if (test_pack_pairs() != 0) return 1;
    hop_opts o;
    EXPECT(hop_opts_default(&o) == HOP_OK && hop_opts_default(nullptr) == HOP_ERR_INVALID_ARG);
    EXPECT(std::strcmp(hop_strerror(HOP_ERR_DEADLOCK), "unknown error") != 0 && hop_strerror(-99) != nullptr);
    long total = 0;
    for (int n : {1, 2, 3, 6}) {
        Graph g = ring(n);
        hop_graph hg{n, g.row_ptr.data(), g.col.data()};
        hop_ctx* c = nullptr;
        // invalid arguments
        EXPECT(hop_init(nullptr, &hg, g.W.data(), n, 8, 1, 0, &o, nullptr) == HOP_ERR_INVALID_ARG);
        EXPECT(hop_init(&c, nullptr, g.W.data(), n, 8, 1, 0, &o, nullptr) == HOP_ERR_INVALID_ARG && c == nullptr);
        EXPECT(hop_init(&c, &hg, nullptr, n, 8, 1, 0, &o, nullptr) == HOP_ERR_INVALID_ARG);
        EXPECT(hop_init(&c, &hg, g.W.data(), n, 0, 1, 0, &o, nullptr) == HOP_ERR_INVALID_ARG);
        EXPECT(hop_init(&c, &hg, g.W.data(), n + 1, 8, 1, 0, &o, nullptr) == HOP_ERR_INVALID_ARG);
        EXPECT(hop_init(&c, &hg, g.W.data(), n, 8, -1, 0, &o, nullptr) == HOP_ERR_INVALID_ARG);
        hop_opts bad = o;
        bad.momentum = 1.0f;
        EXPECT(hop_init(&c, &hg, g.W.data(), n, 8, 1, 0, &bad, nullptr) == HOP_ERR_INVALID_ARG);
        bad = o;
        bad.batch = 5000;
        EXPECT(hop_init(&c, &hg, g.W.data(), n, 8, 1, 0, &bad, nullptr) == HOP_ERR_INVALID_ARG);
        if (n >= 3) {
            EXPECT(hop_init(&c, &hg, g.W.data(), n, 8, 1, 2, &o, nullptr) == HOP_ERR_BAD_BACKUP);
            std::vector<int32_t> col = g.col;
            col[0] = 0;                                  // self edge at node 0
            hop_graph hb{n, g.row_ptr.data(), col.data()};
            EXPECT(hop_init(&c, &hb, g.W.data(), n, 8, 1, 0, &o, nullptr) == HOP_ERR_BAD_GRAPH);
            col = g.col;
            col[1] = n + 3;                              // out of range
            EXPECT(hop_init(&c, &hb, g.W.data(), n, 8, 1, 0, &o, nullptr) == HOP_ERR_BAD_GRAPH);
            std::vector<int32_t> rp = g.row_ptr;
            rp[1] = rp[2] + 1;                           // decreasing row pointer
            hop_graph hr{n, rp.data(), g.col.data()};
            EXPECT(hop_init(&c, &hr, g.W.data(), n, 8, 1, 0, &o, nullptr) == HOP_ERR_BAD_GRAPH);
            std::vector<float> W = g.W;
            W[1] = -0.1f;
            EXPECT(hop_init(&c, &hg, W.data(), n, 8, 1, 0, &o, nullptr) == HOP_ERR_BAD_WEIGHTS);
        }
        // a working host-only context
        o.batch = 3;
        o.skip_on = 1;
        EXPECT(hop_init(&c, &hg, g.W.data(), n, 8, 2, 0, &o, nullptr) == HOP_OK && c != nullptr);
        for (int i = 0; i < n; ++i) EXPECT(hop_set_rows(c, i, 11 + i) == HOP_OK);
        EXPECT(hop_set_rows(c, n, 1) == HOP_ERR_INVALID_ARG && hop_set_rows(c, 0, -1) == HOP_ERR_INVALID_ARG);
        float dummy[4] = {0, 0, 0, 0};
        EXPECT(hop_set_params(c, dummy, 0, 0) == HOP_ERR_NO_DEVICE);
        EXPECT(hop_set_data_dense(c, 0, dummy, dummy, 1) == HOP_ERR_NO_DEVICE);
        EXPECT(hop_set_grad_source(c, 99, 0.f, nullptr) == HOP_ERR_INVALID_ARG);
        EXPECT(hop_set_grad_source(c, HOP_GRAD_EXTERNAL, 0.f, nullptr) == HOP_ERR_INVALID_ARG);
        EXPECT(hop_set_grad_source(c, HOP_GRAD_SYNTH, -1.f, nullptr) == HOP_ERR_INVALID_ARG);
        hop_schedule* s1 = nullptr;
        hop_schedule* s2 = nullptr;
        hop_schedule* s3 = nullptr;
        EXPECT(hop_simulate(c, nullptr, -1, &s1) == HOP_ERR_INVALID_ARG && s1 == nullptr);
        EXPECT(hop_simulate(c, nullptr, 9, nullptr) == HOP_ERR_INVALID_ARG);
        hop_delay_model dm{HOP_DELAY_TABLE, 3, nullptr, nullptr};
        EXPECT(hop_simulate(c, &dm, 9, &s1) == HOP_ERR_INVALID_ARG);
        dm.kind = 17;
        EXPECT(hop_simulate(c, &dm, 9, &s1) == HOP_ERR_INVALID_ARG);
        EXPECT(hop_simulate(c, nullptr, 9, &s1) == HOP_OK && s1 != nullptr);
        std::vector<double> mult((size_t)n, 1.0);
        mult[0] = 3.0;
        hop_delay_model exp1{HOP_DELAY_EXP1, 0, mult.data(), nullptr};
        EXPECT(hop_simulate(c, &exp1, 12, &s2) == HOP_OK);
        EXPECT(hop_simulate(c, &exp1, 0, &s3) == HOP_OK);
        hop_schedule_arrays v;
        EXPECT(hop_schedule_view(s1, &v) == HOP_OK && v.n_records >= n * 9 - 0 * n && v.n_workers == n);
        total += touch(v);
        EXPECT(hop_schedule_view(s2, &v) == HOP_OK);
        total += touch(v);
        EXPECT(hop_schedule_view(s3, &v) == HOP_OK && v.n_records == 0 && v.n_waves == 0);
        total += touch(v);
        EXPECT(hop_schedule_view(nullptr, &v) == HOP_ERR_INVALID_ARG && hop_schedule_view(s1, nullptr) == HOP_ERR_INVALID_ARG);
        EXPECT(hop_step(c, s1, 0, -1) == HOP_ERR_NO_DEVICE);
        EXPECT(hop_schedule_bytes(nullptr) == 0 && hop_schedule_bytes(s1) > 0);
        EXPECT(hop_schedule_bytes(s3) >= 256);                       // an empty schedule still has a size
        alignas(256) static char fake[256];
        EXPECT(hop_schedule_bind(c, s1, nullptr, 1 << 20) == HOP_ERR_INVALID_ARG);
        EXPECT(hop_schedule_bind(c, s1, fake, 1 << 20) == HOP_ERR_NO_DEVICE);
        EXPECT(hop_schedule_bind(nullptr, s1, fake, 1 << 20) == HOP_ERR_INVALID_ARG);
        const float* p = nullptr;
        int32_t it = 0;
        EXPECT(hop_params(c, 0, &p, &it) == HOP_ERR_NO_DEVICE && hop_params(c, -1, &p, &it) == HOP_ERR_INVALID_ARG);
        EXPECT(hop_use_graph(c, 1) == HOP_ERR_NO_DEVICE && hop_profile(c, 1) == HOP_ERR_NO_DEVICE);
        if (n >= 2) {                                   // a frozen worker: the stall is reported, the schedule returned
            std::vector<uint64_t> table((size_t)n * 5, 1u << 20);
            for (int k = 0; k < 5; ++k) table[k] = HOP_TICKS_NEVER;
            hop_delay_model frozen{HOP_DELAY_TABLE, 5, nullptr, table.data()};
            hop_schedule* s4 = nullptr;
            EXPECT(hop_simulate(c, &frozen, 5, &s4) == HOP_ERR_DEADLOCK && s4 != nullptr);
            EXPECT(hop_schedule_view(s4, &v) == HOP_OK && v.stalled == 1);
            total += touch(v);
            EXPECT(hop_schedule_free(s4) == HOP_OK);
        }
        // lifetimes: free the middle schedule, destroy the context, then free what is left
        EXPECT(hop_schedule_free(s2) == HOP_OK);
        EXPECT(hop_destroy(c) == HOP_OK);
        EXPECT(hop_schedule_view(s1, &v) == HOP_OK);
        total += touch(v);
        EXPECT(hop_schedule_free(s1) == HOP_OK && hop_schedule_free(s3) == HOP_OK);
        EXPECT(hop_schedule_free(nullptr) == HOP_ERR_INVALID_ARG && hop_destroy(nullptr) == HOP_ERR_INVALID_ARG);
        o.batch = 0;
        o.skip_on = 0;
    }
    // layout queries and stand-alone entry points with arguments that must be refused before any launch
    int32_t depth = 0;
    int64_t stride = 0;
    EXPECT(hop_layout(100, 3, nullptr, &depth, &stride) == HOP_OK && depth == 4 && stride == 192);
    EXPECT(hop_layout(0, 3, nullptr, &depth, &stride) == HOP_ERR_INVALID_ARG);
    EXPECT(hop_arena_bytes(0, 8, 1, 0, nullptr) == 0 && hop_arena_bytes(4, 8, 1, 0, nullptr) > 0);
    EXPECT(hop_arena_bytes(4, 8, 1, -1, nullptr) == 0 && hop_arena_bytes(4, 8, 1, 1, nullptr) == hop_arena_bytes(4, 8, 1, 0, nullptr));
    EXPECT(hop_mix(nullptr, 1, 8, nullptr) == HOP_ERR_INVALID_ARG);
    hop_mix_job mj;
    std::memset(&mj, 0, sizeof(mj));
    mj.A = 40;
    EXPECT(hop_mix(&mj, 1, 8, nullptr) == HOP_ERR_INVALID_ARG);
    mj.A = 1;
    EXPECT(hop_mix(&mj, 1, 8, nullptr) == HOP_ERR_INVALID_ARG);      // null out
    EXPECT(hop_mix(&mj, 0, 8, nullptr) == HOP_OK);
    EXPECT(hop_svm_grad_dense(nullptr, nullptr, nullptr, nullptr, 1, 8, 0.f, 0, nullptr, nullptr, nullptr, nullptr) ==
           HOP_ERR_INVALID_ARG);
    EXPECT(hop_svm_grad_csr(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1, 8, 0.f, 0, nullptr, nullptr,
                            nullptr) == HOP_ERR_INVALID_ARG);
    EXPECT(hop_synth_grad(1, 0, 0, 1.f, nullptr, 8, nullptr) == HOP_ERR_INVALID_ARG);
    EXPECT(hop_copy(nullptr, nullptr, 16, nullptr) == HOP_ERR_INVALID_ARG);
    EXPECT(hop_download(nullptr, nullptr, 16, nullptr) == HOP_ERR_INVALID_ARG);
    EXPECT(hop_grad_scratch_floats(0, 1) == 0 && hop_grad_scratch_floats(100, 4) >= 4);
    std::printf("ok total=%ld\n", total);
    return 0;
}
