// Walk through the device paths of the C ABI on a real GPU with the HOST code under AddressSanitizer
// (kernels are the product's): contexts on a hipMalloc'ed arena, every gradient source, momentum,
// partial wave ranges, profiling, graph replay, re-simulation, data swaps, frees in awkward orders.
// Checks results only for finiteness and two invariants; element-wise parity is the Python tests' job.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <random>
#include <vector>

#include "hop.h"

#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            std::printf("FAIL line %d: %s\n", __LINE__, #cond);             \
            std::fflush(stdout);                                            \
            return 1;                                                       \
        }                                                                   \
    } while (0)
#define HIP_OK(call) EXPECT((call) == hipSuccess)

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
        int a = (i + n - 1) % n, b = (i + 1) % n;
        if (a > b) std::swap(a, b);
        g.col.push_back(a);
        g.col.push_back(b);
        g.row_ptr.push_back((int32_t)g.col.size());
    }
    g.W.assign((size_t)n * n, 0.f);
    for (int i = 0; i < n; ++i) {
        g.W[(size_t)i * n + i] = 1.0f / 3.0f;
        for (int p = g.row_ptr[i]; p < g.row_ptr[i + 1]; ++p) g.W[(size_t)g.col[p] * n + i] = 1.0f / 3.0f;
    }
    return g;
}

template <class T>
static T* to_device(const std::vector<T>& v) {
    T* p = nullptr;
    if (hipMalloc((void**)&p, v.size() * sizeof(T)) != hipSuccess) return nullptr;
    if (hipMemcpy(p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return nullptr;
    return p;
}

static bool all_finite(hop_ctx* c, int N, int64_t d, std::vector<float>* last) {
    std::vector<float> h((size_t)d);
    for (int i = 0; i < N; ++i) {
        const float* p = nullptr;
        int32_t it = 0;
        if (hop_params(c, i, &p, &it) != HOP_OK) return false;
        if (hop_download(h.data(), p, (size_t)d * 4, nullptr) != HOP_OK) return false;
        for (float v : h)
            if (!std::isfinite(v)) return false;
    }
    if (last) *last = h;
    return true;
}

int main() {
    const int N = 6, B = 8, rows = 50, nnz = 5;
    std::mt19937 gen(7);
    std::normal_distribution<float> nd(0.f, 1.f);
    Graph g = ring(N);
    hop_graph hg{N, g.row_ptr.data(), g.col.data()};
    for (int64_t d : {(int64_t)1003, (int64_t)4096}) {
        for (float momentum : {0.0f, 0.9f}) {
            hop_opts o;
            hop_opts_default(&o);
            o.batch = B;
            o.skip_on = 1;
            o.seed = 11;
            o.momentum = momentum;
            o.grad_ahead = d == 4096 ? 3 : 1;      // synthetic gradients three waves ahead on one of the sizes
            o.lr = 0.05f;
            const int s = 2, b = 1;
            size_t need = hop_arena_bytes(N, d, s, b, &o);
            EXPECT(need > 0);
            void* arena = nullptr;
            HIP_OK(hipMalloc(&arena, need));
            HIP_OK(hipMemset(arena, 0, need));
            hop_device dev{arena, need, nullptr};
            hop_ctx* c = nullptr;
            hop_device small = dev;
            small.arena_bytes = need - 4;
            EXPECT(hop_init(&c, &hg, g.W.data(), N, d, s, b, &o, &small) == HOP_ERR_ARENA_TOO_SMALL);
            EXPECT(hop_init(&c, &hg, g.W.data(), N, d, s, b, &o, &dev) == HOP_OK);
            std::printf("ctx d=%lld momentum=%.1f\n", (long long)d, momentum);
            std::fflush(stdout);
            std::vector<float> p0((size_t)d);
            for (auto& v : p0) v = 0.1f * nd(gen);
            EXPECT(hop_set_params(c, p0.data(), 0, 0) == HOP_OK);
            // data sets: dense rows and CSR rows per worker
            std::vector<float*> Xs, ys, vals;
            std::vector<int64_t*> rps;
            std::vector<int32_t*> cols;
            for (int i = 0; i < N; ++i) {
                std::vector<float> X((size_t)rows * d), y((size_t)rows);
                for (auto& v : X) v = nd(gen);
                for (auto& v : y) v = nd(gen) > 0 ? 1.f : -1.f;
                Xs.push_back(to_device(X));
                ys.push_back(to_device(y));
                std::vector<int64_t> rp((size_t)rows + 1);
                std::vector<int32_t> col((size_t)rows * nnz);
                std::vector<float> val((size_t)rows * nnz);
                for (int r = 0; r <= rows; ++r) rp[r] = (int64_t)r * nnz;
                for (int r = 0; r < rows; ++r)
                    for (int q = 0; q < nnz; ++q) {
                        col[(size_t)r * nnz + q] = (int32_t)((q * (d / nnz) + (r * 7) % (d / nnz)));
                        val[(size_t)r * nnz + q] = nd(gen);
                    }
                rps.push_back(to_device(rp));
                cols.push_back(to_device(col));
                vals.push_back(to_device(val));
                EXPECT(Xs.back() && ys.back() && rps.back() && cols.back() && vals.back());
            }
            std::vector<float> ext((size_t)N * d);
            for (auto& v : ext) v = 0.01f * nd(gen);
            float* ext_dev = nullptr;
            if (d % 4 == 0) ext_dev = to_device(ext);

            std::vector<double> mult(N, 1.0);
            mult[2] = 3.0;
            hop_delay_model dm{HOP_DELAY_EXP1, 0, mult.data(), nullptr};
            hop_schedule* sched = nullptr;
            for (int i = 0; i < N; ++i) EXPECT(hop_set_rows(c, i, rows) == HOP_OK);
            EXPECT(hop_simulate(c, &dm, 12, &sched) == HOP_OK);
            hop_schedule_arrays v;
            EXPECT(hop_schedule_view(sched, &v) == HOP_OK && v.n_waves > 0);
            // the descriptors of a schedule live in memory the caller lends
            EXPECT(hop_step(c, sched, 0, -1) == HOP_ERR_ARENA_TOO_SMALL);
            const size_t ws_bytes = hop_schedule_bytes(sched);
            void* ws = nullptr;
            EXPECT(ws_bytes > 0);
            HIP_OK(hipMalloc(&ws, ws_bytes));
            EXPECT(hop_schedule_bind(c, sched, ws, ws_bytes - 1) == HOP_ERR_ARENA_TOO_SMALL);
            EXPECT(hop_schedule_bind(c, sched, (char*)ws + 16, ws_bytes) == HOP_ERR_INVALID_ARG);
            EXPECT(hop_schedule_bind(c, sched, ws, ws_bytes) == HOP_OK);

            for (int mode : {HOP_GRAD_ZERO, HOP_GRAD_SYNTH, HOP_GRAD_SVM_DENSE, HOP_GRAD_SVM_CSR, HOP_GRAD_EXTERNAL}) {
                if (mode == HOP_GRAD_EXTERNAL && !ext_dev) continue;
                if (mode == HOP_GRAD_SVM_DENSE)
                    for (int i = 0; i < N; ++i) EXPECT(hop_set_data_dense(c, i, Xs[i], ys[i], rows) == HOP_OK);
                if (mode == HOP_GRAD_SVM_CSR)
                    for (int i = 0; i < N; ++i)
                        EXPECT(hop_set_data_csr(c, i, rps[i], cols[i], vals[i], ys[i], rows) == HOP_OK);
                EXPECT(hop_set_grad_source(c, mode, 1e-3f, ext_dev) == HOP_OK);
                EXPECT(hop_set_params(c, p0.data(), 0, 0) == HOP_OK);
                std::printf("  mode %d\n", mode);
                std::fflush(stdout);
                // whole pass, then wave by wave, then profiled, then graph replays
                EXPECT(hop_step(c, sched, 0, -1) == HOP_OK);
                HIP_OK(hipDeviceSynchronize());
                std::vector<float> first;
                EXPECT(all_finite(c, N, d, &first));
                EXPECT(hop_set_params(c, p0.data(), 0, 0) == HOP_OK);
                EXPECT(hop_step(c, sched, 1, 2) == HOP_ERR_STATE);          // out of sequence
                for (int w = 0; w < v.n_waves; ++w) EXPECT(hop_step(c, sched, w, w + 1) == HOP_OK);
                HIP_OK(hipDeviceSynchronize());
                std::vector<float> second;
                EXPECT(all_finite(c, N, d, &second));
                if (mode != HOP_GRAD_SVM_CSR) EXPECT(first == second);      // atomics: CSR only to rounding
                EXPECT(hop_profile(c, 1) == HOP_OK);
                EXPECT(hop_set_params(c, p0.data(), 0, 0) == HOP_OK);
                EXPECT(hop_step(c, sched, 0, -1) == HOP_OK);
                double ms = 0, bytes = 0;
                int64_t launches = 0;
                EXPECT(hop_profile_read(c, HOP_KERNEL_MIX, &ms, &launches, &bytes) == HOP_OK);
                if (mode != HOP_GRAD_SVM_DENSE) {          // dense: the Reduce rides in the gradient launches
                    EXPECT(launches == v.n_waves);
                } else {
                    int64_t grad_launches = 0;
                    EXPECT(hop_profile_read(c, HOP_KERNEL_GRAD, &ms, &grad_launches, &bytes) == HOP_OK);
                    EXPECT(launches + grad_launches == v.n_waves);
                }
                EXPECT(hop_profile(c, 0) == HOP_OK);
                EXPECT(hop_use_graph(c, 1) == HOP_OK);
                for (int rep = 0; rep < 3; ++rep) {
                    EXPECT(hop_set_params(c, p0.data(), 0, 0) == HOP_OK);
                    EXPECT(hop_step(c, sched, 0, -1) == HOP_OK);
                    HIP_OK(hipDeviceSynchronize());
                    std::vector<float> third;
                    EXPECT(all_finite(c, N, d, &third));
                    if (mode != HOP_GRAD_SVM_CSR) EXPECT(first == third);
                }
                EXPECT(hop_use_graph(c, 0) == HOP_OK);
                if (mode == HOP_GRAD_SVM_DENSE || mode == HOP_GRAD_SVM_CSR) {
                    const float* coef = nullptr;
                    EXPECT(hop_coef(c, sched, 0, &coef) == HOP_OK && coef != nullptr);
                    std::vector<float> hc(B);
                    EXPECT(hop_download(hc.data(), coef, B * 4, nullptr) == HOP_OK);
                    EXPECT(hop_coef(c, sched, v.n_records, &coef) == HOP_ERR_INVALID_ARG);
                }
            }
            // a data set of another size after the simulation must be refused, not indexed
            EXPECT(hop_set_data_dense(c, 0, Xs[0], ys[0], rows - 1) == HOP_OK);
            EXPECT(hop_set_grad_source(c, HOP_GRAD_SVM_DENSE, 0.f, nullptr) == HOP_OK);
            EXPECT(hop_step(c, sched, 0, -1) == HOP_ERR_STATE);
            // a second schedule on the same context, identical replicas + zero gradient stay identical
            hop_schedule* again = nullptr;
            EXPECT(hop_simulate(c, nullptr, 5, &again) == HOP_OK);
            void* ws2 = nullptr;
            HIP_OK(hipMalloc(&ws2, hop_schedule_bytes(again)));
            EXPECT(hop_schedule_bind(c, again, ws2, hop_schedule_bytes(again)) == HOP_OK);
            EXPECT(hop_set_grad_source(c, HOP_GRAD_ZERO, 0.f, nullptr) == HOP_OK);
            EXPECT(hop_set_params(c, p0.data(), 0, 0) == HOP_OK);
            EXPECT(hop_step(c, again, 0, -1) == HOP_OK);
            HIP_OK(hipDeviceSynchronize());
            std::vector<float> fixed;
            EXPECT(all_finite(c, N, d, &fixed));
            for (int64_t k = 0; k < d; ++k) EXPECT(std::fabs(fixed[k] - p0[k]) <= 2e-6f * std::fabs(p0[k]) + 1e-12f);
            EXPECT(hop_schedule_free(sched) == HOP_OK);
            EXPECT(hop_destroy(c) == HOP_OK);
            EXPECT(hop_schedule_free(again) == HOP_OK);
            (void)hipFree(ws);
            (void)hipFree(ws2);
            for (int i = 0; i < N; ++i) {
                (void)hipFree(Xs[i]); (void)hipFree(ys[i]); (void)hipFree(rps[i]); (void)hipFree(cols[i]); (void)hipFree(vals[i]);
            }
            if (ext_dev) (void)hipFree(ext_dev);
            HIP_OK(hipFree(arena));
        }
    }
    std::printf("ok\n");
    return 0;
}
