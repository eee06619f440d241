// Drives the library's host simulator (hop_sim.cpp alone, no HIP) over a grid of graphs and modes.
// Built by tests/test_host_sanitizers.py with AddressSanitizer and UBSan; prints one line per run.
#include <cstdio>
#include <cstdlib>
#include <set>
#include <vector>

#include "hop_internal.h"

int hopk_dense_nseg(int64_t) { return 1; }   // the only kernel-side symbol the simulator's header names

static std::vector<std::vector<int>> ring(int n) {
    std::vector<std::vector<int>> nb(n);
    for (int i = 0; i < n; ++i) {
        std::set<int> s{(i + n - 1) % n, (i + 1) % n};
        s.erase(i);
        nb[i].assign(s.begin(), s.end());
    }
    return nb;
}
static std::vector<std::vector<int>> complete(int n) {
    std::vector<std::vector<int>> nb(n);
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            if (j != i) nb[i].push_back(j);
    return nb;
}
static std::vector<std::vector<int>> torus(int r, int c) {
    std::vector<std::vector<int>> nb(r * c);
    for (int a = 0; a < r; ++a)
        for (int b = 0; b < c; ++b) {
            std::set<int> s{((a + r - 1) % r) * c + b, ((a + 1) % r) * c + b, a * c + (b + c - 1) % c,
                            a * c + (b + 1) % c};
            s.erase(a * c + b);
            nb[a * c + b].assign(s.begin(), s.end());
        }
    return nb;
}

int main() {
    std::vector<std::vector<std::vector<int>>> graphs{ring(2), ring(5), complete(4), torus(3, 3), ring(1)};
    long total = 0;
    int runs = 0;
    for (size_t gi = 0; gi < graphs.size(); ++gi)
        for (int s : {0, 1, 3})
            for (int b : {0, 1})
                for (int skip : {0, 1})
                    for (uint32_t lat : {0u, 1u << 20})
                      for (int option : {0, 1, 2})                // 0 token queues, 1 serial approach, 2 NOTIFY-ACK
                        for (int kind : {HOP_DELAY_NONE, HOP_DELAY_EXP1, HOP_DELAY_BERNOULLI6}) {
                            if (option == 2 && (s != 0 || b != 0 || skip || lat > 1)) continue;
                            const auto& nb = graphs[gi];
                            const int N = (int)nb.size();
                            int mindeg = N;
                            for (const auto& l : nb) mindeg = std::min<int>(mindeg, (int)l.size());
                            if (b > 0 && b >= mindeg) continue;
                            hop_ctx c;
                            c.N = N; c.s = s; c.b = b; c.d = 8;
                            hop_opts_default(&c.opts);
                            c.opts.skip_on = skip;
                            c.opts.seed = 17 * gi + s;
                            c.opts.batch = 4;
                            c.opts.max_latency = lat;
                            c.opts.serial = option == 1;
                            c.opts.notify_ack = option == 2;
                            c.max_ig = option == 2 ? 2 : (s > 0 ? s : 1);
                            c.D = s >= 1 ? (lat > 1 ? s + c.max_ig + 2 : c.max_ig + 1) : c.max_ig + 2;
                            c.slots = c.D + (option == 1 ? 1 : 0);
                            c.in_nbrs = nb;
                            c.out_nbrs.assign(N, {});
                            for (int i = 0; i < N; ++i)
                                for (int j : nb[i]) c.out_nbrs[j].push_back(i);
                            c.W.assign((size_t)N * N, 0.f);
                            for (int i = 0; i < N; ++i) {
                                float w = 1.0f / (float)(nb[i].size() + 1);
                                c.W[(size_t)i * N + i] = w;
                                for (int j : nb[i]) c.W[(size_t)j * N + i] = w;
                            }
                            c.data.assign(N, HopData{});
                            for (int i = 0; i < N; ++i) c.data[i].rows = 31 + i;
                            std::vector<double> mult(N, 1.0);
                            if (N > 2) mult[1] = (gi % 2) ? 3.0 : (double)HOP_TICKS_NEVER;
                            hop_delay_model dm{kind, 0, mult.data(), nullptr};
                            hop_schedule sched;
                            int rc = hop_run_protocol(&c, &dm, 12, &sched);
                            if (rc != HOP_OK && rc != HOP_ERR_DEADLOCK) {
                                std::printf("FAIL rc=%d graph=%zu s=%d b=%d\n", rc, gi, s, b);
                                return 1;
                            }
                            total += (long)sched.kind.size() + sched.n_waves;
                            ++runs;
                        }
    std::printf("ok runs=%d records+waves=%ld\n", runs, total);
    return 0;
}

// hop_opts_default lives in hop_api.cpp, which needs HIP; a local copy of its few lines keeps this
// driver free of the GPU runtime.
extern "C" int hop_opts_default(hop_opts* o) {
    *o = hop_opts{};
    o->max_skip = 10;
    o->trigger = 1;
    o->lr = 0.01f;
    o->lambda = 1e-4f;
    return 0;
}
