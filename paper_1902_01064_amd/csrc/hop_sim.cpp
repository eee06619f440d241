// Host discrete-event run of Hop's queue protocol -> schedule of STEP / JUMP records.
//
// Follows, in the paper's notation: Section 3.2 (parallel approach: Send x_k and Compute on
// x_k when iteration k is entered, then Recv, Reduce, Apply), Section 4.1 (update queues with
// (iter, w_id) tags), Section 4.2 (token queues, max_ig), Section 4.3 (backup workers N_buw),
// Section 4.4 (bounded staleness, newest update per in-neighbour, Eq. 2), Section 5 (skipping
// iterations), Section 6.1 (one queue per iteration: version v lives in ring slot v mod D) and
// Section 6.2 (a) (stale updates dropped at dequeue).
//
// Options beside the paper's own design: the serial approach of Section 3.2 (Compute and Apply on x_k, Send
// the result, then Recv and Reduce: two records per iteration, the current parameters in slot D of every
// worker) and NOTIFY-ACK of Section 3.3 (no token queues: Send(k) waits for every out-going neighbour's
// acknowledgement of update k - 1, which leaves right after the Reduce that consumed it; Recv and Reduce run
// beside Compute; standard training only).
//
// Time is integer ticks (2^20 per time unit); an update sent at T is visible at T + 1; Reduce,
// Apply, token moves and jumps take no time; simultaneous events run in the order
// (time, arrival before compute-done, worker, sender, tag).  All randomness is a pure function of
// (seed, stream, a, b, c) through a SplitMix64-style mixer, so nothing depends on event order.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <queue>

#include "hop_internal.h"

namespace hoprng {

static inline uint64_t sm64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint64_t mix(uint64_t seed, uint64_t stream, uint64_t a, uint64_t b, uint64_t c) {
    uint64_t h = sm64(seed);
    h = sm64(h ^ stream);
    h = sm64(h ^ a);
    h = sm64(h ^ b);
    h = sm64(h ^ c);
    return h;
}

void synth_keys(uint64_t seed, int worker, int iter, uint32_t* k0, uint32_t* k1, uint32_t* k2) {
    uint64_t ka = mix(seed, STREAM_SYNTHGRAD, (uint64_t)worker, (uint64_t)iter, 0);
    uint64_t kb = mix(seed, STREAM_SYNTHGRAD, (uint64_t)worker, (uint64_t)iter, 1);
    *k0 = (uint32_t)ka;
    *k1 = (uint32_t)(ka >> 32);
    *k2 = (uint32_t)kb;
}

float synth_scale(float variance) {
    // the centred sum of 12 uniform bytes has variance 12 * (256^2 - 1) / 12 = 65535
    return (float)std::sqrt((double)variance / 65535.0);
}

}  // namespace hoprng

namespace {

constexpr uint64_t TICKS_PER_UNIT = 1ull << 20;
constexpr uint64_t LAT = 1;

enum { EV_ARRIVE = 0, EV_DONE = 1, EV_ACK = 2 };
enum { COMPUTING = 0, WAIT_RECV = 1, WAIT_TOKEN = 2, FINISHED = 3 };

struct Event {
    uint64_t time;
    int kind, worker, sender, tag;
    bool operator>(const Event& o) const {
        if (time != o.time) return time > o.time;
        if (kind != o.kind) return kind > o.kind;
        if (worker != o.worker) return worker > o.worker;
        if (sender != o.sender) return sender > o.sender;
        return tag > o.tag;
    }
};

struct Sim {
    const hop_ctx* c;
    const hop_delay_model* dm;
    hop_schedule* out;
    int N, s, b, K, D, max_ig;
    bool serial = false;
    std::vector<int> in_ptr;                    // in-edge e = in_ptr[i] + position of j in N_in(i)
    std::vector<std::vector<int>> take_edge;    // per worker r: in-edge ids (r -> j), j in N_out(r)
    std::vector<std::vector<int>> queue;        // per in-edge: tags waiting in UpdateQ
    std::vector<int> iter_rcv;                  // per in-edge: newest tag ever dequeued
    std::vector<int> token;                     // per in-edge (r -> h): TokenQ(h -> r), kept at h
    std::vector<int> iter, state, written;
    std::priority_queue<Event, std::vector<Event>, std::greater<Event>> events;
    int err = HOP_OK;

    uint64_t duration(int i, int k) const {
        if (dm && dm->kind == HOP_DELAY_TABLE) return dm->table[(size_t)i * dm->table_iters + k];
        double mult = (dm && dm->mult) ? dm->mult[i] : 1.0;
        if (mult >= (double)HOP_TICKS_NEVER) return HOP_TICKS_NEVER;
        int kind = dm ? dm->kind : HOP_DELAY_NONE;
        uint64_t bits = hoprng::mix(c->opts.seed, hoprng::STREAM_DELAY, (uint64_t)i, (uint64_t)k, 0);
        double u = (double)(bits >> 11) * (1.0 / 9007199254740992.0);
        double base = 1.0;
        if (kind == HOP_DELAY_EXP1) base = -std::log(1.0 - u);
        else if (kind == HOP_DELAY_BERNOULLI6) base = (u < 1.0 / (double)N) ? 6.0 : 1.0;
        volatile double t = base * mult;        // one rounding per product, never fused
        t = t * (double)TICKS_PER_UNIT;
        if (t >= (double)HOP_TICKS_NEVER) return HOP_TICKS_NEVER;
        double f = std::floor(t);
        return f < 1.0 ? 1ull : (uint64_t)f;
    }

    // Ticks from Send to the receiver's queue: 1, or seeded uniform in 1..max_latency (Section 6.1
    // does not assume that the network keeps the order of messages).
    uint64_t latency(int sender, int receiver, int tag) const {
        const uint64_t ml = c->opts.max_latency;
        if (ml <= 1) return LAT;
        return 1 + hoprng::mix(c->opts.seed, hoprng::STREAM_LATENCY, (uint64_t)sender, (uint64_t)receiver,
                               (uint64_t)tag) % ml;
    }

    // Recv(k) at worker i on a snapshot of its queues: can it complete, and what does it take?
    bool recv_eval(int i, int k, std::vector<std::pair<int, int>>& acc) const {
        acc.clear();
        const auto& nb = c->in_nbrs[i];
        int satisfied = 0;
        for (size_t p = 0; p < nb.size(); ++p) {
            int e = in_ptr[i] + (int)p;
            const auto& q = queue[e];
            if (s >= 1) {
                int newest = -1;
                bool any = !q.empty();
                for (int t : q) newest = std::max(newest, t);
                int seen = std::max(iter_rcv[e], any ? newest : -1);
                if (seen >= k - s) ++satisfied;
                // an update no newer than one already reduced carries nothing new (possible only
                // when the network reorders)
                if (any && newest >= k - s && newest > iter_rcv[e]) acc.emplace_back(nb[p], newest);
            } else {
                if (std::find(q.begin(), q.end(), k) != q.end()) {
                    ++satisfied;
                    acc.emplace_back(nb[p], k);
                }
            }
        }
        return satisfied >= (int)nb.size() - b;
    }

    void recv_commit(int i, int k) {
        const auto& nb = c->in_nbrs[i];
        for (size_t p = 0; p < nb.size(); ++p) {
            int e = in_ptr[i] + (int)p;
            auto& q = queue[e];
            if (s >= 1) {
                for (int t : q) iter_rcv[e] = std::max(iter_rcv[e], t);
                q.clear();
            } else {
                q.erase(std::remove_if(q.begin(), q.end(), [k](int t) { return t <= k; }), q.end());
            }
        }
    }

    // Weights of one Reduce: W[j][i] times the Eq. 2 iteration weight, renormalised over what was
    // accepted; doubles, each rounded to fp32 once.
    void emit(int kind, int i, int k_eff, int k_label, int self_slot,
              const std::vector<std::pair<int, int>>& acc, int out_slot, uint64_t T) {
        for (const auto& a : acc)
            if (!(a.second > written[a.first] - D)) err = HOP_ERR_SLOT_DEAD;
        out->kind.push_back(kind);
        out->worker.push_back(i);
        out->iter.push_back(k_label);
        out->time.push_back(T);
        out->out_slot.push_back(out_slot);
        size_t base = out->src_worker.size();
        out->src_worker.push_back(i);
        out->src_tag.push_back(k_eff);
        out->src_slot.push_back(self_slot);
        for (const auto& a : acc) {
            out->src_worker.push_back(a.first);
            out->src_tag.push_back(a.second);
            out->src_slot.push_back(a.second % D);
        }
        size_t n = out->src_worker.size() - base;
        std::vector<double> r(n);
        double tot = 0.0;
        for (size_t a = 0; a < n; ++a) {
            int j = out->src_worker[base + a];
            double f = s >= 1 ? (double)(out->src_tag[base + a] - (k_eff - s) + 1) : 1.0;
            r[a] = (double)c->W[(size_t)j * N + i] * f;
            tot += r[a];
        }
        for (size_t a = 0; a < n; ++a) out->src_weight.push_back((float)(r[a] / tot));
        out->src_begin.push_back((int32_t)out->src_worker.size());
        // minibatch of a STEP: iid sample ids keyed by (seed, worker, iteration, position)
        if (out->batch > 0) {
            int64_t rows = c->data[i].rows;
            for (int m = 0; m < out->batch; ++m) {
                int32_t r_m = 0;
                if ((kind == HOP_STEP || kind == HOP_APPLY) && rows > 0)
                    r_m = (int32_t)(hoprng::mix(c->opts.seed, hoprng::STREAM_BATCH, (uint64_t)i,
                                                (uint64_t)k_label, (uint64_t)m) % (uint64_t)rows);
                out->batch_rows.push_back(r_m);
            }
        }
    }

    bool tokens_ready(int i) const {
        for (int e : take_edge[i])
            if (token[e] < 1) return false;
        return true;
    }

    void send(int i, int k, uint64_t T) {
        for (int j : c->out_nbrs[i]) {
            events.push(Event{T + latency(i, j, k), EV_ARRIVE, j, i, k});
            if (iter[j] > k) out->late_sends += 1;         // Section 6.2 (b): the receiver is already past it
        }
    }

    void enter(int i, int k, uint64_t T) {
        iter[i] = k;
        const auto& nb = c->in_nbrs[i];
        // insert a token into every local token queue: TokenQ(i -> j), j in N_in(i)
        for (size_t p = 0; p < nb.size(); ++p) token[in_ptr[i] + (int)p] += 1;
        if (k >= K) {
            state[i] = FINISHED;
            out->finish_time[i] = T;
        } else {
            if (!serial) send(i, k, T);                    // parallel approach: x_k leaves on entering iteration k
            uint64_t dur = duration(i, k);
            if (dur < HOP_TICKS_NEVER) events.push(Event{T + dur, EV_DONE, i, 0, k});
            state[i] = COMPUTING;
        }
        for (int j : nb)
            if (state[j] == WAIT_TOKEN) try_advance(j, T);
    }

    void try_advance(int i, uint64_t T) {
        if (!tokens_ready(i)) return;
        for (int e : take_edge[i]) token[e] -= 1;
        enter(i, iter[i] + 1, T);
    }

    void try_recv(int i, uint64_t T) {
        const int k0 = iter[i];
        std::vector<std::pair<int, int>> acc;
        if (!recv_eval(i, k0, acc)) return;
        recv_commit(i, k0);
        if (serial) {
            // the sent vectors (the worker's own y_k sits in ring slot k mod D) reduce into its current parameters
            emit(HOP_REDUCE, i, k0, k0, k0 % D, acc, D, T);
        } else {
            emit(HOP_STEP, i, k0, k0, k0 % D, acc, (k0 + 1) % D, T);
            written[i] = k0 + 1;
        }
        if (c->opts.skip_on && !c->out_nbrs[i].empty()) {
            int slowest = iter[c->out_nbrs[i][0]];
            for (int j : c->out_nbrs[i]) slowest = std::min(slowest, iter[j]);
            int behind = slowest - k0;
            if (behind > c->opts.trigger) {
                int J = std::min(std::min(behind, (int)c->opts.max_skip), std::min(max_ig, K - k0));
                if (J >= 2) {
                    int kp = k0 + J;
                    if (recv_eval(i, kp - 1, acc)) {
                        recv_commit(i, kp - 1);
                        if (serial) {
                            emit(HOP_JUMP, i, kp - 1, kp, D, acc, D, T);     // current parameters renewed in place
                        } else {
                            emit(HOP_JUMP, i, kp - 1, kp, (k0 + 1) % D, acc, kp % D, T);
                            written[i] = kp;
                        }
                        for (int e : take_edge[i]) token[e] -= J;
                        const auto& nb = c->in_nbrs[i];
                        for (size_t p = 0; p < nb.size(); ++p) token[in_ptr[i] + (int)p] += J - 1;
                        out->n_jumps += 1;
                        enter(i, kp, T);
                        return;
                    }
                }
            }
        }
        state[i] = WAIT_TOKEN;
        try_advance(i, T);
    }

    // ---- NOTIFY-ACK: per worker, what the current iteration still needs before it may advance (Section 3.3's
    // Assumption: computed, sent, received) and the newest acknowledgement held per out-going edge
    std::vector<char> computed, sent, consumed;
    std::vector<int> ack_rcv;                   // per in-edge (sender -> receiver): newest tag the receiver acknowledged

    void na_try_send(int i, uint64_t T) {
        if (sent[i]) return;
        for (int e : take_edge[i])
            if (ack_rcv[e] < iter[i] - 1) return;
        sent[i] = 1;
        send(i, iter[i], T);
    }

    void na_try_consume(int i, uint64_t T) {
        if (consumed[i]) return;
        const int k = iter[i];
        const auto& nb = c->in_nbrs[i];
        for (size_t p = 0; p < nb.size(); ++p) {
            const auto& q = queue[in_ptr[i] + (int)p];
            if (std::find(q.begin(), q.end(), k) == q.end()) return;
        }
        for (size_t p = 0; p < nb.size(); ++p) {
            auto& q = queue[in_ptr[i] + (int)p];
            q.erase(std::find(q.begin(), q.end(), k));
            events.push(Event{T + LAT, EV_ACK, nb[p], i, k});      // to every sender, right after the Reduce
        }
        consumed[i] = 1;
    }

    void na_enter(int i, int k, uint64_t T) {
        iter[i] = k;
        if (k >= K) {
            state[i] = FINISHED;
            out->finish_time[i] = T;
            return;
        }
        computed[i] = sent[i] = consumed[i] = 0;
        state[i] = COMPUTING;
        uint64_t dur = duration(i, k);
        if (dur < HOP_TICKS_NEVER) events.push(Event{T + dur, EV_DONE, i, 0, k});
        na_try_send(i, T);
        na_try_consume(i, T);
    }

    void na_try_complete(int i, uint64_t T) {
        if (!(computed[i] && sent[i] && consumed[i])) return;
        const int k = iter[i];
        std::vector<std::pair<int, int>> acc;
        for (int j : c->in_nbrs[i]) acc.emplace_back(j, k);
        emit(HOP_STEP, i, k, k, k % D, acc, (k + 1) % D, T);
        written[i] = k + 1;
        na_enter(i, k + 1, T);
    }

    int run_notify_ack() {
        computed.assign(N, 0);
        sent.assign(N, 0);
        consumed.assign(N, 0);
        ack_rcv.assign(in_ptr[N], -1);
        for (int i = 0; i < N; ++i) na_enter(i, 0, 0);
        while (!events.empty() && err == HOP_OK) {
            Event ev = events.top();
            events.pop();
            const int a = ev.worker;
            if (ev.kind == EV_ACK) {
                // `a` is the sender of the update, ev.sender the receiver that consumed it: in-edge (a -> ev.sender)
                const auto& nb = c->in_nbrs[ev.sender];
                int p = (int)(std::lower_bound(nb.begin(), nb.end(), a) - nb.begin());
                int e = in_ptr[ev.sender] + p;
                ack_rcv[e] = std::max(ack_rcv[e], ev.tag);
                if (state[a] != FINISHED) na_try_send(a, ev.time);
            } else if (state[a] == FINISHED) {
                continue;
            } else if (ev.kind == EV_ARRIVE) {
                const auto& nb = c->in_nbrs[a];
                int p = (int)(std::lower_bound(nb.begin(), nb.end(), ev.sender) - nb.begin());
                queue[in_ptr[a] + p].push_back(ev.tag);
                na_try_consume(a, ev.time);
            } else {
                computed[a] = 1;
            }
            if (state[a] != FINISHED) na_try_complete(a, ev.time);
        }
        return finish();
    }

    int run() {
        N = c->N; s = c->s; b = c->b; D = c->D; max_ig = c->max_ig;
        serial = c->opts.serial != 0;
        in_ptr.assign(N + 1, 0);
        for (int i = 0; i < N; ++i) in_ptr[i + 1] = in_ptr[i] + (int)c->in_nbrs[i].size();
        int E = in_ptr[N];
        take_edge.assign(N, {});
        for (int r = 0; r < N; ++r)
            for (int j : c->out_nbrs[r]) {
                const auto& nb = c->in_nbrs[j];
                int p = (int)(std::lower_bound(nb.begin(), nb.end(), r) - nb.begin());
                take_edge[r].push_back(in_ptr[j] + p);
            }
        queue.assign(E, {});
        iter_rcv.assign(E, -1);
        token.assign(E, max_ig - 1);
        iter.assign(N, 0);
        state.assign(N, COMPUTING);
        written.assign(N, 0);
        out->finish_time.assign(N, 0);
        out->src_begin.push_back(0);
        if (c->opts.notify_ack) return run_notify_ack();
        for (int i = 0; i < N; ++i) enter(i, 0, 0);
        while (!events.empty() && err == HOP_OK) {
            Event ev = events.top();
            events.pop();
            if (ev.kind == EV_ARRIVE) {
                const auto& nb = c->in_nbrs[ev.worker];
                int p = (int)(std::lower_bound(nb.begin(), nb.end(), ev.sender) - nb.begin());
                queue[in_ptr[ev.worker] + p].push_back(ev.tag);
                if (state[ev.worker] == WAIT_RECV) try_recv(ev.worker, ev.time);
            } else {
                if (serial) {
                    // Apply, then Send: y_k = x_k - eta g(x_k) into the ring slot that the neighbours will read
                    static const std::vector<std::pair<int, int>> none;
                    emit(HOP_APPLY, ev.worker, ev.tag, ev.tag, D, none, ev.tag % D, ev.time);
                    written[ev.worker] = ev.tag;
                    send(ev.worker, ev.tag, ev.time);
                }
                state[ev.worker] = WAIT_RECV;
                try_recv(ev.worker, ev.time);
            }
        }
        return finish();
    }

    int finish() {
        if (err != HOP_OK) return err;
        out->final_iter.assign(iter.begin(), iter.end());
        for (int i = 0; i < N; ++i)
            if (state[i] != FINISHED) out->stalled = 1;
        return out->stalled ? HOP_ERR_DEADLOCK : HOP_OK;
    }
};

// Level schedule over ring slots: a record runs one wave after the last earlier writer of anything
// it reads, after every earlier reader of the slot it overwrites and after that slot's last writer.
void build_waves(hop_schedule* sc) {
    const int N = sc->N, D = sc->D;
    const int R = (int)sc->kind.size();
    std::vector<int> last_write((size_t)N * D, -1), last_read((size_t)N * D, -1);
    sc->wave.resize(R);
    int n_waves = 0;
    for (int e = 0; e < R; ++e) {
        int w = 0;
        for (int a = sc->src_begin[e]; a < sc->src_begin[e + 1]; ++a)
            w = std::max(w, last_write[(size_t)sc->src_worker[a] * D + sc->src_slot[a]] + 1);
        size_t o = (size_t)sc->worker[e] * D + sc->out_slot[e];
        w = std::max(w, std::max(last_read[o], last_write[o]) + 1);
        for (int a = sc->src_begin[e]; a < sc->src_begin[e + 1]; ++a) {
            size_t x = (size_t)sc->src_worker[a] * D + sc->src_slot[a];
            last_read[x] = std::max(last_read[x], w);
        }
        last_write[o] = w;
        last_read[o] = -1;
        sc->wave[e] = w;
        n_waves = std::max(n_waves, w + 1);
    }
    sc->n_waves = n_waves;
    sc->wave_begin.assign(n_waves + 1, 0);
    for (int e = 0; e < R; ++e) sc->wave_begin[sc->wave[e] + 1] += 1;
    for (int w = 0; w < n_waves; ++w) sc->wave_begin[w + 1] += sc->wave_begin[w];
    sc->wave_order.resize(R);
    std::vector<int> fill(sc->wave_begin.begin(), sc->wave_begin.end() - 1);
    for (int e = 0; e < R; ++e) sc->wave_order[fill[sc->wave[e]]++] = e;
}

}  // namespace

int hop_run_protocol(const hop_ctx* ctx, const hop_delay_model* dm, int K, hop_schedule* out) {
    out->N = ctx->N;
    out->D = ctx->slots;
    out->K = K;
    bool any_rows = false;
    for (const auto& dd : ctx->data) any_rows = any_rows || dd.rows > 0;
    out->batch = any_rows ? ctx->opts.batch : 0;
    out->rows_at_sim.clear();
    for (const auto& dd : ctx->data) out->rows_at_sim.push_back(dd.rows);
    Sim sim{};
    sim.c = ctx;
    sim.dm = dm;
    sim.out = out;
    sim.K = K;
    int rc = sim.run();
    if (rc == HOP_OK || rc == HOP_ERR_DEADLOCK) build_waves(out);
    return rc;
}
