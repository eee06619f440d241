"""Event-driven run of Hop's queue protocol (oracle side, integers only).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

What is followed, in the paper's notation:
  * graph, N_in / N_out, self-loop                      Section 3.1
  * parallel approach: Send x_k and Compute on x_k at the start of iteration k,
    then Recv, Reduce, Apply                             Section 3.2
  * update queues with (iter, w_id) tags                 Section 4.1, Figure
    "Decentralized Training with Update Queue"
  * token queues TokenQ(i->j), max_ig                    Section 4.2, Figure
    "Decentralized Training with Token Queue"
  * backup workers N_buw = b                             Section 4.3
  * bounded staleness s, iter_rcv, newest-per-neighbour  Section 4.4
  * skipping iterations                                  Section 5
  * one queue per iteration, index iter mod #queues      Section 6.1
  * stale updates discarded on dequeue                   Section 6.2 (a)

Readings where the paper is silent or at odds with itself (each also listed in
the repository's design notes):
  - Time is integer ticks; a message sent at T is visible at T+1; Reduce, Apply,
    token operations and a jump take no time.  Simultaneous events are ordered
    by (time, ARRIVE before COMPUTE_DONE, worker, sender, tag).
  - Token queues start with max_ig-1 tokens and get one more when iteration 0
    is entered (the token figure), which is the "max_ig tokens" of the prose.
  - Iterations are k = 0 .. K-1; the result is x_K.
  - s >= 1 ("staleness mode"): per in-neighbour the newest queued tag counts; a
    neighbour is satisfied when the newest tag ever received from it is
    >= k - s (the prose of Section 4.4, not the do-while of its figure, which
    would wait for a new update even when an old one is within the bound); a
    satisfied neighbour with nothing new contributes nothing to this Reduce.
    All neighbours are looked at in one snapshot.  Tags newer than k count.
  - s = 0 ("exact-tag mode"): only tag k counts (update-queue and backup-worker
    figures); tags below k are discarded, tags above k stay queued.
  - b >= 1 together with s >= 1 (the table's "Hybrid" row has no algorithm):
    proceed once deg - b neighbours are satisfied, take every neighbour that
    has something new within the bound.
  - Skipping: after Apply, behind = min over out-neighbours of Iter(j) - k0
    (= min token count - max_ig).  If behind > trigger, jump J = min(behind,
    max_skip, max_ig, K - k0) iterations when J >= 2 and Recv(k0+J-1) would not
    block; otherwise advance normally.  The jump's Reduce averages x_{k0+1}
    with what Recv(k0+J-1) accepts, then J tokens move each way.
  - A worker that reaches iteration K still inserts its tokens, sends nothing.
  - Section 6.1 does not assume that the network keeps messages in order.  With
    max_latency > 1 every update takes a seeded number of ticks in
    1..max_latency, so updates on one edge can overtake each other; the queues
    are multisets of tags, so nothing else changes.  Section 6.2 (b) (do not
    send what the receiver is already past) is kept as a counter, late_sends:
    in exact-tag mode such an update is always dropped at the next dequeue.

Two more options complete the design space of Sections 3.2 and 3.3 (comparison only; the paper's
own design is the parallel approach with token queues):
  - serial=True: the serial approach of Section 3.2.  On entering iteration k a worker Computes
    on its current parameters x_k, Applies (y_k = x_k - eta g), and only then Sends y_k; when
    Recv(k) is satisfied it Reduces the y's (its own included) into x_{k+1}.  Two records per
    iteration: APPLY (x_cur, gradient -> ring slot k mod D, the vector that is sent) and REDUCE
    (ring slots -> x_cur).  x_cur is a slot of its own per worker (index D), never sent.  With
    s = 0, b = 0 this is X_{k+1} = W^T (X_k - eta G_k) whatever the delays.  The queue rules
    (tokens, backup workers, staleness, skipping) are the same; a jump's Reduce reads and
    writes x_cur.
  - notify_ack=True: the NOTIFY-ACK protocol of Section 3.3 on the parallel approach, standard
    training only (s = 0, no backup workers, no skipping, no token queues - Section 3.3 and
    the introduction say it supports none of them).  A worker may not Send(k) before every
    out-going neighbour has acknowledged its update of iteration k - 1; a worker acknowledges
    to all in-coming neighbours right after the Reduce that consumed their updates; Recv and
    Reduce of iteration k run as soon as the updates of iteration k are all there, beside the
    Compute (that is what the parallel approach allows, and what lets a sender get 2 ahead of
    a receiver, the table's figure); the worker advances when it has computed, sent and
    received (the Assumption of Section 3.3).  An acknowledgement travels one tick.  Records
    are those of standard training; only times and order change.  Ring as for max_ig = 2.

Versions live in a ring of D slots per worker, slot = version mod D, with
D = max_ig + 1 in staleness mode (the paper's #queues) and max_ig + 2 in
exact-tag mode (the ring also holds the not yet sent x_{k+1}).  With
out-of-order delivery a reader in iteration k may take a tag as old as k - s
while the sender, at most max_ig iterations ahead, has already produced version
k + max_ig + 1: staleness mode then needs D = s + max_ig + 2.
"""
import heapq
from collections import deque

import numpy as np

from . import rng
from .arith import reduce_weights

STEP = 0      # parallel approach: Reduce + Apply of one iteration
JUMP = 1      # Section 5: Reduce without gradient into the iteration jumped to
APPLY = 2     # serial approach: y_k = x_k - eta g(x_k) into the ring slot that is sent
REDUCE = 3    # serial approach: x_{k+1} = sum_a w'_a y_a into the worker's current parameters

EV_ARRIVE = 0
EV_DONE = 1
EV_ACK = 2

COMPUTING = 0
WAIT_RECV = 1
WAIT_TOKEN = 2
FINISHED = 3

LAT = 1


class ProtocolError(Exception):
    pass


class SlotDead(ProtocolError):
    pass


def transpose(in_nbrs):
    out = [[] for _ in in_nbrs]
    for i, lst in enumerate(in_nbrs):
        for j in lst:
            out[j].append(i)
    return [sorted(o) for o in out]


def shortest_paths(out_nbrs):
    """dist[a][b] = length of the shortest directed path a -> b (inf if none)."""
    n = len(out_nbrs)
    dist = [[float("inf")] * n for _ in range(n)]
    for a in range(n):
        dist[a][a] = 0
        dq = deque([a])
        while dq:
            u = dq.popleft()
            for v in out_nbrs[u]:
                if dist[a][v] == float("inf"):
                    dist[a][v] = dist[a][u] + 1
                    dq.append(v)
    return dist


def ring_depth(s, max_ig, max_latency=1):
    if s >= 1:
        return max_ig + 1 if max_latency <= 1 else s + max_ig + 2
    return max_ig + 2


class Record:
    __slots__ = ("seq", "kind", "worker", "k", "time", "src_worker", "src_tag",
                 "src_slot", "w64", "w32", "out_slot")

    def key(self):
        return (self.kind, self.worker, self.k, tuple(self.src_worker),
                tuple(self.src_tag), tuple(self.src_slot), self.out_slot)


class Hop:
    """One run of the protocol.  in_nbrs[i] lists the non-self in-neighbours of
    i in ascending order; W[j][i] is the weight of sender j at receiver i."""

    def __init__(self, in_nbrs, W, s, b, K, max_ig=0, skip_on=False, max_skip=10,
                 trigger=1, seed=0, delay_kind=rng.DELAY_NONE, mult=None,
                 table=None, check=True, trace=False, max_latency=1, serial=False, notify_ack=False):
        self.N = len(in_nbrs)
        self.in_nbrs = [sorted(l) for l in in_nbrs]
        self.out_nbrs = transpose(self.in_nbrs)
        self.W = np.asarray(W, dtype=np.float32)
        self.s, self.b, self.K = int(s), int(b), int(K)
        self.max_ig = int(max_ig) if max_ig else max(self.s, 1)
        self.skip_on, self.max_skip, self.trigger = bool(skip_on), int(max_skip), int(trigger)
        self.seed, self.delay_kind = int(seed), int(delay_kind)
        self.mult = [1.0] * self.N if mult is None else [float(m) for m in mult]
        self.table = table
        self.max_latency = int(max_latency)
        self.serial, self.notify_ack = bool(serial), bool(notify_ack)
        if self.notify_ack:
            if self.s != 0 or self.b != 0 or self.skip_on or self.serial or self.max_latency > 1:
                raise ProtocolError("NOTIFY-ACK is standard training on the parallel approach only")
            self.max_ig = 2                      # a sender is never more than 2 ahead: ring as for max_ig = 2
        self.D = ring_depth(self.s, self.max_ig, self.max_latency)
        self.slots = self.D + (1 if self.serial else 0)     # slots per worker in memory; slot D = x_cur (serial)
        self.check = check
        for i in range(self.N):
            if self.b > 0 and self.b >= len(self.in_nbrs[i]):
                raise ProtocolError("N_buw(i) must be below |N_in(i)|")
        self.dist = shortest_paths(self.out_nbrs) if check else None
        self.trace = [] if trace else None

    # ---- Recv -------------------------------------------------------------
    def _recv_eval(self, i, k):
        """Decide Recv(k, i) on a snapshot of i's queues, without side effects.
        Returns (proceeds, [(j, tag), ...] ascending j)."""
        s = self.s
        satisfied = 0
        accepted = []
        for j in self.in_nbrs[i]:
            q = self.queue[(j, i)]
            if s >= 1:
                new = max(q) if q else None
                seen = self.iter_rcv[(j, i)]
                if new is not None and new > seen:
                    seen = new
                if seen >= k - s:
                    satisfied += 1
                # an update no newer than one already reduced carries nothing new (it can only
                # show up after a newer one when the network reorders)
                if new is not None and new >= k - s and new > self.iter_rcv[(j, i)]:
                    accepted.append((j, new))
            else:
                if k in q:
                    satisfied += 1
                    accepted.append((j, k))
        return satisfied >= len(self.in_nbrs[i]) - self.b, accepted

    def _recv_commit(self, i, k):
        for j in self.in_nbrs[i]:
            q = self.queue[(j, i)]
            if self.s >= 1:
                if q:
                    self.iter_rcv[(j, i)] = max(self.iter_rcv[(j, i)], max(q))
                    q.clear()
            else:
                q[:] = [t for t in q if t > k]

    # ---- records ------------------------------------------------------------
    def _emit(self, kind, i, k_eff, k_label, self_slot, accepted, out_slot, T):
        for (j, t) in accepted:
            if not (t > self.written[j] - self.D):
                raise SlotDead("version %d of worker %d already overwritten" % (t, j))
        r = Record()
        r.seq = len(self.records)
        r.kind, r.worker, r.k, r.time = kind, i, k_label, T
        r.src_worker = [i] + [j for (j, _) in accepted]
        r.src_tag = [k_eff] + [t for (_, t) in accepted]
        r.src_slot = [self_slot] + [t % self.D for (_, t) in accepted]
        r.w64, r.w32 = reduce_weights(self.W, i, k_eff, self.s, r.src_worker, r.src_tag)
        r.out_slot = out_slot
        self.records.append(r)

    # ---- iteration boundaries -------------------------------------------------
    def _send(self, i, k, T):
        for j in self.out_nbrs[i]:
            lat = rng.latency_ticks(self.seed, self.max_latency, i, j, k)
            heapq.heappush(self.events, (T + lat, EV_ARRIVE, j, i, k))
            if self.Iter[j] > k:
                self.late_sends += 1

    def _enter(self, i, k, T):
        self.Iter[i] = k
        for j in self.in_nbrs[i]:
            self.tokens[(i, j)] += 1
        if self.trace is not None:
            self.trace.append(("enter", i, k))
        if k >= self.K:
            self.state[i] = FINISHED
            self.finish_time[i] = T
        else:
            if not self.serial:
                self._send(i, k, T)              # parallel approach: Send x_k on entering iteration k
            dur = rng.duration_ticks(self.seed, self.delay_kind, self.N, self.mult[i], i, k,
                                     self.table)
            if dur < rng.TICKS_NEVER:
                heapq.heappush(self.events, (T + dur, EV_DONE, i, 0, k))
            self.state[i] = COMPUTING
        for j in self.in_nbrs[i]:
            if self.state[j] == WAIT_TOKEN:
                self._try_advance(j, T)

    def _try_advance(self, i, T):
        if all(self.tokens[(j, i)] >= 1 for j in self.out_nbrs[i]):
            for j in self.out_nbrs[i]:
                self.tokens[(j, i)] -= 1
            self._enter(i, self.Iter[i] + 1, T)

    def _try_recv(self, i, T):
        k = self.Iter[i]
        ok, accepted = self._recv_eval(i, k)
        if not ok:
            return
        self._recv_commit(i, k)
        D = self.D
        if self.serial:
            # Reduce of the sent vectors (own y_k in ring slot k mod D) into the current parameters
            self._emit(REDUCE, i, k, k, k % D, accepted, D, T)
        else:
            self._emit(STEP, i, k, k, k % D, accepted, (k + 1) % D, T)
            self.written[i] = k + 1
        if self.trace is not None:
            self.trace.append(("recv", i, k, tuple(accepted)))
        k0 = k
        if self.skip_on and self.out_nbrs[i]:
            behind = min(self.Iter[j] for j in self.out_nbrs[i]) - k0
            if behind > self.trigger:
                J = min(behind, self.max_skip, self.max_ig, self.K - k0)
                if J >= 2:
                    kp = k0 + J
                    ok2, acc2 = self._recv_eval(i, kp - 1)
                    if ok2:
                        self._recv_commit(i, kp - 1)
                        if self.serial:          # x_cur (= x_{k0+1}) renewed in place
                            self._emit(JUMP, i, kp - 1, kp, D, acc2, D, T)
                        else:
                            self._emit(JUMP, i, kp - 1, kp, (k0 + 1) % D, acc2, kp % D, T)
                            self.written[i] = kp
                        for j in self.out_nbrs[i]:
                            self.tokens[(j, i)] -= J
                            assert self.tokens[(j, i)] >= 0
                        for j in self.in_nbrs[i]:
                            self.tokens[(i, j)] += J - 1
                        self.n_jumps += 1
                        if self.trace is not None:
                            self.trace.append(("jump", i, kp, tuple(acc2)))
                        self._enter(i, kp, T)
                        return
        self.state[i] = WAIT_TOKEN
        self._try_advance(i, T)

    # ---- invariants (token identity, Theorems 1 and 2, the gap table) -------
    def _check(self):
        N, ig = self.N, self.max_ig
        It = self.Iter
        for h in range(N):
            for r in self.in_nbrs[h]:
                t = self.tokens[(h, r)]
                assert t == It[h] - It[r] + ig and t >= 0, "token identity broken"
                assert t <= ig * (self.dist[h][r] + 1), "token queue over capacity"
        for i in range(N):
            for j in range(N):
                if i == j:
                    continue
                gap = It[i] - It[j]
                assert gap <= ig * self.dist[i][j], "token bound (Theorem 2) broken"
                if self.b == 0:
                    fwd = (self.s + 1) * self.dist[j][i] if self.s >= 1 else self.dist[j][i]
                    assert gap <= fwd, "forward gap bound (gap table) broken"
        if self.s == 0 and self.b == 0:
            # Section 4.2's capacity bound is for standard training; with backup
            # workers late updates pile up until the next dequeue (Section 4.3)
            for i in range(N):
                occ = sum(len(self.queue[(j, i)]) for j in self.in_nbrs[i])
                assert occ <= (1 + ig) * len(self.in_nbrs[i]), "update queue over capacity"
        self.max_gap = max(self.max_gap, max(It) - min(It))

    # ---- main loop -------------------------------------------------------------
    def run(self):
        N = self.N
        self.records = []
        self.events = []
        self.Iter = [0] * N
        self.state = [COMPUTING] * N
        self.finish_time = [None] * N
        self.written = [0] * N
        self.queue = {(j, i): [] for i in range(N) for j in self.in_nbrs[i]}
        self.iter_rcv = {(j, i): -1 for i in range(N) for j in self.in_nbrs[i]}
        self.tokens = {(i, j): self.max_ig - 1 for i in range(N) for j in self.in_nbrs[i]}
        self.n_jumps = 0
        self.late_sends = 0
        self.max_gap = 0
        self.max_queue = 0
        if self.notify_ack:
            return self._run_notify_ack()
        for i in range(N):
            self._enter(i, 0, 0)
        if self.check:
            self._check()
        while self.events:
            T, kind, a, snd, tag = heapq.heappop(self.events)
            if kind == EV_ARRIVE:
                self.queue[(snd, a)].append(tag)
                self.max_queue = max(self.max_queue, len(self.queue[(snd, a)]))
                if self.trace is not None:
                    self.trace.append(("deliver", snd, a, tag))
                if self.state[a] == WAIT_RECV:
                    self._try_recv(a, T)
            else:
                assert self.state[a] == COMPUTING and self.Iter[a] == tag
                if self.serial:
                    # Apply, then Send: y_k = x_k - eta g(x_k) goes into ring slot k mod D and out
                    self._emit(APPLY, a, tag, tag, self.D, [], tag % self.D, T)
                    self.written[a] = tag
                    self._send(a, tag, T)
                self.state[a] = WAIT_RECV
                self._try_recv(a, T)
            if self.check:
                self._check()
        self.stalled = any(st != FINISHED for st in self.state)
        return self.records

    # ---- NOTIFY-ACK (Section 3.3) ------------------------------------------------
    def _na_try_send(self, i, T):
        k = self.Iter[i]
        if self.sent[i] or not all(self.ack_rcv[(i, j)] >= k - 1 for j in self.out_nbrs[i]):
            return
        self.sent[i] = True
        self._send(i, k, T)

    def _na_try_consume(self, i, T):
        k = self.Iter[i]
        if self.consumed[i] or not all(k in self.queue[(j, i)] for j in self.in_nbrs[i]):
            return
        for j in self.in_nbrs[i]:
            self.queue[(j, i)].remove(k)
            heapq.heappush(self.events, (T + LAT, EV_ACK, j, i, k))       # ACK after the Reduce, to every sender
        self.consumed[i] = True
        if self.trace is not None:
            self.trace.append(("recv", i, k, tuple((j, k) for j in self.in_nbrs[i])))

    def _na_try_complete(self, i, T):
        k = self.Iter[i]
        if not (self.computed[i] and self.sent[i] and self.consumed[i]):
            return
        D = self.D
        self._emit(STEP, i, k, k, k % D, [(j, k) for j in self.in_nbrs[i]], (k + 1) % D, T)
        self.written[i] = k + 1
        self._na_enter(i, k + 1, T)

    def _na_enter(self, i, k, T):
        self.Iter[i] = k
        if self.trace is not None:
            self.trace.append(("enter", i, k))
        if k >= self.K:
            self.state[i] = FINISHED
            self.finish_time[i] = T
            return
        self.computed[i] = self.sent[i] = self.consumed[i] = False
        self.state[i] = COMPUTING
        dur = rng.duration_ticks(self.seed, self.delay_kind, self.N, self.mult[i], i, k, self.table)
        if dur < rng.TICKS_NEVER:
            heapq.heappush(self.events, (T + dur, EV_DONE, i, 0, k))
        self._na_try_send(i, T)
        self._na_try_consume(i, T)

    def _na_check(self):
        It = self.Iter
        for i in range(self.N):
            for j in self.in_nbrs[i]:
                assert len(self.queue[(j, i)]) <= 1, "a sender has two unconsumed updates at one receiver"
            for j in range(self.N):
                if i != j:
                    assert It[i] - It[j] <= min(self.dist[j][i], 2 * self.dist[i][j]), "NOTIFY-ACK gap bound broken"
        self.max_gap = max(self.max_gap, max(It) - min(It))

    def _run_notify_ack(self):
        N = self.N
        self.ack_rcv = {(j, i): -1 for i in range(N) for j in self.in_nbrs[i]}     # newest ACK j holds from i
        self.computed, self.sent, self.consumed = [False] * N, [False] * N, [False] * N
        for i in range(N):
            self._na_enter(i, 0, 0)
        if self.check:
            self._na_check()
        while self.events:
            T, kind, a, snd, tag = heapq.heappop(self.events)
            if self.state[a] != FINISHED or kind == EV_ACK:
                if kind == EV_ARRIVE:
                    self.queue[(snd, a)].append(tag)
                    self.max_queue = max(self.max_queue, len(self.queue[(snd, a)]))
                    if self.trace is not None:
                        self.trace.append(("deliver", snd, a, tag))
                    self._na_try_consume(a, T)
                elif kind == EV_DONE:
                    assert self.Iter[a] == tag
                    self.computed[a] = True
                else:                            # ACK of receiver `snd` for a's update `tag`
                    self.ack_rcv[(a, snd)] = max(self.ack_rcv[(a, snd)], tag)
                    if self.state[a] != FINISHED:
                        self._na_try_send(a, T)
                if self.state[a] != FINISHED:
                    self._na_try_complete(a, T)
            if self.check:
                self._na_check()
        self.stalled = any(st != FINISHED for st in self.state)
        return self.records
