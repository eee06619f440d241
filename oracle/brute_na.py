"""Exhaustive untimed model of NOTIFY-ACK (Section 3.3) for tiny graphs (oracle side).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

Time is forgotten: any interleaving of the moves below that respects the protocol is a legal execution.
A worker in iteration k may

  send(i)      put update k on every out-going edge, once ACK(k - 1) has come back from every out-going
               neighbour (nothing to wait for at k = 0)
  consume(i)   take update k of every in-coming neighbour out of its queues (its Reduce) once all of them
               are there, and put an ACK(k) on the way back to each of them
  done(i)      finish its Compute
  complete(i)  with send, consume and done behind it: Apply, enter iteration k + 1

and the network may

  deliver(j, i)  hand the oldest update in flight on edge j -> i to i's queue
  ack(i, j)      hand the oldest ACK in flight from i back to j

The walk over all reachable states is a pin for the timed simulator: its runs are walks of this model
(same reading, eager moves), every reachable state must keep at most one unconsumed update per edge and obey
the gap row of the table, min(len(j -> i), 2 len(i -> j)), and no state may be stuck before the end.
"""
from collections import deque


class Model:
    def __init__(self, in_nbrs, K):
        self.n = len(in_nbrs)
        self.inn = [tuple(sorted(l)) for l in in_nbrs]
        outn = [[] for _ in in_nbrs]
        for i, l in enumerate(self.inn):
            for j in l:
                outn[j].append(i)
        self.outn = [tuple(sorted(l)) for l in outn]
        self.edges = tuple((j, i) for i in range(self.n) for j in self.inn[i])      # j sends to i
        self.eidx = {e: x for x, e in enumerate(self.edges)}
        self.K = K

    # state = (it, flags, flight, queue, ackfl, acked)
    #   flags[i]: bit 0 sent, bit 1 consumed, bit 2 computed;  flight / queue / ackfl: tuples of tags per edge;
    #   acked[e] for e = (j, i): newest ACK of i that j holds
    def initial(self):
        ne = len(self.edges)
        return ((0,) * self.n, (0,) * self.n, ((),) * ne, ((),) * ne, ((),) * ne, (-1,) * ne)

    def finished(self, state):
        return all(k >= self.K for k in state[0])

    def moves(self, state):
        it, flags, flight, queue, ackfl, acked = state
        out = []
        for x, (j, i) in enumerate(self.edges):
            if flight[x]:
                out.append(("deliver", j, i))
            if ackfl[x]:
                out.append(("ack", i, j))
        for i in range(self.n):
            k = it[i]
            if k >= self.K:
                continue
            f = flags[i]
            if not f & 1 and all(acked[self.eidx[(i, j)]] >= k - 1 for j in self.outn[i]):
                out.append(("send", i))
            if not f & 2 and all(k in queue[self.eidx[(j, i)]] for j in self.inn[i]):
                out.append(("consume", i))
            if not f & 4:
                out.append(("done", i))
            if f == 7:
                out.append(("complete", i))
        return out

    def apply(self, state, move):
        it, flags, flight, queue, ackfl, acked = (list(x) for x in state)
        kind = move[0]
        if kind == "deliver":
            x = self.eidx[(move[1], move[2])]
            queue[x] = queue[x] + (flight[x][0],)
            flight[x] = flight[x][1:]
        elif kind == "ack":
            x = self.eidx[(move[2], move[1])]               # edge j -> i carries i's ACKs back to j
            acked[x] = max(acked[x], ackfl[x][0])
            ackfl[x] = ackfl[x][1:]
        else:
            i = move[1]
            k = it[i]
            if kind == "send":
                for j in self.outn[i]:
                    x = self.eidx[(i, j)]
                    flight[x] = flight[x] + (k,)
                flags[i] |= 1
            elif kind == "consume":
                for j in self.inn[i]:
                    x = self.eidx[(j, i)]
                    q = list(queue[x])
                    q.remove(k)
                    queue[x] = tuple(q)
                    ackfl[x] = ackfl[x] + (k,)
                flags[i] |= 2
            elif kind == "done":
                flags[i] |= 4
            else:
                it[i] = k + 1
                flags[i] = 0
        return tuple(tuple(x) for x in (it, flags, flight, queue, ackfl, acked))

    def explore(self, limit=2_000_000):
        """Breadth-first over all reachable states.  Returns (number of states, gap[i][j] = largest Iter(i) - Iter(j)
        seen, largest number of unconsumed updates on one edge, number of stuck states)."""
        start = self.initial()
        seen = {start}
        todo = deque([start])
        n = self.n
        gap = [[0] * n for _ in range(n)]
        worst_queue = stuck = 0
        while todo:
            st = todo.popleft()
            it, _, flight, queue, _, _ = st
            for i in range(n):
                for j in range(n):
                    gap[i][j] = max(gap[i][j], it[i] - it[j])
            worst_queue = max(worst_queue, max((len(q) for q in queue), default=0))
            mv = self.moves(st)
            if not mv and not self.finished(st):
                stuck += 1
            for m in mv:
                nx = self.apply(st, m)
                if nx not in seen:
                    if len(seen) >= limit:
                        raise RuntimeError("state space larger than the limit")
                    seen.add(nx)
                    todo.append(nx)
        return len(seen), gap, worst_queue, stuck

    def follows(self, trace):
        """True if the visible events of a timed run - ("enter", i, k), ("recv", i, k, ...), ("deliver", j, i, tag) in
        the order they happened - are one walk of this model.  The moves a trace does not show (send, ack, done) only
        ever enable others and disable none, so they are taken as soon as they are possible."""
        st = self.initial()

        def settle(st):
            moved = True
            while moved:
                moved = False
                for m in self.moves(st):
                    if m[0] in ("send", "ack", "done"):
                        st = self.apply(st, m)
                        moved = True
                        break
            return st

        for ev in trace:
            st = settle(st)
            if ev[0] == "enter":
                i, k = ev[1], ev[2]
                if k == 0:
                    if st[0][i] != 0:
                        return False
                    continue
                if st[0][i] != k - 1 or ("complete", i) not in self.moves(st):
                    return False
                st = self.apply(st, ("complete", i))
            elif ev[0] == "recv":
                i, k = ev[1], ev[2]
                if st[0][i] != k or ("consume", i) not in self.moves(st):
                    return False
                st = self.apply(st, ("consume", i))
            elif ev[0] == "deliver":
                j, i, tag = ev[1], ev[2], ev[3]
                x = self.eidx[(j, i)]
                if not st[2][x] or st[2][x][0] != tag:
                    return False
                st = self.apply(st, ("deliver", j, i))
            else:
                return False
        return self.finished(settle(st))
