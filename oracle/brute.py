"""Exhaustive untimed model of the protocol for tiny graphs (oracle side).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

The paper's Assumption (Section 3.3) says when a worker may advance, not when it
does: any interleaving of message deliveries and worker steps that respects the
queues is a legal execution.  This module forgets time altogether and walks
every such interleaving.  Three kinds of move exist:

  deliver(j, i)  the oldest update in flight on edge j -> i reaches UpdateQ(i)
  fire(i)        worker i, whose Recv(k) can complete, does Recv, Reduce, Apply
                 (and, with skipping on, possibly a jump: Section 5)
  advance(i)     worker i, holding a token from every out-neighbour, removes
                 them and enters the next iteration: inserts its own tokens and
                 Sends (token-queue figure, Section 4.2)
  send(i)        serial approach of Section 3.2 only: the Send is a move of its own,
                 any time after entering the iteration and before the Recv

It serves as a pin for the timed simulator: every timed run must be one walk of
this model, every reachable state must obey the token identity of Theorem 2's
proof and the gap table, and no reachable state may be stuck before the end.
"""
from collections import deque


class Model:
    def __init__(self, in_nbrs, s, b, K, max_ig=0, skip_on=False, max_skip=10, trigger=1, ordered=True, serial=False):
        self.ordered = ordered            # False: any update in flight may arrive next (Section 6.1)
        self.serial = serial              # True: the serial approach of Section 3.2, Send after Compute and Apply
        self.n = len(in_nbrs)
        self.inn = [tuple(sorted(l)) for l in in_nbrs]
        outn = [[] for _ in in_nbrs]
        for i, l in enumerate(self.inn):
            for j in l:
                outn[j].append(i)
        self.outn = [tuple(sorted(l)) for l in outn]
        self.edges = tuple((j, i) for i in range(self.n) for j in self.inn[i])   # j sends to i
        self.eidx = {e: x for x, e in enumerate(self.edges)}
        self.s, self.b, self.K = s, b, K
        self.ig = max_ig if max_ig else max(s, 1)
        self.skip_on, self.max_skip, self.trigger = skip_on, max_skip, trigger

    # state = (it, ph, flight, queue, rcv, tok); ph: 0 running, 1 wants tokens, 2 done, 3 (serial approach only)
    # computing with nothing sent yet
    # tok[e] for e = (j, i) is TokenQ(i -> j): kept at i, taken by j.
    def initial(self):
        ne = len(self.edges)
        st = [[0] * self.n, [0] * self.n, [()] * ne, [()] * ne, [-1] * ne, [self.ig - 1] * ne]
        for i in range(self.n):
            self._enter(st, i, 0, [])
        return self._freeze(st)

    @staticmethod
    def _freeze(st):
        return tuple(tuple(x) for x in st)

    @staticmethod
    def _thaw(state):
        return [list(x) for x in state]

    def _enter(self, st, i, k, out):
        it, ph, flight, queue, rcv, tok = st
        it[i] = k
        for j in self.inn[i]:
            tok[self.eidx[(j, i)]] += 1
        out.append(("enter", i, k))
        if k >= self.K:
            ph[i] = 2
        elif self.serial:
            ph[i] = 3                     # the update of iteration k leaves after Compute and Apply: move "send"
        else:
            ph[i] = 0
            for j in self.outn[i]:
                e = self.eidx[(i, j)]
                flight[e] = flight[e] + (k,)

    def _recv(self, st, i, k):
        """(can complete, accepted) for Recv(k) at worker i."""
        _, _, _, queue, rcv, _ = st
        ok_count, acc = 0, []
        for j in self.inn[i]:
            e = self.eidx[(j, i)]
            q = queue[e]
            if self.s >= 1:
                newest = max(q) if q else -1
                if max(newest, rcv[e]) >= k - self.s:
                    ok_count += 1
                if q and newest >= k - self.s and newest > rcv[e]:
                    acc.append((j, newest))
            elif k in q:
                ok_count += 1
                acc.append((j, k))
        return ok_count >= len(self.inn[i]) - self.b, tuple(acc)

    def _consume(self, st, i, k):
        _, _, _, queue, rcv, _ = st
        for j in self.inn[i]:
            e = self.eidx[(j, i)]
            if self.s >= 1:
                if queue[e]:
                    rcv[e] = max(rcv[e], max(queue[e]))
                queue[e] = ()
            else:
                queue[e] = tuple(t for t in queue[e] if t > k)

    def moves(self, state):
        """All enabled moves as (name, args...)."""
        it, ph, flight, queue, rcv, tok = state
        mv = []
        for x, e in enumerate(self.edges):
            if flight[x] and self.ordered:
                mv.append(("deliver",) + e)
            elif flight[x]:
                mv.extend(("deliver",) + e + (t,) for t in flight[x])
        st = self._thaw(state)
        for i in range(self.n):
            if ph[i] == 0 and self._recv(st, i, it[i])[0]:
                mv.append(("fire", i))
            if ph[i] == 1 and all(tok[self.eidx[(i, j)]] >= 1 for j in self.outn[i]):
                mv.append(("advance", i))
            if ph[i] == 3:
                mv.append(("send", i))
        return mv

    def apply(self, state, move):
        """Returns (new state, what happened as trace items)."""
        st = self._thaw(state)
        it, ph, flight, queue, rcv, tok = st
        out = []
        if move[0] == "deliver":
            e = self.eidx[(move[1], move[2])]
            tag = flight[e][0] if len(move) == 3 else move[3]
            rest = list(flight[e])
            rest.remove(tag)
            flight[e] = tuple(rest)
            # staleness mode only ever looks at the newest queued tag
            queue[e] = (max(queue[e] + (tag,)),) if self.s >= 1 else queue[e] + (tag,)
            out.append(("deliver", move[1], move[2], tag))
        elif move[0] == "send":
            i = move[1]
            for j in self.outn[i]:
                e = self.eidx[(i, j)]
                flight[e] = flight[e] + (it[i],)
            ph[i] = 0
        elif move[0] == "fire":
            i = move[1]
            k = it[i]
            ok, acc = self._recv(st, i, k)
            assert ok
            self._consume(st, i, k)
            out.append(("recv", i, k, acc))
            ph[i] = 1
            if self.skip_on and self.outn[i]:
                behind = min(it[j] for j in self.outn[i]) - k
                if behind > self.trigger:
                    J = min(behind, self.max_skip, self.ig, self.K - k)
                    if J >= 2:
                        ok2, acc2 = self._recv(st, i, k + J - 1)
                        if ok2:
                            self._consume(st, i, k + J - 1)
                            out.append(("jump", i, k + J, acc2))
                            for j in self.outn[i]:
                                tok[self.eidx[(i, j)]] -= J
                            for j in self.inn[i]:
                                tok[self.eidx[(j, i)]] += J - 1
                            self._enter(st, i, k + J, out)
        else:
            i = move[1]
            for j in self.outn[i]:
                tok[self.eidx[(i, j)]] -= 1
            self._enter(st, i, it[i] + 1, out)
        return self._freeze(st), out

    def final(self, state):
        return all(p == 2 for p in state[1])

    def explore(self, limit=2_000_000):
        """Breadth-first closure.  Returns (set of states, list of stuck
        non-final states, list of all fired ("recv"/"jump") items)."""
        start = self.initial()
        seen = {start}
        dq = deque([start])
        stuck, fired = [], set()
        while dq:
            s = dq.popleft()
            mv = self.moves(s)
            if not mv and not self.final(s):
                stuck.append(s)
            for m in mv:
                t, out = self.apply(s, m)
                for o in out:
                    if o[0] in ("recv", "jump"):
                        fired.add(o)
                if t not in seen:
                    if len(seen) >= limit:
                        raise RuntimeError("state space larger than limit")
                    seen.add(t)
                    dq.append(t)
        return seen, stuck, fired

    def replay(self, trace):
        """Walk a timed run's trace through the model; raises AssertionError at
        the first item the model does not allow or does not reproduce."""
        state = self.initial()
        pending = deque()
        n_init = 0
        for item in trace:
            if item[0] == "enter" and item[2] == 0 and n_init < self.n:
                n_init += 1
                continue
            if pending:
                want = pending.popleft()
                assert want == item, (want, item)
                continue
            for i in range(self.n):       # sends leave no trace item and only ever enable other moves: take them at once
                if state[1][i] == 3:
                    state, _ = self.apply(state, ("send", i))
            if item[0] == "deliver":
                mv = ("deliver", item[1], item[2]) if self.ordered else ("deliver", item[1], item[2], item[3])
            elif item[0] == "recv":
                mv = ("fire", item[1])
            elif item[0] == "enter":
                mv = ("advance", item[1])
            else:
                raise AssertionError("unexpected trace item %r" % (item,))
            assert mv in self.moves(state), (mv, item)
            state, out = self.apply(state, mv)
            assert out[0] == item, (out, item)
            pending.extend(out[1:])
        assert not pending
        return state
