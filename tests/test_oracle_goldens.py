"""Hand-worked traces for the two readings the paper gives no algorithm for - backup workers together with
bounded staleness (the gap table's "Hybrid" row) and the skip trigger / size of Section 5 - against the
oracle, and a set of planted mistakes that these traces must catch.  No GPU."""
import importlib
import os
import shutil
import sys
from fractions import Fraction

import numpy as np
import pytest

from conftest import ROOT, golden

KIND = {"STEP": 0, "JUMP": 1}


def parse_trace(name):
    g = golden(name)
    recs = []
    for key in sorted(k for k in g if k.startswith("rec")):
        parts = [p.strip() for p in g[key].split("|")]
        t, kind, worker, k = parts[0].split()
        srcs = [tuple(int(v) for v in item.split(":")) for item in parts[1].split()]
        weights = [Fraction(v) for v in parts[2].split()]
        out_slot = int(parts[3]) if len(parts) > 3 else None
        recs.append((int(t), KIND[kind], int(worker), int(k), srcs, weights, out_slot))
    return recs, [int(v) for v in g["finish"].split()], g


def check_trace(protocol, rng, recs, want, finish):
    """Every record of the oracle against the hand-worked one: time, kind, worker, iteration, the averaged
    (worker, tag[, slot]) list in order, the weights as exact fractions (fp64 to an ulp, fp32 bit for bit)."""
    assert len(recs) == len(want), (len(recs), len(want))
    for r, (t, kind, worker, k, srcs, weights, out_slot) in zip(recs, want):
        assert (r.time, r.kind, r.worker, r.k) == (t, kind, worker, k), (r.seq, r.time, r.kind, r.worker, r.k)
        got = list(zip(r.src_worker, r.src_tag, r.src_slot)) if len(srcs[0]) == 3 else list(zip(r.src_worker, r.src_tag))
        assert got == srcs, (r.seq, got, srcs)
        assert abs(sum(weights) - 1) == 0
        for w64, w32, f in zip(r.w64, r.w32, weights):
            assert abs(w64 - float(f)) <= 2.0 ** -52, (r.seq, w64, f)
            assert np.float32(w32) == np.float32(float(f)), (r.seq, w32, f)
        if out_slot is not None:
            assert r.out_slot == out_slot, (r.seq, r.out_slot, out_slot)
    return True


def run_hybrid(protocol, rng):
    nb = [[1, 2, 3], [0, 2, 3], [0, 1, 3], [0, 1, 2]]
    W = np.full((4, 4), 0.25, dtype=np.float32)
    table = [[10] * 5, [12] * 5, [25] * 5, [100] * 5]
    h = protocol.Hop(nb, W, s=2, b=1, K=5, max_ig=4, delay_kind=rng.DELAY_TABLE, table=table, check=True)
    return h, h.run()


def run_jump(protocol, rng):
    nb = [[1, 2], [0, 2], [0, 1]]
    W = np.array([[0.5, 0.25, 0.25], [0.25, 0.5, 0.25], [0.25, 0.25, 0.5]], dtype=np.float32)
    table = [[35] * 6, [10] * 6, [10] * 6]
    h = protocol.Hop(nb, W, s=0, b=1, K=6, max_ig=5, skip_on=True, max_skip=10, trigger=1,
                     delay_kind=rng.DELAY_TABLE, table=table, check=True)
    return h, h.run()


def both_traces(protocol, rng):
    want, finish, _ = parse_trace("hybrid_trace.txt")
    h, recs = run_hybrid(protocol, rng)
    check_trace(protocol, rng, recs, want, finish)
    assert list(h.finish_time) == finish and not h.stalled and h.n_jumps == 0
    want, finish, g = parse_trace("jump_trace.txt")
    h, recs = run_jump(protocol, rng)
    check_trace(protocol, rng, recs, want, finish)
    assert list(h.finish_time) == finish and not h.stalled and h.n_jumps == int(g["jumps"]) and h.D == int(g["depth"])


def test_hybrid_trace_worked_by_hand():
    """Sections 4.3 + 4.4, gap-table row "Hybrid": 4 workers, s = 2, N_buw = 1, fixed compute times."""
    from oracle import protocol, rng
    want, finish, _ = parse_trace("hybrid_trace.txt")
    assert len(want) == 20
    h, recs = run_hybrid(protocol, rng)
    check_trace(protocol, rng, recs, want, finish)
    assert list(h.finish_time) == finish and not h.stalled
    # what the trace is there to show
    by = {(r.worker, r.k): r for r in recs}
    assert by[(0, 1)].src_worker == [0, 1]            # neighbours 2 and 3 satisfied by an old update: not averaged
    assert by[(0, 3)].time == 40                      # proceeds with 2 of 3 satisfied (worker 3 is not)
    assert by[(0, 4)].time == 51                      # 1 of 3 is not enough: waits one tick for worker 2's update


def test_jump_trace_worked_by_hand():
    """Section 5 with trigger 1 and max_skip 10: the slow worker runs iterations 0 and 3 only, each followed by a
    jump of 3 whose Reduce averages its fresh parameters with both neighbours' updates of iteration k - 1."""
    from oracle import protocol, rng
    want, finish, g = parse_trace("jump_trace.txt")
    h, recs = run_jump(protocol, rng)
    check_trace(protocol, rng, recs, want, finish)
    assert list(h.finish_time) == finish and h.n_jumps == int(g["jumps"]) and h.D == int(g["depth"])
    assert [r.k for r in recs if r.worker == 0] == [0, 3, 3, 6]


# (file, text as it stands, planted mistake): each must make a hand-worked trace fail
MISTAKES = [
    ("protocol.py", "if new is not None and new >= k - s and new > self.iter_rcv[(j, i)]:\n                    accepted.append((j, new))",
     "if seen >= k - s:\n                    accepted.append((j, seen))", "a satisfied neighbour with nothing new is averaged"),
    ("protocol.py", "return satisfied >= len(self.in_nbrs[i]) - self.b, accepted",
     "return satisfied >= len(self.in_nbrs[i]) - self.b - 1, accepted", "one backup worker too many"),
    ("protocol.py", "return satisfied >= len(self.in_nbrs[i]) - self.b, accepted",
     "return satisfied >= len(self.in_nbrs[i]), accepted", "backup workers ignored"),
    ("protocol.py", "if seen >= k - s:\n                    satisfied += 1", "if seen > k - s:\n                    satisfied += 1",
     "staleness bound off by one"),
    ("protocol.py", "new = max(q) if q else None", "new = min(q) if q else None", "oldest instead of newest update"),
    ("arith.py", "f = float(t - (k - s) + 1) if s >= 1 else 1.0", "f = float(t - (k - s)) if s >= 1 else 1.0", "Eq. 2 without its + 1"),
    ("arith.py", "r.append(float(W[j][i]) * f)", "r.append(f)", "mixing weight dropped from the product"),
    ("protocol.py", "J = min(behind, self.max_skip, self.max_ig, self.K - k0)", "J = min(behind + 1, self.max_skip, self.max_ig, self.K - k0)",
     "jump lands one past the slowest neighbour"),
    ("protocol.py", "J = min(behind, self.max_skip, self.max_ig, self.K - k0)", "J = min(behind, 2, self.max_ig, self.K - k0)",
     "max_skip not the stated default"),
    ("protocol.py", "self._emit(JUMP, i, kp - 1, kp, (k0 + 1) % D, acc2, kp % D, T)", "self._emit(JUMP, i, kp - 1, kp, k0 % D, acc2, kp % D, T)",
     "the jump averages x_k0 instead of the fresh x_{k0+1}"),
    ("protocol.py", "ok2, acc2 = self._recv_eval(i, kp - 1)", "ok2, acc2 = self._recv_eval(i, kp)", "the jump receives iteration k instead of k - 1"),
    ("protocol.py", "self.tokens[(i, j)] += J - 1", "self.tokens[(i, j)] += J", "a jump hands out one token too many"),
    ("protocol.py", "if behind > self.trigger:", "if behind > self.trigger + 2:", "trigger not the stated default"),
]
# (Keeping stale tags queued in exact-tag mode changes no record of these two traces; the queue model fed
# from a trace in test_oracle_protocol.py is what catches that one.)


@pytest.mark.parametrize("fname,old,new,what", MISTAKES, ids=[m[3] for m in MISTAKES])
def test_planted_mistake_fails_a_hand_trace(tmp_path, fname, old, new, what):
    """A copy of oracle/ with one plausible mistake planted (on the CPU, in the copy only) must be caught by the
    hand-worked traces: an assertion of the comparison, or of the copy's own invariant checks."""
    pkg = "oracle_planted_%d" % (abs(hash(what)) % 10 ** 8)
    dst = tmp_path / pkg
    shutil.copytree(os.path.join(ROOT, "oracle"), dst, ignore=shutil.ignore_patterns("__pycache__"))
    path = dst / fname
    text = path.read_text()
    assert text.count(old) == 1, "the oracle changed: update the planted mistake '%s'" % what
    path.write_text(text.replace(old, new))
    sys.path.insert(0, str(tmp_path))
    try:
        protocol = importlib.import_module(pkg + ".protocol")
        rng = importlib.import_module(pkg + ".rng")
        with pytest.raises((AssertionError, protocol.ProtocolError, KeyError, IndexError)):
            both_traces(protocol, rng)
    finally:
        sys.path.remove(str(tmp_path))
        for m in [m for m in sys.modules if m.startswith(pkg)]:
            del sys.modules[m]


def test_the_unplanted_copy_passes(tmp_path):
    """The same machinery on an untouched copy: the failures above come from the mistakes."""
    dst = tmp_path / "oracle_copy_clean"
    shutil.copytree(os.path.join(ROOT, "oracle"), dst, ignore=shutil.ignore_patterns("__pycache__"))
    sys.path.insert(0, str(tmp_path))
    try:
        both_traces(importlib.import_module("oracle_copy_clean.protocol"), importlib.import_module("oracle_copy_clean.rng"))
    finally:
        sys.path.remove(str(tmp_path))
        for m in [m for m in sys.modules if m.startswith("oracle_copy_clean")]:
            del sys.modules[m]
