"""Out-of-order delivery (Section 6.1: "we do not assume network preserves the message order") and the
late-update counter of Section 6.2 (b).  No GPU."""
import random

import numpy as np
import pytest

from oracle import brute, protocol, rng, waves
from paper_1902_01064_amd import hop, inputs
from test_host_library import assert_same_schedule, host_ctx, oracle_run

UNIT = rng.TICKS_PER_UNIT


def run(nb, s, b, K, **kw):
    h = protocol.Hop(nb, inputs.uniform_weights(nb), s, b, K, **kw)
    h.run()
    return h


def test_updates_really_overtake_each_other_and_invariants_hold():
    nb = inputs.torus(3, 3)
    h = run(nb, 2, 1, 40, delay_kind=rng.DELAY_EXP1, seed=4, max_latency=2 * UNIT, check=True, trace=True)
    assert not h.stalled and h.D == 2 + 2 + 2                 # s + max_ig + 2
    last, overtakes = {}, 0
    for item in h.trace:
        if item[0] == "deliver":
            e = (item[1], item[2])
            overtakes += item[3] < last.get(e, -1)
            last[e] = max(last.get(e, -1), item[3])
    assert overtakes > 10
    # whatever the order of arrival, a receiver never goes back to an older update of a neighbour
    used = {}
    for r in h.records:
        for j, t in zip(r.src_worker[1:], r.src_tag[1:]):
            assert t > used.get((j, r.worker), -1)
            used[(j, r.worker)] = t
    wv = waves.assign_waves(h.records, h.N, h.D)
    assert waves.check_waves(h.records, wv, h.N, h.D)


def test_ring_depth_covers_the_oldest_tag_that_can_be_taken():
    """With reordering a reader in iteration k can take tag k - s while the sender has produced
    k + max_ig + 1: no version that is read may have been overwritten (SlotDead would raise), across
    many seeds, and the paper's #queues = max_ig + 1 would not be enough."""
    nb = inputs.ring(6)
    span = 0
    for seed in range(40):
        h = run(nb, 3, 0, 30, delay_kind=rng.DELAY_EXP1, seed=seed, max_latency=4 * UNIT,
                mult=[1, 1, 4, 1, 1, 1], check=True)
        newest = [0] * h.N
        for r in h.records:
            for j, t in zip(r.src_worker[1:], r.src_tag[1:]):
                span = max(span, newest[j] - t)
            newest[r.worker] = r.k + 1 if r.kind == protocol.STEP else r.k
    assert span >= 4                                          # beyond what max_ig + 1 = 4 slots could hold
    assert span < 3 + 3 + 2


@pytest.mark.parametrize("lat", [UNIT // 2, 3 * UNIT])
def test_library_matches_oracle_bit_for_bit_under_reordering(lat):
    rnd = random.Random(lat)
    graphs = [inputs.ring(5), inputs.torus(3, 3), inputs.complete(4), inputs.directed_cycle([0, 3, 1, 4, 2])]
    for trial in range(40):
        nb = rnd.choice(graphs)
        s = rnd.choice([0, 1, 2, 4])
        b = rnd.randrange(0, min(len(l) for l in nb))
        c = dict(in_nbrs=nb, W=inputs.uniform_weights(nb), N=len(nb), d=8, s=s, b=b,
                 max_ig=rnd.choice([0, 2, 5]), skip_on=rnd.random() < 0.5 and (s > 0 or b > 0),
                 max_skip=rnd.choice([2, 10]), trigger=1, lr=0.1, lam=0.0, batch=0, rows=0, seed=trial,
                 delay_kind=rnd.choice([0, 1, 2]), mult=[rnd.choice([1.0, 1.0, 3.0]) for _ in nb],
                 max_latency=lat)
        ctx = host_ctx(c)
        sched = hop.hop_simulate(ctx, 14, c["delay_kind"], c["mult"])
        h, recs = oracle_run(c, 14)
        assert_same_schedule(c, sched, h, recs, 14)
        sched.free()
        hop.hop_destroy(ctx)


def test_late_sends_are_never_used_in_exact_tag_mode():
    """Section 6.2 (b): an update whose receiver is already past its iteration is stale on arrival; in
    exact-tag mode it is dropped at the next dequeue, so not sending it would change nothing."""
    nb = inputs.complete(4)
    h = run(nb, 0, 2, 40, max_ig=4, delay_kind=rng.DELAY_EXP1, seed=2, mult=[1, 1, 1, 5], check=True, trace=True)
    assert h.late_sends > 0
    it, late = [0] * 4, set()
    for item in h.trace:
        if item[0] == "enter":
            i, k = item[1], item[2]
            it[i] = k
            if k < 40:
                late |= {(i, j, k) for j in nb[i] if it[j] > k}
    assert len(late) == h.late_sends
    for r in h.records:
        for j, t in zip(r.src_worker[1:], r.src_tag[1:]):
            assert (j, r.worker, t) not in late


UNORDERED = [(inputs.ring(2), 2, 0, 3, 2, True), (inputs.ring(3), 0, 0, 3, 2, False),
             (inputs.complete(3), 0, 1, 2, 2, False)]


@pytest.mark.parametrize("case", range(len(UNORDERED)))
def test_every_timed_run_is_a_walk_of_the_unordered_model(case):
    nb, s, b, K, ig, skip = UNORDERED[case]
    m = brute.Model(nb, s, b, K, max_ig=ig, skip_on=skip, ordered=False)
    seen, stuck, _ = m.explore(limit=600_000)
    assert not stuck
    for state in seen:
        it, ph, flight, queue, rcv, tok = state
        for x, (j, i) in enumerate(m.edges):
            assert tok[x] == it[i] - it[j] + m.ig >= 0
    for seed in range(8):
        h = protocol.Hop(nb, inputs.uniform_weights(nb), s, b, K, max_ig=ig, skip_on=skip, seed=seed,
                         delay_kind=rng.DELAY_EXP1, max_latency=2 * UNIT, check=True, trace=True)
        h.run()
        assert not h.stalled
        end = m.replay(h.trace)
        assert end in seen and m.final(end)
