"""Host side of libhop.so without a GPU: exported symbols, argument checking, and the
library's own protocol simulator against the oracle, bit for bit."""
import ctypes
import os
import random
import re

import numpy as np
import pytest

from oracle import protocol, rng, waves
from paper_1902_01064_amd import hop, inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hop.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hop_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = hop.load()
    names = declared_functions()
    assert len(names) >= 25
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(hop.EXPORTS) == names
    assert hop.hop_version() >= 1
    assert hop.hop_strerror(hop.HOP_ERR_BAD_BACKUP).startswith("backup")


def code(fn):
    with pytest.raises(hop.HopError) as e:
        fn()
    return e.value.code


def host_ctx(c, **over):
    row_ptr, col = inputs.to_csr(c["in_nbrs"])
    o = hop.make_opts(max_ig=c["max_ig"], skip_on=c["skip_on"], max_skip=c["max_skip"],
                      trigger=c["trigger"], lr=c["lr"], lam=c["lam"], batch=c["batch"], seed=c["seed"],
                      max_latency=c.get("max_latency", 0), serial=c.get("serial", False),
                      notify_ack=c.get("notify_ack", False))
    ctx = hop.hop_init(row_ptr, col, c["W"], c["N"], c["d"], c["s"], c["b"], o)
    for i in range(c["N"]):
        if c["batch"]:
            hop.hop_set_rows(ctx, i, c["rows"])
    return ctx


def oracle_run(c, K):
    h = protocol.Hop(c["in_nbrs"], c["W"], c["s"], c["b"], K, max_ig=c["max_ig"], skip_on=c["skip_on"],
                     max_skip=c["max_skip"], trigger=c["trigger"], seed=c["seed"],
                     delay_kind=c["delay_kind"], mult=c["mult"], check=False,
                     max_latency=c.get("max_latency", 1), serial=c.get("serial", False),
                     notify_ack=c.get("notify_ack", False))
    return h, h.run()


def assert_same_schedule(c, sched, h, recs, K):
    assert sched.n_records == len(recs) and sched.depth == h.slots
    assert sched.stalled == h.stalled and sched.n_jumps == h.n_jumps and sched.late_sends == h.late_sends
    assert list(sched.kind) == [r.kind for r in recs]
    assert list(sched.worker) == [r.worker for r in recs]
    assert list(sched.iter) == [r.k for r in recs]
    assert list(sched.time) == [r.time for r in recs]
    assert list(sched.out_slot) == [r.out_slot for r in recs]
    assert list(sched.src_begin) == list(np.cumsum([0] + [len(r.src_worker) for r in recs]))
    assert list(sched.src_worker) == [j for r in recs for j in r.src_worker]
    assert list(sched.src_tag) == [t for r in recs for t in r.src_tag]
    assert list(sched.src_slot) == [t for r in recs for t in r.src_slot]
    w_ref = np.concatenate([r.w32 for r in recs]) if recs else np.zeros(0, np.float32)
    assert np.array_equal(sched.src_weight.view(np.uint32), w_ref.view(np.uint32))   # bit-exact fp32
    assert list(sched.final_iter) == h.Iter
    assert list(sched.finish_time) == [t or 0 for t in h.finish_time]
    wv = waves.assign_waves(recs, h.N, h.slots)
    assert list(sched.wave) == wv
    assert waves.check_waves(recs, list(sched.wave), h.N, h.slots)
    assert sched.n_waves == (max(wv) + 1 if wv else 0)
    order = list(sched.wave_order)
    assert sorted(order) == list(range(len(recs)))
    for w in range(sched.n_waves):
        seg = order[sched.wave_begin[w]:sched.wave_begin[w + 1]]
        assert seg == sorted(seg) and all(sched.wave[e] == w for e in seg)
    if c["batch"]:
        assert sched.batch == c["batch"]
        for e in random.Random(0).sample(range(len(recs)), min(40, len(recs))):
            r = recs[e]
            want = rng.batch_rows(c["seed"], r.worker, r.k, c["batch"], c["rows"]) \
                if r.kind in (protocol.STEP, protocol.APPLY) else np.zeros(c["batch"], np.int64)
            assert np.array_equal(sched.batch_rows[e], want)


@pytest.mark.parametrize("cfgn", [1, 2, 3, 4, 5])
def test_schedule_is_bit_exact_at_full_size(cfgn):
    c = inputs.config(cfgn)
    ctx = host_ctx(c)
    sched = hop.hop_simulate(ctx, c["K"], c["delay_kind"], c["mult"])
    h, recs = oracle_run(c, c["K"])
    assert_same_schedule(c, sched, h, recs, c["K"])
    assert not sched.stalled
    sched.free()
    hop.hop_destroy(ctx)


def test_schedule_is_bit_exact_in_random_modes():
    rnd = random.Random(11)
    graphs = [inputs.ring(5), inputs.torus(3, 3), inputs.complete(4),
              inputs.ring_with_chords(8, 1, 11), inputs.directed_cycle([0, 3, 1, 4, 2])]
    for trial in range(80):
        nb = rnd.choice(graphs)
        s = rnd.choice([0, 0, 1, 2, 4])
        b = rnd.randrange(0, min(len(l) for l in nb))
        c = dict(in_nbrs=nb, W=inputs.uniform_weights(nb), N=len(nb), d=8, s=s, b=b,
                 max_ig=rnd.choice([0, 0, 1, 2, 5]), skip_on=rnd.random() < 0.5,
                 max_skip=rnd.choice([2, 10]), trigger=rnd.choice([0, 1, 2]), lr=0.1, lam=0.0,
                 batch=rnd.choice([0, 4]), rows=37, seed=trial, delay_kind=rnd.choice([0, 1, 2]),
                 mult=[rnd.choice([1.0, 1.0, 2.5, float(1 << 62)]) if rnd.random() < 0.3 else 1.0
                       for _ in nb])
        ctx = host_ctx(c)
        sched = hop.hop_simulate(ctx, 14, c["delay_kind"], c["mult"])
        h, recs = oracle_run(c, 14)
        assert_same_schedule(c, sched, h, recs, 14)
        sched.free()
        hop.hop_destroy(ctx)


def test_serial_and_notify_ack_schedules_are_bit_exact():
    """The two comparison options (Sections 3.2 and 3.3) in the library's simulator against the oracle: record
    kinds, times, slots (the serial approach's current-parameter slot included), weights, waves, minibatches,
    stalls with frozen workers."""
    rnd = random.Random(23)
    graphs = [inputs.ring(5), inputs.torus(3, 3), inputs.complete(4),
              inputs.ring_with_chords(8, 1, 11), inputs.directed_cycle([0, 3, 1, 4, 2])]
    kinds = set()
    for trial in range(60):
        nb = rnd.choice(graphs)
        serial = trial % 2 == 0
        s = rnd.choice([0, 0, 1, 3]) if serial else 0
        b = rnd.randrange(0, min(len(l) for l in nb)) if serial else 0
        c = dict(in_nbrs=nb, W=inputs.uniform_weights(nb), N=len(nb), d=8, s=s, b=b,
                 max_ig=rnd.choice([0, 0, 2, 5]), skip_on=serial and rnd.random() < 0.5,
                 max_skip=rnd.choice([2, 10]), trigger=rnd.choice([0, 1]), lr=0.1, lam=0.0,
                 batch=rnd.choice([0, 4]), rows=37, seed=500 + trial, delay_kind=rnd.choice([0, 1, 2]),
                 mult=[rnd.choice([1.0, 1.0, 2.5, float(1 << 62)]) if rnd.random() < 0.3 else 1.0 for _ in nb],
                 serial=serial, notify_ack=not serial)
        ctx = host_ctx(c)
        sched = hop.hop_simulate(ctx, 12, c["delay_kind"], c["mult"])
        h, recs = oracle_run(c, 12)
        assert_same_schedule(c, sched, h, recs, 12)
        kinds.update(r.kind for r in recs)
        sched.free()
        hop.hop_destroy(ctx)
    assert kinds == {protocol.STEP, protocol.JUMP, protocol.APPLY, protocol.REDUCE}
    # NOTIFY-ACK with anything it cannot support is refused
    nb = inputs.ring(4)
    row_ptr, col = inputs.to_csr(nb)
    for kw, s, b in ((dict(), 1, 0), (dict(), 0, 1), (dict(skip_on=True), 0, 0), (dict(serial=True), 0, 0),
                     (dict(max_latency=5), 0, 0)):
        o = hop.make_opts(notify_ack=True, **kw)
        assert code(lambda: hop.hop_init(row_ptr, col, inputs.uniform_weights(nb), 4, 8, s, b, o)) == hop.HOP_ERR_INVALID_ARG


def test_delay_table_and_frozen_worker_stall():
    nb = inputs.complete(3)
    c = dict(in_nbrs=nb, W=inputs.uniform_weights(nb), N=3, d=4, s=0, b=1, max_ig=2, skip_on=False,
             max_skip=10, trigger=1, lr=0.1, lam=0.0, batch=0, rows=0, seed=1)
    ctx = host_ctx(c)
    table = np.full((3, 10), 1 << 20, dtype=np.uint64)
    table[0, :] = hop.HOP_TICKS_NEVER
    sched = hop.hop_simulate(ctx, 10, hop.HOP_DELAY_TABLE, None, table)
    assert sched.rc == hop.HOP_ERR_DEADLOCK and sched.stalled
    assert list(sched.final_iter) == [0, 2, 2]            # stopped by the token queues at max_ig
    h = protocol.Hop(nb, c["W"], 0, 1, 10, max_ig=2, delay_kind=rng.DELAY_TABLE, table=table, check=True)
    recs = h.run()
    assert_same_schedule(c, sched, h, recs, 10)
    sched.free()
    hop.hop_destroy(ctx)


def test_argument_checking():
    nb = inputs.ring(4)
    row_ptr, col = inputs.to_csr(nb)
    W = inputs.uniform_weights(nb)
    o = hop.make_opts()

    assert code(lambda: hop.hop_init(row_ptr, col, W, 4, 8, 1, 2, o)) == hop.HOP_ERR_BAD_BACKUP
    # two separate pairs, and a one-way chain 0 -> 1 -> 2: no path between every two nodes
    for nb2 in ([[1], [0], [3], [2]], [[], [0], [1]]):
        rp2, col2 = inputs.to_csr(nb2)
        assert code(lambda: hop.hop_init(rp2, col2, inputs.uniform_weights(nb2), len(nb2), 8, 1, 0, o)) == hop.HOP_ERR_BAD_GRAPH
    off = W.copy()
    off[0, 0] += 3e-6                                      # a column that sums to 1 + 3e-6
    assert code(lambda: hop.hop_init(row_ptr, col, off, 4, 8, 1, 0, o)) == hop.HOP_ERR_BAD_WEIGHTS
    bad = col.copy()
    bad[0] = 0                                             # self edge at node 0
    assert code(lambda: hop.hop_init(row_ptr, bad, W, 4, 8, 1, 0, o)) == hop.HOP_ERR_BAD_GRAPH
    W2 = W.copy()
    W2[0, 0] = 0.5
    assert code(lambda: hop.hop_init(row_ptr, col, W2, 4, 8, 1, 0, o)) == hop.HOP_ERR_BAD_WEIGHTS
    W3 = W.copy()
    W3[2, 0] = 0.1                                         # weight on a non-edge
    assert code(lambda: hop.hop_init(row_ptr, col, W3, 4, 8, 1, 0, o)) == hop.HOP_ERR_BAD_WEIGHTS
    assert code(lambda: hop.hop_init(row_ptr, col, W, 4, 0, 1, 0, o)) == hop.HOP_ERR_INVALID_ARG
    ctx = hop.hop_init(row_ptr, col, W, 4, 8, 1, 0, o)
    sched = hop.hop_simulate(ctx, 3)
    assert code(lambda: hop.hop_step(ctx, sched)) == hop.HOP_ERR_NO_DEVICE
    assert code(lambda: hop.hop_params(ctx, 0)) == hop.HOP_ERR_NO_DEVICE
    assert code(lambda: hop.hop_set_rows(ctx, 9, 1)) == hop.HOP_ERR_INVALID_ARG
    assert hop.hop_layout(1 << 20, 3, o) == (4, (1 << 20) + 64)
    assert hop.hop_layout(100, 0, hop.make_opts(max_ig=3)) == (5, 192)
    need = hop.hop_arena_bytes(4, 8, 1, 0, o)
    ahead = hop.make_opts(grad_ahead=4)
    depth, stride = hop.hop_layout(8, 1, ahead)
    assert hop.hop_arena_bytes(4, 8, 1, 0, ahead) == need + 3 * 4 * stride * 4        # three more gradient buffers per worker
    assert hop.hop_arena_bytes(4, 8, 1, 0, hop.make_opts(grad_ahead=17)) == 0 and hop.hop_arena_bytes(4, 8, 1, 0, hop.make_opts(grad_ahead=-1)) == 0
    assert need >= 4 * (2 + 1) * 8 * 4
    sched.free()
    hop.hop_destroy(ctx)


def test_schedule_may_outlive_its_context():
    """A schedule is host data: freeing it after hop_destroy of its context must be harmless, and
    several schedules of one context can be freed in any order."""
    c = inputs.config(1)
    ctx = host_ctx(c)
    a = hop.hop_simulate(ctx, 5, c["delay_kind"], c["mult"])
    b = hop.hop_simulate(ctx, 7, c["delay_kind"], c["mult"])
    keep = list(b.iter)
    a.free()
    hop.hop_destroy(ctx)
    assert list(b.iter) == keep and b.n_records == 4 * 7
    b.free()
