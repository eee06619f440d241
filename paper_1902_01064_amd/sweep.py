"""Heterogeneity sweeps in simulated time with the library's host simulator (no GPU needed).

Re-runs the settings of the paper's Section 7.3 as far as the protocol alone decides them: how long
an iteration takes on average when workers are slowed down at random (6x with probability 1/n per
iteration, Section 7.3.1) or one worker is 4x slower (Section 7.3.5), with and without backup
workers, bounded staleness and skipping.  Only time is simulated: there is no model and no loss,
so the figures to hold against the paper are its per-iteration speed ratios (up to 1.81x for one
backup worker; the straggler's 3.9x slowdown cut to about 1.1x by skipping), not its loss curves.

    python -m paper_1902_01064_amd.sweep
"""
import numpy as np

from . import hop, inputs

TICKS = float(1 << 20)


def mean_iteration_time(in_nbrs, s, b, K, kind, mult=None, seed=1, max_ig=0, skip_on=False, max_skip=10,
                        exclude=()):
    """Simulated time units per iteration: latest finish time over the workers not in `exclude`,
    divided by K.  Returns (time per iteration, number of jumps, stalled)."""
    n = len(in_nbrs)
    row_ptr, col = inputs.to_csr(in_nbrs)
    o = hop.make_opts(max_ig=max_ig, skip_on=skip_on, max_skip=max_skip, trigger=1, seed=seed)
    ctx = hop.hop_init(row_ptr, col, inputs.uniform_weights(in_nbrs), n, 4, s, b, o)
    try:
        sched = hop.hop_simulate(ctx, K, kind, mult)
        ft = [float(t) for i, t in enumerate(sched.finish_time) if i not in exclude]
        out = (max(ft) / TICKS / K, int(sched.n_jumps), bool(sched.stalled))
        sched.free()
        return out
    finally:
        hop.hop_destroy(ctx)


def random_slowdown_table(n=16, K=400, seeds=(1, 2, 3)):
    """Rows: graph, setting, mean time per iteration, speed-up over standard on the same graph."""
    rows = []
    graphs = (("ring", inputs.ring(n)), ("ring-based", inputs.ring_based(n)), ("double-ring", inputs.double_ring(n)))
    settings = (("standard", dict(s=0, b=0)), ("no slowdown", dict(s=0, b=0, kind=hop.HOP_DELAY_NONE)),
                ("1 backup worker", dict(s=0, b=1, max_ig=5)), ("staleness 5", dict(s=5, b=0)),
                ("backup + staleness 5", dict(s=5, b=1)))
    for gname, nb in graphs:
        base = None
        for sname, kw in settings:
            kw = dict(kw)
            kind = kw.pop("kind", hop.HOP_DELAY_BERNOULLI6)
            t = float(np.mean([mean_iteration_time(nb, K=K, kind=kind, seed=sd, **kw)[0] for sd in seeds]))
            if sname == "standard":
                base = t
            rows.append((gname, sname, t, base / t))
    return rows


def straggler_table(n=16, K=400, factor=4.0):
    """One worker `factor` times slower on the ring-based graph (Section 7.3.5): time per iteration
    of the other workers, relative to a run without the straggler."""
    nb = inputs.ring_based(n)
    mult = [1.0] * n
    mult[n // 3] = factor
    rows = []
    for name, kw in (("standard", dict(s=0, b=0)),
                     ("1 backup worker, max_ig 10", dict(s=0, b=1, max_ig=10)),
                     ("backup + skip at most 2", dict(s=0, b=1, max_ig=10, skip_on=True, max_skip=2)),
                     ("backup + skip at most 10", dict(s=0, b=1, max_ig=10, skip_on=True, max_skip=10)),
                     ("staleness 5 + skip at most 10", dict(s=5, b=0, max_ig=10, skip_on=True, max_skip=10))):
        t, jumps, stalled = mean_iteration_time(nb, K=K, kind=hop.HOP_DELAY_NONE, mult=mult,
                                                exclude=(n // 3,), **kw)
        rows.append((name, t, jumps, stalled))
    return rows


def main():
    print("random slowdown: every worker 6x slower with probability 1/16 per iteration, 16 workers")
    print("%-12s %-22s %12s %10s" % ("graph", "setting", "time/iter", "speed-up"))
    for g, s, t, sp in random_slowdown_table():
        print("%-12s %-22s %12.3f %10.2f" % (g, s, t, sp))
    print()
    print("one worker 4x slower, ring-based graph, 16 workers (time per iteration of the other 15)")
    print("%-32s %12s %8s" % ("setting", "time/iter", "jumps"))
    for name, t, jumps, stalled in straggler_table():
        print("%-32s %12.3f %8d%s" % (name, t, jumps, "  (stalled)" if stalled else ""))


if __name__ == "__main__":
    main()
