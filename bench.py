"""Benchmark of the Hop hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4]

A step is one pass of the whole hot path over the workload's schedule: every wave of
hop_step (gradient kernels + fused Reduce/Apply) for all iterations of all workers.  The
default workload is config 4 of the synthetic suite: 32 workers on a ring with chords,
Metropolis weights, staleness 4, one backup worker, two 3x stragglers with skipping,
d = 25 000 000 fp32 parameters per replica, synthetic gradients, 100 iterations.
Inputs (initial replicas, data, schedule, job descriptors) are resident in HBM before the
timed region.  Prints ONE JSON line; the other four configs of the suite are run briefly
afterwards and reported under "other_configs" (not part of value).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "worker-updates/sec and mixing-kernel HBM GB/s (% of peak) at N workers, d params"


def read_traffic(name):
    """HBM bytes per launch measured with rocprofv3 counters, if a summary has been committed."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        line = line.split("#", 1)[0].strip()
        if "=" in line:
            k, v = line.split("=", 1)
            vals[k.strip()] = v.strip()
    try:
        return float(vals["fetch_bytes_per_launch"]) + float(vals["write_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def _oracle_slice(args):
    """The oracle's Reduce + Apply on the columns [lo, hi) of the first `n_records` STEP records (all of the
    method's arithmetic is separable by column, and the synthetic gradient can be generated per column)."""
    import numpy as np

    from oracle import arith
    c, recs, p0n, lo, hi, n_records = args
    p0s = p0n[lo:hi]
    slots = {}

    def get(j, sl):
        if (j, sl) in slots:
            return slots[(j, sl)]
        assert sl == 0, "sample reaches past the versions it has produced"
        return p0s
    grad = arith.GradSynth(c["seed"], c["grad_var"], np.arange(lo, hi))
    done = 0
    for r in recs:
        if r.kind != 0:
            continue
        vecs = [get(j, sl) for j, sl in zip(r.src_worker, r.src_slot)]
        slots[(r.worker, r.out_slot)] = arith.reduce_apply(vecs, r.w32, grad(r.worker, r.k, vecs[0]), c["lr"])
        done += 1
        if done >= n_records:
            break
    return done


def cpu_baseline(c, recs, p0):
    """The oracle as it stands (numpy, fp64 accumulation), timed on this host on the first STEP records of the
    same schedule at full d: on one core, then with the columns split over all the cores this process may use
    (at most 16, a one-GPU machine's share).  Runs before anything touches the GPU, so the worker processes can be
    plain forks."""
    import multiprocessing as mp

    p0n = p0.numpy()
    d = c["d"]
    t0 = time.perf_counter()
    one = _oracle_slice((c, recs, p0n, 0, d, 12))
    t_one = time.perf_counter() - t0
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:
        avail = os.cpu_count() or 1
    cores = max(1, min(avail, 16))
    n_all = 64
    bounds = [d * q // cores for q in range(cores + 1)]
    with mp.get_context("fork").Pool(cores) as pool:
        pool.map(_oracle_slice, [(c, recs, p0n, 0, 1024, 1)] * cores)          # start the workers before the clock
        t0 = time.perf_counter()
        done = pool.map(_oracle_slice, [(c, recs, p0n, bounds[q], bounds[q + 1], n_all) for q in range(cores)])
        t_all = time.perf_counter() - t0
    return {"value": done[0] / t_all, "unit": "worker-updates/s", "cores": cores, "kind": "oracle",
            "one_core_value": one / t_one, "host_cpu_count": os.cpu_count(),
            "sample": "first %d STEP records of the same schedule at full d=%d, columns split over %d processes, "
                      "%.1f s; one core: first %d records, %.1f s (numpy, fp64 accumulation)"
                      % (done[0], d, cores, t_all, one, t_one)}


def wave_compulsory_bytes(sched, d, mode, momentum):
    """HBM bytes one Reduce + Apply launch cannot avoid, per wave, from the schedule itself: every distinct
    (worker, slot) vector the wave reads once, one result per record, one gradient per STEP record where the
    kernel reads a dense one (synthetic, external), the velocity read and written.  With large dense minibatches
    ("dense_fused") the gradient kernel reduces its own records and the mix launch holds the jumps only."""
    import numpy as np
    out = np.zeros(int(sched.n_waves))
    for w in range(int(sched.n_waves)):
        members = sched.wave_order[sched.wave_begin[w]:sched.wave_begin[w + 1]]
        srcs = set()
        vectors = 0
        for e in members:
            if mode == "dense_fused" and sched.kind[e] in (0, 2):
                continue
            a0, a1 = int(sched.src_begin[e]), int(sched.src_begin[e + 1])
            srcs.update(zip(sched.src_worker[a0:a1].tolist(), sched.src_slot[a0:a1].tolist()))
            vectors += 1
            if sched.kind[e] == 0 and mode == "synth":
                vectors += 1 + (2 if momentum else 0)
        out[w] = 4.0 * d * (len(srcs) + vectors)
    return out


def run_config(cfgn, steps, warmup, graph, over=None, external=False):
    """Sets one workload up on cuda:0, times `steps` passes, returns (result dict, config, p0).
    external: gradients from a buffer the caller filled once (config 4 only), so no generator kernel runs."""
    import torch

    from paper_1902_01064_amd import hop, inputs
    from paper_1902_01064_amd.session import Session, make_data

    c = inputs.config(cfgn, **(over or {}))
    dev = "cuda:0"
    sess = Session(c, dev)
    try:
        p0, data = make_data(c, dev)
        if c["model"] == "dense":
            sess.set_dense(*data)
        elif c["model"] == "csr":
            sess.set_csr(data)
        elif external:
            gen = torch.Generator(device=dev)
            gen.manual_seed(c["seed"])
            gext = torch.randn(c["N"] * c["d"], generator=gen, device=dev, dtype=torch.float32) * (c["grad_var"] ** 0.5)
            hop.hop_set_grad_source(sess.ctx, hop.HOP_GRAD_EXTERNAL, 0.0, gext.data_ptr())
        else:
            hop.hop_set_grad_source(sess.ctx, hop.HOP_GRAD_SYNTH, c["grad_var"])
        sess.set_params(p0)
        sched = sess.simulate()
        mix_mode = "synth" if c["model"] == "synth" else ("dense_fused" if c["model"] == "dense" and c["batch"] * c["d"] * 4 > (2 << 20) else "none")
        compulsory = wave_compulsory_bytes(sched, c["d"], mix_mode, c.get("momentum", 0.0) > 0)
        n_step = int((sched.kind == hop.HOP_STEP).sum())
        n_jump = int((sched.kind == hop.HOP_JUMP).sum())
        A = (sched.src_begin[1:] - sched.src_begin[:-1])
        if graph:
            hop.hop_use_graph(sess.ctx, 1)
        for _ in range(warmup):
            sess.step()
        sess.sync()
        if not graph:
            hop.hop_profile(sess.ctx, 1)     # HIP events around every kernel group, inside the timed region
        sess.sync()
        t0 = time.perf_counter()
        for _ in range(steps):
            sess.step()
        sess.sync()
        t1 = time.perf_counter()
        if graph:                            # graph replays cannot be timed per kernel: one extra pass
            hop.hop_profile(sess.ctx, 1)
            sess.step()
            sess.sync()
        mix_ms, mix_n, mix_bytes = hop.hop_profile_read(sess.ctx, hop.HOP_KERNEL_MIX)
        grad_ms, grad_n, grad_bytes = hop.hop_profile_read(sess.ctx, hop.HOP_KERNEL_GRAD)
        syn_ms, syn_n, syn_bytes = hop.hop_profile_read(sess.ctx, hop.HOP_KERNEL_SYNTH)
        hop.hop_profile(sess.ctx, 0)
        elapsed = t1 - t0

        def rate(b, ms):
            return b / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        res = {
            "value": n_step * steps / elapsed,
            "ms_per_step": elapsed * 1e3 / steps,
            "config": {
                "workload": c["name"] + (" (config %d of the synthetic suite)" % cfgn),
                "N": c["N"], "d": c["d"], "s": c["s"], "b": c["b"], "iterations": c["K"], "seed": c["seed"],
                "step_records": n_step, "jump_records": n_jump, "waves": int(sched.n_waves),
                "mean_A": float(A.mean()), "min_A": int(A.min()), "max_A": int(A.max()),
                "records_per_wave": float(len(A)) / max(int(sched.n_waves), 1),
                "simulated_makespan_units": float(max(sched.finish_time)) / float(1 << 20),
                "step_definition": "one pass of hop_step over the whole schedule",
                "launch": "hip graph replay" if graph else "kernel by kernel",
            },
            "mix": {"ms": mix_ms, "launches": int(mix_n), "bytes": mix_bytes, "GBps": rate(mix_bytes, mix_ms),
                    "compulsory_bytes_per_pass": float(compulsory.sum()),
                    "passes_timed": 1 if graph else steps},
            "grad": {"ms": grad_ms, "launches": int(grad_n), "GBps": rate(grad_bytes, grad_ms)},
            "synth": {"ms": syn_ms, "launches": int(syn_n), "GBps": rate(syn_bytes, syn_ms)},
        }
        return res, c, p0
    finally:
        sess.close()
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--d", type=int, default=0, help="override the parameter count (not a valid bench line)")
    ap.add_argument("--momentum", type=float, default=0.0, help="per-worker momentum (not the default bench line)")
    ap.add_argument("--log-loss", action="store_true", help="log loss instead of hinge (SVM configs)")
    ap.add_argument("--seed", type=int, default=0, help="seed of graph, slow set, delays and data (default: the suite's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the brief runs of the other configs")
    ap.add_argument("--graph", action="store_true",
                    help="time HIP-graph replays of the pass (kernel figures then come from one extra, "
                         "untimed kernel-by-kernel pass)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="only run the plain copy kernel on BYTES (for scaling rocprofv3 traffic counters)")
    args = ap.parse_args()
    if args.copy_calibration:
        import torch
        from paper_1902_01064_amd import hop
        n = args.copy_calibration // 4
        a = torch.ones(n, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        for _ in range(5):
            hop.hop_copy(b.data_ptr(), a.data_ptr(), n * 4, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": n * 4, "launches": 5}))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    over = {"d": args.d} if args.d else {}
    if args.momentum:
        over["momentum"] = args.momentum
    if args.log_loss:
        over["loss"] = 1
    if args.seed:
        over["seed"] = args.seed
    cpu = None
    if not args.no_cpu_baseline:
        # the oracle first, while no GPU runtime is alive in this process (its all-cores leg forks workers)
        from oracle import protocol
        from paper_1902_01064_amd import inputs
        c0 = inputs.config(args.config, **over)
        if c0["model"] == "synth" and not args.momentum:
            h = protocol.Hop(c0["in_nbrs"], c0["W"], c0["s"], c0["b"], c0["K"], max_ig=c0["max_ig"],
                             skip_on=c0["skip_on"], max_skip=c0["max_skip"], trigger=c0["trigger"], seed=c0["seed"],
                             delay_kind=c0["delay_kind"], mult=c0["mult"], check=False)
            cpu = cpu_baseline(c0, h.run(), inputs.initial_params(c0["seed"], c0["d"], 0.01))
    res, c, p0 = run_config(args.config, args.steps, args.warmup, args.graph, over or None)
    del p0
    mix = res["mix"]
    launches = max(mix["launches"], 1)
    avg_us = mix["ms"] * 1e3 / launches
    compulsory = mix["compulsory_bytes_per_pass"] * mix["passes_timed"] / launches      # per launch
    hbm_GBps = compulsory / (avg_us * 1e-6) / 1e9 if avg_us > 0 else 0.0
    counters = None if over else read_traffic("hop_mix_cfg%d_traffic.txt" % args.config)
    note = None
    if counters is not None and abs(counters - compulsory) > 0.03 * compulsory:
        note = ("profiles/hop_mix_cfg%d_traffic.txt holds %.4g bytes per launch, the schedule of this run needs %.4g: "
                "the counter figure belongs to another schedule or kernel and is not quoted"
                % (args.config, counters, compulsory))
        counters = None
    out = {
        "metric": METRIC,
        "value": res["value"],
        "unit": "worker-updates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": res["config"],
        # HBM side: the bytes a launch cannot avoid (every distinct source of the wave once, one gradient and one
        # result per record; from this run's schedule) over the launch time measured in this run.  The rate at which
        # the records' 4 d (A + 2) bytes reach the CUs is higher (sources shared through L2) and is no HBM figure.
        "roofline": {
            "bound": "hbm", "kernel": "pair_mix_kernel", "achieved": hbm_GBps, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": hbm_GBps / HBM_PEAK_GBS,
            "traffic": counters,
            "launches": mix["launches"], "avg_launch_us": avg_us,
            "compulsory_bytes_per_launch": compulsory,
            "algorithmic_bytes_per_launch": mix["bytes"] / launches,
            "l2_side_GBps": mix["GBps"],
        },
        "kernels": {k: {kk: vv for kk, vv in res[k].items() if kk not in ("bytes", "compulsory_bytes_per_pass", "passes_timed")}
                    for k in ("mix", "grad", "synth")},
    }
    r = out["roofline"]
    grad = res["grad"]
    if grad["ms"] > res["mix"]["ms"] and c["model"] == "dense":
        # dense SVM configs: the gradient launches (margins; second pass + Reduce + Apply) are the dominant group;
        # their algorithmic bytes are the minibatch rows once plus the vectors of the record's Reduce and Apply
        n_g = max(grad["launches"], 1)
        us = grad["ms"] * 1e3 / n_g
        out["roofline"] = r = {
            "bound": "hbm",
            "kernel": ("dense_margin4_kernel + dense_grad_kernel (one group per wave)" if c["batch"] * c["d"] * 4 > (2 << 20)
                       else "pair_dense_margin_kernel + dense_grad_kernel (one group per wave; bound by launches)"),
            "achieved": grad["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": grad["GBps"] / HBM_PEAK_GBS,
            "traffic": None, "launches": grad["launches"], "avg_launch_us": us,
            "algorithmic_bytes_per_launch": grad["GBps"] * 1e9 * us * 1e-6,
        }
    if note:
        r["traffic_note"] = note
    if counters and avg_us > 0:
        r["traffic_GBps"] = counters / (avg_us * 1e-6) / 1e9
        r["traffic_frac"] = r["traffic_GBps"] / HBM_PEAK_GBS
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu
    if not args.no_others and not over:
        others = {}
        bound = {1: "launches (80 KB per wave)", 2: "gradient: hbm (its kernel also does the Reduce; a mix launch only for jumps)",
                 3: "launches (3.4 records of 4 MB per wave)", 4: "hbm", 5: "hbm"}
        for n in (1, 2, 3, 5):
            if n == args.config:
                continue
            r, _, _ = run_config(n, 2, 1, True)
            m = r["mix"]
            passes = max(m["passes_timed"], 1)
            n_launch = (m["launches"] + r["grad"]["launches"] + r["synth"]["launches"]) / passes
            others[r["config"]["workload"]] = {
                "worker_updates_per_s": r["value"], "ms_per_step": r["ms_per_step"], "launch": r["config"]["launch"],
                "records": r["config"]["step_records"] + r["config"]["jump_records"], "waves": r["config"]["waves"],
                "timed_kernel_groups_per_pass": n_launch, "bound": bound[n],
                "mix_l2_side_GBps": m["GBps"],
                "mix_hbm_GBps": m["compulsory_bytes_per_pass"] * passes / (m["ms"] * 1e-3) / 1e9 if m["ms"] > 0 else 0.0,
                "grad_GBps": r["grad"]["GBps"]}
        if args.config == 4:
            # the same schedule with gradients the caller provides: no arithmetic kernel runs in front of the mixes
            r, _, _ = run_config(4, 2, 1, False, external=True)
            m = r["mix"]
            n_l = max(m["launches"], 1)
            us = m["ms"] * 1e3 / n_l
            comp = m["compulsory_bytes_per_pass"] * m["passes_timed"] / n_l
            others["cfg4 with caller-provided gradients (no generator kernel between the mixes)"] = {
                "worker_updates_per_s": r["value"], "ms_per_step": r["ms_per_step"], "launch": r["config"]["launch"],
                "mix_avg_launch_us": us, "mix_hbm_GBps": comp / (us * 1e-6) / 1e9 if us > 0 else 0.0,
                "mix_hbm_frac": comp / (us * 1e-6) / 1e9 / HBM_PEAK_GBS if us > 0 else 0.0,
                "mix_l2_side_GBps": m["GBps"]}
        out["other_configs"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
