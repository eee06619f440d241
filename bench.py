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


def cpu_baseline(c, recs, p0, budget_s=20.0):
    """The oracle as it stands, timed on this host on the first records of the same schedule at
    full d.  Rings are built lazily (every slot 0 is p0) so the sample needs no 16 GB of host RAM."""
    import numpy as np

    from oracle import arith
    p0n = p0.cpu().numpy()
    slots = {}

    def get(j, sl):
        if (j, sl) in slots:
            return slots[(j, sl)]
        assert sl == 0, "sample reaches past the first versions"
        return p0n
    grad = arith.GradSynth(c["seed"], c["grad_var"], np.arange(c["d"])) if c["model"] == "synth" else None
    done, t0 = 0, time.perf_counter()
    for r in recs:
        if r.kind != 0:
            continue
        vecs = [get(j, sl) for j, sl in zip(r.src_worker, r.src_slot)]
        g = grad(r.worker, r.k, vecs[0]) if grad is not None else None
        slots[(r.worker, r.out_slot)] = arith.reduce_apply(vecs, r.w32, g, c["lr"])
        done += 1
        if time.perf_counter() - t0 > budget_s or done >= 28:
            break
    dt = time.perf_counter() - t0
    return {"value": done / dt, "unit": "worker-updates/s", "cores": 1, "kind": "oracle",
            "sample": "first %d STEP records of the same schedule at full d=%d (numpy, fp64 accumulate), %.1f s"
                      % (done, c["d"], dt)}


def run_config(cfgn, steps, warmup, graph, over=None):
    """Sets one workload up on cuda:0, times `steps` passes, returns (result dict, config, p0)."""
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
        else:
            hop.hop_set_grad_source(sess.ctx, hop.HOP_GRAD_SYNTH, c["grad_var"])
        sess.set_params(p0)
        sched = sess.simulate()
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
            "mix": {"ms": mix_ms, "launches": int(mix_n), "bytes": mix_bytes, "GBps": rate(mix_bytes, mix_ms)},
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
    res, c, p0 = run_config(args.config, args.steps, args.warmup, args.graph, over or None)
    mix = res["mix"]
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
        "roofline": {
            "bound": "hbm", "kernel": "mix_kernel", "achieved": mix["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": mix["GBps"] / HBM_PEAK_GBS,
            "traffic": None if over else read_traffic("hop_mix_cfg%d_traffic.txt" % args.config),
            "launches": mix["launches"], "avg_launch_us": mix["ms"] * 1e3 / max(mix["launches"], 1),
            "algorithmic_bytes_per_launch": mix["bytes"] / max(mix["launches"], 1),
        },
        "kernels": {k: {kk: vv for kk, vv in res[k].items() if kk != "bytes"} for k in ("mix", "grad", "synth")},
    }
    r = out["roofline"]
    if r["traffic"] and r["avg_launch_us"] > 0:
        # the same launches seen from the HBM side: counter bytes over the measured duration
        r["traffic_GBps"] = r["traffic"] / (r["avg_launch_us"] * 1e-6) / 1e9
        r["traffic_frac"] = r["traffic_GBps"] / HBM_PEAK_GBS
    if not args.no_cpu_baseline:
        from oracle import protocol
        if c["model"] == "synth" and not args.momentum:
            h = protocol.Hop(c["in_nbrs"], c["W"], c["s"], c["b"], c["K"], max_ig=c["max_ig"],
                             skip_on=c["skip_on"], max_skip=c["max_skip"], trigger=c["trigger"], seed=c["seed"],
                             delay_kind=c["delay_kind"], mult=c["mult"], check=False)
            out["cpu_baseline"] = cpu_baseline(c, h.run(), p0)
        else:
            out["cpu_baseline"] = None
    del p0
    if not args.no_others and not over:
        others = {}
        for n in (1, 2, 3, 5):
            if n == args.config:
                continue
            r, _, _ = run_config(n, 2, 1, True)
            others[r["config"]["workload"]] = {
                "worker_updates_per_s": r["value"], "ms_per_step": r["ms_per_step"], "launch": r["config"]["launch"],
                "records": r["config"]["step_records"] + r["config"]["jump_records"], "waves": r["config"]["waves"],
                "mix_GBps": r["mix"]["GBps"], "grad_GBps": r["grad"]["GBps"]}
        out["other_configs"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
