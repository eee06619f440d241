"""Benchmark of the Hop hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4]

A step is one pass of the whole hot path over the workload's schedule: every wave of
hop_step (gradient kernels + fused Reduce/Apply) for all iterations of all workers.  The
default workload is config 4 of the synthetic suite: 32 workers on a ring with chords,
Metropolis weights, staleness 4, one backup worker, two 3x stragglers with skipping,
d = 25 000 000 fp32 parameters per replica, synthetic gradients, 100 iterations.
Inputs (initial replicas, schedule, job descriptors) are resident in HBM before the
timed region.  Prints ONE JSON line.
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
        if time.perf_counter() - t0 > budget_s or done >= 16:
            break
    dt = time.perf_counter() - t0
    return {"value": done / dt, "unit": "worker-updates/s", "cores": 1, "kind": "oracle",
            "sample": "first %d STEP records of the same schedule at full d=%d (numpy, fp64 accumulate), %.1f s"
                      % (done, c["d"], dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--d", type=int, default=0, help="override the parameter count (not a valid bench line)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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

    import torch

    from oracle import protocol
    from paper_1902_01064_amd import hop, inputs
    from paper_1902_01064_amd.session import Session, make_data

    over = {"d": args.d} if args.d else {}
    c = inputs.config(args.config, **over)
    dev = "cuda:0"
    sess = Session(c, dev)
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

    if args.graph:
        hop.hop_use_graph(sess.ctx, 1)
    for _ in range(args.warmup):
        sess.step()
    sess.sync()
    if not args.graph:
        hop.hop_profile(sess.ctx, 1)
    sess.sync()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sess.step()
    sess.sync()
    t1 = time.perf_counter()
    if args.graph:
        hop.hop_profile(sess.ctx, 1)
        sess.step()
        sess.sync()
    mix_ms, mix_n, mix_bytes = hop.hop_profile_read(sess.ctx, hop.HOP_KERNEL_MIX)
    grad_ms, grad_n, grad_bytes = hop.hop_profile_read(sess.ctx, hop.HOP_KERNEL_GRAD)
    syn_ms, syn_n, syn_bytes = hop.hop_profile_read(sess.ctx, hop.HOP_KERNEL_SYNTH)
    hop.hop_profile(sess.ctx, 0)

    elapsed = t1 - t0
    achieved = mix_bytes / (mix_ms * 1e-3) / 1e9 if mix_ms > 0 else 0.0
    out = {
        "metric": "worker-updates/sec and mixing-kernel HBM GB/s (% of peak) at N workers, d params",
        "value": n_step * args.steps / elapsed,
        "unit": "worker-updates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": c["name"] + (" (config %d of the synthetic suite)" % args.config),
            "N": c["N"], "d": c["d"], "s": c["s"], "b": c["b"], "iterations": c["K"],
            "step_records": n_step, "jump_records": n_jump, "waves": int(sched.n_waves),
            "mean_A": float(A.mean()), "max_A": int(A.max()),
            "step_definition": "one pass of hop_step over the whole schedule",
            "launch": "hip graph replay" if args.graph else "kernel by kernel",
        },
        "roofline": {
            "bound": "hbm", "kernel": "mix_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": read_traffic("hop_mix_cfg%d_traffic.txt" % args.config),
            "launches": int(mix_n), "avg_launch_us": mix_ms * 1e3 / max(mix_n, 1),
            "algorithmic_bytes_per_launch": mix_bytes / max(mix_n, 1),
        },
        "kernels": {
            "mix": {"ms": mix_ms, "launches": int(mix_n), "GBps": achieved},
            "grad": {"ms": grad_ms, "launches": int(grad_n),
                     "GBps": grad_bytes / (grad_ms * 1e-3) / 1e9 if grad_ms > 0 else 0.0},
            "synth": {"ms": syn_ms, "launches": int(syn_n),
                      "GBps": syn_bytes / (syn_ms * 1e-3) / 1e9 if syn_ms > 0 else 0.0},
        },
    }
    if not args.no_cpu_baseline:
        h = protocol.Hop(c["in_nbrs"], c["W"], c["s"], c["b"], c["K"], max_ig=c["max_ig"],
                         skip_on=c["skip_on"], max_skip=c["max_skip"], trigger=c["trigger"], seed=c["seed"],
                         delay_kind=c["delay_kind"], mult=c["mult"], check=False)
        recs = h.run()
        if c["model"] == "synth":
            out["cpu_baseline"] = cpu_baseline(c, recs, p0)
        else:
            out["cpu_baseline"] = None
    sess.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
