"""Host-side parts of bench.py: the one-GPU rule, the compulsory-byte count of a wave taken from a schedule,
and the reader of the committed counter summaries.  No GPU."""
import os
import subprocess
import sys

import numpy as np

from conftest import ROOT

sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_1902_01064_amd import hop, inputs  # noqa: E402
from test_host_library import host_ctx  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_compulsory_bytes_of_a_lock_step_ring():
    """Ring of 4, standard mode, no delays: every wave holds 4 records that read the 4 current replicas (each one
    three times) and write 4 new ones; with a gradient buffer per STEP that is 4 + 4 + 4 vectors, without 4 + 4."""
    c = inputs.config(1, K=5)
    ctx = host_ctx(c)
    try:
        s = hop.hop_simulate(ctx, c["K"], c["delay_kind"], c["mult"])
        d = 1000
        got = bench.wave_compulsory_bytes(s, d, "synth", False)
        assert s.n_waves == 5 and np.all(got == 4.0 * d * 12)
        assert np.all(bench.wave_compulsory_bytes(s, d, "none", False) == 4.0 * d * 8)
        assert np.all(bench.wave_compulsory_bytes(s, d, "synth", True) == 4.0 * d * 20)     # + velocity read and written
        assert np.all(bench.wave_compulsory_bytes(s, d, "dense_fused", False) == 0)        # no record left for the mix
        s.free()
    finally:
        hop.hop_destroy(ctx)


def test_counter_summaries_parse_and_match_their_own_text():
    for name, low, high in (("hop_mix_cfg4_traffic.txt", 7.9e9, 8.3e9), ("hop_mix_cfg5_traffic.txt", 2.1e9, 2.3e9)):
        v = bench.read_traffic(name)
        assert v is not None and low < v < high, (name, v)
    assert bench.read_traffic("no_such_summary.txt") is None
