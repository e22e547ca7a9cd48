"""Host-side pieces of bench.py that need no GPU: the algorithmic-byte accounting (the denominator
of every bandwidth figure), the cpu_baseline leg on a tiny workload, the refusal of --gpus > 1."""
import os
import subprocess
import sys

import bench
from paper_2601_02360_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_algorithmic_bytes_of_the_headline_workload():
    n = sum(W.numels(2))
    n_chunks = sum((x + 4095) // 4096 for x in W.numels(2))
    assert (n, n_chunks, len(W.numels(2))) == (887_687_168, 216_737, 146)
    c, a, u = bench.algorithmic_bytes(n, n_chunks, 64, 8, False)
    payload = n_chunks * (2 * 64 + 8)
    assert c == 16 * n + payload and a == 4 * n + 8 * payload and u == 12 * n
    step = 8 * c + a + u
    assert step == 16 * n * 9 + 16 * payload
    assert abs(step / 1e9 - 128.3) < 0.05                      # 127.8 GB of dense traffic + 0.47 GB of messages
    # bf16 pseudo-gradient given directly: 2 + 4 + 4 bytes per parameter
    assert bench.algorithmic_bytes(n, n_chunks, 64, 8, True)[0] == 10 * n + payload
    # Q = identity: 2-byte index + 4-byte value per kept entry
    assert bench.algorithmic_bytes(n, n_chunks, 64, 8, False, quant=False)[0] == 16 * n + n_chunks * 6 * 64


def test_workload_shapes_match_the_stated_sizes():
    assert sum(W.numels(0)) == 4_194_304
    assert (len(W.numels(1)), sum(W.numels(1))) == (110, 151_898_880)
    assert (len(W.numels(4)), sum(W.numels(4))) == (146, 888_557_599)
    assert all(x % 4096 != 0 for x in W.numels(4))             # every tensor ends in a partial chunk


def test_cpu_baseline_leg_on_a_tiny_replica_set():
    rs = W.ReplicaSet(0, device="cpu", replicas=2)
    out = bench.cpu_baseline(rs, dict(W.WORKLOADS[0]), [0], True)
    assert out["kind"] == "oracle" and out["unit"] == "params/s" and out["value"] > 0 and out["cores"] >= 1
    assert out["single_thread_value"] > 0 and "threads" in out["sample"]


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and not r.stdout.strip()
