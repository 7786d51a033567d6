"""Command-line contract of bench.py that needs no GPU: more than one GPU is
refused with a message, and the byte accounting of the JSON line is what the
workload shapes say."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2 and "one GPU" in res.stderr and res.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="4")
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, env=env)
    assert res.returncode == 2 and "one GPU" in res.stderr


def test_algorithmic_bytes():
    sys.path.insert(0, ROOT)
    import bench
    from workloads import CONFIGS
    w = CONFIGS["cfg3_gradient"]
    ell = w.W // w.r
    # one pass: all of V, every coded packet, the outputs
    assert bench.algorithmic_bytes_pipeline(w, ell) == 2_867_200_000 + 1_075_200_000 + 102_400_000
    assert bench.algorithmic_bytes_pipeline(w, ell, 2) * 2 == bench.algorithmic_bytes_pipeline(w, ell)
    # fused shuffle: the (K-r)/K of V that is sent, the coded and the decoded packets
    assert bench.algorithmic_bytes_shuffle(w, ell) == 2_150_400_000 + 1_075_200_000 + 2_150_400_000
    w5 = CONFIGS["cfg5_k24"]
    assert bench.algorithmic_bytes_pipeline(w5, 512) == 2_089_156_608 + 435_240_960 + 24 * 2048 * 4
    # measured traffic is only quoted for the kernel sources it was measured on
    key = next(iter(bench.TRAFFIC))
    assert bench.measured_traffic("no such workload", "f32", "pipeline") == (None, None)
    t = bench.TRAFFIC[key]
    assert (bench.measured_traffic(*key)[0] is not None) == (t["source_hash"] == bench.kernel_source_hash(key[2]))
    # every recorded figure names the summary under profiles/ it was taken from
    for rec in bench.TRAFFIC.values():
        assert os.path.exists(os.path.join(ROOT, rec["profile"])), rec["profile"]
    # the default run also reports the other large workloads and the per-node-faithful accounting
    assert ("cfg5_k24", "f32", "pipeline") in bench.ALSO and ("cfg5_k24", "u32", "pipeline") in bench.ALSO
    assert ("cfg3_gradient", "f32", "node") in bench.ALSO
