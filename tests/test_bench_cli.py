"""bench.py's command line without a GPU: more than one GPU is refused with a message, and there is no
CPU fallback; its CPU-baseline helper really runs the oracle."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300)


def test_more_than_one_gpu_is_refused():
    r = _run("--gpus", "2")
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_no_gpu_means_no_result():
    import torch
    if torch.cuda.is_available():
        return
    r = _run("--steps", "1", "--warmup", "0")
    assert r.returncode == 2 and "no CPU fallback" in r.stderr and r.stdout.strip() == ""


def test_cpu_baseline_helper_times_the_oracle():
    sys.path.insert(0, ROOT)
    import bench
    import tc_workloads as W
    shape = W.CONFIGS[1].with_blocks(200)
    rng = W.rng_for(1, salt=60)
    a = W.pick_ids(rng, 200, 16)
    b = W.pick_ids(rng, 200, 16, exclude=a)
    res = bench.cpu_baseline(shape, a, b, budget_s=0.5)
    assert res["kind"] == "oracle" and res["cores"] == 1 and res["unit"] == "GB/s"
    assert res["value"] > 0 and res["parallel_calls"]["value"] > 0
    assert np.isfinite(res["upload_ms_per_1k_tokens"])
