"""The roofline accounting of bench.py against the figures of the workload table it is quoted on
(parameters, algorithmic flops and HBM bytes per agent-step of the five workloads), and the
one-GPU contract of its command line.  No GPU is used."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench
from paper_2205_05248_amd import workloads as wl


def test_per_agent_step_figures_of_the_five_workloads():
    params = [27721, 31566, 32203, 29644, 146856]
    flops = [54144, 61184, 62848, 57728, 283648]          # 2 D H + 12 H^2 + 2 H A
    act_bytes = [681, 906, 955, 796, 2428]                # obs, avail, h in, h out, action, Q
    for i in range(5):
        dims = wl.dims(wl.config(i))
        assert wl.param_count(*dims) == params[i]
        assert bench.flops_per_agent_step(*dims) == flops[i]
        assert bench.act_bytes_per_agent_step(*dims) == act_bytes[i]


def test_published_peaks():
    assert bench.PEAK["hbm_GBs"] == 8000.0 and bench.PEAK["bf16_TFs"] == 2500.0


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
