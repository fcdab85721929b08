"""Host-side pieces of the benchmark's contract (no GPU): more than one GPU is refused with a
message, and the HBM-traffic figure of the roofline comes from the committed counter summary of
the workload that is timed -- or is absent when there is none."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one gpu" in (r.stdout + r.stderr).lower()


def test_traffic_comes_from_the_committed_summary_of_the_same_workload():
    total, source = bench.profile_traffic("cfg4", 0.3, "expert_up")
    assert source == os.path.join("profiles", "dmoe_forward_cfg4_tau0.3_hbm_traffic.txt")
    # the wide up-projection: about 1.8 GB read + 53 MB written per launch
    assert 1.5e9 < total < 2.2e9
    # every line the benchmark reads is there for the workloads that have a summary
    for name, tau, kernels in [("cfg2", 0.5, ("router", "expert_up", "expert_down")),
                               ("cfg3", 0.5, ("expert_up", "expert_down")),
                               ("cfg4", 0.6, ("expert_up", "expert_down")),
                               ("cfg5a", 0.5, ("small_up", "small_down"))]:
        for k in kernels:
            t, src = bench.profile_traffic(name, tau, k)
            assert t is not None and t > 0 and os.path.exists(os.path.join(ROOT, src)), (name, k)


def test_no_summary_means_no_traffic_figure():
    assert bench.profile_traffic("cfg2", 0.7, "expert_up") == (None, None)
    assert bench.profile_traffic("cfg4", 0.3, "no_such_kernel") == (None, None)
