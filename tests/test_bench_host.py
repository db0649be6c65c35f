"""Host-side checks of bench.py that need no GPU: the workloads it offers follow the benchmark configurations'
statements (batch, draft policy, acceptance mode), and a request for more than one GPU is refused with a message."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_workloads_follow_the_benchmark_configurations():
    import bench
    from paper_2508_18588_amd import HS_ACCEPT_REJECTION, HS_K_AIMD, HS_K_FIXED, HS_K_MATCHLEN
    w2, w3, w5 = bench.workload_params(2), bench.workload_params(3), bench.workload_params(5)
    assert (w2["batch"], w2["policy"]["k_mode"], w2["policy"]["k_fixed"], w2["p_iid"], w2["p_span"]) == \
        (64, HS_K_FIXED, 8, [0.20], 0.05)
    assert (w3["batch"], w3["policy"]["k_mode"], w3["k_max"], w3["ctx"]) == (128, HS_K_MATCHLEN, 16, ("uniform", 2048, 16384))
    assert abs((1 - w3["p_iid"][0]) * (1 - w3["p_span"]) - 0.70) < 0.005          # 70 % of the history copied
    for reuse in (0.0, 0.5, 0.9):
        w4 = bench.workload_params(4, reuse)
        assert (w4["batch"], w4["policy"]["k_mode"], w4["k_max"]) == (256, HS_K_AIMD, 32)
        assert w4["p_iid"] == [1.0 - reuse] and w4["p_span"] == 0.0
        assert w4["ctx"][:5] == ("lognormal", 4000.0, 0.8, 512, 32768)
    assert (w5["batch"], w5["ctx"], w5["p_iid"], w5["mode"], w5["temperature"]) == \
        (64, ("fixed", 8192), [0.4, 0.6], HS_ACCEPT_REJECTION, 1.0)
    assert w5["policy"]["k_fixed"] == 8 and w5["snapshot"] and "FIRST SPECULATIVE STEP" in w5["name"]
    for w in (w2, w3, w5):
        assert w["policy"]["k_max"] == w["k_max"] and w["window_tokens"] >= 64
    with pytest.raises(SystemExit):
        bench.workload_params(1)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)
