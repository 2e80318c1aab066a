"""CPU checks of bench.py's host-side helpers (no GPU, no library call)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_table_parses_and_covers_the_default_workloads():
    sys.path.insert(0, ROOT)
    import bench
    for kernel in ("fwd_gemm_lse", "bwd_gemm_dlogits", "bwd_gemm_dh", "bwd_gemm_dw"):
        for config in (2, 3):
            t = bench.pmc_traffic_bytes("lmhead", config, "blocks", kernel)
            assert t is not None and 1e9 < t < 1e11, (config, kernel, t)
    # per 1024 rows the forward launch fetches what one mini-sequence's launch used to: about 1.6 GB
    assert 1.5e9 < bench.pmc_traffic_bytes("lmhead", 3, "blocks", "fwd_gemm_lse") / 32 < 1.8e9
    assert bench.pmc_traffic_bytes("mlp", 2, "anything", "dw") > 3e9          # schedule column "-" matches any
    assert bench.pmc_traffic_bytes("lmhead", 4, "blocks", "bwd_gemm_dw") is None
    assert bench.pmc_traffic_bytes("lmhead", 3, "pairs", "bwd_gemm_dw") is None


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
