"""Host-side checks of the benchmark's accounting (no GPU): the algorithmic bytes and operations
that the roofline line is built from, which bound is reported for which workload, and that a run
on more than one GPU is refused."""
import os
import subprocess
import sys

import bench
from paper_2605_00422_amd import inputs as syn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_linear_forward_bytes_of_the_default_workload():
    """cfg1 (one token, 4096 -> 11008, rank 32): sign bits 5.64 MB + fp16 alpha and V + the codes,
    scale and code sum of one token + T + the fp32 output row = 6.41 MB, counted term by term."""
    cfg = syn.CONFIGS["cfg1_decode7b"]
    assert (cfg.M, cfg.K, cfg.N, cfg.r) == (1, 4096, 11008, 32)
    bits, alpha, V = 11008 * 4096 // 8, 2 * 11008, 2 * 11008 * 32
    codes, scale_qsum, T, Y = 4096, 8, 4 * 32, 4 * 11008
    assert bench.linear_forward_bytes(cfg) == bits + alpha + V + codes + scale_qsum + T + Y == 6410888
    assert bench.gemm_ops(cfg) == 2 * 11008 * 4096


def test_roofline_fields_and_bound_selection():
    cfg1 = syn.CONFIGS["cfg1_decode7b"]
    r = bench.roofline_for(cfg1, 5.0)
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["achieved"] - 6410888 / 5e-6 / 1e9) < 1e-6 and abs(r["frac"] - r["achieved"] / 8000.0) < 1e-12
    assert r["traffic"] == bench.MEASURED_TRAFFIC_BYTES["cfg1_decode7b"] >= 6410888
    cfg3 = syn.CONFIGS["cfg3_qwen32b_down_m2048"]
    r3 = bench.roofline_for(cfg3, 200.0)
    assert r3["bound"] == "mfma" and r3["unit"] == "TOP/s" and r3["peak"] == 5000.0
    assert abs(r3["achieved"] - 2 * 2048 * cfg3.N * cfg3.K / 200e-6 / 1e12) < 1e-9
    # the same rule at the crossover: bytes / 8 TB/s against ops / 5 POP/s
    for cfg in (cfg1, cfg3, syn.CONFIGS["cfg2_qwen32b_up_m16"]):
        hbm_t = bench.linear_forward_bytes(cfg) / 8e12
        mfma_t = bench.gemm_ops(cfg) / 5e15
        assert bench.roofline_for(cfg, 10.0)["bound"] == ("hbm" if hbm_t >= mfma_t else "mfma")


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode == 2
    assert "one GPU" in p.stderr and p.stdout.strip() == ""
