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
    traffic = bench.measured_traffic()
    # two launches per layer: the dominant kernel is the GEMM of bwla_linear_forward, the layer beside it
    r = bench.roofline_for(cfg1, 2, 13.0, 5.0, None, traffic)
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert r["kernel"] == "gemm_decode_bs_kernel"
    assert abs(r["achieved"] - 6410888 / 5e-6 / 1e9) < 1e-6 and abs(r["frac"] - r["achieved"] / 8000.0) < 1e-12
    assert abs(r["layer"]["achieved"] - bench.layer_bytes(cfg1) / 13e-6 / 1e9) < 1e-6 and r["layer"]["launches"] == 2
    # the measured traffic comes from the tracked counter summary, and is no less than the algorithmic bytes
    assert r["traffic"] == traffic[("cfg1_decode7b", "gemm_decode_bs_kernel")] >= 6410888
    # one launch per layer: the kernel is the layer
    r1 = bench.roofline_for(cfg1, 1, 7.0, 5.0, None, traffic)
    assert r1["kernel"] == "decode_layer_kernel" and r1["bytes_per_launch"] == bench.layer_bytes(cfg1)
    assert abs(r1["achieved"] - bench.layer_bytes(cfg1) / 7e-6 / 1e9) < 1e-6 and r1["layer"]["frac"] == r1["frac"]
    assert r1["traffic"] == traffic[("cfg1_decode7b", "decode_layer_kernel")] >= bench.layer_bytes(cfg1)
    cfg3 = syn.CONFIGS["cfg3_qwen32b_down_m2048"]
    r3 = bench.roofline_for(cfg3, 2, 450.0, 200.0, None, traffic)
    assert r3["bound"] == "mfma" and r3["unit"] == "TOP/s" and r3["peak"] == 5000.0
    assert abs(r3["achieved"] - 2 * 2048 * cfg3.N * cfg3.K / 200e-6 / 1e12) < 1e-9
    assert abs(r3["layer"]["achieved"] - 2 * 2048 * cfg3.N * cfg3.K / 450e-6 / 1e12) < 1e-9
    # the same rule at the crossover: bytes / 8 TB/s against ops / 5 POP/s
    for cfg in (cfg1, cfg3, syn.CONFIGS["cfg2_qwen32b_up_m16"]):
        hbm_t = bench.layer_bytes(cfg) / 8e12
        mfma_t = bench.gemm_ops(cfg) / 5e15
        assert bench.roofline_for(cfg, 2, 20.0, 10.0, None, traffic)["bound"] == ("hbm" if hbm_t >= mfma_t else "mfma")


def test_layer_bytes_are_both_calls_bytes():
    cfg = syn.CONFIGS["cfg1_decode7b"]
    rq = 2 * 4096 + 4 * (64 * 64 + 64 * 64) + 2 * 4096 * 32 + 4096 + 8 + 4 * 32
    assert bench.rotate_quant_bytes(cfg) == rq
    assert bench.layer_bytes(cfg) == 6410888 + rq == 6718224


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode == 2
    assert "one GPU" in p.stderr and p.stdout.strip() == ""
