"""Host-side checks of bench.py that need no GPU: the committed counter summary yields a traffic figure for every
kernel kind of every benchmarked workload, the roofline arithmetic is what the documentation says, and a request
for more than one GPU is refused with a message."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402


def test_traffic_table_covers_every_workload_and_kind():
    table = bench.hbm_traffic_table()
    for cfg in (2, 3, 4, 5):
        for kind in ("project_pack", "fwd", "mvue_pack", "wgrad", "wgrad_reduce"):
            assert (cfg, kind) in table, (cfg, kind)
            assert table[(cfg, kind)] > 0
    # the forward launches of the 8-bit block must at least move their compulsory bytes
    # (X + packed weight + bf16 Z, mean over the four layers: 265 MB) and not absurdly more
    assert 265e6 <= table[(5, "fwd")] <= 3 * 265e6


def test_roofline_objects_follow_the_stated_arithmetic():
    flops = 2.0 * 32768 * 1280 * 5120                       # dense-equivalent flops of one GEMM launch
    kernels = {"project_pack": {"ms": 0.015, "GB_per_s": 3000.0}, "fwd": {"ms": 0.120}, "wgrad": {"ms": 0.100},
               "mvue_pack": {"ms": 0.050, "GB_per_s": 2800.0}, "wgrad_reduce": {"ms": 0.012},
               "wgrad_row": {"ms": 0.162}}
    roof, row = bench.roofline_of(kernels, flops, "e4m3", 5, {(5, "fwd"): 4.0e8, (5, "mvue_pack"): 1.0e8, (5, "wgrad"): 2.0e8,
                                                                (5, "wgrad_reduce"): 0.5e8})
    assert roof["kernel"] == "fwd" and roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == 5000.0
    # executed flops are half of the dense-equivalent ones (2:4), held against the dense peak of the operand type
    assert abs(roof["achieved"] - 0.5 * flops / 0.120e-3 * 1e-12) < 1e-6
    assert abs(roof["frac"] - roof["achieved"] / 5000.0) < 1e-12
    assert roof["traffic"] == 4.0e8
    assert abs(row["achieved"] - 0.5 * flops / 0.162e-3 * 1e-12) < 1e-6 and row["traffic"] == 3.5e8


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr
