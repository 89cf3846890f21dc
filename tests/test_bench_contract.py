"""Host-side checks of bench.py's contract: the parts that need no GPU."""
import json
import os
import subprocess
import sys

import pytest

import synth_inputs as si
from oracle import hmar_attn_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr or "--gpus 1" in res.stderr
    assert res.stdout.strip() == ""          # no JSON line is printed for a refused run


def test_kernel_byte_and_flop_models_match_the_schedule_arithmetic():
    sys.path.insert(0, ROOT)
    import bench
    w = si.WORKLOADS[bench.WORKLOAD]
    A = orc.allowed_pairs(w.sides)
    n_heads = w.B * w.H
    m = bench.kernel_models(n_heads, w.L, w.D, A)
    rows = n_heads * w.L
    # forward: Q, K, V in, O out (bf16 rows of 128 bytes) and LSE (4 bytes) per row
    assert m["hmar_fwd_kernel"]["bytes"] == rows * (4 * 128 + 4) == 269_475_840
    # per kernel: the contractions it performs over the unmasked pairs, 2*D*A flops each per head
    # (forward S and PV; dK/dV kernel S, dP, dV, dK; dQ kernel S, dP, dQ -- S and dP are formed by
    # both backward kernels, while the headline metric counts them once: 4 + 10 per pair and D)
    unit = 2 * w.D * A * n_heads
    assert m["hmar_fwd_kernel"]["flops"] == 2 * unit
    assert m["hmar_dkdv_kernel"]["flops"] == 4 * unit
    assert m["hmar_dq_kernel"]["flops"] == 3 * unit
    # useful flops: the recomputed S and dP count once, so the per-kernel figures add up to the
    # 2 + 5 contractions of the headline metric
    assert sum(k["useful_flops"] for k in m.values()) == (2 + 5) * unit
    assert m["hmar_dkdv_kernel"]["useful_flops"] == 2 * unit
    assert abs((2 + 5) * unit / 1e9 - 124.43) < 0.01              # the headline figure per step
    assert bench.METRIC.startswith("useful TFLOP/s fwd+bwd (680 tok, H=24, D=64)")


def test_traffic_file_is_readable_and_close_to_the_algorithmic_bytes():
    sys.path.insert(0, ROOT)
    import bench
    w = si.WORKLOADS[bench.WORKLOAD]
    m = bench.kernel_models(w.B * w.H, w.L, w.D, orc.allowed_pairs(w.sides))
    for kernel, model in m.items():
        t = bench.read_traffic(kernel)
        assert t is not None, kernel
        assert 0.9 * model["bytes"] <= t <= 1.25 * model["bytes"], (kernel, t, model["bytes"])
