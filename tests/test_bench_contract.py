"""Host-side checks of bench.py's contract: more than one GPU is refused with a message, and the model of
algorithmic work it prices the kernels with agrees with the count model of the oracle package (App. F)."""
import os
import subprocess
import sys

import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       cwd=ROOT, timeout=300)
    assert p.returncode != 0
    assert "one GPU" in p.stderr
    assert p.stdout.strip() == ""


def test_algorithmic_flops_match_the_count_model():
    sys.path.insert(0, ROOT)
    import bench
    from oracle import count_model as cm
    w = wl.CONFIGS["c4"]
    per_kernel, fwd_total, bwd_total = bench.algorithmic_flops(w)
    # forward and backward matmul FLOPs per token and head (App. F.1, causal factor 0.5)
    fwd = 4 * w.dqk * w.dhv + 0.5 * 2 * w.chunk * (w.dqk + w.dhv)
    bwd = 8 * w.dqk * w.dhv + 0.5 * 2 * w.chunk * (3 * w.dqk + 2 * w.dhv)
    units = w.B * w.NH * w.T
    assert abs(fwd_total - fwd * units) <= 1e-9 * fwd_total
    assert abs(bwd_total - bwd * units) <= 1e-9 * bwd_total
    # the per-kernel figures are the products each kernel performs itself
    assert per_kernel["recurrent_fwd"] == 2 * w.dqk * w.dhv * units
    assert abs(per_kernel["tile_H"] - (2 * w.dqk * w.dhv + 0.5 * 2 * w.chunk * (w.dqk + w.dhv)) * units) < 1.0
    # the generation benchmark prices its kernel with the recurrent formulation's memory operations (App. F.2)
    assert cm.bytes_recurrent_step_exp(256, 512) > 2 * 256 * 512 * 4
