"""Host-side logic of bench.py (no GPU): the algorithmic byte / flop counts behind the roofline
object, the traffic lookup in the committed counter summary, the oracle leg, and the refusal of
more than one GPU."""
import subprocess
import sys
import os

import numpy as np
import pytest

import bench
import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_algorithmic_counts_at_the_headline_shape():
    w = bench.WORKLOAD
    assert (w["N"], w["d"], w["m"], w["k"], w["r"]) == (32768, 2048, 2048, 128, 128)
    # compress: X 134.2 MB + P 1.0 MB + C 16.8 MB; C^T dY: C 16.8 + dY 134.2 MB + one fp32 T (2.1 MB)
    assert bench.algorithmic_bytes("compress", w) == 2 * (32768 * 2048 + 2048 * 256 + 32768 * 256)
    assert bench.algorithmic_bytes("compress", w) / 1e6 == pytest.approx(152.0, abs=0.1)
    assert bench.algorithmic_bytes("ct_dy", w) / 1e6 == pytest.approx(153.1, abs=0.1)
    assert bench.algorithmic_flops("compress", w) == 2.0 * 32768 * 2048 * 256
    assert bench.algorithmic_flops("ct_dy", w) == 2.0 * 32768 * 256 * 2048
    assert bench.algorithmic_flops("p_t", w) == 2.0 * 2048 * 256 * 2048
    # both main kernels sit below the ridge of 2.5 PFLOP/s over 8 TB/s (312 flop per byte): HBM-bound
    for kind in ("compress", "ct_dy"):
        assert bench.algorithmic_flops(kind, w) / bench.algorithmic_bytes(kind, w) < 2500e12 / 8000e9
    with pytest.raises(KeyError):
        bench.algorithmic_bytes("nope", w)


def test_traffic_lookup_reads_the_committed_summary():
    t = bench.read_traffic("ct_dy", bench.WORKLOAD["name"])
    assert t is not None and 0.9 * bench.algorithmic_bytes("ct_dy", bench.WORKLOAD) < t < 2e9
    assert bench.read_traffic("ct_dy", "no_such_workload") is None


def test_every_named_workload_is_a_baseline_shape():
    names = [bench.WORKLOAD["name"], *bench.OTHER_WORKLOADS, bench.BLOCK_WORKLOAD]
    assert len(set(names)) == len(names)
    for w in bench.OTHER_WORKLOADS.values():
        assert w["k"] + w["r"] <= w["d"] and w["N"] % 128 == 0


def test_cpu_baseline_runs_the_oracle_on_a_small_sample():
    X = si.round_to(si.activation(512, 64, 0.8, seed=1)[0], "bf16")
    dY = si.round_to(si.grad_output(512, 48, 1e-3, seed=2), "bf16")
    out = bench.cpu_baseline(X, dY, 8, 8, 500)
    assert out["kind"] == "oracle" and out["unit"] == "tokens/s" and out["cores"] >= 1
    assert np.isfinite(out["value"]) and out["value"] > 0 and "512 tokens" in out["sample"]


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode == 2 and "one GPU" in p.stderr and p.stdout.strip() == ""
