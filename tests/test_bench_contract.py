"""Host-side checks of the measurement program (no GPU): what it refuses, the roofline arithmetic it prints,
and the algorithmic byte and FLOP counts it divides by - recomputed here from the workload definitions."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_roofline_objects_divide_algorithmic_work_by_kernel_time():
    h = bench.hbm_roofline("k", 108_350_720, 21.7, traffic=109.9e6)
    assert h["bound"] == "hbm" and h["peak"] == 8000.0 and h["unit"] == "GB/s"
    assert h["achieved"] == pytest.approx(108_350_720 / 21.7e-6 / 1e9, rel=1e-3)
    assert h["frac"] == pytest.approx(h["achieved"] / 8000.0, abs=1e-4) and h["traffic"] == 109.9e6
    m = bench.mfma_roofline("k", 2.0 ** 42, 4000.0)
    assert m["bound"] == "mfma" and m["peak"] == 2500.0 and m["unit"] == "TFLOP/s"
    assert m["achieved"] == pytest.approx(2.0 ** 42 / 4000e-6 / 1e12, rel=1e-3)
    assert m["frac"] == pytest.approx(m["achieved"] / 2500.0, abs=1e-4) and m["traffic"] is None


def test_config2_algorithmic_bytes_follow_from_the_shapes():
    """Reuse layer: every selected (K row, V row, index) once plus Q and O; anchor sweep: every K row once, an
    fp32 logit per (query head, key), plus Q (Sec. 3.6; bf16 rows of 128 elements)."""
    class WL:   # the shape of config 2, nothing else
        B, Hq, Hkv, d = 8, 32, 8, 128
        seqlens = [32768] * 8
        k_per_seq = [3277] * 8
    leg = bench.DecodeLeg.__new__(bench.DecodeLeg)
    leg.wl = WL
    gather, stream = leg.bytes()
    assert gather == 8 * 8 * 3277 * (2 * 128 * 2 + 4) + 2 * 8 * 32 * 128 * 2 == 108_350_720
    assert stream == 8 * 32768 * 8 * 128 * 2 + 8 * 32768 * 32 * 4 + 8 * 32 * 128 * 2 == 570_490_880


def test_traffic_table_is_read_from_the_tracked_summary():
    t = bench.load_traffic()
    for kernel in ("decode_stream", "decode_gather", "prefill_sweep1", "prefill_sweep2", "prefill_sparse",
                   "decode_gather_cfg3"):
        assert kernel in t and t[kernel] > 0
    # counter traffic of the decode kernels stays within a few percent of the algorithmic bytes
    assert 0.95 < t["decode_gather"] / 108_350_720 < 1.10
    assert 0.95 < t["decode_stream"] / 570_490_880 < 1.10
