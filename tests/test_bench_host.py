"""Host-side checks of bench.py's accounting (no GPU): the algorithmic bytes per parameter behind the roofline
figure and the static memory per parameter (Sec. 4.2 "Memory and Runtime": master weights + m + v = 12 bytes
per parameter, FP8 weights + m + v = 9)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench          # noqa: E402
import workloads      # noqa: E402


def test_static_memory_matches_the_papers_accounting():
    wl = workloads.config4()
    eco = bench.static_bytes_per_param(wl, "adam-sr")
    master = bench.static_bytes_per_param(wl, "adam-master-sr")
    assert eco == pytest.approx(9.0 + 4.0 / 128)                 # 1 (FP8) + 4 (m) + 4 (v) + one fp32 scale per 128
    assert master - eco == pytest.approx(4.0)                    # the fp32 master copy the method removes
    assert master - (1.0 + 4.0 / 128) == pytest.approx(12.0)     # master + m + v, without the quantized copy
    assert bench.static_bytes_per_param(workloads.config5(), "adam-sr") == pytest.approx(0.5 + 2 + 2 + 2.0 / 128)


def test_algorithmic_bytes_per_parameter():
    wl = workloads.config4()
    n = wl.numel
    assert bench.algorithmic_bytes(wl, "adam-sr") / n == pytest.approx(20.0625)
    assert bench.algorithmic_bytes(wl, "sgdm-sr") / n == pytest.approx(12.0625)
    assert bench.algorithmic_bytes(wl, "adam-master-sr") / n == pytest.approx(27.03125)
    assert bench.algorithmic_bytes(wl, "sgdm-exact-sr") / n == pytest.approx(20.0625)
    assert bench.algorithmic_bytes(workloads.config5(), "adam-sr") / workloads.config5().numel == pytest.approx(11.03125)
    tw = workloads.with_granularity(workloads.config4(), "tensor")
    assert bench.algorithmic_bytes(tw, "adam-sr") / n == pytest.approx(31.0, abs=1e-3)   # inputs read twice
    # the two-launch configuration counts its bf16 norm vectors at 22 bytes per parameter
    c2 = workloads.config2()
    q = sum(t.numel for t in c2.tensors if t.fmt == "fp8")
    p = sum(t.numel for t in c2.tensors if t.fmt == "bf16_plain")
    assert bench.algorithmic_bytes(c2, "adam-sr") == pytest.approx(20.0625 * q + 22.0 * p)


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
