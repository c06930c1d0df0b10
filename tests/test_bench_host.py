"""Host-side checks of bench.py (no GPU): the accounting of compulsory work per configuration, the roofline
arithmetic, the one-GPU rule and the rule that stored counter traffic is dropped once its kernel source changed."""
import importlib.util
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
bench = importlib.util.module_from_spec(spec)
spec.loader.exec_module(bench)

MIB = float(1 << 20)


def test_accounting_matches_the_compulsory_traffic_of_every_configuration():
    # worked expression at 8192 x 8192 x 5: write f, read df, read f, write the dense dc: 4 x 256 MiB plus the small tensors
    elems, nbytes, dom = bench.accounting("cfg3", bench.workload("cfg3"))
    assert 1024 * MIB < nbytes < 1026 * MIB and elems * 4 == nbytes
    assert dom == dict(kernel="k_worked_backward", bound="hbm", per_launch=2 * 8192 * 8192 * 4, launches=1)
    # the three patterns of the introduction: 128 MiB, 256 MiB (dense dx), 128 MiB
    for name, lo in (("cfg2_1", 128), ("cfg2_2", 256), ("cfg2_3", 128)):
        _, nbytes, dom = bench.accounting(name, bench.workload(name))
        assert lo * MIB <= nbytes < (lo + 0.2) * MIB, (name, nbytes / MIB)
        assert dom["bound"] == "hbm" and dom["per_launch"] in (64 * MIB, 256 * MIB)
    # strided map: x read twice (forward, dw), dx written, f written once and read with df: 31.7 MB
    _, nbytes, dom = bench.accounting("cfg5", bench.workload("cfg5"))
    assert 31.6e6 < nbytes < 31.7e6
    assert dom["per_launch"] == (2 * 32 * 128 * 128 + 2 * 32 * 257 * 257) * 4
    # long summed index and the plain product: three contractions of 2 I J K flop each
    for name, (i, j, k) in (("cfg4", (4096, 4096, 256)), ("matmul", (4096, 4096, 4096))):
        _, _, dom = bench.accounting(name, bench.workload(name))
        assert dom["bound"] == "mfma" and dom["per_launch"] == 2.0 * i * j * k and dom["step_flops"] == 6.0 * i * j * k


def test_roofline_entry_arithmetic():
    r = dict(name="cfg3", dominant=dict(kernel="k", bound="hbm", per_launch=8e9, launches=1), dominant_ms=2.0,
             dominant_launches=4, timed_every=25)
    out = bench.roofline(r)
    assert out["achieved"] == pytest.approx(4000.0) and out["peak"] == 8000.0 and out["frac"] == pytest.approx(0.5)
    r["dominant"] = dict(kernel="k", bound="mfma", per_launch=157.3e12 * 1e-3, launches=1)
    r["dominant_ms"] = 2.0
    out = bench.roofline(r)
    assert out["unit"] == "TFLOP/s" and out["frac"] == pytest.approx(0.5)
    r["dominant_ms"] = None                       # nothing timed: no figures
    assert bench.roofline(r)["frac"] is None


def test_stored_traffic_is_dropped_when_the_kernel_source_changed(monkeypatch):
    assert bench.measured_traffic("no such workload") is None
    name, entry = next(iter(bench.MEASURED_TRAFFIC.items()))
    monkeypatch.setitem(bench.MEASURED_TRAFFIC, name, dict(entry, sha256="0" * 16))
    assert bench.measured_traffic(name) is None


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode == 2 and "ONE GPU" in p.stderr and p.stdout.strip() == ""
