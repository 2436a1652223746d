"""The two stand-alone measurement programs (practical ceilings quoted beside the kernels' figures) run and
print what they say they print."""
import json
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2201_05596_amd")


def _lines(cmd):
    out = subprocess.run(cmd, capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stderr
    return [json.loads(l) for l in out.stdout.splitlines() if l.startswith("{")]


def test_mfma_rate_program():
    exe = os.path.join(PKG, "mfma_rate")
    if not os.path.exists(exe):
        pytest.fail("paper_2201_05596_amd/mfma_rate is not built (python -m paper_2201_05596_amd.build)")
    rows = _lines([exe, "2000"])
    assert [r["operands"] for r in rows] == ["zeros", "random bf16"]
    for r in rows:
        assert 100.0 < r["TFLOPs"] < 2600.0          # never above the 2.5 PFLOP/s the chip is specified with


def test_hbm_rate_program():
    exe = os.path.join(PKG, "hbm_rate")
    if not os.path.exists(exe):
        pytest.fail("paper_2201_05596_amd/hbm_rate is not built (python -m paper_2201_05596_amd.build)")
    rows = _lines([exe])
    assert sum(r["pattern"] == "linear" for r in rows) == 2 and sum(r["pattern"] == "strips" for r in rows) == 4
    for r in rows:
        rates = [v for k, v in r.items() if k.endswith("_TBps")]
        assert rates and all(0.5 < v < 8.0 for v in rates)        # never above the 8 TB/s of the HBM
