"""Host-side parts of bench.py that need no GPU: argument handling and the oracle-timing leg."""
import importlib.util
import os
import subprocess
import sys

import pytest

from oracle import pab_oracle as orc
from paper_2408_12588_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and res.stdout.strip() == ""


@pytest.mark.parametrize("wl", [W.TINY, W.LATTE_512], ids=lambda w: w.name)
def test_cpu_baseline_extrapolates_a_video_from_per_kind_times(wl):
    small = W.Workload(**{**wl.__dict__, "S": 48, "T": min(wl.T, 4)})
    out = _bench().cpu_baseline(small, 0.3)
    assert out["kind"] == "oracle" and out["unit"] == "TFLOP/s" and out["cores"] >= 1
    kinds = [k for k in range(3) if small.intervals[k] > 0]
    assert set(out["sec_per_call"]) == {W.KIND_NAMES[k] for k in kinds}
    # rebuild the extrapolation from the reported per-call times and the schedule (Eq. 1)
    for name, ivals in (("pab", small.intervals), ("no_pab", (1, 1, 1))):
        sec = 0.0
        flops = 0.0
        for k in kinds:
            computed = sum(orc.schedule(s, small.lo, small.hi, ivals[k]) == orc.COMPUTE for s in range(small.n_steps))
            blocks = sum(1 for b in range(small.n_blocks) if k in small.kinds_of_block(b))
            sec += out["sec_per_call"][W.KIND_NAMES[k]] * computed * blocks
            flops += small.flops(k) * computed * blocks
        assert out["video_seconds_extrapolated"][name] == pytest.approx(sec, rel=0.02, abs=2e-3)
        if name == "pab":
            assert out["value"] == pytest.approx(flops / sec / 1e12, rel=0.1)
    assert out["video_seconds_extrapolated"]["pab"] < out["video_seconds_extrapolated"]["no_pab"]
