import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the library that is built; only a tree in which nothing is built yet gets built here
    from paper_2408_12588_amd import build as pab_build
    pab_build.ensure_built()


def golden_path(name):
    return os.path.join(ROOT, "tests", "golden", name)


@pytest.fixture(scope="session")
def golden_schedule_rows():
    rows = []
    with open(golden_path("schedule_tables.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, n_steps, lo, hi, n, pattern = line.split()
            rows.append((name, int(n_steps), int(lo), int(hi), int(n), pattern))
    return rows


@pytest.fixture(scope="session")
def golden_attention():
    out = {}
    with open(golden_path("attention_worked.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            out[parts[0]] = [float(x) for x in parts[1:]]
    return out


@pytest.fixture(scope="session")
def golden_timestep_windows():
    """(windows, rows, presets) of tests/golden/timestep_windows.txt."""
    windows, rows, presets = [], [], []
    with open(golden_path("timestep_windows.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            p = line.split()
            if p[0] == "row":
                rows.append((p[1], int(p[2]), p[3]))
            elif p[0] == "mlp":
                continue   # MLP broadcast rows: read by tests/test_oracle_module.py
            elif p[0] == "preset":
                presets.append((p[1], int(p[2]), tuple(int(x) for x in p[3:6]), float(p[6]), float(p[7])))
            else:
                windows.append((p[0],) + tuple(int(x) for x in p[1:]))
    return windows, rows, presets
