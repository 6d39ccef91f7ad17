"""Pins for the oracle's mapping of a timestep window onto sampler steps (paper App. A.2.1)."""
import math
import random

from oracle import pab_oracle as orc


def evenly_spaced(n_steps, first, stride):
    return [first - s * stride for s in range(n_steps)]


def test_golden_windows(golden_timestep_windows):
    windows, _, _ = golden_timestep_windows
    assert len(windows) >= 6
    for name, n_steps, first, stride, t_start, t_end, lo, hi in windows:
        got = orc.window_from_timesteps(evenly_spaced(n_steps, first, stride), t_start, t_end)
        assert got == (None if lo < 0 else (lo, hi)), name


def test_golden_rows_on_the_open_sora_window(golden_timestep_windows):
    windows, rows, _ = golden_timestep_windows
    name, n_steps, first, stride, t_start, t_end, lo, hi = windows[0]
    assert name == "os30_930_450"
    got = orc.window_from_timesteps(evenly_spaced(n_steps, first, stride), t_start, t_end)
    assert len(rows) == 9
    for rname, n, pattern in rows:
        assert len(pattern) == n_steps, rname
        assert orc.schedule_row(n_steps, got[0], got[1], n) == pattern, rname


def test_closed_form_for_evenly_spaced_lists():
    # timestep of step s is first - s*stride, so the window is
    # ceil((first - t_start)/stride) <= s <= floor((first - t_end)/stride), clipped to the steps
    rng = random.Random(99)
    for _ in range(2000):
        n_steps = rng.randint(1, 200)
        stride = rng.randint(1, 40)
        first = rng.randint(stride * (n_steps - 1), stride * (n_steps - 1) + 60)
        t_end = rng.randint(-20, first + 20)
        t_start = rng.randint(t_end, first + 40)
        lo = max(0, -((t_start - first) // stride))          # ceil((first - t_start) / stride)
        hi = min(n_steps - 1, (first - t_end) // stride)     # floor
        want = (lo, hi) if lo <= hi else None
        assert orc.window_from_timesteps(evenly_spaced(n_steps, first, stride), t_start, t_end) == want


def test_brute_force_on_irregular_lists():
    # membership test written out per step, on lists with repeats and uneven gaps (float timesteps too)
    rng = random.Random(5)
    for _ in range(500):
        n = rng.randint(1, 40)
        ts = sorted((rng.choice([rng.randint(0, 1000), rng.uniform(0, 1000)]) for _ in range(n)), reverse=True)
        a, b = sorted((rng.uniform(-50, 1050), rng.uniform(-50, 1050)))
        inside = [s for s in range(n) if b >= ts[s] >= a]
        want = (inside[0], inside[-1]) if inside else None
        assert orc.window_from_timesteps(ts, b, a) == want
        if inside:   # a non-increasing list puts the in-window steps next to each other
            assert inside == list(range(inside[0], inside[-1] + 1))


def test_ends_are_inclusive_and_errors():
    ts = [1000, 750, 500, 250, 0]
    assert orc.window_from_timesteps(ts, 750, 250) == (1, 3)
    assert orc.window_from_timesteps(ts, 749, 251) == (2, 2)
    assert orc.window_from_timesteps(ts, 1000, 0) == (0, 4)
    assert orc.window_from_timesteps(ts, 400, 300) is None
    import pytest
    with pytest.raises(ValueError):
        orc.window_from_timesteps(ts, 100, 200)          # start below end
    with pytest.raises(ValueError):
        orc.window_from_timesteps([0, 500, 1000], 900, 100)   # list runs the wrong way


def test_window_fraction_of_the_papers_settings(golden_timestep_windows):
    # Sec. 2.2 / App. A.2.1: broadcasting covers the stable middle of the run, roughly half to
    # three quarters of the steps, never the first or the last one for these settings
    windows, _, _ = golden_timestep_windows
    for name, n_steps, first, stride, t_start, t_end, lo, hi in windows[:2]:
        frac = (hi - lo + 1) / n_steps
        assert 0.4 <= frac <= 0.8, name
        assert lo > 0 and hi < n_steps - 1, name
