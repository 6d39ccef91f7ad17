"""Pins for the oracle's broadcast schedule (paper Sec. 2.3, Eq. 1; App. A.2.1)."""
import math
import random

import pytest

from oracle import pab_oracle as orc
from paper_2408_12588_amd import workloads as W


def eq1_literal(n_steps, lo, hi, n):
    """Eq. 1 built as text, without modular arithmetic: outside the stable
    segment everything is computed; inside, runs of one 'C' followed by n-1 'R',
    cut off at the segment end."""
    inside = ("C" + "R" * (n - 1)) * (hi - lo + 1)
    inside = inside[: hi - lo + 1]
    row = "C" * lo + inside + "C" * n_steps
    return row[:n_steps]


def test_golden_tables(golden_schedule_rows):
    assert len(golden_schedule_rows) >= 10
    for name, n_steps, lo, hi, n, pattern in golden_schedule_rows:
        assert len(pattern) == n_steps, name
        assert orc.schedule_row(n_steps, lo, hi, n) == pattern, name


def test_eq1_literal_agrees_with_golden(golden_schedule_rows):
    # the text construction itself must reproduce the hand tables, else it pins nothing
    for name, n_steps, lo, hi, n, pattern in golden_schedule_rows:
        assert eq1_literal(n_steps, lo, hi, n) == pattern, name


def test_fuzz_against_eq1_literal():
    rng = random.Random(1234)
    for _ in range(3000):
        n_steps = rng.randint(1, 160)
        lo = rng.randint(0, n_steps - 1)
        hi = rng.randint(lo, n_steps + 5)
        n = rng.randint(1, 12)
        assert orc.schedule_row(n_steps, lo, hi, n) == eq1_literal(n_steps, lo, hi, n)


@pytest.mark.parametrize("wl", W.CONFIGS, ids=lambda w: w.name)
def test_closed_form_counts(wl):
    # in-segment computes = ceil(W / n); total = steps - W + ceil(W / n)
    Wn = wl.hi - wl.lo + 1
    for kind in range(3):
        n = wl.intervals[kind]
        if n == 0:
            continue
        row = orc.schedule_row(wl.n_steps, wl.lo, wl.hi, n)
        assert row.count("C") == wl.n_steps - Wn + math.ceil(Wn / n)


def test_counts_of_the_five_workloads():
    # numbers worked out by hand from the closed form
    expect = {"tiny": (7, 5, 5), "opensora_480p": (18, 12, 10), "latte_512": (30, 23, None),
              "osp_512_long": (60, 40, 33), "stress_720p": (18, 12, 10)}
    for wl in W.CONFIGS:
        for kind, want in enumerate(expect[wl.name]):
            if want is None:
                assert wl.intervals[kind] == 0
                continue
            row = orc.schedule_row(wl.n_steps, wl.lo, wl.hi, wl.intervals[kind])
            assert row.count("C") == want, (wl.name, kind)


def test_pyramid_ordering():
    # Sec. 2.3: the less an attention kind varies, the longer its broadcast range, so
    # reuse fractions order spatial < temporal < cross for the paper's 2/4/6 setting.
    wl = W.OPENSORA_480P
    reuse = [orc.schedule_row(wl.n_steps, wl.lo, wl.hi, n).count("R") for n in wl.intervals]
    assert reuse[0] < reuse[1] < reuse[2]
    assert reuse == [12, 18, 20]


def test_invariants():
    rng = random.Random(7)
    for _ in range(500):
        n_steps = rng.randint(2, 120)
        lo = rng.randint(0, n_steps - 1)
        hi = rng.randint(lo, n_steps - 1)
        n = rng.randint(1, 10)
        row = orc.schedule_row(n_steps, lo, hi, n)
        if n == 1:
            assert "R" not in row
        if n >= hi - lo + 1:
            assert row[lo:hi + 1].count("C") == 1 and row[lo] == "C"
        if lo > 0:
            assert row[0] == "C"
        if hi < n_steps - 1:
            assert row[-1] == "C"
        for s in range(n_steps):
            src = orc.source_step(s, lo, hi, n)
            if row[s] == "C":
                assert src == s
            else:
                assert lo <= src < s and row[src] == "C" and s - src <= n - 1
                assert "C" not in row[src + 1:s + 1]   # the latest computed step


def test_bad_arguments():
    for args in [(-1, 0, 5, 2), (0, 0, 5, 0), (0, 6, 5, 2), (3, 0, 5, -2)]:
        with pytest.raises(ValueError):
            orc.schedule(*args)
        with pytest.raises(ValueError):
            orc.source_step(*args)
