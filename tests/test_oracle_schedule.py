"""Pins for the checker's alpha-beta fit and Algorithm 1 (Section V)."""
import os

import numpy as np
import pytest

from oracle import schedule_oracle as SO

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "alpha_beta.txt")


def _paper_ag():
    out = {}
    for line in open(GOLD):
        if line.strip() and not line.startswith("#"):
            name, a, b = line.split()
            out[name] = (float(a), float(b))
    return out


def test_fit_recovers_the_papers_line_exactly():
    for a, b in _paper_ag().values():
        xs = [2.0 ** p for p in range(16, 28)]
        ts = [a + b * x for x in xs]
        fa, fb = SO.alpha_beta_fit(xs, ts)
        assert fa == pytest.approx(a, rel=1e-9) and fb == pytest.approx(b, rel=1e-12)


def test_fit_matches_textbook_routine_on_noisy_data():
    rng = np.random.default_rng(0)
    xs = rng.uniform(1e5, 1e8, 40)
    ts = 3e-4 + 6e-10 * xs + rng.normal(0, 1e-5, 40)
    fa, fb = SO.alpha_beta_fit(xs, ts)
    pb, pa = np.polyfit(xs, ts, 1)
    assert fa == pytest.approx(pa, rel=1e-7) and fb == pytest.approx(pb, rel=1e-9)
    # residuals are orthogonal to the regressors (the normal equations)
    res = ts - (fa + fb * xs)
    assert abs(res.sum()) < 1e-12 and abs((res * xs).sum()) < 1e-4


def test_fit_rejects_degenerate_input():
    with pytest.raises(ValueError):
        SO.alpha_beta_fit([1.0], [2.0])
    with pytest.raises(ValueError):
        SO.alpha_beta_fit([3.0, 3.0, 3.0], [1.0, 2.0, 3.0])
    with pytest.raises(ValueError):
        SO.alpha_beta_fit([1.0, 2.0], [1.0])


def test_times_by_hand():
    """B=2, L=4, M=8, E=4, k=2, f=1.5, N_ESP=2, N_MP=2: x = 64, T = 2*1.5*8/4 = 6, y = 4*6*8*2 = 384."""
    t1, t2 = SO.schedule_times(1.0, 0.5, 2.0, 0.25, 3.0, 0.125, 2, 4, 4, 8, 2, 1.5, 2, 2)
    assert t1 == 2 * (2.0 + 0.25 * 384 / 2) + 1.0 + 0.5 * 64 == 133.0
    assert t2 == 2.0 + 0.25 * 384 / 2 + 3.0 + 0.125 * 384 == 101.0
    assert SO.choose_schedule(1.0, 0.5, 2.0, 0.25, 3.0, 0.125, 2, 4, 4, 8, 2, 1.5, 2, 2) == 2


def test_limits_named_in_the_paper():
    """Section IV-B: with N_ESP = 1 and a vanishing capacity S2 wins (S1 still pays the AllGather of
    B L M elements); for a large capacity S1 wins, because that AllGather does not grow with T."""
    a_ag, b_ag = _paper_ag()["A"]
    common = dict(B=8, L=1024, E=8, M=1024, k=2, n_esp=1, n_mp=4)
    args = lambda f: (a_ag, b_ag, 2e-4, 6e-10, 2e-4, 6e-10, common["B"], common["L"], common["E"], common["M"],
                      common["k"], f, common["n_esp"], common["n_mp"])
    assert SO.choose_schedule(*args(1e-9)) == 2
    assert SO.choose_schedule(*args(64.0)) == 1
    # the switch-over point is where the two expressions meet; they are linear in f
    t = [SO.schedule_times(*args(f)) for f in (1.0, 2.0, 3.0)]
    d = [a - b for a, b in t]
    assert d[1] - d[0] == pytest.approx(d[2] - d[1], rel=1e-9)


def test_tie_goes_to_s1_and_nmp_one():
    # all constants zero: both times are zero -> S1
    assert SO.choose_schedule(0, 0, 0, 0, 0, 0, 4, 128, 8, 64, 2, 1.2, 2, 2) == 1
    # N_MP = 1, equal collectives, no start-up costs: t_D1 = 2 b y + b_ag x > t_D2 = 2 b y  -> S2
    assert SO.choose_schedule(0.0, 1e-9, 0.0, 1e-9, 0.0, 1e-9, 4, 128, 8, 64, 2, 1.2, 2, 1) == 2
