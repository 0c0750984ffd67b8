"""The library's host-side schedule selection (Section V) against the CPU checker: no GPU involved."""
import numpy as np
import pytest

from oracle import schedule_oracle as SO
from paper_2407_00599_amd import api


def test_fit_matches_checker():
    rng = np.random.default_rng(4)
    for n in (2, 3, 17, 200):
        xs = rng.uniform(1e4, 1e9, n)
        ts = 5e-4 + 7e-10 * xs + rng.normal(0, 2e-5, n)
        a, b = api.moe_alpha_beta_fit(xs, ts)
        ra, rb = SO.alpha_beta_fit(xs, ts)
        assert a == pytest.approx(ra, rel=1e-9, abs=1e-15) and b == pytest.approx(rb, rel=1e-9)


def test_fit_errors():
    with pytest.raises(api.MoEError):
        api.moe_alpha_beta_fit([1.0], [1.0])
    with pytest.raises(api.MoEError):
        api.moe_alpha_beta_fit([2.0, 2.0, 2.0], [1.0, 2.0, 3.0])
    with pytest.raises(api.MoEError):
        api.moe_alpha_beta_fit([1.0, 2.0, 3.0], [1.0, 2.0])


def test_choice_matches_checker_over_a_grid():
    rng = np.random.default_rng(8)
    n_s1 = n_s2 = 0
    for _ in range(400):
        consts = [float(v) for v in rng.uniform(0, 1e-3, 1)] + [float(rng.uniform(1e-10, 1e-9))] + \
                 [float(rng.uniform(0, 1e-3)), float(rng.uniform(1e-10, 1e-9)), float(rng.uniform(0, 1e-3)),
                  float(rng.uniform(1e-10, 2e-9))]
        B, L = int(rng.choice([2, 4, 8])), int(rng.choice([512, 1024, 2048]))
        E, M = int(rng.choice([4, 8, 16, 64])), int(rng.choice([1024, 2048, 4096]))
        k, f = int(rng.choice([1, 2])), float(rng.choice([0.05, 1.2, 2.4, 8.0]))
        n_esp, n_mp = int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 4, 8]))
        got, t1, t2 = api.moe_choose_schedule(*consts, B, L, E, M, k, f, n_esp, n_mp)
        r1, r2 = SO.schedule_times(*consts, B, L, E, M, k, f, n_esp, n_mp)
        assert t1 == pytest.approx(r1, rel=1e-12) and t2 == pytest.approx(r2, rel=1e-12)
        if abs(r1 - r2) > 1e-12 * max(r1, r2):
            assert got == SO.choose_schedule(*consts, B, L, E, M, k, f, n_esp, n_mp)
        n_s1 += got == 1; n_s2 += got == 2
    assert n_s1 > 20 and n_s2 > 20          # the grid exercises both outcomes


def test_choice_errors_and_tie():
    assert api.moe_choose_schedule(0, 0, 0, 0, 0, 0, 4, 128, 8, 64, 2, 1.2, 2, 2)[0] == 1
    for bad in [dict(B=0), dict(E=0), dict(f=0.0), dict(n_mp=0), dict(k=0)]:
        kw = dict(B=4, L=128, E=8, M=64, k=2, f=1.2, n_esp=2, n_mp=2); kw.update(bad)
        with pytest.raises(api.MoEError):
            api.moe_choose_schedule(1e-4, 1e-9, 1e-4, 1e-9, 1e-4, 1e-9, kw["B"], kw["L"], kw["E"], kw["M"], kw["k"], kw["f"],
                                    kw["n_esp"], kw["n_mp"])
