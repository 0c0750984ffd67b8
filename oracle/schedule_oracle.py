"""CPU checker for the schedule selection of Section V ("Solution"): the alpha-beta model of a
collective's time and Algorithm 1, which picks S1 or S2.  TEST INFRASTRUCTURE ONLY, like the rest
of this package: the library never imports it.

Readings of the paper taken here:
  * Section V-A: a collective over x elements costs alpha + beta * x; alpha and beta come from an
    ordinary least-squares fit of measured (x, time) pairs.
  * Algorithm 1 prints T = k f B L M / E and then y = E T M N_ESP.  Section II-A defines the
    capacity as T = k f B L / E, and y is the element count of the [E, T, M] buffer times N_ESP, so
    the M in the listing's T is taken as a slip: T = k f B L / E (real-valued, as in the listing).
  * t_D1 and t_D2 are the listing's expressions.  (The prose of Section V-B writes t_D2 with an
    explicit MP-AllGather term and divides the overlapped size by N_MP; the listing folds both into
    the fitted pair (alpha_o, beta_o) of the overlapped collective measured on y elements.)
  * Ties go to S1 (the listing tests t_D1 <= t_D2).
"""
from __future__ import annotations


def alpha_beta_fit(xs, ts):
    """Least squares for t = alpha + beta x over the given samples (normal equations, float64)."""
    xs = [float(v) for v in xs]
    ts = [float(v) for v in ts]
    n = len(xs)
    if n != len(ts) or n < 2:
        raise ValueError("need at least two samples")
    mx = sum(xs) / n
    mt = sum(ts) / n
    sxx = sum((x - mx) ** 2 for x in xs)
    if sxx == 0.0:
        raise ValueError("all sizes equal: beta is undetermined")
    beta = sum((x - mx) * (t - mt) for x, t in zip(xs, ts)) / sxx
    return mt - beta * mx, beta


def schedule_times(a_ag, b_ag, a_a2a, b_a2a, a_o, b_o, B, L, E, M, k, f, n_esp, n_mp):
    """(t_D1, t_D2) of Algorithm 1."""
    x = float(B) * L * M                         # elements of the MP-AllGather under S1
    T = k * f * B * L / E                        # expert capacity (Section II-A)
    y = E * T * M * n_esp                        # elements entering the EP&ESP-AlltoAll before the MP split
    t_d1 = 2.0 * (a_a2a + b_a2a * y / n_mp) + a_ag + b_ag * x
    t_d2 = a_a2a + b_a2a * y / n_mp + a_o + b_o * y
    return t_d1, t_d2


def choose_schedule(*args):
    """1 for S1, 2 for S2."""
    t_d1, t_d2 = schedule_times(*args)
    return 1 if t_d1 <= t_d2 else 2
