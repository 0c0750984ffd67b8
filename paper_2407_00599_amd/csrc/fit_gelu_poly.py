#!/usr/bin/env python3
"""Writes the polynomial coefficients GELU_PHI / GELU_DG used by the bf16 epilogues in ffn.hip.

On |z| <= Z0 the odd functions Phi(z) - 1/2 and GeLU'(z) - 1/2 = Phi(z) + z phi(z) - 1/2 (Phi, phi:
standard normal CDF and density) are fitted by z * P(z^2) in the minimax sense (Lawson's iteratively
reweighted least squares, fp64, basis scaled to [0, 1]); the kernel clamps z to [-Z0, Z0].  Run it to
print the tables and the errors of their fp32 Horner evaluation:  python fit_gelu_poly.py
"""
import numpy as np
from scipy.special import erf

Z0, N_PHI, N_DG = 4.25, 9, 10


def Phi(z):
    return 0.5 * (1.0 + erf(z / np.sqrt(2.0)))


def phi(z):
    return np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


def fit_odd(f, nterms, iters=300):
    z = np.linspace(1e-6, Z0, 8001)
    u = (z / Z0) ** 2
    A = np.stack([z * u ** k for k in range(nterms)], 1)
    w = np.ones_like(z)
    for _ in range(iters):
        c, *_ = np.linalg.lstsq(A * w[:, None], f(z) * w, rcond=None)
        r = np.abs(A @ c - f(z))
        w = w * (0.5 + r / r.max())
        w /= w.mean()
    return np.array([c[k] / Z0 ** (2 * k) for k in range(nterms)]).astype(np.float32)


def horner32(c, z):
    """0.5 + zc * P(zc^2) with zc = clamp(z), every operation rounded to fp32 as in the kernel."""
    zc = np.clip(z.astype(np.float32), np.float32(-Z0), np.float32(Z0))
    u = (zc * zc).astype(np.float32)
    p = np.full_like(u, c[-1])
    for k in range(len(c) - 2, -1, -1):
        p = (p * u + c[k]).astype(np.float32)
    return (np.float32(0.5) + zc * p).astype(np.float32)


def tables():
    return fit_odd(lambda t: Phi(t) - 0.5, N_PHI), fit_odd(lambda t: Phi(t) + t * phi(t) - 0.5, N_DG)


if __name__ == "__main__":
    cP, cD = tables()
    print("GELU_PHI[%d] = {%s}" % (N_PHI, ", ".join("%.9ef" % c for c in cP)))
    print("GELU_DG[%d] = {%s}" % (N_DG, ", ".join("%.9ef" % c for c in cD)))
    z = np.linspace(-9, 9, 400001).astype(np.float32)
    zz = z.astype(np.float64)
    ge = z * np.clip(horner32(cP, z), 0, 1)
    print("max |GeLU error| %.2e   max |GeLU' error| %.2e" % (
        np.abs(ge - zz * Phi(zz)).max(), np.abs(horner32(cD, z) - (Phi(zz) + zz * phi(zz))).max()))
