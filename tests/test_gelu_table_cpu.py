"""The GeLU polynomial tables compiled into the bf16 FFN epilogues, checked on the CPU: the numbers in
csrc/ffn.hip are the ones the fitting script beside it produces, and their fp32 Horner evaluation stays
within the documented distance of the checker's exact (erf) GeLU and GeLU'."""
import importlib.util
import os
import re

import numpy as np

from oracle import moe_oracle as O

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2407_00599_amd", "csrc")


def _source_table(name):
    src = open(os.path.join(CSRC, "ffn.hip")).read()
    body = re.search(name + r"\[\d+\] = \{([^}]*)\}", src).group(1)
    return np.array([float(t.strip().rstrip("f")) for t in body.split(",")], dtype=np.float32)


def _fit_module():
    spec = importlib.util.spec_from_file_location("fit_gelu_poly", os.path.join(CSRC, "fit_gelu_poly.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_tables_in_source_are_the_fitted_ones():
    fit = _fit_module()
    cP, cD = fit.tables()
    np.testing.assert_allclose(_source_table("GELU_PHI"), cP, rtol=2e-6)
    np.testing.assert_allclose(_source_table("GELU_DG"), cD, rtol=2e-6)


def test_tables_against_exact_gelu():
    fit = _fit_module()
    cP, cD = _source_table("GELU_PHI"), _source_table("GELU_DG")
    assert len(cP) == fit.N_PHI and len(cD) == fit.N_DG
    z = np.linspace(-12.0, 12.0, 480001).astype(np.float32)
    ge = z * np.clip(fit.horner32(cP, z), 0, 1)       # what the kernel computes, op by op in fp32
    dg = fit.horner32(cD, z)
    zz = z.astype(np.float64)
    assert np.abs(ge - O.gelu(zz)).max() < 6e-5
    big = zz > 1.0
    assert (np.abs(ge - O.gelu(zz))[big] / O.gelu(zz)[big]).max() < 2e-5
    assert np.abs(dg - O.gelu_grad(zz)).max() < 2e-4
    # limits: identity / zero far from the origin, slope 1/2 at it
    assert ge[-1] == z[-1] and ge[0] == 0.0 and abs(dg[len(z) // 2] - 0.5) < 1e-6
