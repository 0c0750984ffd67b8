"""GPU parity: dispatch, combine forward/backward (incl. the N_ESP partial-sum form) against the
CPU checker.  Plain row copies are compared bit for bit; weighted sums to the dtype's tolerance."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2407_00599_amd import api, synth
from util import DEV, TOL, to_dev, to_host, rel_err, torch_dtype

pytestmark = pytest.mark.gpu


def routing(S, E, k, C, seed, skew=1.0):
    logits = synth.synthetic_logits(S, E, seed=seed, sigma=1.0) + skew * np.linspace(0, 1, E, dtype=np.float32)[None]
    idx = O.topk_select(logits, k)
    slot, inv, counts = O.capacity_slots(idx, E, C)
    w = O.combine_weights(logits, idx, True).astype(np.float32)
    return idx, slot, inv, w


@pytest.mark.parametrize("S,M,E,k,C,dtype", [
    (1, 8, 1, 1, 1, "f32"), (100, 64, 4, 2, 30, "f32"), (300, 520, 8, 2, 60, "bf16"), (1000, 1024, 16, 3, 150, "bf16"),
    (257, 4096, 8, 2, 70, "bf16"), (513, 72, 64, 8, 50, "f32"),
])
def test_dispatch_and_combine(S, M, E, k, C, dtype):
    idx, slot, inv, w = routing(S, E, k, C, seed=S + M)
    rng = np.random.default_rng(S)
    x = synth.store(rng.standard_normal((S, M)).astype(np.float32), dtype)
    tdt = torch_dtype(dtype)
    d_inv, d_idx, d_slot, d_w = to_dev(inv), to_dev(idx), to_dev(slot), to_dev(w)
    buf = torch.full((E, C, M), 7.0, dtype=tdt, device=DEV)
    api.moe_dispatch(to_dev(x), S, M, E, k, C, d_inv, None, buf)
    ref = O.dispatch(x.val, inv, k)
    assert np.array_equal(to_host(buf), ref)                      # pure copy: exact
    bufw = torch.full((E, C, M), 7.0, dtype=tdt, device=DEV)
    api.moe_dispatch(to_dev(x), S, M, E, k, C, d_inv, d_w, bufw)
    assert rel_err(to_host(bufw), O.dispatch(x.val, inv, k, w)) <= (1e-6 if dtype == "f32" else 4e-3)

    for n_part in (1, 2, 3, 4):
        Y = synth.store(rng.standard_normal((n_part, E, C, M)).astype(np.float32), dtype)
        y = torch.full((S, M), 7.0, dtype=tdt, device=DEV)
        api.moe_combine_fwd(to_dev(Y), n_part, S, M, E, k, C, d_idx, d_slot, d_w, y)
        ref = O.combine_fwd(Y.val, idx, slot, w)
        assert rel_err(to_host(y), ref) <= TOL[dtype] * (0.1 if dtype == "f32" else 0.25)
        dropped = (slot < 0).all(axis=1)
        assert np.all(to_host(y)[dropped] == 0.0)
        # unit weights: backward of dispatch
        y1 = torch.empty((S, M), dtype=tdt, device=DEV)
        api.moe_combine_fwd(to_dev(Y), n_part, S, M, E, k, C, d_idx, d_slot, None, y1)
        assert rel_err(to_host(y1), O.combine_fwd(Y.val, idx, slot, None)) <= TOL[dtype] * 0.25
        # backward
        dy = synth.store(rng.standard_normal((S, M)).astype(np.float32), dtype)
        dY = torch.full((E, C, M), 7.0, dtype=tdt, device=DEV); dw = torch.full((S, k), 7.0, device=DEV)
        api.moe_combine_bwd(to_dev(dy), to_dev(Y), n_part, S, M, E, k, C, d_idx, d_slot, d_inv, d_w, dY, dw)
        rdY, rdw = O.combine_bwd(dy.val, Y.val, idx, slot, w)
        assert rel_err(to_host(dY), rdY) <= (1e-6 if dtype == "f32" else 4e-3)
        assert rel_err(to_host(dw), rdw) <= 2e-6 * np.sqrt(M)
        assert np.all(to_host(dw)[slot < 0] == 0.0)
    torch.cuda.synchronize()


def test_identity_round_trip_on_device():
    # dispatch then unit-weight combine returns (number of surviving choices) * x
    S, M, E, k, C = 500, 256, 8, 2, 100
    idx, slot, inv, w = routing(S, E, k, C, seed=3, skew=2.0)
    x = synth.store(np.random.default_rng(0).standard_normal((S, M)).astype(np.float32) , "f32")
    buf = torch.empty((E, C, M), device=DEV); y = torch.empty((S, M), device=DEV)
    api.moe_dispatch(to_dev(x), S, M, E, k, C, to_dev(inv), None, buf)
    api.moe_combine_fwd(buf, 1, S, M, E, k, C, to_dev(idx), to_dev(slot), None, y)
    surv = (slot >= 0).sum(1)
    assert (surv < k).any()
    assert np.array_equal(to_host(y), surv[:, None] * x.val.astype(np.float64))
