"""GPU parity for schedule S2 (Section III-B): the slot-range dispatch against slices of the checker's
dispatch buffer, bit for bit, and the whole S2 composition of an MP group against the checker's S2
layer (which equals the plain layer on all tokens of the group)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2407_00599_amd import api, synth
from s2_group import MoES2Group
from util import DEV, TOL, to_dev, to_host, rel_err, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("S,M,E,k,C,n,dtype", [
    (100, 64, 4, 2, 30, 3, "f32"), (300, 520, 8, 2, 61, 4, "bf16"), (1000, 1024, 16, 3, 150, 8, "bf16"),
    (64, 8, 2, 1, 3, 4, "f32"),     # ranks with an empty range (C < n) are rejected by the call
])
def test_dispatch_slots(S, M, E, k, C, n, dtype):
    rng = np.random.default_rng(S + C)
    logits = synth.synthetic_logits(S, E, seed=S, sigma=1.0)
    idx = O.topk_select(logits, k)
    slot, inv, counts = O.capacity_slots(idx, E, C)
    w = O.combine_weights(logits, idx, True).astype(np.float32)
    x = synth.store(rng.standard_normal((S, M)).astype(np.float32), dtype)
    full = O.dispatch(x.val, inv, k)
    fullw = O.dispatch(x.val, inv, k, w)
    d_x, d_inv, d_w = to_dev(x), to_dev(inv), to_dev(w)
    tdt = torch_dtype(dtype)
    seen = 0
    for r in range(n):
        c0, c1 = O.slot_range(C, r, n)
        if c1 == c0:
            with pytest.raises(api.MoEError):
                api.moe_dispatch_slots(d_x, S, M, E, k, C, c0, c1, d_inv, None, torch.empty(8, dtype=tdt, device=DEV))
            continue
        part = torch.full((E, c1 - c0, M), 7.0, dtype=tdt, device=DEV)
        api.moe_dispatch_slots(d_x, S, M, E, k, C, c0, c1, d_inv, None, part)
        assert np.array_equal(to_host(part), full[:, c0:c1])               # pure copy: exact
        assert np.array_equal(to_host(part), O.dispatch(x.val, inv[:, c0:c1], k))
        partw = torch.full((E, c1 - c0, M), 7.0, dtype=tdt, device=DEV)
        api.moe_dispatch_slots(d_x, S, M, E, k, C, c0, c1, d_inv, d_w, partw)
        assert rel_err(to_host(partw), fullw[:, c0:c1]) <= (1e-6 if dtype == "f32" else 4e-3)
        seen += c1 - c0
    assert seen == C
    with pytest.raises(api.MoEError):
        api.moe_dispatch_slots(d_x, S, M, E, k, C, 0, C + 1, d_inv, None, torch.empty(8, dtype=tdt, device=DEV))


@pytest.mark.parametrize("name,n_mp,n_esp", [("tiny_fp32", 2, 1), ("tiny_fp32", 3, 2), ("mp4_ep", 4, 1)])
def test_s2_group_matches_checker(name, n_mp, n_esp):
    cfg = synth.CONFIGS[name]
    x = synth.tokens(cfg); Wg = synth.gate_weight(cfg); bias = synth.gate_bias(cfg)
    W1, W2 = synth.expert_weights(cfg, cfg.E)
    S = cfg.S_total                                   # S2 gates every token of the MP group
    rng = np.random.default_rng(cfg.cfg_id)
    dy = synth.store(rng.standard_normal((S, cfg.M)).astype(np.float32), cfg.dtype)
    norm = 1
    L = MoES2Group(S, cfg.M, cfg.H, cfg.E, cfg.k, cfg.f, dtype=torch_dtype(cfg.dtype), n_mp=n_mp, n_esp=n_esp,
                   norm_topk=norm, device=DEV)
    L.forward(to_dev(x), to_dev(Wg), to_dev(bias) if bias is not None else None, to_dev(W1), to_dev(W2))
    L.backward(to_dev(dy))
    torch.cuda.synchronize()
    r = O.layer_fwd_s2(x.val, Wg, bias, W1.val, W2.val, cfg.k, cfg.f, bool(norm), n_mp, n_esp)
    r["buf"] = np.concatenate(r["buf_parts"], axis=1)
    g = O.layer_bwd(r, dy.val, x.val, Wg, W1.val, W2.val, cfg.k, bool(norm), n_esp)
    assert L.C == r["C"]
    assert np.array_equal(to_host(L.logits).astype(np.float32), r["logits"])
    for n in ("idx", "slot", "inv", "counts"):
        assert np.array_equal(to_host(getattr(L, n)), r[n]), n
    for rank, (c0, c1) in enumerate(L.ranges):
        assert (c0, c1) == O.slot_range(r["C"], rank, n_mp)
        if c1 > c0:
            assert np.array_equal(to_host(L.parts[rank]), r["buf_parts"][rank])
    tol = TOL[cfg.dtype]
    for nm, a, b in [("Yret", L.Yret, r["Yret"]), ("y", L.y, r["y"]), ("dw", L.dw, g["dw"]), ("dbuf", L.dbuf, None),
                     ("dW1", L.dW1, g["dW1"]), ("dW2", L.dW2, g["dW2"]), ("dlogits", L.dlogits, g["dlogits"]),
                     ("dWg", L.dWg, g["dWg"]), ("dx", L.dx, g["dx"])]:
        if b is not None:
            e = rel_err(to_host(a), b)
            assert e <= tol, (nm, e)
