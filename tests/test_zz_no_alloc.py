"""The gate entry point that allocates nothing (its histograms live in the library's static device array)
against moe_gate_topk with a caller's workspace: the same kernels on the same inputs, so every output must
agree bit for bit, on two calls in a row, the second on a smaller problem (the array keeps the first call's
contents), through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2407_00599_amd import api, synth
from util import DEV, to_dev

pytestmark = pytest.mark.gpu


def outputs(S, E, k, C):
    i32, f32 = torch.int32, torch.float32
    return dict(logits=torch.full((S, E), -7.0, dtype=f32, device=DEV), idx=torch.full((S, k), -7, dtype=i32, device=DEV),
                slot=torch.full((S, k), -7, dtype=i32, device=DEV), w=torch.full((S, k), -7.0, dtype=f32, device=DEV),
                inv=torch.full((E, C), -7, dtype=i32, device=DEV), counts=torch.full((E,), -7, dtype=i32, device=DEV))


def both(S_total, M, E, k, f, n_mp, mp_idx, seed, from_logits=False):
    S = S_total // n_mp
    C = api.moe_capacity(S, E, k, f)
    rng = np.random.default_rng(seed)
    x = to_dev(synth.store(rng.standard_normal((S_total, M)).astype(np.float32), "bf16"))
    Wg = to_dev((rng.standard_normal((M, E)) * 0.1).astype(np.float32))
    bias = to_dev(rng.standard_normal(E).astype(np.float32))
    a, b = outputs(S, E, k, C), outputs(S, E, k, C)
    if from_logits:
        lg = to_dev(synth.synthetic_logits(S, E, seed=seed, ties=True))
        a["logits"].copy_(lg); b["logits"].copy_(lg)
        x = Wg = None
    ws = torch.empty(api.moe_gate_workspace_bytes(S, E, k), dtype=torch.uint8, device=DEV)
    api.moe_gate_topk(x, Wg, bias, S_total, M, E, k, C, mp_idx, n_mp, 1, a["logits"], a["idx"], a["slot"], a["w"],
                      a["inv"], a["counts"], ws)
    api.moe_gate_topk_static(x, Wg, bias, S_total, M, E, k, C, mp_idx, n_mp, 1, b["logits"], b["idx"], b["slot"], b["w"],
                             b["inv"], b["counts"])
    torch.cuda.synchronize()
    for n in a:
        assert torch.equal(a[n], b[n]), (n, S, E, k)
    assert (a["slot"] >= 0).any() and int(a["counts"].sum()) == S * k


def test_static_gate_matches_workspace_gate_twice_in_a_row():
    both(16384, 256, 64, 2, 1.25, 1, 0, seed=1)            # scan + slots kernels, 256 token blocks
    both(3 * 700, 136, 8, 2, 1.0, 3, 1, seed=2)             # smaller, right after: stale histograms in the array
    both(300, 8, 5, 3, 0.5, 1, 0, seed=3, from_logits=True)  # logits given, ties, the single-kernel slot path


def test_static_gate_rejects_what_does_not_fit():
    S, E, k = 1 << 20, 256, 8                               # 16384 blocks x 2048 counters x 2 halves: far too much
    assert api.moe_gate_workspace_bytes(S, E, k) > api.MOE_GATE_STATIC_SCRATCH_BYTES
    t = torch.empty(64, dtype=torch.float32, device=DEV)
    with pytest.raises(api.MoEError) as err:
        api.moe_gate_topk_static(None, None, None, S, 8, E, k, 100, 0, 1, 1, t, t.view(torch.int32), t.view(torch.int32), t,
                                 t.view(torch.int32), t.view(torch.int32))
    assert err.value.code == -7
