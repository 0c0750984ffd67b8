"""GPU parity: backward of the gate against the CPU checker."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2407_00599_amd import api, synth
from util import DEV, ROWS, assert_close, to_dev, to_host, rel_err, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("S,M,E,k,norm,dtype,acc", [
    (1, 8, 1, 1, 0, "f32", 0), (256, 64, 4, 1, 0, "f32", 1), (300, 72, 8, 2, 1, "f32", 1), (1000, 1024, 8, 2, 1, "bf16", 1),
    (777, 264, 16, 4, 0, "bf16", 0), (513, 128, 64, 2, 1, "bf16", 1), (400, 200, 100, 8, 0, "f32", 0),
    (2100, 2048, 17, 3, 1, "bf16", 1), (64, 64, 256, 8, 1, "f32", 1),
    # bf16, at most 8 experts, thousands of tokens (blocks of the fused kernel walk several 16-token stages): ragged
    # token and column tails, fewer than 8 experts, both weight normalisations, more than 65536 tokens
    (2048, 256, 8, 1, 0, "bf16", 1), (2049, 264, 8, 2, 1, "bf16", 1), (4099, 1032, 5, 2, 0, "bf16", 0),
    (3000, 520, 1, 1, 0, "bf16", 1), (70001, 72, 8, 2, 1, "bf16", 1),
])
def test_gate_bwd(S, M, E, k, norm, dtype, acc):
    rng = np.random.default_rng(S + E)
    x = synth.store(rng.standard_normal((S, M)).astype(np.float32), dtype)
    Wg = (rng.standard_normal((M, E)) * 0.1).astype(np.float32)
    logits = synth.synthetic_logits(S, E, seed=S)
    idx = O.topk_select(logits, k)
    w = O.combine_weights(logits, idx, bool(norm)).astype(np.float32)
    dw = rng.standard_normal((S, k)).astype(np.float32)
    dx0 = synth.store(rng.standard_normal((S, M)).astype(np.float32), dtype)
    tdt = torch_dtype(dtype)
    dl = torch.empty(S, E, device=DEV); dWg = torch.empty(M, E, device=DEV); db = torch.empty(E, device=DEV)
    dx = to_dev(dx0).clone()
    # a workspace full of 0xFF bytes (NaN as bf16 or fp32): nothing may be read from it that the call has not written
    ws = torch.full((api.moe_gate_bwd_workspace_bytes(S, M, E),), 255, dtype=torch.uint8, device=DEV)
    api.moe_gate_bwd(to_dev(dw), to_dev(w), to_dev(idx), to_dev(logits), to_dev(x), to_dev(Wg), S, M, E, k, norm,
                     dl, dWg, db, dx, acc, ws)
    torch.cuda.synchronize()
    rdl, rdWg, rdb, rdx = O.gate_bwd(dw, logits, idx, bool(norm), x.val, Wg)
    assert rel_err(to_host(dl), rdl) <= 1e-5
    assert rel_err(to_host(dWg), rdWg) <= 1e-5
    assert rel_err(to_host(db), rdb) <= 1e-5
    ref_dx = rdx + (dx0.val if acc else 0.0)
    assert rel_err(to_host(dx), ref_dx) <= (1e-5 if dtype == "f32" else 4e-3)
    assert_close(to_host(dWg), rdWg, 1e-5, "dWg")
    assert_close(to_host(db), rdb, 1e-5, "dbias")
    assert_close(to_host(dx), ref_dx, 1e-5 if dtype == "f32" else 4e-3, "dx", ROWS)
    if k == 1 and norm:
        assert np.all(to_host(dl) == 0)
