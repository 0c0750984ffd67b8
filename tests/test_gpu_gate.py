"""GPU parity: gate (logits, top-k, weights, capacity slots) against the CPU checker.

Integer outputs are compared bit for bit.  The routing decision is taken on fp32 logits on both
sides: either the very same logits are handed to both (logits-in mode), or both compute them
with double accumulation from the same inputs, in which case the fp32 results are required to
agree to 1e-5 of the largest logit and the integers are compared wherever the two logit rows
are bit-identical (everywhere, in practice)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2407_00599_amd import api, synth
from util import DEV, to_dev, to_host, rel_err

pytestmark = pytest.mark.gpu


def run_gate(logits_np, k, C, norm, x=None, Wg=None, bias=None, S_total=None, mp=(0, 1), M=8):
    S, E = logits_np.shape if logits_np is not None else (S_total // mp[1], Wg.shape[1])
    i32, f32 = torch.int32, torch.float32
    logits = to_dev(logits_np) if logits_np is not None else torch.empty(S, E, dtype=f32, device=DEV)
    idx = torch.full((S, k), -7, dtype=i32, device=DEV); slot = torch.full((S, k), -7, dtype=i32, device=DEV)
    w = torch.full((S, k), -7.0, dtype=f32, device=DEV); inv = torch.full((E, C), -7, dtype=i32, device=DEV)
    counts = torch.full((E,), -7, dtype=i32, device=DEV)
    ws = torch.empty(api.moe_gate_workspace_bytes(S, E, k), dtype=torch.uint8, device=DEV)
    api.moe_gate_topk(x, Wg, bias, S_total if S_total else S, M, E, k, C, mp[0], mp[1], norm,
                      logits, idx, slot, w, inv, counts, ws)
    torch.cuda.synchronize()
    return dict(logits=to_host(logits), idx=to_host(idx), slot=to_host(slot), w=to_host(w), inv=to_host(inv),
                counts=to_host(counts))


def check_routing(got, logits_np, k, C, norm):
    E = logits_np.shape[1]
    idx = O.topk_select(logits_np, k)
    slot, inv, counts = O.capacity_slots(idx, E, C)
    assert np.array_equal(got["idx"], idx)
    assert np.array_equal(got["slot"], slot)
    assert np.array_equal(got["inv"], inv)
    assert np.array_equal(got["counts"], counts)
    w = O.combine_weights(logits_np, idx, bool(norm))
    assert rel_err(got["w"], w) <= 1e-5
    assert np.abs(got["w"] - w).max() <= 1e-6


CASES = [
    # S, E, k, C, ties, norm
    (1, 1, 1, 1, False, 0), (2, 2, 2, 1, False, 1), (64, 4, 1, 20, False, 0), (255, 8, 2, 64, False, 1),
    (256, 8, 2, 77, True, 1), (257, 8, 3, 5, True, 0), (1000, 5, 2, 300, False, 1), (1000, 16, 4, 250, True, 1),
    (777, 17, 8, 400, False, 0), (513, 64, 2, 17, True, 1), (2049, 100, 6, 100, False, 1), (1500, 256, 8, 40, True, 0),
    (300, 3, 3, 300, False, 1), (4096, 8, 2, 1229, False, 1), (70000, 64, 2, 2000, True, 1),
]


@pytest.mark.parametrize("S,E,k,C,ties,norm", CASES)
def test_routing_from_given_logits(S, E, k, C, ties, norm):
    logits = synth.synthetic_logits(S, E, seed=S + E + k, sigma=1.5, ties=ties)
    if E >= 8:
        logits = logits + np.linspace(0.0, 1.0, E, dtype=np.float32)[None]     # some imbalance -> drops
    got = run_gate(logits, k, C, norm)
    check_routing(got, logits, k, C, norm)
    assert np.array_equal(got["logits"].astype(np.float32), logits)            # input left untouched


def test_all_equal_logits_and_auto_norm():
    S, E, k, C = 300, 8, 2, 100
    logits = np.zeros((S, E), dtype=np.float32)
    got = run_gate(logits, k, C, -1)         # -1: renormalise because k >= 2
    check_routing(got, logits, k, C, 1)
    assert np.array_equal(got["idx"], np.tile(np.arange(k, dtype=np.int32), (S, 1)))
    got1 = run_gate(synth.synthetic_logits(S, E, seed=1), 1, C, -1)   # -1 with k = 1: raw probability
    assert (got1["w"] < 1.0).all()


@pytest.mark.parametrize("name", synth.CONFIG_ORDER)
def test_gate_from_activations_on_benchmark_shapes(name):
    cfg = synth.CONFIGS[name]
    x = synth.tokens(cfg); Wg = synth.gate_weight(cfg); bias = synth.gate_bias(cfg)
    C = O.capacity(cfg.S, cfg.E, cfg.k, cfg.f)
    assert C == api.moe_capacity(cfg.S, cfg.E, cfg.k, cfg.f)
    norm = 0 if cfg.k == 1 else 1
    got = run_gate(None, cfg.k, C, norm, x=to_dev(x), Wg=to_dev(Wg), bias=to_dev(bias) if bias is not None else None,
                   S_total=cfg.S_total, mp=(cfg.mp_idx, cfg.n_mp), M=cfg.M)
    ref = O.gate_logits(x.val[O.mp_slice(cfg.S_total, cfg.mp_idx, cfg.n_mp)], Wg, bias)
    assert rel_err(got["logits"], ref) <= 1e-5
    same = (got["logits"].astype(np.float32) == ref)
    assert same.mean() > 0.999
    if same.all():
        check_routing(got, ref, cfg.k, C, norm)
    else:   # a last-bit difference somewhere: the integers must still be the routing of the GPU's own fp32 logits
        check_routing(got, got["logits"].astype(np.float32), cfg.k, C, norm)
        rows = same.all(axis=1)
        assert np.array_equal(got["idx"][rows], O.topk_select(ref, cfg.k)[rows])
    if cfg.bias != "none" or cfg.f <= 1.0:
        assert (got["slot"] < 0).any()          # these workloads are built to drop tokens


@pytest.mark.parametrize("E,M,dtype", [(3, 64, "f32"), (12, 200, "bf16"), (24, 136, "bf16"), (64, 512, "f32"),
                                       (130, 72, "bf16")])
def test_gate_logits_odd_shapes(E, M, dtype):
    S, k = 333, min(E, 3)
    rng = np.random.default_rng(E * M)
    x = synth.store(rng.standard_normal((S * 3, M)).astype(np.float32), dtype)
    Wg = (rng.standard_normal((M, E)) * 0.3).astype(np.float32)
    bias = rng.standard_normal(E).astype(np.float32)
    got = run_gate(None, k, 50, 1, x=to_dev(x), Wg=to_dev(Wg), bias=to_dev(bias), S_total=S * 3, mp=(2, 3), M=M)
    ref = O.gate_logits(x.val[2 * S:], Wg, bias)
    assert rel_err(got["logits"], ref) <= 1e-6
    if (got["logits"].astype(np.float32) == ref).all():
        check_routing(got, ref, k, 50, 1)


@pytest.mark.parametrize("S,E,M,n_mp", [(9000, 12, 200, 1), (20001, 7, 1096, 1), (35000, 16, 520, 2), (70001, 3, 72, 1),
                                        (16384, 8, 1024, 1), (8192, 9, 64, 1)])
def test_gate_logits_many_tokens(S, E, M, n_mp):
    """bf16 activations, at most 16 experts, many tokens: the logits kernel on the 4-block fp64 matrix cores, with
    every block size it is launched with, token counts off every tile, and M off the 64- and 512-wide steps."""
    k = min(E, 2)
    rng = np.random.default_rng(S + E)
    x = synth.store(rng.standard_normal((S * n_mp, M)).astype(np.float32), "bf16")
    Wg = (rng.standard_normal((M, E)) * 0.3).astype(np.float32)
    bias = rng.standard_normal(E).astype(np.float32)
    C = O.capacity(S, E, k, 1.0)
    got = run_gate(None, k, C, 1, x=to_dev(x), Wg=to_dev(Wg), bias=to_dev(bias), S_total=S * n_mp, mp=(n_mp - 1, n_mp), M=M)
    ref = O.gate_logits(x.val[(n_mp - 1) * S:], Wg, bias)
    assert rel_err(got["logits"], ref) <= 1e-6
    same = got["logits"].astype(np.float32) == ref
    assert same.mean() > 0.9999
    if same.all():
        check_routing(got, ref, k, C, 1)
