"""GPU parity: the whole layer (all experts local, ESP shards run in turn) against the CPU
checker, tensor by tensor, forward and backward; plus run-to-run determinism."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2407_00599_amd import synth
from paper_2407_00599_amd.layer import MoERankLayer
from util import DEV, TOL, ROWS, EXPERT, to_dev, to_host, rel_err, assert_close, torch_dtype

pytestmark = pytest.mark.gpu

INT_NAMES = ("idx", "slot", "inv", "counts")


def run_layer(cfg, n_esp, norm):
    x = synth.tokens(cfg); Wg = synth.gate_weight(cfg); bias = synth.gate_bias(cfg)
    W1, W2 = synth.expert_weights(cfg, cfg.E); dy = synth.upstream_grad(cfg)
    L = MoERankLayer(cfg.S_total, cfg.M, cfg.H, cfg.E, cfg.k, cfg.f, dtype=torch_dtype(cfg.dtype), n_mp=cfg.n_mp,
                     mp_idx=cfg.mp_idx, n_esp=n_esp, norm_topk=norm, device=DEV)
    L.dW1.fill_(0); L.dW2.fill_(0)
    args = (to_dev(x), to_dev(Wg), to_dev(bias) if bias is not None else None, to_dev(W1), to_dev(W2))
    L.forward(*args); L.backward(to_dev(dy))
    torch.cuda.synchronize()
    xs = x.val[O.mp_slice(cfg.S_total, cfg.mp_idx, cfg.n_mp)]
    r = O.layer_fwd(xs, Wg, bias, W1.val, W2.val, cfg.k, cfg.f, bool(norm), n_esp)
    g = O.layer_bwd(r, dy.val, xs, Wg, W1.val, W2.val, cfg.k, bool(norm), n_esp)
    return L, r, g, args, to_dev(dy)


def compare(L, r, g, dtype, has_bias):
    assert np.array_equal(to_host(L.logits).astype(np.float32), r["logits"])
    for n in INT_NAMES:
        assert np.array_equal(to_host(getattr(L, n)), r[n]), n
    tol = TOL[dtype]
    assert rel_err(to_host(L.w), r["w"]) <= 1e-5
    assert np.array_equal(to_host(L.buf), r["buf"])
    pairs = [("Yret", L.Yret, r["Yret"], ROWS), ("y", L.y, r["y"], ROWS), ("dYret", L.dYret, g["dYret"], ROWS),
             ("dw", L.dw, g["dw"], None), ("dW1", L.dW1, g["dW1"], EXPERT), ("dW2", L.dW2, g["dW2"], EXPERT),
             ("dlogits", L.dlogits, g["dlogits"], None), ("dWg", L.dWg, g["dWg"], None), ("dx", L.dx, g["dx"], ROWS)]
    for name, a, b, group in pairs:
        assert_close(to_host(a), b, tol, name, group)
    if has_bias:
        assert_close(to_host(L.dbias), g["dbias"], tol, "dbias")
    # a token whose every choice was dropped gets a zero output row
    dropped = (r["slot"] < 0).all(axis=1)
    assert np.all(to_host(L.y)[dropped] == 0)


@pytest.mark.parametrize("name,n_esp,norm", [("tiny_fp32", 1, 0), ("tiny_fp32", 1, 1), ("tiny_fp32", 2, 0),
                                             ("layer_bf16", 1, 1), ("mp4_ep", 1, 1), ("mp4_ep", 2, 1)])
def test_layer_matches_checker(name, n_esp, norm):
    cfg = synth.CONFIGS[name]
    L, r, g, _, _ = run_layer(cfg, n_esp, norm)
    compare(L, r, g, cfg.dtype, cfg.bias != "none")
    if name == "tiny_fp32" and norm == 1:
        assert np.all(to_host(L.w) == 1.0) and np.all(to_host(L.dlogits) == 0)    # renormalised top-1 is 1


def test_small_bf16_layer_with_mp_slice_and_esp():
    cfg = synth.MoEConfig("small", 1536, 256, 512, 8, 2, 1.0, n_mp=3, mp_idx=2, bias="normal", cfg_id=9)
    L, r, g, _, _ = run_layer(cfg, 2, 1)
    compare(L, r, g, "bf16", True)
    assert (r["slot"] < 0).any()


def test_two_runs_are_bit_identical():
    cfg = synth.CONFIGS["layer_bf16"]
    L, r, g, args, dy = run_layer(cfg, 1, 1)
    first = {n: getattr(L, n).clone() for n in ("y", "dx", "dW1", "dW2", "dWg", "slot", "inv")}
    L.forward(*args); L.backward(dy)
    torch.cuda.synchronize()
    for n, t in first.items():
        assert torch.equal(getattr(L, n), t), n


@pytest.mark.parametrize("name,n_esp", [("tiny_fp32", 2), ("layer_bf16", 1), ("mp4_ep", 2)])
def test_forward_with_fused_dispatch_is_the_same_forward(name, n_esp):
    """Real routing from the gate: the forward that reads token rows through the inverse slot map gives the
    bits of the forward that dispatches first, and matches the checker."""
    cfg = synth.CONFIGS[name]
    L, r, g, args, run_dy = run_layer(cfg, n_esp, 1)
    ref = {n: getattr(L, n).clone() for n in ("Z", "A", "Yret", "y")}
    for n in ref:
        getattr(L, n).fill_(5.0)
    L.buf.fill_(float("nan"))                  # the fused path must not read the dispatch buffer
    L.forward_fused_dispatch(*args)
    torch.cuda.synchronize()
    for n, t in ref.items():
        assert torch.equal(getattr(L, n), t), n
    assert rel_err(to_host(L.y), r["y"]) <= TOL[cfg.dtype]
    # and the backward that reads the rows of X through the map: the same gradients, bit for bit
    gref = {n: getattr(L, n).clone() for n in ("dx", "dW1", "dW2", "dWg", "dbuf", "dw")}
    for n in gref:
        getattr(L, n).fill_(5.0)
    L.backward_fused_dispatch(run_dy)
    torch.cuda.synchronize()
    for n, t in gref.items():
        assert torch.equal(getattr(L, n), t), n
