"""Pins for the floating-point part of the CPU checker: expert FFN, combine, gradients.

Anchors outside the checker: torch's CPU double-precision linear algebra / GeLU / autograd
for the dense special case, the sharding identity of the paper's "Model Parallelism"
paragraph, a per-token pure-Python evaluation of the layer definition, and central finite
differences of the scalar L = <y, dy> in float64 for every gradient.
"""
import math

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2407_00599_amd import synth


def small_layer(seed=0, S=24, M=5, H=8, E=4, k=2, skew=1.5, sigma_w=0.5):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((S, M))
    Wg = rng.standard_normal((M, E)) * 0.7
    bias = np.linspace(skew, 0, E)
    W1 = rng.standard_normal((E, M, H)) * sigma_w
    W2 = rng.standard_normal((E, H, M)) * sigma_w
    dy = rng.standard_normal((S, M))
    return x, Wg, bias, W1, W2, dy


def test_gelu_and_its_derivative():
    z = np.linspace(-6, 6, 241)
    # exact GeLU = z * Phi(z), checked against math.erf and torch
    ref = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in z])
    assert np.allclose(O.gelu(z), ref, rtol=1e-15, atol=1e-300)
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    gt = torch.nn.functional.gelu(zt)               # erf form
    assert np.allclose(O.gelu(z), gt.detach().numpy(), rtol=1e-13, atol=1e-16)
    gt.sum().backward()
    assert np.allclose(O.gelu_grad(z), zt.grad.numpy(), rtol=1e-12, atol=1e-15)
    h = 1e-6
    fd = (O.gelu(z + h) - O.gelu(z - h)) / (2 * h)
    assert np.allclose(O.gelu_grad(z), fd, rtol=0, atol=1e-9)
    assert O.gelu(np.array([0.0]))[0] == 0.0


def test_single_expert_is_a_dense_mlp():
    # E = 1, k = 1, f = 1: every token goes to the only expert with weight 1 and nothing drops,
    # so the layer is the two-layer MLP  y = GeLU(x W1) W2.
    rng = np.random.default_rng(4)
    S, M, H = 19, 7, 11
    x = rng.standard_normal((S, M)); W1 = rng.standard_normal((1, M, H)); W2 = rng.standard_normal((1, H, M))
    Wg = rng.standard_normal((M, 1)); dy = rng.standard_normal((S, M))
    r = O.layer_fwd(x, Wg, None, W1, W2, k=1, f=1.0, norm_topk=False)
    assert r["C"] == S and (r["slot"][:, 0] == np.arange(S)).all() and np.all(r["w"] == 1.0)
    xt = torch.tensor(x, requires_grad=True); w1 = torch.tensor(W1[0], requires_grad=True)
    w2 = torch.tensor(W2[0], requires_grad=True)
    yt = torch.nn.functional.gelu(xt @ w1) @ w2
    assert np.allclose(r["y"], yt.detach().numpy(), rtol=1e-12, atol=1e-13)
    (yt * torch.tensor(dy)).sum().backward()
    g = O.layer_bwd(r, dy, x, Wg, W1, W2, k=1, norm_topk=False)
    assert np.allclose(g["dW1"][0], w1.grad.numpy(), rtol=1e-11, atol=1e-12)
    assert np.allclose(g["dW2"][0], w2.grad.numpy(), rtol=1e-11, atol=1e-12)
    assert np.allclose(g["dx"], xt.grad.numpy(), rtol=1e-11, atol=1e-12)   # softmax over one expert: no gate grad
    assert np.allclose(g["dWg"], 0, atol=1e-14)


def test_ffn_matches_torch_per_expert_and_layouts():
    rng = np.random.default_rng(5)
    n_src, G, C, M, H = 3, 2, 5, 4, 6
    X = rng.standard_normal((n_src, G, C, M)); dY = rng.standard_normal((n_src, G, C, M))
    W1 = rng.standard_normal((G, M, H)); W2 = rng.standard_normal((G, H, M))
    Z, Y = O.expert_ffn_fwd(X, W1, W2)
    dX, dW1, dW2 = O.expert_ffn_bwd(dY, X, W1, W2)
    for g in range(G):
        rows = torch.tensor(X[:, g].reshape(n_src * C, M), requires_grad=True)
        w1 = torch.tensor(W1[g], requires_grad=True); w2 = torch.tensor(W2[g], requires_grad=True)
        z = rows @ w1
        y = torch.nn.functional.gelu(z) @ w2
        assert np.allclose(Z[:, g].reshape(-1, H), z.detach().numpy(), rtol=1e-13, atol=1e-14)
        assert np.allclose(Y[:, g].reshape(-1, M), y.detach().numpy(), rtol=1e-12, atol=1e-13)
        (y * torch.tensor(dY[:, g].reshape(-1, M))).sum().backward()
        assert np.allclose(dX[:, g].reshape(-1, M), rows.grad.numpy(), rtol=1e-11, atol=1e-12)
        assert np.allclose(dW1[g], w1.grad.numpy(), rtol=1e-11, atol=1e-12)
        assert np.allclose(dW2[g], w2.grad.numpy(), rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("n_esp", [2, 4])
def test_esp_shards_sum_to_the_unsharded_expert(n_esp):
    # Y = sum_p W2^(p) f(W1^(p) X): columns of W1 / rows of W2 split n_esp ways.
    rng = np.random.default_rng(6)
    n_src, G, C, M, H = 2, 3, 4, 5, 8
    X = rng.standard_normal((n_src, G, C, M)); dY = rng.standard_normal((n_src, G, C, M))
    W1 = rng.standard_normal((G, M, H)); W2 = rng.standard_normal((G, H, M))
    Z, Y = O.expert_ffn_fwd(X, W1, W2)
    dX, dW1, dW2 = O.expert_ffn_bwd(dY, X, W1, W2)
    Hl = H // n_esp
    Ysum = 0; dXsum = 0
    for j in range(n_esp):
        Zj, Yj = O.expert_ffn_fwd(X, W1, W2, j, n_esp)
        assert Zj.shape[-1] == Hl and np.allclose(Zj, Z[..., j * Hl:(j + 1) * Hl], rtol=1e-14)
        dXj, dW1j, dW2j = O.expert_ffn_bwd(dY, X, W1, W2, j, n_esp)
        assert np.allclose(dW1j, dW1[:, :, j * Hl:(j + 1) * Hl], rtol=1e-13)       # disjoint slices
        assert np.allclose(dW2j, dW2[:, j * Hl:(j + 1) * Hl, :], rtol=1e-13)
        Ysum = Ysum + Yj; dXsum = dXsum + dXj
    assert np.allclose(Ysum, Y, rtol=1e-12, atol=1e-13)
    assert np.allclose(dXsum, dX, rtol=1e-12, atol=1e-13)


def test_padding_rows_stay_zero_and_idle_expert_gets_no_gradient():
    rng = np.random.default_rng(7)
    X = np.zeros((1, 2, 3, 4)); X[0, 0, :2] = rng.standard_normal((2, 4))      # expert 1 has no rows
    W1 = rng.standard_normal((2, 4, 6)); W2 = rng.standard_normal((2, 6, 4))
    Z, Y = O.expert_ffn_fwd(X, W1, W2)
    assert np.all(Y[0, 0, 2] == 0) and np.all(Y[0, 1] == 0)
    dY = np.zeros_like(X); dY[0, 0, :2] = rng.standard_normal((2, 4))
    dX, dW1, dW2 = O.expert_ffn_bwd(dY, X, W1, W2)
    assert np.all(dW1[1] == 0) and np.all(dW2[1] == 0) and np.all(dX[0, 1] == 0)
    assert np.abs(dW1[0]).max() > 0


def per_token_layer(x, Wg, bias, W1, W2, k, f, norm_topk):
    """The layer written out token by token in pure Python floats:
    y[t] = sum over surviving choices of w * FFN_e(x[t]) with the sequential slot rule."""
    S, M = x.shape; E = Wg.shape[1]; H = W1.shape[2]
    C = max(1, math.ceil(k * S * f / E))
    logits = [[float(np.float32(sum(x[t, m] * Wg[m, e] for m in range(M)) + (bias[e] if bias is not None else 0)))
               for e in range(E)] for t in range(S)]
    choice = [sorted(range(E), key=lambda e: (-logits[t][e], e))[:k] for t in range(S)]
    fill = [0] * E
    alive = [[False] * k for _ in range(S)]
    for j in range(k):
        for t in range(S):
            e = choice[t][j]
            alive[t][j] = fill[e] < C
            fill[e] += 1
    y = np.zeros((S, M))
    for t in range(S):
        ex = [math.exp(v - max(logits[t])) for v in logits[t]]
        den = sum(ex[e] for e in choice[t]) if norm_topk else sum(ex)
        for j, e in enumerate(choice[t]):
            if not alive[t][j]:
                continue
            h = [sum(x[t, m] * W1[e, m, q] for m in range(M)) for q in range(H)]
            a = [0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in h]
            for m in range(M):
                y[t, m] += ex[e] / den * sum(a[q] * W2[e, q, m] for q in range(H))
    return y, alive


@pytest.mark.parametrize("k,norm", [(1, False), (2, True), (2, False), (3, True)])
def test_layer_equals_per_token_definition(k, norm):
    x, Wg, bias, W1, W2, dy = small_layer(seed=10 + k, S=20, E=4, k=k)
    f = 1.0
    r = O.layer_fwd(x, Wg, bias, W1, W2, k=k, f=f, norm_topk=norm, n_esp=2)
    y, alive = per_token_layer(x, Wg, bias, W1, W2, k, f, norm)
    assert np.array_equal(np.array(alive), r["slot"] >= 0)
    assert not np.all(alive)                       # the bias makes some assignments drop
    assert np.allclose(r["y"], y, rtol=1e-11, atol=1e-12)


def _loss(x, Wg, bias, W1, W2, dy, k, f, norm, n_esp, C):
    # unrounded logits: fp32 rounding of the logits would show up as noise in the differences
    r = O.layer_fwd(x, Wg, bias, W1, W2, k=k, f=f, norm_topk=norm, n_esp=n_esp, C=C,
                    logits_dtype=np.float64)
    return float((r["y"] * dy).sum()), r


@pytest.mark.parametrize("k,norm,n_esp", [(1, False, 1), (2, True, 2), (2, False, 1), (3, True, 1), (1, True, 1)])
def test_gradients_by_central_finite_differences(k, norm, n_esp):
    x, Wg, bias, W1, W2, dy = small_layer(seed=20 + 3 * k + n_esp, S=16, M=4, H=6, E=4, k=k)
    f = 1.0
    L0, r = _loss(x, Wg, bias, W1, W2, dy, k, f, norm, n_esp, None)
    C = r["C"]
    assert (r["slot"] < 0).any()
    g = O.layer_bwd(r, dy, x, Wg, W1, W2, k=k, norm_topk=norm, n_esp=n_esp)
    # margin between the k-th and (k+1)-th logit: skip nothing, but require it is comfortable
    srt = np.sort(r["logits"].astype(np.float64), axis=1)[:, ::-1]
    assert (srt[:, k - 1] - srt[:, k]).min() > 1e-3
    eps = 1e-6
    args = dict(x=x, Wg=Wg, bias=bias, W1=W1, W2=W2)
    names = {"x": "dx", "Wg": "dWg", "bias": "dbias", "W1": "dW1", "W2": "dW2"}
    rng = np.random.default_rng(0)
    for name, gname in names.items():
        a = args[name]
        flat_idx = rng.choice(a.size, size=min(a.size, 40), replace=False)
        for fi in flat_idx:
            pos = np.unravel_index(fi, a.shape)
            old = a[pos]
            a[pos] = old + eps; Lp, rp = _loss(**args, dy=dy, k=k, f=f, norm=norm, n_esp=n_esp, C=C)
            a[pos] = old - eps; Lm, rm = _loss(**args, dy=dy, k=k, f=f, norm=norm, n_esp=n_esp, C=C)
            a[pos] = old
            assert np.array_equal(rp["idx"], r["idx"]) and np.array_equal(rm["idx"], r["idx"])
            fd = (Lp - Lm) / (2 * eps)
            an = g[gname][pos]
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an)), (name, pos, fd, an)
    if k == 1 and norm:
        assert np.all(g["dlogits"] == 0) and np.all(g["dWg"] == 0)      # weight is identically 1


def test_backward_is_linear_in_dy_and_combine_bwd_pieces():
    x, Wg, bias, W1, W2, dy = small_layer(seed=31, S=18, E=4, k=2)
    r = O.layer_fwd(x, Wg, bias, W1, W2, k=2, f=1.0, norm_topk=True)
    g1 = O.layer_bwd(r, dy, x, Wg, W1, W2, k=2, norm_topk=True)
    g2 = O.layer_bwd(r, -2.5 * dy, x, Wg, W1, W2, k=2, norm_topk=True)
    for key in ("dx", "dWg", "dW1", "dW2", "dw", "dYret"):
        assert np.allclose(g2[key], -2.5 * g1[key], rtol=1e-12, atol=1e-14)
    # dYret is the weighted dispatch of dy; dw is zero exactly where the choice was dropped
    assert np.allclose(g1["dYret"], O.dispatch(dy, r["inv"], 2, r["w"]), rtol=1e-15)
    assert np.all(g1["dw"][r["slot"] < 0] == 0) and np.all(g1["dw"][r["slot"] >= 0] != 0)
    # dx of dispatch alone = unweighted combine of the returned gradient
    assert np.allclose(g1["dx"], g1["dx_disp"] + g1["dx_gate"])


def test_mp_ranks_partition_the_layer_when_nothing_drops():
    # Schedule S1: each MP rank gates its own token block; with a capacity that drops
    # nothing the concatenation of the ranks' outputs is the layer output on all tokens.
    x, Wg, bias, W1, W2, dy = small_layer(seed=40, S=24, E=4, k=2, skew=0.0)
    full = O.layer_fwd(x, Wg, None, W1, W2, k=2, f=2.0, norm_topk=True)
    assert (full["slot"] >= 0).all()
    parts = []
    for p in range(3):
        sl = O.mp_slice(24, p, 3)
        rp = O.layer_fwd(x[sl], Wg, None, W1, W2, k=2, f=2.0, norm_topk=True)
        assert (rp["slot"] >= 0).all()
        parts.append(rp["y"])
    assert np.allclose(np.concatenate(parts), full["y"], rtol=1e-12, atol=1e-13)


def test_row_and_hidden_unit_forms_agree_with_the_full_expert():
    rng = np.random.default_rng(50)
    n_src, G, C, M, H = 2, 2, 6, 5, 8
    X = rng.standard_normal((n_src, G, C, M)); dY = rng.standard_normal((n_src, G, C, M))
    W1 = rng.standard_normal((G, M, H)); W2 = rng.standard_normal((G, H, M))
    Z, Y = O.expert_ffn_fwd(X, W1, W2, 1, 2)
    dX, dW1, dW2 = O.expert_ffn_bwd(dY, X, W1, W2, 1, 2)
    g = 1
    w1s, w2s = W1[g][:, 4:], W2[g][4:, :]
    z, y, dx = O.expert_ffn_rows(X[1, g, 2:4], dY[1, g, 2:4], w1s, w2s)
    assert np.allclose(z, Z[1, g, 2:4], rtol=1e-13) and np.allclose(y, Y[1, g, 2:4], rtol=1e-12)
    assert np.allclose(dx, dX[1, g, 2:4], rtol=1e-12, atol=1e-13)
    a, b = O.expert_ffn_hidden_unit(X[:, g].reshape(-1, M), dY[:, g].reshape(-1, M), w1s[:, 3], w2s[3, :])
    assert np.allclose(a, dW1[g][:, 3], rtol=1e-12, atol=1e-13) and np.allclose(b, dW2[g][3, :], rtol=1e-12, atol=1e-13)
