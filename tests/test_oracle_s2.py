"""Pins for the checker's schedule-S2 functions (Section III-B): the slot ranges partition the
capacity, the per-rank buffers are the slices of the full dispatch buffer, and -- PauseMP changes
no arithmetic -- the S2 layer equals the plain layer on the whole token block; plus a brute-force
evaluation on a tiny case."""
import math

import numpy as np
import pytest

from oracle import moe_oracle as O


@pytest.mark.parametrize("C", [1, 2, 7, 64, 77, 1229])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 8])
def test_slot_ranges_partition_the_capacity(C, n):
    edges = [O.slot_range(C, r, n) for r in range(n)]
    assert edges[0][0] == 0 and edges[-1][1] == C
    for (a0, a1), (b0, b1) in zip(edges, edges[1:]):
        assert a1 == b0 and a0 <= a1
    sizes = [b - a for a, b in edges]
    assert max(sizes) - min(sizes) <= 1 and sum(sizes) == C
    with pytest.raises(ValueError):
        O.slot_range(C, n, n)


def _case(S=96, M=16, H=24, E=4, k=2, seed=5):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((S, M)).astype(np.float32)
    Wg = (rng.standard_normal((M, E)) * 0.5).astype(np.float32)
    W1 = (rng.standard_normal((E, M, H)) / math.sqrt(M)).astype(np.float32)
    W2 = (rng.standard_normal((E, H, M)) / math.sqrt(H)).astype(np.float32)
    return x, Wg, W1, W2


@pytest.mark.parametrize("n_mp,n_esp,f", [(1, 1, 1.0), (2, 1, 1.2), (4, 2, 0.5), (3, 3, 2.0)])
def test_s2_layer_equals_plain_layer(n_mp, n_esp, f):
    x, Wg, W1, W2 = _case()
    bias = np.linspace(-0.5, 0.5, Wg.shape[1]).astype(np.float32)
    a = O.layer_fwd_s2(x, Wg, bias, W1, W2, 2, f, True, n_mp, n_esp)
    b = O.layer_fwd(x, Wg, bias, W1, W2, 2, f, True, n_esp)
    assert a["C"] == b["C"] == O.capacity(x.shape[0], Wg.shape[1], 2, f)     # capacity from ALL tokens
    np.testing.assert_array_equal(a["inv"], b["inv"])
    np.testing.assert_array_equal(np.concatenate(a["buf_parts"], axis=1), b["buf"])
    np.testing.assert_allclose(a["Yret"], b["Yret"], rtol=0, atol=1e-12)
    np.testing.assert_allclose(a["y"], b["y"], rtol=0, atol=1e-12)


def test_s2_differs_from_s1_in_capacity():
    """S1 gates each MP slice on its own (capacity from B*L/N_MP tokens), S2 gates the whole block:
    with a tight capacity the two drop different tokens."""
    x, Wg, W1, W2 = _case(S=64, E=2, k=1, seed=11)
    n_mp, f = 2, 0.75
    s2 = O.layer_fwd_s2(x, Wg, None, W1, W2, 1, f, False, n_mp)
    assert s2["C"] == O.capacity(64, 2, 1, f) == 24
    halves = [O.layer_fwd(x[O.mp_slice(64, r, n_mp)], Wg, None, W1, W2, 1, f, False) for r in range(n_mp)]
    assert all(h["C"] == 12 for h in halves)
    kept_s1 = sum(int((h["slot"] >= 0).sum()) for h in halves)
    kept_s2 = int((s2["slot"] >= 0).sum())
    assert kept_s1 <= 48 and kept_s2 <= 48
    y_s1 = np.concatenate([h["y"] for h in halves], axis=0)
    assert not np.allclose(y_s1, s2["y"])          # the schedules agree only when nothing is dropped
    s2_loose = O.layer_fwd_s2(x, Wg, None, W1, W2, 1, 4.0, False, n_mp)
    halves_loose = [O.layer_fwd(x[O.mp_slice(64, r, n_mp)], Wg, None, W1, W2, 1, 4.0, False) for r in range(n_mp)]
    np.testing.assert_allclose(np.concatenate([h["y"] for h in halves_loose], axis=0), s2_loose["y"], atol=1e-12)


def test_s2_brute_force_tiny():
    """Token by token, straight from the definitions: y[t] = sum_j w_j FFN_{e_j}(x[t]) over the
    choices that found a slot, slots handed out choice-major then in token order."""
    x, Wg, W1, W2 = _case(S=10, M=4, H=6, E=3, k=2, seed=3)
    f, n_mp = 0.9, 2
    r = O.layer_fwd_s2(x, Wg, None, W1, W2, 2, f, True, n_mp)
    S, E, k = 10, 3, 2
    C = max(1, math.ceil(k * S * f / E))
    logits = x.astype(np.float64) @ Wg.astype(np.float64)
    logits = logits.astype(np.float32).astype(np.float64)
    chosen = [sorted(range(E), key=lambda e: (-logits[t, e], e))[:k] for t in range(S)]
    load = [0] * E
    keep = {}
    for j in range(k):
        for t in range(S):
            e = chosen[t][j]
            if load[e] < C:
                keep[(t, j)] = True
                load[e] += 1
    y = np.zeros((S, 4))
    for t in range(S):
        p = np.exp(logits[t, chosen[t]] - logits[t, chosen[t]].max())
        wts = p / p.sum()
        for j in range(k):
            if (t, j) in keep:
                e = chosen[t][j]
                z = x[t].astype(np.float64) @ W1[e].astype(np.float64)
                a = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in z])
                y[t] += wts[j] * (a @ W2[e].astype(np.float64))
    np.testing.assert_allclose(r["y"], y, rtol=1e-9, atol=1e-12)
