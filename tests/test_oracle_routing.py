"""Pins for the routing part of the CPU checker: capacity, top-k, weights, slots.

None of these retype the checker's own vectorised formulas: they use the paper's printed
formula evaluated by hand (golden file), a sequential queue simulation in pure Python,
closed forms for degenerate inputs, invariants, and scipy's softmax.
"""
import os

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import moe_oracle as O
from paper_2407_00599_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_capacity_matches_paper_formula_on_benchmark_shapes():
    rows = []
    for line in open(os.path.join(GOLDEN, "capacity.txt")):
        line = line.split("#")[0].split()
        if line:
            rows.append(line)
    assert len(rows) == 5
    for S, E, k, f, T in rows:
        assert O.capacity(int(S), int(E), int(k), float(f)) == int(T)
    # the five configs of the generator agree with the table
    for name, row in zip(synth.CONFIG_ORDER, rows):
        c = synth.CONFIGS[name]
        assert (c.S, c.E, c.k, c.f) == (int(row[0]), int(row[1]), int(row[2]), float(row[3]))


def test_capacity_edge_cases():
    assert O.capacity(1, 64, 1, 1.0) == 1          # never below one row
    assert O.capacity(8, 4, 2, 1.0) == 4
    assert O.capacity(7, 4, 1, 1.0) == 2           # 1.75 -> 2
    assert O.capacity(100, 8, 2, 2.4) == 60        # paper's second capacity factor


def brute_topk(l_row, k):
    order = sorted(range(len(l_row)), key=lambda e: (-float(l_row[e]), e))
    return order[:k]


def brute_slots(idx, E, C):
    """Sequential simulation: serve all first choices in token order, then all second
    choices, ...; each expert hands out slots 0,1,2,.. until C are taken."""
    S, k = idx.shape
    fill = [0] * E
    slot = -np.ones((S, k), dtype=np.int32)
    inv = -np.ones((E, C), dtype=np.int32)
    counts = np.zeros(E, dtype=np.int32)
    for j in range(k):
        for t in range(S):
            e = int(idx[t, j])
            counts[e] += 1
            if fill[e] < C:
                slot[t, j] = fill[e]
                inv[e, fill[e]] = t * k + j
            fill[e] += 1
    return slot, inv, counts


@pytest.mark.parametrize("S,E,k,C,ties", [
    (1, 1, 1, 1, False), (7, 3, 1, 2, False), (33, 4, 2, 9, False), (64, 8, 3, 11, True),
    (50, 5, 5, 50, False), (64, 8, 2, 1, True), (40, 6, 2, 200, False), (64, 64, 2, 3, True),
])
def test_routing_equals_bruteforce(S, E, k, C, ties):
    for seed in range(3):
        logits = synth.synthetic_logits(S, E, seed=seed + 17 * S, ties=ties)
        idx = O.topk_select(logits, k)
        for t in range(S):
            assert list(idx[t]) == brute_topk(logits[t], k)
        slot, inv, counts = O.capacity_slots(idx, E, C)
        bs, bi, bc = brute_slots(idx, E, C)
        assert np.array_equal(slot, bs) and np.array_equal(inv, bi) and np.array_equal(counts, bc)


def test_routing_invariants():
    S, E, k = 300, 8, 2
    logits = synth.synthetic_logits(S, E, seed=5) + np.linspace(0, 2, E, dtype=np.float32)[None]
    C = O.capacity(S, E, k, 1.0)
    idx = O.topk_select(logits, k)
    slot, inv, counts = O.capacity_slots(idx, E, C)
    # each token goes to k distinct experts
    assert all(len(set(r)) == k for r in idx.tolist())
    assert counts.sum() == S * k
    for e in range(E):
        used = int(((idx == e) & (slot >= 0)).sum())
        assert used == min(int(counts[e]), C)                      # never more than C
        assert np.all(inv[e, :used] >= 0) and np.all(inv[e, used:] == -1)   # dense from slot 0
    assert (slot < 0).any()                                        # skew makes some drop
    # inv o slot = identity on surviving assignments
    t, j = np.nonzero(slot >= 0)
    assert np.array_equal(inv[idx[t, j], slot[t, j]], t * k + j)
    # choice-major priority: a dropped first choice implies that expert took no second choices
    for e in range(E):
        if ((idx[:, 0] == e) & (slot[:, 0] < 0)).any():
            assert not ((idx[:, 1] == e) & (slot[:, 1] >= 0)).any()


def test_all_equal_logits_closed_form():
    # Every token's j-th choice is expert j (ties -> lowest index), so expert j only sees
    # j-th choices and slot[t,j] = t while t < C.
    S, E, k, C = 20, 6, 3, 7
    logits = np.zeros((S, E), dtype=np.float32)
    idx = O.topk_select(logits, k)
    assert np.array_equal(idx, np.tile(np.arange(k, dtype=np.int32), (S, 1)))
    slot, inv, counts = O.capacity_slots(idx, E, C)
    want = np.where(np.arange(S) < C, np.arange(S), -1)
    for j in range(k):
        assert np.array_equal(slot[:, j], want)
    assert np.array_equal(counts, [S, S, S, 0, 0, 0])
    assert np.all(inv[k:] == -1)
    w = O.combine_weights(logits, idx, True)
    assert np.allclose(w, 1.0 / k, rtol=0, atol=1e-15)
    assert np.allclose(O.combine_weights(logits, idx, False), 1.0 / E, rtol=0, atol=1e-15)


def test_large_capacity_factor_drops_nothing():
    S, E, k = 128, 8, 2
    logits = synth.synthetic_logits(S, E, seed=9) * 3
    C = O.capacity(S, E, k, E / k)         # f = E/k  ->  C = S: an expert can take every token
    assert C == S
    slot, _, _ = O.capacity_slots(O.topk_select(logits, k), E, C)
    assert (slot >= 0).all()


def test_permuting_experts_permutes_selection():
    S, E, k = 64, 8, 3
    logits = synth.synthetic_logits(S, E, seed=21)
    perm = np.random.default_rng(0).permutation(E)
    idx = O.topk_select(logits, k)
    idx_p = O.topk_select(logits[:, perm], k)         # column c of the permuted logits is expert perm[c]
    assert np.array_equal(perm[idx_p], idx)           # no ties here, so order is preserved too


def test_weights_against_library_softmax():
    S, E, k = 96, 16, 4
    logits = synth.synthetic_logits(S, E, seed=3) * 2
    idx = O.topk_select(logits, k)
    w = O.combine_weights(logits, idx, True)
    sel = np.take_along_axis(logits.astype(np.float64), idx.astype(np.int64), 1)
    assert np.allclose(w, scipy_softmax(sel, axis=1), rtol=1e-13, atol=0)
    assert np.allclose(w.sum(1), 1.0, rtol=0, atol=1e-14)
    assert np.all(np.diff(w, axis=1) <= 0)            # best expert first
    p = scipy_softmax(logits.astype(np.float64), axis=1)
    w0 = O.combine_weights(logits, idx, False)
    assert np.allclose(w0, np.take_along_axis(p, idx.astype(np.int64), 1), rtol=1e-13)
    # E == k: renormalising changes nothing
    idx_all = O.topk_select(logits, E)
    assert np.allclose(O.combine_weights(logits, idx_all, True), O.combine_weights(logits, idx_all, False),
                       rtol=1e-13)
    # top-1 renormalised is identically one
    assert np.all(O.combine_weights(logits, O.topk_select(logits, 1), True) == 1.0)


def test_gate_logits_is_a_linear_layer_and_slices_tokens():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((12, 5)).astype(np.float32)
    Wg = rng.standard_normal((5, 3)).astype(np.float32)
    b = rng.standard_normal(3).astype(np.float32)
    l = O.gate_logits(x, Wg, b)
    assert l.dtype == np.float32
    for t in range(12):
        for e in range(3):
            ref = sum(float(x[t, m]) * float(Wg[m, e]) for m in range(5)) + float(b[e])
            assert abs(l[t, e] - ref) <= 1e-6 * max(1.0, abs(ref))
    sl = O.mp_slice(12, 2, 3)
    assert (sl.start, sl.stop) == (8, 12)
    assert np.array_equal(O.gate_logits(x[sl], Wg, b), l[8:12])


def test_dispatch_combine_round_trip_and_zero_padding():
    S, E, k, M = 40, 4, 2, 6
    rng = np.random.default_rng(2)
    x = rng.standard_normal((S, M))
    logits = synth.synthetic_logits(S, E, seed=2) + np.array([2, 0, 0, 0], np.float32)
    C = O.capacity(S, E, k, 1.0)
    idx = O.topk_select(logits, k)
    slot, inv, counts = O.capacity_slots(idx, E, C)
    buf = O.dispatch(x, inv, k)
    assert buf.shape == (E, C, M)
    for e in range(E):
        for c in range(C):
            if inv[e, c] < 0:
                assert np.all(buf[e, c] == 0.0)
            else:
                assert np.array_equal(buf[e, c], x[inv[e, c] // k])
    # identity experts + unit weights: every token comes back once per surviving choice
    y = O.combine_fwd(buf, idx, slot, None)
    surv = (slot >= 0).sum(1)
    assert (surv == 0).any() or (surv < k).any()
    assert np.allclose(y, surv[:, None] * x, rtol=1e-15, atol=0)
    assert np.all(y[surv == 0] == 0.0)
    # weighted dispatch scales rows by the gate weight
    w = O.combine_weights(logits, idx, True)
    bw = O.dispatch(x, inv, k, w)
    t, j = np.nonzero(slot >= 0)
    assert np.allclose(bw[idx[t, j], slot[t, j]], w[t, j][:, None] * x[t], rtol=1e-15)
    # n_part partial sums are added before the weighted gather
    parts = np.stack([0.25 * buf, 0.75 * buf])
    assert np.allclose(O.combine_fwd(parts, idx, slot, w), O.combine_fwd(buf, idx, slot, w), rtol=1e-14)
