"""CPU checker for one rank's share of a Parm MoE layer -- TEST INFRASTRUCTURE ONLY.

This is a plain, slow, float64 restatement of what the per-rank path of an
MP+EP+ESP mixture-of-experts layer computes (gate -> dispatch -> sharded expert
FFN -> combine, and the chain rule through each).  It exists so that the HIP
library can be checked against something written independently of it.  Only the
tests, the smoke entry and the benchmark's cpu_baseline leg may call it; the
product path never does, and this file imports nothing from the product.

Every function names the passage of the paper it restates.  Where the paper is
silent the chosen reading is stated next to the code (and pinned by the CPU
tests, since the paper prints no worked example of these steps):

  * capacity T = k*f*S/E is rounded up, evaluated in double as ((k*S)*f)/E, min 1;
  * S is the number of tokens this rank gates: the MP slice under schedule S1;
  * top-k is taken on the fp32 logits, equal logits go to the lower expert index;
  * capacity slots are handed out choice-major (every first choice before any
    second choice), then in token order;
  * combine weights are the softmax over the k selected logits (norm_topk) or the
    full-softmax probabilities of the selected experts; they do not depend on drops;
  * a dropped (token, choice) contributes zero; a token with every choice dropped
    gets a zero output row;
  * the expert is  Y = GeLU(X W1) W2  with the exact (erf) GeLU and no biases;
  * ESP shard j owns columns [j*H/N, (j+1)*H/N) of W1 and the same rows of W2.

Parity pins: see tests/test_oracle_*.py (brute-force routing on tiny inputs,
closed forms, invariants, library cross-checks of the dense special case, central
finite differences of every gradient).  The conventions listed above are choices,
not facts of the paper: "parity unpinned" applies to them and to nothing else.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# --------------------------------------------------------------------------- #
# Section II-A, "Gating Function": T := k * f * B * L / E
# --------------------------------------------------------------------------- #
def capacity(S: int, E: int, k: int, f: float) -> int:
    """Maximum number of tokens one expert accepts (the paper's T), for S gated tokens."""
    t = (float(k * S) * float(f)) / float(E)
    c = int(np.ceil(t))
    return max(c, 1)


def mp_slice(S_total: int, mp_idx: int, n_mp: int) -> slice:
    """Section III-B (PauseMP, schedule S1): MP rank mp_idx keeps one contiguous
    1/N_MP block of the flattened B*L tokens."""
    assert S_total % n_mp == 0 and 0 <= mp_idx < n_mp
    S = S_total // n_mp
    return slice(mp_idx * S, (mp_idx + 1) * S)


# --------------------------------------------------------------------------- #
# Section II-A: the gate is one linear layer followed by softmax and top-k.
# --------------------------------------------------------------------------- #
def gate_logits(x, Wg, bias=None, out_dtype=np.float32):
    """logits[t,e] = sum_m x[t,m] Wg[m,e] (+ bias[e]); float64 sum, rounded once to fp32 (the
    precision the routing decision is taken in).  out_dtype=float64 skips that rounding; only
    the finite-difference tests use it, so that the loss is smooth in the inputs."""
    l = np.asarray(x, F64) @ np.asarray(Wg, F64)
    if bias is not None:
        l = l + np.asarray(bias, F64)[None, :]
    return l.astype(out_dtype)


def topk_select(logits, k: int):
    """For each token the k experts with the largest logits, best first; among equal
    logits the lower expert index wins.  (Softmax is monotone, so this is the top-k
    of the softmax layer.)"""
    l = np.array(logits, dtype=F64, copy=True)
    S, E = l.shape
    assert 1 <= k <= E
    idx = np.empty((S, k), dtype=np.int32)
    rows = np.arange(S)
    for j in range(k):
        e = np.argmax(l, axis=1)          # first occurrence of the maximum = lowest index
        idx[:, j] = e
        l[rows, e] = -np.inf
    return idx


def softmax(logits):
    l = np.asarray(logits, F64)
    z = np.exp(l - l.max(axis=1, keepdims=True))
    return z / z.sum(axis=1, keepdims=True)


def combine_weights(logits, idx, norm_topk: bool):
    """Gate weight of each selected expert: full-softmax probability, renormalised over
    the k selected experts when norm_topk (== softmax over the selected logits only)."""
    p = softmax(logits)
    sel = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if norm_topk:
        sel = sel / sel.sum(axis=1, keepdims=True)
    return sel


# --------------------------------------------------------------------------- #
# Section II-A: f limits the number of tokens assigned to an expert to T.
# --------------------------------------------------------------------------- #
def capacity_slots(idx, E: int, C: int):
    """Queue position of every (token t, choice j) at its expert e = idx[t,j]:
        pos = #{first..(j-1)-th choices that picked e} + #{t' < t : idx[t',j] = e}
    slot = pos if pos < C else -1 (dropped).  inv[e,c] = t*k+j for the occupant of slot c
    of expert e, -1 if empty.  counts[e] = number of (t,j) that asked for e."""
    idx = np.asarray(idx)
    S, k = idx.shape
    slot = np.full((S, k), -1, dtype=np.int32)
    inv = np.full((E, C), -1, dtype=np.int32)
    counts = np.zeros(E, dtype=np.int32)
    for e in range(E):
        before = 0                                    # demand from earlier choices
        for j in range(k):
            want = idx[:, j] == e
            rank = np.cumsum(want) - 1                # tokens t' < t with the same wish
            pos = before + rank
            ok = want & (pos < C)
            t_ok = np.nonzero(ok)[0]
            slot[t_ok, j] = pos[t_ok]
            inv[e, pos[t_ok]] = t_ok * k + j
            before += int(want.sum())
        counts[e] = before
    return slot, inv, counts


# --------------------------------------------------------------------------- #
# Section II-A: row G[i,:,:] holds the tokens dispatched to expert i.
# --------------------------------------------------------------------------- #
def dispatch(x, inv, k: int, w=None):
    """buf[e,c,:] = x[t,:] for the occupant (t,j) of slot (e,c) (times w[t,j] if given),
    zero rows where the slot is empty."""
    x = np.asarray(x, F64)
    E, C = inv.shape
    buf = np.zeros((E, C, x.shape[1]), dtype=F64)
    e_i, c_i = np.nonzero(inv >= 0)
    a = inv[e_i, c_i].astype(np.int64)
    t, j = a // k, a % k
    rows = x[t]
    if w is not None:
        rows = rows * np.asarray(w, F64)[t, j][:, None]
    buf[e_i, c_i] = rows
    return buf


# --------------------------------------------------------------------------- #
# Section II-A "Experts" and the sharding identity of "Model Parallelism":
#   Y = sum_p W2^(p) f(W1^(p) X), W1 split by columns and W2 by rows.
# --------------------------------------------------------------------------- #
def gelu(z):
    z = np.asarray(z, F64)
    return 0.5 * z * (1.0 + _erf(z / np.sqrt(2.0)))


def gelu_grad(z):
    z = np.asarray(z, F64)
    return 0.5 * (1.0 + _erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


def _shard(H: int, esp_idx: int, n_esp: int) -> slice:
    assert H % n_esp == 0 and 0 <= esp_idx < n_esp
    Hl = H // n_esp
    return slice(esp_idx * Hl, (esp_idx + 1) * Hl)


def expert_ffn_fwd(X, W1, W2, esp_idx: int = 0, n_esp: int = 1):
    """X [n_src,G,C,M], W1 [G,M,H], W2 [G,H,M]  ->  Z [n_src,G,C,H/n_esp], Y [n_src,G,C,M].
    Local expert g sees the rows X[:,g]; shard esp_idx produces a partial sum of Y."""
    X = np.asarray(X, F64)
    n_src, G, C, M = X.shape
    hs = _shard(W1.shape[2], esp_idx, n_esp)
    Z = np.empty((n_src, G, C, hs.stop - hs.start), dtype=F64)
    Y = np.empty((n_src, G, C, M), dtype=F64)
    for g in range(G):
        w1 = np.asarray(W1[g][:, hs], F64)
        w2 = np.asarray(W2[g][hs, :], F64)
        for s in range(n_src):
            z = X[s, g] @ w1
            Z[s, g] = z
            Y[s, g] = gelu(z) @ w2
    return Z, Y


def expert_ffn_bwd(dY, X, W1, W2, esp_idx: int = 0, n_esp: int = 1):
    """Chain rule through the shard: dA = dY W2^T, dW2 = A^T dY, dZ = dA * GeLU'(Z),
    dW1 = X^T dZ, dX = dZ W1^T.  Returns dX [n_src,G,C,M] and the shard's slices
    dW1 [G,M,H/n_esp], dW2 [G,H/n_esp,M] (reduction over all n_src*C rows of an expert)."""
    X = np.asarray(X, F64)
    dY = np.asarray(dY, F64)
    n_src, G, C, M = X.shape
    hs = _shard(W1.shape[2], esp_idx, n_esp)
    Hl = hs.stop - hs.start
    dX = np.empty_like(X)
    dW1 = np.zeros((G, M, Hl), dtype=F64)
    dW2 = np.zeros((G, Hl, M), dtype=F64)
    for g in range(G):
        w1 = np.asarray(W1[g][:, hs], F64)
        w2 = np.asarray(W2[g][hs, :], F64)
        for s in range(n_src):
            z = X[s, g] @ w1
            a = gelu(z)
            dA = dY[s, g] @ w2.T
            dW2[g] += a.T @ dY[s, g]
            dZ = dA * gelu_grad(z)
            dW1[g] += X[s, g].T @ dZ
            dX[s, g] = dZ @ w1.T
    return dX, dW1, dW2


# --------------------------------------------------------------------------- #
# Section II-A: expert outputs [Q_1..Q_E] are combined back to token order;
# Section III-C: partial sums of the N_ESP shards are summed locally first.
# --------------------------------------------------------------------------- #
def combine_fwd(Yret, idx, slot, w=None):
    """y[t,:] = sum over surviving choices j of w[t,j] * Yret[idx[t,j], slot[t,j], :].
    Yret is [E,C,M] or [n_part,E,C,M] (n_part partial sums, added first).  w=None means
    unit weights (this is then the backward of dispatch)."""
    Yret = np.asarray(Yret, F64)
    if Yret.ndim == 4:
        Yret = Yret.sum(axis=0)
    S, k = idx.shape
    y = np.zeros((S, Yret.shape[2]), dtype=F64)
    for j in range(k):
        ok = slot[:, j] >= 0
        t = np.nonzero(ok)[0]
        rows = Yret[idx[t, j], slot[t, j]]
        if w is not None:
            rows = rows * np.asarray(w, F64)[t, j][:, None]
        y[t] += rows
    return y


def combine_bwd(dy, Yret, idx, slot, w):
    """dYret[e,c,:] = w[t,j] dy[t,:] for the occupant of (e,c), zero for empty slots (the
    same gradient goes to every one of the n_part partial sums);
    dw[t,j] = <dy[t,:], Yret[idx[t,j], slot[t,j], :]> (0 if dropped)."""
    dy = np.asarray(dy, F64)
    Yret = np.asarray(Yret, F64)
    if Yret.ndim == 4:
        Yret = Yret.sum(axis=0)
    E, C, M = Yret.shape
    S, k = idx.shape
    w = np.asarray(w, F64)
    dYret = np.zeros((E, C, M), dtype=F64)
    dw = np.zeros((S, k), dtype=F64)
    for j in range(k):
        t = np.nonzero(slot[:, j] >= 0)[0]
        e, c = idx[t, j], slot[t, j]
        dYret[e, c] = w[t, j][:, None] * dy[t]
        dw[t, j] = np.einsum("tm,tm->t", dy[t], Yret[e, c])
    return dYret, dw


def gate_bwd(dw, logits, idx, norm_topk: bool, x, Wg):
    """Chain rule through the gate with the selection held fixed.
    norm_topk:  w_j = exp(l_j) / sum_{j' selected} exp(l_j')
                dl[e_j] = w_j (dw_j - sum_j' w_j' dw_j'),  0 for unselected experts.
    otherwise:  w_j = p[e_j], p = softmax(l):  dl[e] = sum_j dw_j p[e_j] (delta(e,e_j) - p[e]).
    Then dWg = x^T dl, dbias = sum_t dl, dx = dl Wg^T."""
    dw = np.asarray(dw, F64)
    S, k = idx.shape
    E = logits.shape[1]
    ii = idx.astype(np.int64)
    dl = np.zeros((S, E), dtype=F64)
    if norm_topk:
        w = combine_weights(logits, idx, True)
        inner = (w * dw).sum(axis=1, keepdims=True)
        np.put_along_axis(dl, ii, w * (dw - inner), axis=1)
    else:
        p = softmax(logits)
        pe = np.take_along_axis(p, ii, axis=1)                  # [S,k]
        dl -= p * (dw * pe).sum(axis=1, keepdims=True)
        cur = np.take_along_axis(dl, ii, axis=1)
        np.put_along_axis(dl, ii, cur + dw * pe, axis=1)
    x = np.asarray(x, F64)
    dWg = x.T @ dl
    dbias = dl.sum(axis=0)
    dx = dl @ np.asarray(Wg, F64).T
    return dl, dWg, dbias, dx


# --------------------------------------------------------------------------- #
# Whole layer on one rank's tokens, all E experts local (stands in for the two
# AlltoAlls of Section III-C): y[t] = sum_j w[t,j] FFN_{idx[t,j]}(x[t]).
# --------------------------------------------------------------------------- #
def route(x, Wg, bias, k: int, f: float, norm_topk: bool, C: int | None = None,
          logits_dtype=np.float32):
    logits = gate_logits(x, Wg, bias, logits_dtype)
    S, E = logits.shape
    if C is None:
        C = capacity(S, E, k, f)
    idx = topk_select(logits, k)
    w = combine_weights(logits, idx, norm_topk)
    slot, inv, counts = capacity_slots(idx, E, C)
    return dict(logits=logits, idx=idx, w=w, slot=slot, inv=inv, counts=counts, C=C)


def layer_fwd(x, Wg, bias, W1, W2, k: int, f: float, norm_topk: bool, n_esp: int = 1, C=None,
              logits_dtype=np.float32):
    """Returns the routing record r and y [S,M].  The expert FFN is evaluated as the sum of
    its n_esp shards (each a partial sum), as the local combine of Section III-C does."""
    r = route(x, Wg, bias, k, f, norm_topk, C, logits_dtype)
    buf = dispatch(x, r["inv"], k)                                # [E,C,M]
    parts = []
    for j in range(n_esp):
        _, Yj = expert_ffn_fwd(buf[None], W1, W2, j, n_esp)
        parts.append(Yj[0])
    Yret = np.stack(parts, axis=0)                                # [n_esp,E,C,M]
    y = combine_fwd(Yret, r["idx"], r["slot"], r["w"])
    r.update(buf=buf, Yret=Yret, y=y)
    return r


def layer_bwd(r, dy, x, Wg, W1, W2, k: int, norm_topk: bool, n_esp: int = 1):
    """Gradients of L = <y, dy> w.r.t. x, Wg, gate bias, W1, W2 (routing held fixed)."""
    dYret, dw = combine_bwd(dy, r["Yret"], r["idx"], r["slot"], r["w"])
    E = dYret.shape[0]
    H = W1.shape[2]
    Hl = H // n_esp
    dW1 = np.zeros((E, W1.shape[1], H), dtype=F64)
    dW2 = np.zeros((E, H, W2.shape[2]), dtype=F64)
    dbuf = np.zeros_like(dYret)
    for j in range(n_esp):
        dXj, dW1j, dW2j = expert_ffn_bwd(dYret[None], r["buf"][None], W1, W2, j, n_esp)
        dbuf += dXj[0]
        dW1[:, :, j * Hl:(j + 1) * Hl] = dW1j
        dW2[:, j * Hl:(j + 1) * Hl, :] = dW2j
    dx_disp = combine_fwd(dbuf, r["idx"], r["slot"], None)        # backward of dispatch
    dl, dWg, dbias, dx_gate = gate_bwd(dw, r["logits"], r["idx"], norm_topk, x, Wg)
    return dict(dYret=dYret, dw=dw, dbuf=dbuf, dW1=dW1, dW2=dW2, dlogits=dl, dWg=dWg,
                dbias=dbias, dx=dx_disp + dx_gate, dx_disp=dx_disp, dx_gate=dx_gate)


# --------------------------------------------------------------------------- #
# Schedule S2 of Section III-B ("Dedicated Schedules"): MP is paused AFTER the gate and
# resumed BEFORE the combine.  Gate and dispatch see all B*L tokens of the MP group (the
# capacity comes from B*L); the MP-Split then leaves MP rank r one part of the dispatched
# [E,C,M] buffer, the experts work on that part, and the MP-AllGather puts the parts back
# together before the combine.  The paper does not say how the buffer is cut; here rank r
# of n takes the contiguous slot range [floor(r C / n), floor((r+1) C / n)) of every expert.
# --------------------------------------------------------------------------- #
def slot_range(C: int, mp_idx: int, n_mp: int):
    if not (n_mp >= 1 and 0 <= mp_idx < n_mp):
        raise ValueError("bad MP rank")
    return (mp_idx * C) // n_mp, ((mp_idx + 1) * C) // n_mp


def layer_fwd_s2(x_full, Wg, bias, W1, W2, k: int, f: float, norm_topk: bool, n_mp: int, n_esp: int = 1):
    """All n_mp ranks of one MP group, one after the other: returns the routing record (with the
    per-rank buffers in r["buf_parts"]) and y for ALL tokens of the group."""
    r = route(x_full, Wg, bias, k, f, norm_topk)
    C = r["C"]
    E = r["inv"].shape[0]
    Yret = np.zeros((n_esp, E, C, W2.shape[2]), dtype=F64)
    parts = []
    for rank in range(n_mp):
        c0, c1 = slot_range(C, rank, n_mp)
        if c1 == c0:
            parts.append(np.zeros((E, 0, x_full.shape[1]), dtype=F64))
            continue
        part = dispatch(x_full, r["inv"][:, c0:c1], k)           # MP-Split of the dispatched buffer
        parts.append(part)
        for j in range(n_esp):
            _, Yj = expert_ffn_fwd(part[None], W1, W2, j, n_esp)
            Yret[j, :, c0:c1] = Yj[0]                             # MP-AllGather: the parts side by side
    y = combine_fwd(Yret, r["idx"], r["slot"], r["w"])
    r.update(buf_parts=parts, Yret=Yret, y=y)
    return r


# --------------------------------------------------------------------------- #
# The same expert FFN evaluated for single rows / single hidden units, so that
# outputs of a full-size run can be checked one by one.
# --------------------------------------------------------------------------- #
def expert_ffn_rows(x_rows, dy_rows, w1s, w2s):
    """Rows of ONE expert shard: w1s [M,H_l], w2s [H_l,M].  Returns z, y and dx of those rows."""
    x = np.asarray(x_rows, F64); dy = np.asarray(dy_rows, F64)
    w1s = np.asarray(w1s, F64); w2s = np.asarray(w2s, F64)
    z = x @ w1s
    y = gelu(z) @ w2s
    dx = ((dy @ w2s.T) * gelu_grad(z)) @ w1s.T
    return z, y, dx


def expert_ffn_hidden_unit(Xg, dYg, w1_col, w2_row):
    """One hidden unit h of ONE expert over all of its rows Xg [R,M], dYg [R,M]:
    returns dW1[:, h] (length M) and dW2[h, :] (length M)."""
    Xg = np.asarray(Xg, F64); dYg = np.asarray(dYg, F64)
    z = Xg @ np.asarray(w1_col, F64)
    dz = (dYg @ np.asarray(w2_row, F64)) * gelu_grad(z)
    return Xg.T @ dz, gelu(z) @ dYg
