"""GPU parity at the two largest benchmark workloads ("esp4": S = 16384, M = 2048, E = 64, 4 partial
sums; "large": S = 32768, M = 4096, E = 8, 2 partial sums) for every step of the path except the expert
FFN (which test_gpu_ffn.py covers at these sizes): gate, dispatch, combine forward (weighted and with unit
weights = dispatch backward), combine backward, gate backward.  The kernels run at full size in the launch
configuration the benchmark uses.  Each step is given the CPU checker's own routing tensors as input, so a
step is judged on its own.  Plain copies and the gate backward are compared over the whole tensors; the
combine is compared on sampled tokens (the checker then only needs the rows those tokens touch) plus
properties that hold at any size (dropped tokens and empty slots give exact zeros)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2407_00599_amd import api, synth
from util import DEV, TOL, ROWS, to_dev, to_host, rel_err, assert_close

pytestmark = pytest.mark.gpu

N_SAMPLE = 384


@pytest.fixture(scope="module", params=["esp4", "large"])
def work(request):
    """Inputs of one workload, the checker's routing, and the same tensors on the device."""
    cfg = synth.CONFIGS[request.param]
    x = synth.tokens(cfg); Wg = synth.gate_weight(cfg); bias = synth.gate_bias(cfg); dy = synth.upstream_grad(cfg)
    xs = x.val[O.mp_slice(cfg.S_total, cfg.mp_idx, cfg.n_mp)]
    r = O.route(xs, Wg, bias, cfg.k, cfg.f, True)
    C = r["C"]
    w32 = r["w"].astype(np.float32)
    d = dict(cfg=cfg, x=x, xs=xs, Wg=Wg, bias=bias, dy=dy, r=r, C=C, w32=w32,
             d_x=to_dev(x), d_dy=to_dev(dy), d_idx=to_dev(r["idx"]), d_slot=to_dev(r["slot"]), d_inv=to_dev(r["inv"]),
             d_w=to_dev(w32))
    yield d
    d.clear()
    torch.cuda.empty_cache()


def sample_tokens(r, S, rng):
    """Random tokens plus some of every drop pattern the routing has (none, some, all choices dropped)."""
    dropped = (r["slot"] < 0).sum(axis=1)
    pick = [rng.choice(S, N_SAMPLE, replace=False), np.array([0, S - 1])]
    for n in np.unique(dropped):
        cand = np.nonzero(dropped == n)[0]
        pick.append(cand[:16])
    return np.unique(np.concatenate(pick))


def compact(r, toks, Yret_dev, C):
    """The rows of Yret [n_part, E, C, M] that the sampled tokens touch, as a small [n_part, 1, n, M]
    problem of its own: every surviving (token, choice) is given the next row of a single expert."""
    idx, slot = r["idx"][toks], r["slot"][toks]
    live = slot >= 0
    e, c = idx[live].astype(np.int64), slot[live].astype(np.int64)
    rows = Yret_dev[:, torch.from_numpy(e).to(DEV), torch.from_numpy(c).to(DEV)]        # [n_part, n, M]
    idx_c = np.zeros_like(idx)
    slot_c = np.full_like(slot, -1)
    slot_c[live] = np.arange(live.sum(), dtype=np.int32)
    return to_host(rows)[:, None], idx_c, slot_c, (e, c)


def test_gate_integers(work):
    cfg, r, C = work["cfg"], work["r"], work["C"]
    S, E, k = cfg.S, cfg.E, cfg.k
    i32, f32 = torch.int32, torch.float32
    logits = torch.empty(S, E, dtype=f32, device=DEV)
    idx = torch.empty(S, k, dtype=i32, device=DEV); slot = torch.empty(S, k, dtype=i32, device=DEV)
    w = torch.empty(S, k, dtype=f32, device=DEV); inv = torch.empty(E, C, dtype=i32, device=DEV)
    counts = torch.empty(E, dtype=i32, device=DEV)
    ws = torch.empty(api.moe_gate_workspace_bytes(S, E, k), dtype=torch.uint8, device=DEV)
    api.moe_gate_topk(work["d_x"], to_dev(work["Wg"]), to_dev(work["bias"]) if work["bias"] is not None else None,
                      cfg.S_total, cfg.M, E, k, C, cfg.mp_idx, cfg.n_mp, 1, logits, idx, slot, w, inv, counts, ws)
    torch.cuda.synchronize()
    same = to_host(logits).astype(np.float32) == r["logits"]
    assert same.mean() > 0.999
    if same.all():
        for n, t in (("idx", idx), ("slot", slot), ("inv", inv), ("counts", counts)):
            assert np.array_equal(to_host(t), r[n]), n
        assert np.abs(to_host(w) - r["w"]).max() <= 1e-6
    assert (r["slot"] < 0).any()                                  # these workloads drop tokens


def test_dispatch_whole_buffer(work):
    cfg, r, C = work["cfg"], work["r"], work["C"]
    S, M, E, k = cfg.S, cfg.M, cfg.E, cfg.k
    buf = torch.full((E, C, M), 7.0, dtype=torch.bfloat16, device=DEV)
    api.moe_dispatch(work["d_x"], S, M, E, k, C, work["d_inv"], None, buf)
    torch.cuda.synchronize()
    ref = O.dispatch(work["xs"], r["inv"], k)
    assert np.array_equal(to_host(buf), ref)                      # a plain copy: every element exact
    del ref
    assert not buf[work["d_inv"] < 0].any()                       # empty slots are zero rows


@pytest.mark.parametrize("weighted", [True, False])
def test_combine_fwd_sampled(work, weighted):
    cfg, r, C = work["cfg"], work["r"], work["C"]
    S, M, E, k, n_part = cfg.S, cfg.M, cfg.E, cfg.k, cfg.n_esp
    gen = torch.Generator(device=DEV); gen.manual_seed(synth.BASE_SEED + 50 + cfg.cfg_id)
    Yret = torch.empty(n_part, E, C, M, dtype=torch.bfloat16, device=DEV)
    for p in range(n_part):
        Yret[p] = (torch.randn(E, C, M, generator=gen, device=DEV, dtype=torch.float32) * 0.5).to(torch.bfloat16)
    y = torch.full((S, M), 7.0, dtype=torch.bfloat16, device=DEV)
    api.moe_combine_fwd(Yret, n_part, S, M, E, k, C, work["d_idx"], work["d_slot"], work["d_w"] if weighted else None, y)
    torch.cuda.synchronize()
    toks = sample_tokens(r, S, np.random.default_rng(cfg.cfg_id))
    Ysub, idx_c, slot_c, _ = compact(r, toks, Yret, C)
    ref = O.combine_fwd(Ysub, idx_c, slot_c, work["w32"][toks] if weighted else None)
    got = to_host(y[torch.from_numpy(toks).to(DEV)])
    assert_close(got, ref, TOL["bf16"] * 0.25, "y", ROWS)
    all_dropped = torch.from_numpy((r["slot"] < 0).all(axis=1)).to(DEV)
    assert not y[all_dropped].any()                               # at any size: no surviving choice, zero row


def test_combine_bwd(work):
    cfg, r, C = work["cfg"], work["r"], work["C"]
    S, M, E, k, n_part = cfg.S, cfg.M, cfg.E, cfg.k, cfg.n_esp
    gen = torch.Generator(device=DEV); gen.manual_seed(synth.BASE_SEED + 60 + cfg.cfg_id)
    Yret = torch.empty(n_part, E, C, M, dtype=torch.bfloat16, device=DEV)
    for p in range(n_part):
        Yret[p] = (torch.randn(E, C, M, generator=gen, device=DEV, dtype=torch.float32) * 0.5).to(torch.bfloat16)
    dYret = torch.full((E, C, M), 7.0, dtype=torch.bfloat16, device=DEV)
    dw = torch.full((S, k), 7.0, dtype=torch.float32, device=DEV)
    api.moe_combine_bwd(work["d_dy"], Yret, n_part, S, M, E, k, C, work["d_idx"], work["d_slot"], work["d_inv"],
                        work["d_w"], dYret, dw)
    torch.cuda.synchronize()
    # sampled tokens through the checker's combine backward
    toks = sample_tokens(r, S, np.random.default_rng(10 + cfg.cfg_id))
    Ysub, idx_c, slot_c, (e, c) = compact(r, toks, Yret, C)
    rdY, rdw = O.combine_bwd(work["dy"].val[toks], Ysub, idx_c, slot_c, work["w32"][toks])
    got_rows = to_host(dYret[torch.from_numpy(e).to(DEV), torch.from_numpy(c).to(DEV)])
    assert_close(got_rows, rdY[0, :len(e)], 4e-3, "dYret rows", ROWS)   # one product rounded to bf16: 2^-9 per element
    got_dw = to_host(dw)[toks]
    assert rel_err(got_dw, rdw) <= 2e-6 * np.sqrt(M)
    assert np.all(got_dw[r["slot"][toks] < 0] == 0.0)
    # the whole buffer: the gradient of the returned rows is the weighted dispatch of dy
    ref = O.dispatch(work["dy"].val, r["inv"], k, work["w32"])
    assert rel_err(to_host(dYret), ref) <= 4e-3
    del ref
    assert not dYret[work["d_inv"] < 0].any()
    assert not dw[work["d_slot"] < 0].any()


def test_gate_bwd_whole_tensors(work):
    """Every output of the gate backward over all tokens: at these sizes a block of the fused kernel walks
    128 tokens in eight stages (E <= 16), and the wide kernels sum 256 tokens per partial sum (E = 64)."""
    cfg, r = work["cfg"], work["r"]
    S, M, E, k = cfg.S, cfg.M, cfg.E, cfg.k
    rng = np.random.default_rng(20 + cfg.cfg_id)
    dwn = rng.standard_normal((S, k)).astype(np.float32)
    dx0 = synth.store(rng.standard_normal((S, M)).astype(np.float32), "bf16")
    dl = torch.empty(S, E, device=DEV); dWg = torch.empty(M, E, device=DEV); db = torch.empty(E, device=DEV)
    dx = to_dev(dx0).clone()
    ws = torch.empty(api.moe_gate_bwd_workspace_bytes(S, M, E), dtype=torch.uint8, device=DEV)
    api.moe_gate_bwd(to_dev(dwn), work["d_w"], work["d_idx"], to_dev(r["logits"]), work["d_x"], to_dev(work["Wg"]),
                     S, M, E, k, 1, dl, dWg, db, dx, 1, ws)
    torch.cuda.synchronize()
    rdl, rdWg, rdb, rdx = O.gate_bwd(dwn, r["logits"], r["idx"], True, work["xs"], work["Wg"])
    assert_close(to_host(dl), rdl, 1e-5, "dlogits")
    assert_close(to_host(dWg), rdWg, 1e-5, "dWg")
    assert_close(to_host(db), rdb, 1e-5, "dbias")
    assert_close(to_host(dx), rdx + dx0.val, 4e-3, "dx", ROWS)
