#!/usr/bin/env python3
"""Benchmark of one rank's MoE-layer step (gate, dispatch, expert FFN, combine; fwd+bwd) on ONE MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config large] [--no-cpu-baseline] [--no-secondary]

A step is one pass of the whole hot path over one batch of seeded synthetic input that is already
resident in HBM.  Prints ONE JSON line: tokens/s of the layer fwd+bwd on the largest single-GPU workload
("large"), the roofline of the dominant kernel family (the six grouped bf16 MFMA GEMMs of the expert FFN:
executed flops per GEMM / mean time per GEMM, timed with HIP events on the launch stream inside the timed
steps), the achieved HBM rate of every memory-bound call against the HBM peak (`memory_kernels`), the CPU
checker timed on the host cores on a stated sample of the same workload (`cpu_baseline`), and the same
measurement on the small single-rank workload "layer_bf16" (`secondary`).

A rank that holds only a part of the experts or of their hidden dimension receives its expert inputs
through an AlltoAll that one GPU cannot run.  The receive buffers are then stand-ins built once, before
the timed region, from the rank's own data: source chunk s of the receive buffer is send chunk s mod N_EP of
the rank's own dispatched buffer, with the occupancy counts the gate produced for it (a peer's tokens
are distributed like the rank's own), and the returned buffers are the rank's own expert outputs.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0


def measured_traffic(name):
    """HBM bytes per grouped GEMM (mean of the 6 per step) from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    summary of this workload under profiles/, scaled there by the copy calibration; None if there is none."""
    path = os.path.join(ROOT, "profiles", f"bench_{name}_gemm_pmc.md")
    try:
        m = re.search(r"^traffic_bytes_per_gemm:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def measure(name, steps, warmup, settle, fused_ok=True, extras=False, tile=0):
    """Builds the workload on the device, runs settle + warmup untimed steps and `steps` timed ones."""
    import numpy as np
    import torch
    from paper_2407_00599_amd import api, synth
    from paper_2407_00599_amd.layer import MoERankShape

    dev = "cuda:0"
    cfg = synth.CONFIGS[name]
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    norm = 0 if cfg.k == 1 else 1
    L = MoERankShape(cfg.S_total, cfg.M, cfg.H, cfg.E, cfg.k, cfg.f, dtype=tdt, n_mp=cfg.n_mp, mp_idx=cfg.mp_idx,
                     n_ep=cfg.n_ep, n_esp=cfg.n_esp, esp_idx=cfg.esp_idx, norm_topk=norm, device=dev, tile=tile)

    def dev_t(st):
        if isinstance(st, synth.Stored):
            if st.bits is None:
                return torch.from_numpy(st.val).to(dev)
            return torch.from_numpy(st.bits.view(np.int16)).to(dev).view(torch.bfloat16)
        return None if st is None else torch.from_numpy(np.ascontiguousarray(st)).to(dev)

    if cfg.cfg_id <= 3:              # host-generated inputs (small enough)
        x, Wg, bias = dev_t(synth.tokens(cfg)), dev_t(synth.gate_weight(cfg)), dev_t(synth.gate_bias(cfg))
        w1, w2 = synth.expert_weights(cfg, L.G)
        W1, W2, dy = dev_t(w1), dev_t(w2), dev_t(synth.upstream_grad(cfg))
        del w1, w2
    else:                            # large shapes: the same distributions, drawn on the device
        gen = torch.Generator(device=dev); gen.manual_seed(synth.BASE_SEED + cfg.cfg_id)
        rn = lambda *s, sig=1.0, dt=tdt: (torch.randn(*s, generator=gen, device=dev, dtype=torch.float32) * sig).to(dt)
        x = rn(cfg.S_total, cfg.M, sig=cfg.sigma_x); Wg = rn(cfg.M, cfg.E, sig=cfg.sigma_w, dt=torch.float32)
        bias = dev_t(synth.gate_bias(cfg))
        W1 = torch.empty(L.G, cfg.M, cfg.H, dtype=tdt, device=dev); W2 = torch.empty(L.G, cfg.H, cfg.M, dtype=tdt, device=dev)
        for g in range(L.G):
            W1[g] = rn(cfg.M, cfg.H, sig=cfg.sigma_w); W2[g] = rn(cfg.H, cfg.M, sig=cfg.sigma_w)
        dy = rn(L.S, cfg.M)
    L.bind(x, Wg, bias, W1, W2, dy)
    if not L.closed:
        L.fill_stand_ins()           # one untimed pass that builds what the AlltoAlls would deliver

    # With every expert on this rank no AlltoAll separates the gate from the experts, and the dispatch is
    # fused into the expert GEMMs (token rows read through the inverse slot map: the same values, one
    # launch and one [E, C, M] buffer less); otherwise the dispatch writes the send buffer.
    fused_step = L.closed and fused_ok
    names = MoERankShape.STEPS_FUSED if fused_step else MoERankShape.STEPS
    for _ in range(settle + warmup):
        L.step(fused_step)
    torch.cuda.synchronize()

    K = steps
    # Per-call HIP events (for the roofline figures and the per-call breakdown) go into every fourth timed
    # step only: an event record between two launches costs the GPU a few microseconds of idle queue, and
    # the other steps run as a training loop would issue them.
    probed = [s for s in range(K) if s % 4 == 0]
    ev = {s: [torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)] for s in probed}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(K):
        if s in ev:
            ev[s][0].record()
            for i, n in enumerate(names):
                getattr(L, n)()
                ev[s][i + 1].record()
        else:
            L.step(fused_step)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    per_call = {n: sum(ev[s][i].elapsed_time(ev[s][i + 1]) for s in probed) / len(probed) for i, n in enumerate(names)}

    # FLOPs = what the six launches multiply out: row tiles that are all capacity padding are skipped by the
    # kernels and not counted (moe_ffn_executed_flops mirrors the kernels' skipping rule on a host copy of the counts)
    rows = L.n_src * L.G * L.C
    cnt_host = None if L.row_counts is None else L.row_counts.cpu().numpy()
    dtc = api.MOE_BF16 if cfg.dtype == "bf16" else api.MOE_F32
    fl_fwd, fl_bwd = (api.moe_ffn_executed_flops(dtc, L.n_src, L.G, L.C, cfg.M, cfg.H, L.n_esp, cnt_host, b, tile) for b in (0, 1))
    flops_per_launch = (fl_fwd + fl_bwd) / 6.0
    occupied = rows if cnt_host is None else int(np.minimum(cnt_host, L.C).sum())
    fwd_name, bwd_name = ("ffn_fwd_gather", "ffn_bwd_gather") if fused_step else ("ffn_fwd", "ffn_bwd")
    gemm_ms = (per_call[fwd_name] + per_call[bwd_name]) / 6.0
    achieved = flops_per_launch / (gemm_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": measured_traffic(cfg.name),
                "kernel": "ffn_gemm_dma x3 + ffn_bwd_trio (6 grouped GEMMs in 4 launches per step)", "gemm_ms": round(gemm_ms, 4),
                "flops_per_gemm": flops_per_launch, "occupied_rows": occupied, "capacity_rows": rows,
                "flops_if_all_capacity_rows": 2.0 * rows * cfg.M * L.Hl,
                "fwd_frac": round(fl_fwd / (per_call[fwd_name] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                "bwd_frac": round(fl_bwd / (per_call[bwd_name] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
    if cfg.dtype == "f32":
        roofline.update({"bound": "alu", "peak": 78.6, "frac": round(achieved / 78.6, 5),
                         "kernel": "ffn_gemm_f32 (6 grouped GEMMs per step)"})

    # Memory-bound calls: algorithmic bytes of one call over its mean duration, against the HBM peak.
    # valid = occupied slots of the rank's own [E, C, M] buffer (from the gate's demand counts).
    b = 2 if cfg.dtype == "bf16" else 4
    S, M, E, k, C, P = L.S, cfg.M, cfg.E, cfg.k, L.C, L.n_esp
    valid = int(np.minimum(L.counts.cpu().numpy(), C).sum())
    alg = {"gate": S * M * b + 4 * M * E + 4 * S * E + 12 * S * k + 4 * E * C,
           "dispatch": valid * M * b + E * C * M * b + 4 * E * C,
           "combine": valid * P * M * b + S * M * b + 12 * S * k,
           "combine_bwd": valid * M * b + E * C * M * b + S * M * b + valid * P * M * b + 16 * S * k,
           "dispatch_bwd": valid * P * M * b + S * M * b + 8 * S * k,
           "gate_bwd": 3 * S * M * b + 8 * S * E + 4 * M * E}
    memory_kernels = {n: {"bytes": int(alg[n]), "ms": round(per_call[n], 4),
                          "GBps": round(alg[n] / (per_call[n] * 1e-3) / 1e9, 1),
                          "frac_of_hbm_peak": round(alg[n] / (per_call[n] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
                      for n in alg if n in per_call}

    # Forward / backward with the dispatch fused into the GEMMs against the unfused pair (outside the timed
    # region, every expert local): events around 20 repetitions of each
    fused = None
    if L.closed and extras:
        def timed(fn, reps=20):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fn(); torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record(); torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps
        fused = {"dispatch_plus_ffn_fwd_ms": round(timed(lambda: (L.dispatch(), L.ffn_fwd())), 4),
                 "ffn_fwd_gather_ms": round(timed(L.ffn_fwd_gather), 4),
                 "ffn_bwd_ms": round(timed(L.ffn_bwd), 4), "ffn_bwd_gather_ms": round(timed(L.ffn_bwd_gather), 4)}

    workload = (f"{cfg.name}: S={L.S} tokens, M={cfg.M}, H={cfg.H} (H_local={L.Hl}), E={cfg.E} "
                f"(G={L.G} local, n_src={L.n_src}), top-{cfg.k}, f={cfg.f}, C={L.C}; gate+dispatch+FFN+combine fwd+bwd"
                + (" (dispatch fused into the expert GEMMs)" if fused_step else "")
                + ("" if L.closed else "; receive buffers = the rank's own dispatched chunks and counts"))
    res = {"workload": workload, "ms_per_step": round(ms_per_step, 4), "tokens_per_s": round(L.S / (ms_per_step * 1e-3), 1),
           "roofline": roofline, "memory_kernels": memory_kernels, "per_call_ms": {k_: round(v, 4) for k_, v in per_call.items()},
           "per_call_steps": len(probed), "fused_dispatch": fused, "S": L.S, "dtype": cfg.dtype}
    del L, x, W1, W2, dy
    torch.cuda.empty_cache()
    return res


def cpu_baseline(name):
    """The CPU checker on a bounded sample of the workload: the rank-shaped sequence of its functions (route,
    dispatch, sharded expert FFN forward and backward over n_src source chunks, combine forward and backward,
    dispatch backward, gate backward) for the first S_s tokens of the rank at the workload's own M, H_local,
    E, k, f, N_ESP.  Per-token work is the same as in the full workload (the capacity scales with the token
    count), so tokens/s of the sample is the figure for the whole; S_s is chosen for roughly 10-30 s."""
    import dataclasses
    import numpy as np
    from oracle import moe_oracle as O
    from paper_2407_00599_amd import synth
    cfg = synth.CONFIGS[name]
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    flops_per_token = 12.0 * cfg.k * cfg.f * cfg.n_esp * cfg.M * cfg.H_local      # expert FFN fwd+bwd, this rank
    S_s = int(min(cfg.S, max(256, 2.5e12 // flops_per_token)))                     # about 2.5 TFLOP of float64 work
    S_s = max(cfg.E, S_s // 256 * 256) if S_s >= 256 else S_s
    small = dataclasses.replace(cfg, S_total=S_s, n_mp=1, mp_idx=0, H=cfg.H_local, n_esp=1, esp_idx=0)
    norm = cfg.k > 1
    x = synth.tokens(small).val; Wg = synth.gate_weight(small); bias = synth.gate_bias(small)
    W1, W2 = synth.expert_weights(small, cfg.G)            # the rank's G experts, H_local columns each
    dy = synth.upstream_grad(small).val
    W1, W2 = W1.val, W2.val
    n_ep, n_esp, G, n_src = cfg.n_ep, cfg.n_esp, cfg.G, cfg.n_src
    t0 = time.perf_counter()
    r = O.route(x, Wg, bias, cfg.k, cfg.f, norm)
    C = r["C"]
    buf = O.dispatch(x, r["inv"], cfg.k)                                           # [E, C, M] = [n_ep, G, C, M]
    send = buf.reshape(n_ep, G, C, cfg.M)
    Xrecv = np.stack([send[s % n_ep] for s in range(n_src)])                       # [n_src, G, C, M]
    _, Y = O.expert_ffn_fwd(Xrecv, W1, W2)
    Yret = Y.reshape(n_esp, cfg.E, C, cfg.M)
    O.combine_fwd(Yret, r["idx"], r["slot"], r["w"])
    dYret, dw = O.combine_bwd(dy, Yret, r["idx"], r["slot"], r["w"])
    dsend = dYret.reshape(n_ep, G, C, cfg.M)
    dYrecv = np.stack([dsend[s % n_ep] for s in range(n_src)])
    dX, _, _ = O.expert_ffn_bwd(dYrecv, Xrecv, W1, W2)
    O.combine_fwd(dX.reshape(n_esp, cfg.E, C, cfg.M), r["idx"], r["slot"], None)
    O.gate_bwd(dw, r["logits"], r["idx"], norm, x, Wg)
    t = time.perf_counter() - t0
    return {"value": round(S_s / t, 1), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"one fwd+bwd pass of the checker's per-rank sequence (numpy float64) over {S_s} of the {cfg.S} tokens "
                      f"of {cfg.name} at its M, H_local, E, k, f and source-chunk count (capacity {C}); per-token work equals "
                      f"the full workload's, so no further scaling; {t:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--settle-steps", type=int, default=-1,
                    help="untimed steps before the warm-up steps (the GPU's clocks need about a second of this load to "
                         "settle); default: what fills about one second, at least 10; reported as settle_steps")
    ap.add_argument("--config", default="large", help="workload name from synth.CONFIGS")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true", help="skip the second measurement on the layer_bf16 workload")
    ap.add_argument("--tile", type=int, default=0, help="tile hint of the FFN GEMMs (MOE_TILE_*, 0 = auto)")
    ap.add_argument("--unfused-dispatch", action="store_true",
                    help="write the dispatched [E, C, M] buffer even when every expert is local (default: fused into the GEMMs)")
    ap.add_argument("--extras", action="store_true", help="also time fused against unfused dispatch after the timed region")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy 5 times (known traffic, used to scale the "
                         "FETCH_SIZE / WRITE_SIZE counters when the run is profiled with rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one rank on one GPU: this build has no inter-GPU collectives and never uses a second "
              "GPU; run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2407_00599_amd import api, synth

    api.lib()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists)", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    # about one second of settling: ~40 ms per step for "large", ~0.6 ms for "layer_bf16"
    est_ms = max(0.3, 12.0 * cfg.k * cfg.f * cfg.n_esp * cfg.M * cfg.H_local * cfg.S / 1.0e15 * 1e3)
    settle = args.settle_steps if args.settle_steps >= 0 else max(10, int(1000.0 / est_ms))

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0"); dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    main_res = measure(args.config, args.steps, args.warmup, settle, fused_ok=not args.unfused_dispatch,
                       extras=args.extras, tile=args.tile)
    secondary = None
    if not args.no_secondary and args.config != "layer_bf16":
        r2 = measure("layer_bf16", 200, 10, 200, fused_ok=not args.unfused_dispatch, tile=args.tile)
        secondary = {k_: r2[k_] for k_ in ("workload", "ms_per_step", "tokens_per_s", "roofline", "memory_kernels", "per_call_ms")}
        secondary.update({"steps": 200, "warmup": 10, "settle_steps": 200})
    cpu = None if args.no_cpu_baseline else cpu_baseline(args.config)

    out = {
        "metric": "MoE-layer fwd+bwd tokens/s (1 GPU)", "value": main_res["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_steps": settle, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if main_res["dtype"] == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": main_res["workload"]},
        "roofline": main_res["roofline"], "cpu_baseline": cpu, "memory_kernels": main_res["memory_kernels"],
        "per_call_ms": main_res["per_call_ms"], "per_call_steps": main_res["per_call_steps"],
        "fused_dispatch": main_res["fused_dispatch"], "secondary": secondary,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
