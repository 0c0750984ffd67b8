#!/usr/bin/env python3
"""Benchmark of one rank's MoE-layer step (gate, dispatch, expert FFN, combine; fwd+bwd) on ONE MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config layer_bf16] [--no-cpu-baseline] [--unfused-dispatch]

A step is one pass of the whole hot path over one batch of seeded synthetic input that is
already resident in HBM.  Prints ONE JSON line: tokens/s of the layer fwd+bwd, the roofline of
the dominant kernel family (the six grouped bf16 MFMA GEMMs of the expert FFN: executed flops per GEMM /
mean time per GEMM, timed with HIP events on the launch stream inside the timed steps) and the
CPU checker timed on the host cores on the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0
# HBM bytes per grouped GEMM (mean of the 6 per step), from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this command scaled by the copy calibration; None where no such run has been made (see profiles/).
MEASURED_TRAFFIC = {"layer_bf16": 222.9e6}   # profiles/bench_layer_bf16_gemm_pmc.md


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--settle-steps", type=int, default=200,
                    help="untimed steps before the warm-up steps: the GPU needs about 50 steps (30 ms) of this load "
                         "before its clocks settle; reported as settle_steps")
    ap.add_argument("--config", default="layer_bf16", help="workload name from synth.CONFIGS")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tile", type=int, default=0, help="FFN GEMM variant, see moe_ffn_set_tile (0 = auto)")
    ap.add_argument("--unfused-dispatch", action="store_true",
                    help="write the dispatched [E, C, M] buffer even when every expert is local (default: fused into the GEMMs)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the fused / unfused dispatch comparison after the timed region (profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy 5 times (known traffic, used to scale the "
                         "FETCH_SIZE / WRITE_SIZE counters when the run is profiled with rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one rank on one GPU: this build has no inter-GPU collectives, "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2407_00599_amd import api, synth
    from paper_2407_00599_amd.layer import MoERankShape

    api.lib()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists)", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    api.moe_ffn_set_tile(args.tile)
    cfg = synth.CONFIGS[args.config]
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    norm = 0 if cfg.k == 1 else 1

    L = MoERankShape(cfg.S_total, cfg.M, cfg.H, cfg.E, cfg.k, cfg.f, dtype=tdt, n_mp=cfg.n_mp, mp_idx=cfg.mp_idx,
                     n_ep=cfg.n_ep, n_esp=cfg.n_esp, esp_idx=cfg.esp_idx, norm_topk=norm, device=dev)

    def dev_t(st):
        if isinstance(st, synth.Stored):
            if st.bits is None:
                return torch.from_numpy(st.val).to(dev)
            return torch.from_numpy(st.bits.view(np.int16)).to(dev).view(torch.bfloat16)
        return None if st is None else torch.from_numpy(np.ascontiguousarray(st)).to(dev)

    host = {}
    small = cfg.cfg_id <= 3          # host-generated inputs, shared with the CPU baseline
    if small:
        host["x"] = synth.tokens(cfg); host["Wg"] = synth.gate_weight(cfg); host["bias"] = synth.gate_bias(cfg)
        host["W1"], host["W2"] = synth.expert_weights(cfg, L.G); host["dy"] = synth.upstream_grad(cfg)
        x, Wg, bias = dev_t(host["x"]), dev_t(host["Wg"]), dev_t(host["bias"])
        W1, W2, dy = dev_t(host["W1"]), dev_t(host["W2"]), dev_t(host["dy"])
    else:                            # large shapes: same distributions, drawn on the device
        gen = torch.Generator(device=dev); gen.manual_seed(synth.BASE_SEED + cfg.cfg_id)
        rn = lambda *s, sig=1.0, dt=tdt: (torch.randn(*s, generator=gen, device=dev, dtype=torch.float32) * sig).to(dt)
        x = rn(cfg.S_total, cfg.M, sig=cfg.sigma_x); Wg = rn(cfg.M, cfg.E, sig=cfg.sigma_w, dt=torch.float32)
        b = synth.gate_bias(cfg); bias = dev_t(b)
        W1 = torch.empty(L.G, cfg.M, cfg.H, dtype=tdt, device=dev); W2 = torch.empty(L.G, cfg.H, cfg.M, dtype=tdt, device=dev)
        for g in range(L.G):
            W1[g] = rn(cfg.M, cfg.H, sig=cfg.sigma_w); W2[g] = rn(cfg.H, cfg.M, sig=cfg.sigma_w)
        dy = rn(L.S, cfg.M)
    L.bind(x, Wg, bias, W1, W2, dy)
    if not L.closed:
        # stand-ins for what the two EP&ESP-AlltoAlls would deliver (rows ~N(0,1), 80 % occupied)
        gen = torch.Generator(device=dev); gen.manual_seed(synth.BASE_SEED + 77)
        for t in (L.Xrecv, L.dYrecv):
            t.copy_(torch.randn(t.shape, generator=gen, device=dev, dtype=torch.float32).to(tdt))
            t[:, :, int(0.8 * L.C):, :] = 0
        L.row_counts = torch.full((L.n_src, L.G), int(0.8 * L.C), dtype=torch.int32, device=dev)
        for t in (L.Yret, L.dbuf):
            t.copy_((torch.randn(t.shape, generator=gen, device=dev, dtype=torch.float32) * 0.5).to(tdt))

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev); dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # With every expert on this rank no AlltoAll separates the gate from the experts, and the dispatch is
    # fused into the expert GEMMs (token rows read through the inverse slot map: the same values, one
    # launch and one [E, C, M] buffer less); otherwise the dispatch writes the send buffer.
    fused_step = L.closed and not args.unfused_dispatch
    names = MoERankShape.STEPS_FUSED if fused_step else MoERankShape.STEPS
    for _ in range(args.settle_steps + args.warmup):
        L.step(fused_step)
    torch.cuda.synchronize()

    K = args.steps
    # Per-call HIP events (for the roofline figure and the per-call breakdown) go into every fourth timed
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
    executed = sum(api.moe_ffn_executed_flops(dtc, L.n_src, L.G, L.C, cfg.M, cfg.H, L.n_esp, cnt_host, b) for b in (0, 1))
    flops_per_launch = executed / 6.0
    occupied = rows if cnt_host is None else int(np.minimum(cnt_host, L.C).sum())
    fwd_name, bwd_name = ("ffn_fwd_gather", "ffn_bwd_gather") if fused_step else ("ffn_fwd", "ffn_bwd")
    gemm_ms = (per_call[fwd_name] + per_call[bwd_name]) / 6.0
    achieved = flops_per_launch / (gemm_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": MEASURED_TRAFFIC.get(cfg.name),
                "kernel": "ffn_gemm_dma x3 + ffn_bwd_trio (6 grouped GEMMs in 4 launches per step)", "gemm_ms": round(gemm_ms, 4),
                "flops_per_gemm": flops_per_launch, "occupied_rows": occupied, "capacity_rows": rows,
                "flops_if_all_capacity_rows": 2.0 * rows * cfg.M * L.Hl}
    if cfg.dtype == "f32":
        roofline.update({"bound": "alu", "peak": 78.6, "frac": round(achieved / 78.6, 5),
                         "kernel": "ffn_gemm_f32 (6 grouped GEMMs per step)"})

    # Forward with the dispatch fused into the first GEMM (outside the timed region, every expert local):
    # the pair of calls it replaces against the one call, events around 20 repetitions of each
    fused = None
    if L.closed and not args.no_extras:
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

    cpu = None
    if small and not args.no_cpu_baseline and L.closed:
        from oracle import moe_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        xs = host["x"].val[O.mp_slice(cfg.S_total, cfg.mp_idx, cfg.n_mp)]
        passes, tcpu = 0, 0.0
        while passes < 5 and tcpu < 10.0:
            c0 = time.perf_counter()
            r = O.layer_fwd(xs, host["Wg"], host["bias"], host["W1"].val, host["W2"].val, cfg.k, cfg.f, bool(norm), 1)
            O.layer_bwd(r, host["dy"].val, xs, host["Wg"], host["W1"].val, host["W2"].val, cfg.k, bool(norm), 1)
            tcpu += time.perf_counter() - c0
            passes += 1
        cpu = {"value": round(L.S * passes / tcpu, 1), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": f"{passes} full fwd+bwd passes of the same {cfg.name} workload (numpy float64)"}

    out = {
        "metric": "MoE-layer fwd+bwd tokens/s (1 GPU)", "value": round(L.S / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "settle_steps": args.settle_steps, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: S={L.S} tokens, M={cfg.M}, H={cfg.H} (H_local={L.Hl}), E={cfg.E} "
                               f"(G={L.G} local, n_src={L.n_src}), top-{cfg.k}, f={cfg.f}, C={L.C}; "
                               f"gate+dispatch+FFN+combine fwd+bwd" + (" (dispatch fused into the expert GEMMs)" if fused_step else "")},
        "roofline": roofline, "cpu_baseline": cpu,
        "per_call_ms": {k: round(v, 4) for k, v in per_call.items()}, "per_call_steps": len(probed),
        "fused_dispatch_fwd": fused,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
