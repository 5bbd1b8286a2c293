#!/usr/bin/env python3
"""Benchmark of one GPU's MoE layer, forward + backward, on seeded synthetic input.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3]

A step is one pass of the whole hot path over one batch resident in HBM: gate
projection, softmax/top-k/capacity+RTS routing, dispatch, expert FFN forward,
combine, then combine backward, expert FFN backward, dispatch backward, gate
backward and gate-projection backward.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2.5e15      # dense bf16 MFMA, FLOP/s (MI355X datasheet)
PEAK_F32_MFMA = 157.3e12     # fp32 matrix
PEAK_HBM = 8.0e12            # B/s


def cpu_baseline(w, d, budget_flops=2.0e12, forward_only=False):
    """The CPU oracle, as it stands, on a bounded sample of the same workload:
    the first Ts tokens (all of them if the whole layer is below ~2e12 flop),
    capacity scaled with Ts.  Timed on this host's cores."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import moe_oracle as O
    full = 12.0 * w.k * w.T * w.d_model * w.d_ff
    Ts = w.T if full <= budget_flops else max(w.E * 8, int(w.T * budget_flops / full))
    C = w.capacity if Ts == w.T else O.capacity(Ts, w.E, w.k, w.capacity_factor)
    t0 = time.time()
    O.moe_layer(d["x"][:Ts], d["Wg"], d["bias"], d["W1"], d["W2"], d["rts_keys"][:Ts],
                None if forward_only else d["dy"][:Ts], w.k, C, w.act)
    dt = time.time() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": Ts / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {Ts} of {w.T} tokens, all {w.E} experts, capacity {C}, "
                      f"{'fwd' if forward_only else 'fwd+bwd'} in fp64, "
                      f"{dt:.1f} s on {os.cpu_count()} visible cpus"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--aux-coef", type=float, default=0.0,
                    help="weight of the balancing auxiliary loss (Sec. 5.1 uses 0.01); 0 = the plain hot path")
    ap.add_argument("--jitter-eps", type=float, default=0.0, help="gate jitter (Sec. 5.1, Switch: 0.01); 0 = off")
    ap.add_argument("--drop-p", type=float, default=0.0, help="expert dropout (Sec. 5.4: 0.4 in fine-tuning); 0 = off")
    ap.add_argument("--groups", type=int, default=1,
                    help="grouped token selection inside groups of T/groups consecutive tokens (Sec. 3.1); 1 = plain")
    ap.add_argument("--forward-only", action="store_true",
                    help="evaluation path: forward only, capacity factor 2.0, utilisation counting (not the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--breakdown", action="store_true", help="also print per-call timings to stderr")
    ap.add_argument("--vendor-reference", action="store_true",
                    help="after the timed region, also time the vendor library's batched GEMM (torch.bmm) on the two "
                         "forward products at this workload's shape (dense, plain store), for scale")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device copy (to scale rocprofv3's FETCH_SIZE/WRITE_SIZE) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2109_10465_amd import binding as B
    from paper_2109_10465_amd import inputs as I
    from paper_2109_10465_amd.layer import MoELayer

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    if args.copy_calibration:
        # a plain copy kernel of known size: reads 1 GiB, writes 1 GiB
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4, "copies": 3}))
        return
    B.lib()
    w = I.WORKLOADS[args.workload]
    if args.forward_only:
        import dataclasses
        w = dataclasses.replace(w, capacity=B.moe_capacity(w.T, w.E, w.k, 2.0), capacity_factor=2.0)
    d = I.make_inputs(w, seed=0)
    adt = torch.bfloat16 if w.dtype == I.BF16 else torch.float32

    def dev(a, dt=torch.float32):
        return None if a is None else torch.from_numpy(a).cuda().to(dt)

    x, dy, W1, W2 = dev(d["x"], adt), dev(d["dy"], adt), dev(d["W1"], adt), dev(d["W2"], adt)
    Wg, bias, keys = dev(d["Wg"]), dev(d["bias"]), dev(d["rts_keys"])
    layer = MoELayer(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act, forward_only=args.forward_only,
                     groups=args.groups)
    s = layer.shape
    L = layer

    calls = [
        ("gate_logits", lambda: B.moe_gate_logits_jitter(s, x, Wg, bias, args.jitter_eps, 7, L.logits)),
        ("gate_route", lambda: B.moe_gate_route_grouped(s, args.groups, L.logits, keys, L.probs, L.expert_idx,
                                                        L.gate_w, L.slot, L.expert_count, L.expert_demand,
                                                        L.slot_src, L.ws)),
        ("dispatch", lambda: B.moe_dispatch_tokens(s, x, L.expert_idx, L.slot, L.xd)),
        ("expert_ffn_fwd", (lambda: B.moe_expert_ffn_fwd_dropout(s, L.xd, L.expert_count, W1, W2, args.drop_p, 7,
                                                                 L.h, L.dact, L.yd))
         if args.drop_p > 0 else
         (lambda: B.moe_expert_ffn_fwd(s, L.xd, L.expert_count, W1, W2, L.h, L.dact, L.yd))),
        ("combine_fwd", lambda: B.moe_combine_fwd(s, L.yd, L.expert_idx, L.slot, L.gate_w, L.y)),
        ("combine_bwd", lambda: B.moe_combine_bwd(s, dy, L.yd, L.expert_idx, L.slot, L.gate_w, L.dyd, L.dgate_w)),
        ("expert_ffn_bwd", lambda: B.moe_expert_ffn_bwd(s, L.dyd, L.xd, L.h, L.dact, L.expert_count, W1, W2,
                                                        L.dxd, L.dW1, L.dW2, L.ws)),
        ("gate_bwd", (lambda: B.moe_gate_bwd(s, L.dgate_w, L.probs, L.expert_idx, L.slot, L.dlogits))
         if args.aux_coef == 0.0 else
         (lambda: B.moe_gate_bwd_aux(s, L.dgate_w, L.probs, L.expert_idx, L.slot, L.first_frac, args.aux_coef,
                                     L.dlogits))),
        ("dispatch_gate_logits_bwd", lambda: B.moe_dispatch_gate_logits_bwd(s, x, Wg, L.dlogits, L.dxd, L.expert_idx, L.slot,
                                                                            args.jitter_eps, 7, L.dWg, L.dx, L.ws)),
    ]
    if args.aux_coef != 0.0 and not args.forward_only:
        calls.insert(2, ("aux_loss", lambda: B.moe_aux_loss(s, L.probs, L.expert_idx, L.first_frac, L.mean_prob,
                                                            L.aux_loss, L.ws)))
    if args.forward_only:
        calls = calls[:[n for n, _ in calls].index("combine_fwd") + 1]
        calls.insert(2, ("utilisation", lambda: B.moe_utilisation_accumulate(s, L.expert_demand, L.utilisation)))
    gemm_calls = {"expert_ffn_fwd", "expert_ffn_bwd"}

    for _ in range(args.warmup):
        for _, fn in calls:
            fn()
    torch.cuda.synchronize()

    # timed region: exactly K steps; HIP events (torch's current stream is the
    # stream the kernels are launched on) bracket the expert-GEMM calls
    # and, for the HBM-bound steps the metric also names, the route / dispatch / combine calls
    hbm_calls = ("gate_logits", "gate_route", "dispatch", "combine_fwd", "combine_bwd", "dispatch_gate_logits_bwd")
    timed = [n for n, _ in calls if n in gemm_calls or n in hbm_calls]
    ev = [{n: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for n in timed}
          for _ in range(args.steps)]
    step_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step_ev[i][0].record()
        for name, fn in calls:
            if name in ev[i]:
                ev[i][name][0].record()
                fn()
                ev[i][name][1].record()
            else:
                fn()
        step_ev[i][1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    step_ms = sorted(a.elapsed_time(b) for a, b in step_ev)     # per step, HIP events on the same stream
    call_ms = {n: sum(e[n][0].elapsed_time(e[n][1]) for e in ev) / args.steps for n in timed}
    gemm_ms = sum(v for n, v in call_ms.items() if n in gemm_calls)

    M = int(L.expert_count.sum().item())                      # kept assignments actually routed
    n_gemm = 2 if args.forward_only else 6
    flops = 2.0 * n_gemm * M * w.d_model * w.d_ff             # grouped GEMMs of 2*M*d*f each
    peak = PEAK_BF16_MFMA if w.dtype == I.BF16 else PEAK_F32_MFMA
    sb = 2 if w.dtype == I.BF16 else 4
    # algorithmic HBM bytes of the expert FFN (what the method must move on kept rows, each tensor once):
    # forward: xd, yd, the saved activation, W1, W2; backward adds dyd, xd, the saved activation, W1, W2 read and
    # dxd and the fp32 dW1, dW2 written
    ffn_bytes = M * (2 * w.d_model + w.d_ff) * sb + 2 * w.E * w.d_model * w.d_ff * sb
    if not args.forward_only:
        ffn_bytes += M * (3 * w.d_model + w.d_ff) * sb + 2 * w.E * w.d_model * w.d_ff * sb + 8 * w.E * w.d_model * w.d_ff
    t_mfma, t_hbm = flops / peak, ffn_bytes / PEAK_HBM        # the two floors of the GEMM phase
    gemm_s = gemm_ms * 1e-3
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", f"grouped_gemm_{w.name}_hbm_traffic.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch"):
                traffic = float(line.split("=")[1])
            if line.startswith("measured_at_commit"):
                traffic_source = f"profiles/{os.path.basename(tpath)} (rocprofv3 counters, kernels of commit {line.split('=')[1].strip()})"
    if t_mfma >= t_hbm:
        roofline = {"bound": "mfma", "achieved": flops / gemm_s / 1e12, "peak": peak / 1e12, "unit": "TFLOP/s",
                    "frac": flops / gemm_s / peak}
    else:       # few rows per expert: weight and weight-gradient traffic, not the matrix pipe, bounds the FFN
        roofline = {"bound": "hbm", "achieved": ffn_bytes / gemm_s / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                    "frac": ffn_bytes / gemm_s / PEAK_HBM}
    roofline.update({"kernel": f"grouped_gemm_kernel ({n_gemm} launches per step)", "traffic": traffic,
                     "traffic_source": traffic_source,
                     "flops_per_launch": flops / n_gemm, "algorithmic_bytes_per_launch": ffn_bytes / n_gemm,
                     "avg_launch_ms": gemm_ms / n_gemm, "kept_assignments": M,
                     "floor_ms": {"mfma": t_mfma * 1e3, "hbm": t_hbm * 1e3},
                     "frac_of_mfma_peak": flops / gemm_s / peak, "frac_of_hbm_peak": ffn_bytes / gemm_s / PEAK_HBM})

    # algorithmic HBM bytes per call (each tensor once; gathered rows counted per use)
    Tn, dm, E, k, C = w.T, w.d_model, w.E, w.k, w.capacity
    kept_tok = int((L.slot >= 0).any(dim=1).sum().item())
    alg = {
        "gate_logits": Tn * dm * sb + dm * E * 4 + Tn * E * 4,
        "gate_route": Tn * E * 4 * 2 + 12 * Tn * k + 4 * Tn + 4 * Tn * k + 4 * E * C + 8 * E,
        "dispatch": kept_tok * dm * sb + 8 * Tn * k + M * dm * sb,
        "combine_fwd": M * dm * sb + 12 * Tn * k + Tn * dm * sb,
        "combine_bwd": Tn * dm * sb + M * dm * sb + M * dm * sb + 4 * Tn * k,
        "gate_bwd": Tn * E * 4 * 2 + 16 * Tn * k,
        "aux_loss": Tn * E * 4 + 4 * Tn * k,
        # x and dlogits for dWg; the kept rows of dxd, dlogits and Wg for dx; dx written once
        "dispatch_gate_logits_bwd": Tn * dm * sb + 2 * Tn * E * 4 + M * dm * sb + 8 * Tn * k + Tn * dm * sb
                                    + dm * E * 8,
    }
    hbm = {n: {"us": call_ms[n] * 1e3, "GBps": alg[n] / (call_ms[n] * 1e-3) / 1e9,
               "frac_of_8TBps": alg[n] / (call_ms[n] * 1e-3) / PEAK_HBM}
           for n in hbm_calls if n in call_ms}

    if "gate_logits" in hbm and "gate_route" in hbm:
        # the gate projection, softmax/top-k and the capacity rank together: the only part of "route" with real
        # HBM traffic is the projection's read of x; the rank itself is integer work on data that lives in L2
        us = hbm["gate_logits"]["us"] + hbm["gate_route"]["us"]
        by = alg["gate_logits"] + alg["gate_route"]
        hbm["route_a0_a3"] = {"us": us, "GBps": by / (us * 1e-6) / 1e9, "frac_of_8TBps": by / (us * 1e-6) / PEAK_HBM}

    breakdown = None
    if args.breakdown:
        n = len(calls)
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(n + 1)] for _ in range(args.steps)]
        for i in range(args.steps):
            for j, (_, fn) in enumerate(calls):
                evs[i][j].record()
                fn()
            evs[i][n].record()
        torch.cuda.synchronize()
        breakdown = {}
        for j, (name, _) in enumerate(calls):
            ts = sorted(evs[i][j].elapsed_time(evs[i][j + 1]) for i in range(args.steps))
            breakdown[name] = {"median_us": ts[len(ts) // 2] * 1e3, "min_us": ts[0] * 1e3}
        for name, b in alg.items():
            if name not in breakdown:
                continue
            us = breakdown[name]["median_us"]
            breakdown[name]["alg_MB"] = b / 1e6
            breakdown[name]["GBps"] = b / (us * 1e-6) / 1e9
            breakdown[name]["hbm_frac"] = b / (us * 1e-6) / PEAK_HBM
        for name, fl in (("expert_ffn_fwd", 4.0), ("expert_ffn_bwd", 8.0)):
            if name not in breakdown:
                continue
            us = breakdown[name]["median_us"]
            breakdown[name]["TFLOPs"] = fl * M * dm * w.d_ff / (us * 1e-6) / 1e12
            breakdown[name]["mfma_frac"] = fl * M * dm * w.d_ff / (us * 1e-6) / peak
        for name, v in breakdown.items():
            print(f"[breakdown] {name:16s} " + " ".join(f"{k}={val:.4g}" for k, val in v.items()), file=sys.stderr)

    out = {
        "metric": "MoE layer fwd+bwd tokens/sec on 1 MI355X; expert-GEMM MFMA util; route HBM GB/s",
        "value": w.T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_median": step_ms[len(step_ms) // 2],
        "ms_per_step_min": step_ms[0],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if w.dtype == I.BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "T": w.T, "d_model": w.d_model, "d_ff": w.d_ff, "E": w.E, "k": w.k,
                   "capacity": w.capacity, "capacity_factor": w.capacity_factor,
                   "act": "gelu" if w.act == I.GELU else "relu", "aux_coef": args.aux_coef, "groups": args.groups, "jitter_eps": args.jitter_eps,
                   "drop_p": args.drop_p,
                   "mode": "forward-only (evaluation)" if args.forward_only else "forward+backward (training)",
                   "kept_assignments": M,
                   "tokens_fully_dropped": int((L.slot < 0).all(dim=1).sum().item()),
                   "gate_skew": gate_skew(w, d["bias"]),
                   "expert_demand_max": int(L.expert_demand.max().item()),
                   "expert_demand_min": int(L.expert_demand.min().item()),
                   "expert_demand": [int(v) for v in L.expert_demand.cpu().tolist()]},
        "roofline": roofline,
        # the metric's other two parts: MFMA utilisation of the expert GEMMs = roofline.frac; achieved
        # algorithmic HBM rate of the route / dispatch / combine calls (HIP events inside the timed region)
        "expert_gemm_mfma_util": roofline["frac_of_mfma_peak"],
        "hbm_calls": hbm,
    }
    if breakdown is not None:
        out["breakdown"] = breakdown
    out["measured_peaks"] = measured_peaks(torch, B)
    mp = out["measured_peaks"]
    if w.dtype == I.BF16 and "mfma_bf16_TFLOPs_random_operands" in mp:
        # context beside the headline fraction (which is against the published peak): what a register-resident
        # MFMA loop on random operands sustains on this machine, and a plain copy
        out["roofline"]["frac_of_measured_mfma_random_operands"] = flops / gemm_s / 1e12 / mp["mfma_bf16_TFLOPs_random_operands"]
        out["roofline"]["frac_of_measured_copy_rate"] = ffn_bytes / gemm_s / 1e12 / mp["copy_TBps"]
    if args.vendor_reference:
        out["vendor_reference"] = vendor_reference(torch, w)
    if not args.no_cpu_baseline:
        del x, dy, W1, W2, layer, L
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(w, d, forward_only=args.forward_only)
    print(json.dumps(out), flush=True)


def gate_skew(w, bias):
    """How the workload's routing skew was synthesised: the logit bias b = beta * onehot(0) (one hot expert) or
    b_e = tau * ln q_e with q_e ~ rank^-a (Zipf), recovered from the generator's bias array."""
    import math
    if bias is None:
        return {"kind": "none"}
    if w.skew == "hot0":
        return {"kind": "hot0", "target_top1_share": w.skew_param, "beta": float(bias[0])}
    q0 = 1.0 / sum(r ** -w.skew_param for r in range(1, w.E + 1))
    return {"kind": "zipf", "exponent": w.skew_param, "tau": float(bias.max()) / math.log(q0)}


def vendor_reference(torch, w):
    """The vendor library's batched GEMM on the two forward products of this workload's shape, every expert full
    (capacity rows), bf16 in and out, no activation, no second output: what a plain library call reaches on this
    box, for scale beside the expert GEMM's own figures.  Row-major operands as the layer holds them (no transposed
    views).  Outside the timed region; never part of `value`."""
    try:
        from paper_2109_10465_amd import inputs as I
        if w.dtype != I.BF16:
            return {"skipped": "bf16 workloads only"}
        E, C, d, f = w.E, w.capacity, w.d_model, w.d_ff
        g = torch.Generator(device="cuda")
        g.manual_seed(0)
        mk = lambda *sh: torch.randn(*sh, device="cuda", generator=g).to(torch.bfloat16)
        xd, h, W1, W2 = mk(E, C, d), mk(E, C, f), mk(E, d, f) * 0.02, mk(E, f, d) * 0.02
        res = {"shape": {"E": E, "rows_per_expert": C, "d_model": d, "d_ff": f}, "library": "torch.bmm"}
        flop = 2.0 * E * C * d * f
        for name, fn in (("fwd1_xd_W1", lambda: torch.bmm(xd, W1)), ("fwd2_h_W2", lambda: torch.bmm(h, W2))):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                fn()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / 20 * 1e3
            res[name] = {"us": us, "TFLOPs": flop / us / 1e6, "frac_of_mfma_peak": flop / us / 1e6 / 2500.0}
        return res
    except Exception as exc:      # noqa: BLE001 - report, never fail the line
        return {"error": repr(exc)}


def measured_peaks(torch, B):
    """What this machine sustains, for scale beside the published peaks the fractions are quoted against: a plain
    device-to-device copy (read + write bytes) and a register-resident bf16 MFMA loop (random and all-equal
    operands: the clock under matrix load depends on the data).  Outside the timed region; a failure here never
    costs the benchmark line."""
    try:
        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e-3 / reps
        src = torch.empty(1 << 27, dtype=torch.float32, device="cuda").normal_()      # 512 MiB
        dst = torch.empty_like(src)
        t_copy = timed(lambda: dst.copy_(src), 5)
        del dst
        n_wg = 4 * torch.cuda.get_device_properties(0).multi_processor_count         # 4 waves per SIMD
        outb = torch.empty(n_wg * 256, dtype=torch.float32, device="cuda")
        iters = 20000
        flop = n_wg * 4 * iters * 8 * 32768.0
        res = {"copy_TBps": 2 * src.numel() * 4 / t_copy / 1e12, "published": {"hbm_TBps": 8.0, "mfma_bf16_TFLOPs": 2500.0}}
        for name, rnd in (("mfma_bf16_TFLOPs_random_operands", 1), ("mfma_bf16_TFLOPs_equal_operands", 0)):
            res[name] = flop / timed(lambda: B.moe_microbench_mfma_bf16(n_wg, iters, rnd, outb), 3) / 1e12
        return res
    except Exception as exc:      # noqa: BLE001 - report, never fail the line
        return {"error": repr(exc)}


if __name__ == "__main__":
    main()
