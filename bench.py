#!/usr/bin/env python3
"""Benchmark of the GLA forward hot path on one MI355X.

A step is one call of the whole path (gla_fwd_ex: span states, carry, outputs)
on one batch of synthetic DiG-XL/2 activations at 2048 px (B=1, H=16, T=16384,
dk=36, dv=72, bf16 q/k/v, fp32 log_alpha, fp32 out), inputs resident in HBM.
Steps rotate over several independent buffer sets so that every call streams
from HBM rather than from the 256 MB last-level cache.

Prints ONE JSON line (metric, value, unit, timing, workload, roofline, cpu_baseline).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def algorithmic_bytes_per_token_head(dk, dv, qkv_bytes, out_bytes):
    # q, k, v read once, log_alpha (fp32) read once, out written once
    return 2 * dk * qkv_bytes + dk * 4 + dv * qkv_bytes + dv * out_bytes


def algorithmic_flops_per_token_head(dk, dv, chunk=64):
    # state update + state read: 4*dk*dv ; causal half of the in-chunk scores and their use: (C+1)(dk+dv)
    return 4 * dk * dv + (chunk + 1) * (dk + dv)


def measured_traffic(config_name, kernel, args):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary (None if absent or if
    this run does not use the configuration the summary was taken with)."""
    if (args.out_dtype != "f32" or args.scan != 0 or args.chunks_per_span != 0 or args.engine != 0
            or args.layout != "bhtd"):
        return None
    path = os.path.join(ROOT, "profiles", f"gla_fwd_{config_name}_hbm_traffic.md")
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) >= 3 and parts[0] == "TRAFFIC_BYTES_PER_LAUNCH" and parts[1] == kernel:
                return int(float(parts[2]))
    except OSError:
        pass
    return None


def time_forward(name, scan, gla, gi, torch, np, steps=200, warmup=20, nsets=4, check=True):
    """One line of the `configs` table: gla_fwd_ex on a contract workload over rotating buffer sets (every call
    streams from HBM), whole-call time, algorithmic bytes, fraction of the HBM peak, parity against the oracle."""
    cfg = gi.CONFIGS[name]
    dev = torch.device("cuda:0")
    d = gi.make_config_inputs(cfg)
    B, H, T, dk, dv = cfg.B, cfg.H, cfg.T, cfg.dk, cfg.dv
    bf16 = cfg.dtype == "bf16"
    if bf16:
        host = [torch.from_numpy(d[n + "_bits"].view(np.int16)).view(torch.bfloat16) for n in ("q", "k", "v")]
    else:
        host = [torch.from_numpy(d[n]) for n in ("q", "k", "v")]
    host.append(torch.from_numpy(d["log_alpha"]))
    ws_bytes = gla.gla_fwd_workspace_bytes(B, H, T, dk, dv, gla.DT_BF16 if bf16 else gla.DT_F32)
    sets = []
    for _ in range(nsets):
        q, k, v, la = (t.to(dev) for t in host)
        sets.append((q, k, v, la, torch.empty((B, H, T, dv), dtype=torch.float32, device=dev),
                     torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev),
                     torch.empty((ws_bytes,), dtype=torch.uint8, device=dev)))

    def step(i):
        q, k, v, la, out, fin, ws = sets[i % nsets]
        gla.gla_fwd_ex(q, k, v, la, cfg.grid_h, cfg.grid_w, scan, out=out, final_state=fin, workspace=ws)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    alg_bytes = algorithmic_bytes_per_token_head(dk, dv, 2 if bf16 else 4, 4) * B * H * T
    row = {"workload": name, "scan": scan, "ms_per_step": round(ms, 5), "tokens_per_s": round(B * T / (ms * 1e-3), 1),
           "algorithmic_bytes": alg_bytes,
           "whole_path_frac": round(alg_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    if check:
        from oracle import gla_oracle
        ref, ref_fin = gla_oracle.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], cfg.grid_h, cfg.grid_w, scan)
        step(0)
        torch.cuda.synchronize()
        rms = float(np.sqrt(np.mean(ref.astype(np.float64) ** 2)))
        row["max_err_over_rms"] = round(float(np.abs(sets[0][4].cpu().numpy() - ref).max() / rms), 6)
    del sets
    torch.cuda.empty_cache()
    return row


# the contract workloads (scan order 0 unless named) and the throughput-only shapes, as timed for the `configs` table
TABLE = [("tiny_f32", 0), ("dig_s2_256", 0), ("dig_xl2_512", 0), ("dig_xl2_1024", 0), ("dig_xl2_2048", 0),
         ("dig_xl2_2048_longmem", 0), ("dig_xl2_2048", 2), ("dig_xl2_2048", 3), ("dig_s2_1792", 0)]


def bench_fused(args, cfg, gla, gi, torch, np):
    """gla_fwd_fused on the workload (gates from bf16 pre-activations, Swish gate times LayerNorm before a bf16
    store): whole-call timing over rotating buffer sets, parity figure against the oracle."""
    dev = torch.device("cuda:0")
    B, H, T, dk, dv = cfg.B, cfg.H, cfg.T, cfg.dk, cfg.dv
    d = gi.make_fused_inputs(B, H, T, dk, dv, cfg.dtype, seed=cfg.seed, z_mean=cfg.z_mean)
    bf16 = cfg.dtype == "bf16"
    if bf16:
        to = lambda bits: torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)
        host = [to(d[n + "_bits"]) for n in ("q", "k", "v", "z", "r")]
    else:
        host = [torch.from_numpy(d[n]) for n in ("q", "k", "v", "z", "r")]
    host += [torch.from_numpy(d["ln_w"]), torch.from_numpy(d["ln_b"])]
    odt = torch.bfloat16 if args.out_dtype == "bf16" else torch.float32
    qdt = gla.DT_BF16 if bf16 else gla.DT_F32
    ws_bytes = gla.gla_fwd_workspace_bytes(B, H, T, dk, dv, qdt)
    sets = []
    for _ in range(max(1, args.sets)):
        sets.append([t.to(dev) for t in host] + [torch.empty((B, H, T, dv), dtype=odt, device=dev),
                                                 torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev),
                                                 torch.empty((ws_bytes,), dtype=torch.uint8, device=dev)])

    epi = not args.no_epilogue

    def step(i):
        q, k, v, z, r, lw, lb, out, fin, ws = sets[i % len(sets)]
        return gla.gla_fwd_fused(q, k, v, z, 16.0, cfg.grid_h, cfg.grid_w, args.scan, r_pre=r if epi else None,
                                 ln_weight=lw if epi else None, ln_bias=lb if epi else None, ln_eps=1e-5, out=out,
                                 final_state=fin, workspace=ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    qb = 2 if bf16 else 4
    ob = 2 if args.out_dtype == "bf16" else 4
    alg_bytes = (3 * dk * qb + (2 if epi else 1) * dv * qb + dv * ob) * B * H * T   # q, k, z, v (, r) read once; y written once
    achieved = alg_bytes / (ms * 1e-3) / 1e9
    result = {
        "metric": "GLA fwd (gate prologue + Swish/LayerNorm epilogue) tokens/s at DiG-XL/2 shape T=16384" if epi
        else "GLA fwd (gate prologue: gates from bf16 pre-activations) tokens/s at DiG-XL/2 shape T=16384",
        "value": round(B * T / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} fused: B={B} H={H} T={T} ({cfg.grid_h}x{cfg.grid_w}) dk={dk} dv={dv} "
                               f"{cfg.dtype} q/k/v/z/r, {args.out_dtype} out, scan={args.scan}",
                   "buffer_sets": len(sets)},
        "roofline": {"bound": "hbm", "kernel": "whole_call", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes": alg_bytes, "kernel_ms": round(ms, 5)},
    }
    if not args.no_check:
        from oracle import gla_oracle_fused as fo
        ref, ref_fin = fo.gla_fused(d["q"], d["k"], d["v"], d["z"], 16.0, d["r"] if epi else None,
                                    d["ln_w"] if epi else None, d["ln_b"] if epi else None, 1e-5,
                                    cfg.grid_h, cfg.grid_w, args.scan)
        got, fin = step(0)
        torch.cuda.synchronize()
        rms = float(np.sqrt(np.mean(ref ** 2)))
        result["max_err_over_rms"] = round(float(np.abs(got.float().cpu().numpy() - ref).max() / rms), 6)
    print(json.dumps(result), flush=True)


def bench_multi(args, cfg, d, gla, gi, torch, np, dirs):
    """gla_fwd_multi (sum over scan orders) on the workload: whole-call timing over rotating buffer sets."""
    dev = torch.device("cuda:0")
    B, H, T, dk, dv = cfg.B, cfg.H, cfg.T, cfg.dk, cfg.dv
    bf16 = cfg.dtype == "bf16"
    if bf16:
        host = [torch.from_numpy(d[n + "_bits"].view(np.int16)).view(torch.bfloat16) for n in ("q", "k", "v")]
    else:
        host = [torch.from_numpy(d[n]) for n in ("q", "k", "v")]
    host.append(torch.from_numpy(d["log_alpha"]))
    qdt = gla.DT_BF16 if bf16 else gla.DT_F32
    ws_bytes = gla.gla_fwd_workspace_bytes(B, H, T, dk, dv, qdt)
    sets = []
    for _ in range(max(1, args.sets)):
        sets.append([t.to(dev) for t in host] + [torch.empty((B, H, T, dv), dtype=torch.float32, device=dev),
                                                 torch.empty((ws_bytes,), dtype=torch.uint8, device=dev)])

    def step(i):
        q, k, v, la, out, ws = sets[i % len(sets)]
        return gla.gla_fwd_multi(q, k, v, la, cfg.grid_h, cfg.grid_w, dirs, out=out, workspace=ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    qb = 2 if bf16 else 4
    alg_bytes = (2 * dk * qb + dk * 4 + dv * qb + dv * 4) * B * H * T   # inputs read once, the sum written once
    achieved = alg_bytes / (ms * 1e-3) / 1e9
    result = {
        "metric": f"GLA fwd, {len(dirs)} scan orders summed, tokens/s at DiG-XL/2 shape T=16384",
        "value": round(B * T / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} scan orders {list(dirs)}: B={B} H={H} T={T} ({cfg.grid_h}x{cfg.grid_w}) "
                               f"dk={dk} dv={dv} {cfg.dtype} q/k/v, fp32 log_alpha, fp32 out",
                   "buffer_sets": len(sets)},
        "roofline": {"bound": "hbm", "kernel": "whole_call", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes": alg_bytes, "kernel_ms": round(ms, 5)},
    }
    if not args.no_check:
        from oracle import gla_oracle
        ref = gla_oracle.gla_fwd_multi(d["q"], d["k"], d["v"], d["log_alpha"], cfg.grid_h, cfg.grid_w, dirs)
        got = step(0)
        torch.cuda.synchronize()
        rms = float(np.sqrt(np.mean(ref ** 2)))
        result["max_err_over_rms"] = round(float(np.abs(got.cpu().numpy() - ref).max() / rms), 6)
    print(json.dumps(result), flush=True)


def bench_gates(args, cfg, gla, gi, torch, np):
    """gla_fwd_gates (two-sided gate alpha_t^T beta_t) at the workload's shape, or (--pass fusedgates)
    gla_fwd_fused_gates: both gates from bf16 pre-activations plus the Swish / LayerNorm epilogue."""
    dev = torch.device("cuda:0")
    B, H, T, dk, dv = cfg.B, cfg.H, cfg.T, cfg.dk, cfg.dv
    fused = args.which == "fusedgates"
    bf16 = cfg.dtype == "bf16"
    if fused:
        d = gi.make_fused_gate_inputs(B, H, T, dk, dv, cfg.dtype, cfg.seed, cfg.z_mean)
        names = ("q", "k", "v", "z", "zb", "r")
    else:
        d = gi.make_gate_inputs(B, H, T, dk, dv, cfg.dtype, cfg.seed, cfg.z_mean)
        names = ("q", "k", "v")
    if bf16:
        host = [torch.from_numpy(d[n + "_bits"].view(np.int16)).view(torch.bfloat16) for n in names]
    else:
        host = [torch.from_numpy(d[n]) for n in names]
    if fused:
        lnw, lnb = torch.from_numpy(d["ln_w"]).to(dev), torch.from_numpy(d["ln_b"]).to(dev)
    else:
        host += [torch.from_numpy(d["log_alpha"]), torch.from_numpy(d["log_beta"])]
    qdt = gla.DT_BF16 if bf16 else gla.DT_F32
    ws_bytes = gla.gla_fwd_workspace_bytes(B, H, T, dk, dv, qdt)
    sets = []
    for _ in range(max(1, args.sets)):
        sets.append([t.to(dev) for t in host] + [torch.empty((ws_bytes,), dtype=torch.uint8, device=dev),
                                                 torch.empty((B, H, T, dv), dtype=torch.float32, device=dev),
                                                 torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev)])

    def step(i):
        if fused:
            q, k, v, z, zb, r, ws, out, fin = sets[i % len(sets)]
            return gla.gla_fwd_fused_gates(q, k, v, z, zb, 16.0, cfg.grid_h, cfg.grid_w, args.scan, r_pre=r,
                                           ln_weight=lnw, ln_bias=lnb, ln_eps=1e-5, out=out, final_state=fin,
                                           workspace=ws)
        q, k, v, la, lb, ws, out, fin = sets[i % len(sets)]
        return gla.gla_fwd_gates(q, k, v, la, lb, cfg.grid_h, cfg.grid_w, args.scan, out=out, final_state=fin,
                                 workspace=ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    qb = 2 if bf16 else 4
    if fused:
        alg_bytes = (3 * dk * qb + 3 * dv * qb + dv * 4) * B * H * T    # q, k, z_alpha; v, z_beta, r; y
    else:
        alg_bytes = (2 * dk * qb + dk * 4 + dv * qb + dv * 4 + dv * 4) * B * H * T   # q, k, log_alpha, v, log_beta, out
    alg_flops = 5 * dk * dv * B * H * T      # per state element and token: gate product, decay FMA, k*v, read FMA
    achieved = alg_flops / (ms * 1e-3) / 1e12
    result = {
        "metric": ("GLA fwd with both gates from pre-activations and the output epilogue" if fused else
                   "GLA fwd with the two-sided gate") + ", tokens/s at DiG-XL/2 shape T=16384",
        "value": round(B * T / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} + {'z_beta, r' if fused else 'log_beta'}: B={B} H={H} T={T} ({cfg.grid_h}x{cfg.grid_w}) dk={dk} dv={dv} "
                               f"{cfg.dtype} q/k/v, {cfg.dtype + ' gate pre-activations' if fused else 'fp32 gates'}, fp32 out, "
                               f"scan {args.scan}", "buffer_sets": len(sets)},
        "roofline": {"bound": "alu", "kernel": "whole_call", "achieved": round(achieved, 2), "peak": 157.3,
                     "unit": "TFLOP/s", "frac": round(achieved / 157.3, 4), "traffic": None,
                     "algorithmic_flops": alg_flops, "algorithmic_bytes": alg_bytes, "kernel_ms": round(ms, 5)},
    }
    if not args.no_check:
        from oracle import gla_oracle_gates, gla_oracle_fused
        if fused:
            ref, _ = gla_oracle_fused.gla_fused_gates(d["q"], d["k"], d["v"], d["z"], d["zb"], 16.0, d["r"], d["ln_w"],
                                                      d["ln_b"], 1e-5, cfg.grid_h, cfg.grid_w, args.scan)
        else:
            ref, _ = gla_oracle_gates.gla_fwd_gates(d["q"], d["k"], d["v"], d["log_alpha"], d["log_beta"],
                                                    cfg.grid_h, cfg.grid_w, args.scan)
        got, _ = step(0)
        torch.cuda.synchronize()
        rms = float(np.sqrt(np.mean(ref ** 2)))
        result["max_err_over_rms"] = round(float(np.abs(got.cpu().numpy() - ref).max() / rms), 6)
    print(json.dumps(result), flush=True)


def bench_bwd_gates(args, cfg, gla, gi, torch, np):
    """gla_bwd_gates (backward of the two-sided-gate recurrence) at the workload's shape."""
    dev = torch.device("cuda:0")
    B, H, T, dk, dv = cfg.B, cfg.H, cfg.T, cfg.dk, cfg.dv
    d = gi.make_gate_inputs(B, H, T, dk, dv, cfg.dtype, cfg.seed, cfg.z_mean)
    w = np.random.Generator(np.random.PCG64(cfg.seed + 1000)).standard_normal((B, H, T, dv), dtype=np.float32)
    bf16 = cfg.dtype == "bf16"
    if bf16:
        wb = gi.round_to_bf16_bits(w)
        w = gi.bf16_bits_to_f32(wb)
        host = [torch.from_numpy(d[n + "_bits"].view(np.int16)).view(torch.bfloat16) for n in ("q", "k", "v")]
        host.append(torch.from_numpy(wb.view(np.int16)).view(torch.bfloat16))
    else:
        host = [torch.from_numpy(d[n]) for n in ("q", "k", "v")] + [torch.from_numpy(w)]
    host += [torch.from_numpy(d["log_alpha"]), torch.from_numpy(d["log_beta"])]
    qdt = gla.DT_BF16 if bf16 else gla.DT_F32
    ws_bytes = gla.gla_bwd_gates_workspace_bytes(B, H, T, dk, dv, qdt)
    sets = [[t.to(dev) for t in host] + [torch.empty((ws_bytes,), dtype=torch.uint8, device=dev)]
            for _ in range(max(1, min(args.sets, 2)))]

    outs = None
    if args.reuse_fwd:      # the fp32 outputs of the forward call are handed over instead of being recomputed
        outs = [gla.gla_fwd_gates(s_[0], s_[1], s_[2], s_[4], s_[5], cfg.grid_h, cfg.grid_w, args.scan)[0] for s_ in sets]

    def step(i):
        q, k, v, wt, la, lb, ws = sets[i % len(sets)]
        return gla.gla_bwd_gates(q, k, v, la, lb, wt, cfg.grid_h, cfg.grid_w, args.scan, workspace=ws,
                                 out_fwd=outs[i % len(sets)] if outs else None)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    qb = 2 if bf16 else 4
    # q, k, v, dO, both gates read once; five gradients written once
    alg_bytes = ((2 * dk + 2 * dv) * qb + (dk + dv) * 4 + (3 * dk + 2 * dv) * 4) * B * H * T
    achieved = alg_bytes / (ms * 1e-3) / 1e9
    result = {
        "metric": "GLA bwd with the two-sided gate, tokens/s at DiG-XL/2 shape T=16384",
        "value": round(B * T / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} + log_beta, backward: B={B} H={H} T={T} ({cfg.grid_h}x{cfg.grid_w}) dk={dk} "
                               f"dv={dv} {cfg.dtype} q/k/v/dO, fp32 gates and gradients, scan {args.scan}",
                   "buffer_sets": len(sets)},
        "roofline": {"bound": "hbm", "kernel": "whole_call", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes": alg_bytes, "kernel_ms": round(ms, 5)},
    }
    if not args.no_check:
        # the oracle keeps every state of a sequence: check the first two heads (heads are independent)
        from oracle import gla_oracle_gates
        hs = slice(0, min(H, 2))
        ref = gla_oracle_gates.gla_bwd_gates(d["q"][:1, hs], d["k"][:1, hs], d["v"][:1, hs], d["log_alpha"][:1, hs],
                                             d["log_beta"][:1, hs], w[:1, hs], cfg.grid_h, cfg.grid_w, args.scan)
        got = step(0)
        torch.cuda.synchronize()
        errs = {}
        for name, g, r in zip(("dq", "dk", "dv", "dlog_alpha", "dlog_beta"), got, ref):
            rms = float(np.sqrt(np.mean(r ** 2)))
            errs[name] = round(float(np.abs(g[:1, hs].cpu().numpy() - r).max() / rms), 6)
        result["err_over_rms_first_two_heads"] = errs
    print(json.dumps(result), flush=True)


def bench_srem(args, cfg, gla, gi, torch, np):
    """gla_srem_dwconv on the token matrix of the workload ([B, T, H*dv] bf16 in and out)."""
    dev = torch.device("cuda:0")
    B, T, D = cfg.B, cfg.T, cfg.H * cfg.dv
    rng = np.random.Generator(np.random.PCG64(cfg.seed + 3000))
    x = rng.standard_normal((B, T, D), dtype=np.float32)
    bits = gi.round_to_bf16_bits(x)
    x = gi.bf16_bits_to_f32(bits)
    w = (rng.standard_normal((D, 3, 3), dtype=np.float32) * np.float32(0.3)).astype(np.float32)
    w[:, 1, 1] += np.float32(1)
    b = (rng.standard_normal((D,), dtype=np.float32) * np.float32(0.1)).astype(np.float32)
    wt, bt = torch.from_numpy(w).to(dev), torch.from_numpy(b).to(dev)
    sets = []
    for _ in range(max(1, args.sets)):
        xt = torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
        sets.append((xt, torch.empty_like(xt)))

    def step(i):
        xt, yt = sets[i % len(sets)]
        return gla.gla_srem_dwconv(xt, wt, bt, cfg.grid_h, cfg.grid_w, args.scan, out=yt)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    alg_bytes = 2 * 2 * B * T * D        # every element read once and written once, bf16
    achieved = alg_bytes / (ms * 1e-3) / 1e9
    result = {
        "metric": "SREM 3x3 depth-wise convolution tokens/s at DiG-XL/2 shape T=16384",
        "value": round(B * T / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name} token matrix: B={B} {cfg.grid_h}x{cfg.grid_w} D={D} bf16 in/out, "
                               f"orient={args.scan}", "buffer_sets": len(sets)},
        "roofline": {"bound": "hbm", "kernel": "srem_dwconv_kernel", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes": alg_bytes, "kernel_ms": round(ms, 5)},
    }
    if not args.no_check:
        from oracle import srem_oracle as so
        ref = so.srem_dwconv(x, w, b, cfg.grid_h, cfg.grid_w, args.scan)
        got = step(0).float().cpu().numpy()
        rms = float(np.sqrt(np.mean(ref ** 2)))
        result["max_err_over_rms"] = round(float(np.abs(got - ref).max() / rms), 6)
    print(json.dumps(result), flush=True)


def bench_backward(args, cfg, d, gla, gi, torch, np):
    """gla_bwd on the workload: whole-call timing over rotating buffer sets, oracle timing, parity figure."""
    dev = torch.device("cuda:0")
    B, H, T, dk, dv = cfg.B, cfg.H, cfg.T, cfg.dk, cfg.dv
    rng = np.random.Generator(np.random.PCG64(cfg.seed + 1000))
    w = rng.standard_normal((B, H, T, dv), dtype=np.float32)
    bf16 = cfg.dtype == "bf16"
    if bf16:
        w_bits = gi.round_to_bf16_bits(w)
        w = gi.bf16_bits_to_f32(w_bits)
        to = lambda bits: torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)
        host = [to(d["q_bits"]), to(d["k_bits"]), to(d["v_bits"]), torch.from_numpy(d["log_alpha"]), to(w_bits)]
    else:
        host = [torch.from_numpy(d[n]) for n in ("q", "k", "v", "log_alpha")] + [torch.from_numpy(w)]
    qdt = gla.DT_BF16 if bf16 else gla.DT_F32
    ws_bytes = gla.gla_bwd_workspace_bytes(B, H, T, dk, dv, qdt)
    sets = []
    for _ in range(max(1, args.sets)):
        sets.append([t.to(dev) for t in host] + [torch.empty((ws_bytes,), dtype=torch.uint8, device=dev)])
    train = args.which == "train"     # a step = forward call + backward call that reuses its span states
    fwd_ws = []
    if args.reuse_fwd or train:   # the forward pass of the same step leaves its span states behind
        for q, k, v, la, do, ws in sets:
            fws = torch.empty((gla.gla_fwd_workspace_bytes(B, H, T, dk, dv, qdt),), dtype=torch.uint8, device=dev)
            gla.gla_fwd_ex(q, k, v, la, cfg.grid_h, cfg.grid_w, args.scan, workspace=fws)
            fwd_ws.append(fws)

    fwd_out = [(torch.empty((B, H, T, dv), device=dev), torch.empty((B, H, dk, dv), device=dev)) for _ in sets] if train else []

    def step(i):
        q, k, v, la, do, ws = sets[i % len(sets)]
        if train:
            o, f = fwd_out[i % len(sets)]
            gla.gla_fwd_ex(q, k, v, la, cfg.grid_h, cfg.grid_w, args.scan, out=o, final_state=f,
                           workspace=fwd_ws[i % len(sets)])
        return gla.gla_bwd(q, k, v, la, do, cfg.grid_h, cfg.grid_w, args.scan, workspace=ws,
                           fwd_workspace=fwd_ws[i % len(sets)] if fwd_ws else None)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    qb = 2 if bf16 else 4
    # q, k, v, d_out and log_alpha read once; dq, dk, dlog_alpha, dv (fp32) written once
    alg_bytes = (2 * dk * qb + 2 * dv * qb + dk * 4 + 3 * dk * 4 + dv * 4) * B * H * T
    if train:   # plus the forward call: q, k, v, log_alpha read, out written
        alg_bytes += (2 * dk * qb + dk * 4 + dv * qb + dv * 4) * B * H * T
    achieved = alg_bytes / (ms * 1e-3) / 1e9
    result = {
        "metric": ("GLA fwd+bwd tokens/s at DiG-XL/2 shape T=16384" if train else "GLA bwd tokens/s at DiG-XL/2 shape T=16384"),
        "value": round(B * T / (ms * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} {'forward + backward' if train else 'backward'}: B={B} H={H} T={T} ({cfg.grid_h}x{cfg.grid_w}) dk={dk} dv={dv} "
                               f"{cfg.dtype} q/k/v/d_out, fp32 log_alpha, fp32 gradients, scan={args.scan}"
                               + (", span states of S reused from the forward call" if args.reuse_fwd else ""),
                   "buffer_sets": len(sets)},
        "roofline": {"bound": "hbm", "kernel": "whole_call", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes": alg_bytes, "kernel_ms": round(ms, 5)},
    }
    if not args.no_check or not args.no_cpu_baseline:
        from oracle import gla_oracle
        c0 = time.perf_counter()
        ref = gla_oracle.gla_bwd(d["q"], d["k"], d["v"], d["log_alpha"], w, cfg.grid_h, cfg.grid_w, args.scan)
        c1 = time.perf_counter()
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = {"value": round(B * T / (c1 - c0), 1), "unit": "tokens/s",
                                      "cores": min(gla_oracle.threads(), B * H), "kind": "oracle",
                                      "sample": f"the whole workload ({B * H} sequences of {T} tokens), one run, "
                                                "fp64 step-by-step reverse-mode C loop, OpenMP over batch*head"}
        if not args.no_check:
            got = step(0)
            torch.cuda.synchronize()
            floors = [0.0, 0.0, 0.0, float(np.sqrt(np.mean((d["q"].astype(np.float64) * ref[0]) ** 2)))]
            errs = []
            for g, r, f in zip(got, ref, floors):
                rms = max(float(np.sqrt(np.mean(r ** 2))), f)
                errs.append(float(np.abs(g.cpu().numpy() - r).max() / rms))
            result["max_err_over_rms"] = round(max(errs), 6)
            result["err_over_rms"] = {n: float("%.3g" % e) for n, e in zip(("dq", "dk", "dv", "dlog_alpha"), errs)}
    print(json.dumps(result), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", default="dig_xl2_2048")
    ap.add_argument("--scan", type=int, default=0)
    ap.add_argument("--out-dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--sets", type=int, default=4, help="independent buffer sets rotated over (1 = cache-warm)")
    ap.add_argument("--chunks-per-span", type=int, default=0)
    ap.add_argument("--engine", type=int, default=0)
    ap.add_argument("--pass", dest="which", default="fwd", choices=["fwd", "bwd", "train", "fused", "bidir", "4dir", "srem", "gates", "fusedgates", "bwdgates"],
                    help="fwd: the forward hot path (the headline); bwd: gla_bwd on the same workload; "
                         "train: gla_fwd_ex followed by gla_bwd_reuse; "
                         "fused: gla_fwd_fused (gate prologue, Swish/LayerNorm epilogue) on the same workload; "
                         "bidir / 4dir: gla_fwd_multi over scan orders (0, 1) / (0, 1, 2, 3); "
                         "srem: gla_srem_dwconv on the workload's token matrix; "
                         "gates: gla_fwd_gates (two-sided gate) on the same workload plus a log_beta tensor; "
                         "fusedgates: gla_fwd_fused_gates (both gates from pre-activations, Swish/LayerNorm epilogue); "
                         "bwdgates: gla_bwd_gates (backward of the two-sided-gate recurrence)")
    ap.add_argument("--layout", default="bhtd", choices=["bhtd", "bthd"],
                    help="memory order of q, k, v, log_alpha, out: [B,H,T,d] (the headline) or [B,T,H,d]")
    ap.add_argument("--reuse-fwd", action="store_true",
                    help="with --pass bwd: take the span states of S from the forward call's workspace (gla_bwd_reuse); "
                         "with --pass bwdgates: hand the forward outputs to gla_bwd_gates")
    ap.add_argument("--no-range-fallback", action="store_true",
                    help="skip the launch that recomputes spans outside the fp16 engine's range (none in these workloads)")
    ap.add_argument("--no-epilogue", action="store_true",
                    help="with --pass fused: gate prologue only (plain o is stored)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-table", action="store_true",
                    help="skip the `configs` table (the other contract workloads, timed and checked after the headline)")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--no-cache-resident", action="store_true",
                    help="skip the extra timed loop on one buffer set (keeps a profile of this command to HBM-streaming calls)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy 10 times (a known-size reference for rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters); not part of the timed region")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (no collectives or sharding exist here)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2405_18428_amd as gla
    from paper_2405_18428_amd import inputs as gi

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    gla.load_library()  # raises if the HIP library is not built; there is no fallback
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, args.chunks_per_span)
    gla.gla_set_option(gla.OPT_ENGINE, args.engine)
    gla.gla_set_option(gla.OPT_RANGE_FALLBACK, 0 if args.no_range_fallback else 1)

    cfg = gi.CONFIGS[args.config]
    dev = torch.device("cuda:0")
    d = gi.make_config_inputs(cfg)
    if args.which in ("bwd", "train"):
        bench_backward(args, cfg, d, gla, gi, torch, np)
        return
    if args.which == "fused":
        bench_fused(args, cfg, gla, gi, torch, np)
        return
    if args.which == "bwdgates":
        bench_bwd_gates(args, cfg, gla, gi, torch, np)
        return
    if args.which in ("gates", "fusedgates"):
        bench_gates(args, cfg, gla, gi, torch, np)
        return
    if args.which == "srem":
        bench_srem(args, cfg, gla, gi, torch, np)
        return
    if args.which in ("bidir", "4dir"):
        bench_multi(args, cfg, d, gla, gi, torch, np, (0, 1) if args.which == "bidir" else (0, 1, 2, 3))
        return
    B, H, T, dk, dv = cfg.B, cfg.H, cfg.T, cfg.dk, cfg.dv
    if cfg.dtype == "bf16":
        host = [torch.from_numpy(d[n + "_bits"].view(np.int16)).view(torch.bfloat16) for n in ("q", "k", "v")]
    else:
        host = [torch.from_numpy(d[n]) for n in ("q", "k", "v")]
    host.append(torch.from_numpy(d["log_alpha"]))
    bthd = args.layout == "bthd"
    if bthd:
        host = [t.permute(0, 2, 1, 3).contiguous() for t in host]
    out_dt = torch.float32 if args.out_dtype == "f32" else torch.bfloat16
    qdt = gla.DT_BF16 if cfg.dtype == "bf16" else gla.DT_F32
    ws_bytes = gla.gla_fwd_workspace_bytes(B, H, T, dk, dv, qdt)

    sets = []
    for _ in range(max(1, args.sets)):
        q, k, v, la = (t.to(dev) for t in host)
        sets.append(dict(q=q, k=k, v=v, la=la,
                         out=torch.empty((B, T, H, dv) if bthd else (B, H, T, dv), dtype=out_dt, device=dev),
                         fin=torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev),
                         ws=torch.empty((ws_bytes,), dtype=torch.uint8, device=dev)))

    def step(i):
        s = sets[i % len(sets)]
        if bthd:
            gla.gla_fwd_layout(s["q"], s["k"], s["v"], s["la"], cfg.grid_h, cfg.grid_w, args.scan,
                               layout=gla.LAYOUT_BTHD, out=s["out"], final_state=s["fin"], workspace=s["ws"])
        else:
            gla.gla_fwd_ex(s["q"], s["k"], s["v"], s["la"], cfg.grid_h, cfg.grid_w, args.scan,
                           out=s["out"], final_state=s["fin"], workspace=s["ws"])

    # a plain 256 MiB device copy: the known-size reference of the rocprofv3 HBM counters (--copy-calibration keeps
    # it in the profiled run) and, timed, the bandwidth a streaming kernel reaches on this machine (read + write bytes)
    src = torch.empty((256 << 20,), dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(10 if args.copy_calibration else 3):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * (256 << 20) / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = B * T / (ms_per_step * 1e-3)

    # the same call on one buffer set only (inputs resident in the last-level cache): context, never `value`
    warm_ms = None
    if not args.no_cache_resident:
        for i in range(10):
            step(0)
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        for i in range(args.steps):
            step(0)
        torch.cuda.synchronize()
        warm_ms = (time.perf_counter() - w0) * 1e3 / args.steps

    # per-kernel durations with HIP events on the launch stream, rotating over the same sets
    phase = np.zeros(4)
    reps = 0
    for r in range(0 if bthd else 8):  # (the timing aid covers the headline memory order only)
        for s in sets:
            ms = gla.gla_fwd_timed(s["q"], s["k"], s["v"], s["la"], cfg.grid_h, cfg.grid_w, args.scan,
                                   s["out"], s["fin"], s["ws"], iters=1)
            if r >= 2:
                phase += np.array(ms)
                reps += 1
    phase /= max(reps, 1)
    names = ["span_state", "carry", "output"]
    if bthd:
        phase[:] = [0.0, 0.0, ms_per_step, ms_per_step]
        names = ["span_state", "carry", "whole_call"]
    dom = int(np.argmax(phase[:3]))
    qb = 2 if cfg.dtype == "bf16" else 4
    ob = 4 if args.out_dtype == "f32" else 2
    alg_bytes = algorithmic_bytes_per_token_head(dk, dv, qb, ob) * B * H * T
    alg_flops = algorithmic_flops_per_token_head(dk, dv) * B * H * T
    # `achieved` / `frac` price the WHOLE call (every kernel of the path) on the algorithmic bytes; the dominant
    # kernel by itself (the same bytes over its own duration: it reads every input and writes every output once)
    # is reported beside it as kernel_achieved / kernel_frac
    achieved = alg_bytes / (ms_per_step * 1e-3) / 1e9
    kernel_achieved = alg_bytes / (phase[dom] * 1e-3) / 1e9
    traffic = measured_traffic(cfg.name, names[dom], args)
    parts_traffic = [measured_traffic(cfg.name, n, args) for n in ("span_state", "output")]
    call_traffic = None if (traffic is None or None in parts_traffic) else int(sum(parts_traffic))
    roofline = {
        "bound": "hbm", "kernel": names[dom], "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": traffic,
        "traffic_source": None if traffic is None else f"profiles/gla_fwd_{cfg.name}_hbm_traffic.md (rocprofv3 "
                                                       f"FETCH_SIZE / WRITE_SIZE of this command, committed; not re-measured here)",
        "algorithmic_bytes": alg_bytes, "kernel_ms": round(float(phase[dom]), 5),
        "kernel_achieved": round(kernel_achieved, 1), "kernel_frac": round(kernel_achieved / HBM_PEAK_GBS, 4),
        "phase_ms": {n: round(float(x), 5) for n, x in zip(names + ["whole_call"], phase)},
        "whole_path_frac": round(achieved / HBM_PEAK_GBS, 4),
        "measured_copy_gbs": round(copy_gbs, 1),
        "frac_of_measured_copy": round(achieved / copy_gbs, 4),
        # every kernel of the call: the HBM bytes the committed counter runs measured, moved in ms_per_step
        "call_traffic": call_traffic,
        "call_traffic_gbs": None if call_traffic is None else round(call_traffic / (ms_per_step * 1e-3) / 1e9, 1),
        "call_traffic_frac_of_copy": None if call_traffic is None
        else round(call_traffic / (ms_per_step * 1e-3) / 1e9 / copy_gbs, 4),
        "mfma_tflops": round(alg_flops / (ms_per_step * 1e-3) / 1e12, 2),
        "mfma_frac": round(alg_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 5),
        "mfma_peak_nominal_tflops": MFMA_BF16_PEAK_TFLOPS,
        "mfma_peak_measured_tflops": round(gla.gla_calibrate_mfma(), 1),
    }

    result = {
        "metric": "GLA fwd tokens/s at DiG-XL/2 shape T=16384; % bf16 MFMA roofline",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={B} H={H} T={T} ({cfg.grid_h}x{cfg.grid_w}) dk={dk} dv={dv} "
                               f"{cfg.dtype} q/k/v, fp32 log_alpha, {args.out_dtype} out, scan={args.scan}, layout={args.layout}",
                   "buffer_sets": len(sets), "token_heads_per_s": round(B * H * T / (ms_per_step * 1e-3), 1),
                   "cache_resident_ms_per_step": None if warm_ms is None else round(warm_ms, 5),
                   "engine": gla.gla_get_option(gla.OPT_ENGINE),
                   "chunks_per_span": gla.gla_get_option(gla.OPT_CHUNKS_PER_SPAN)},
        "roofline": roofline,
    }

    if not args.no_check or not args.no_cpu_baseline:
        from oracle import gla_oracle
        q64, k64, v64, g64 = (np.asarray(d[n], dtype=np.float64) for n in ("q", "k", "v", "log_alpha"))
        best = None
        runs = 1 if args.no_cpu_baseline else 3
        for _ in range(runs):
            c0 = time.perf_counter()
            ref, ref_fin = gla_oracle.gla_fwd(q64, k64, v64, g64, cfg.grid_h, cfg.grid_w, args.scan)
            c1 = time.perf_counter()
            best = c1 - c0 if best is None else min(best, c1 - c0)
        if not args.no_cpu_baseline:
            c0 = time.perf_counter()
            gla_oracle.gla_fwd(q64, k64, v64, g64, cfg.grid_h, cfg.grid_w, args.scan, nthreads=1)
            single = time.perf_counter() - c0
            result["cpu_baseline"] = {
                "value": round(B * T / best, 1), "unit": "tokens/s",
                "cores": min(gla_oracle.threads(), B * H), "kind": "oracle",
                "single_thread_value": round(B * T / single, 1),
                "sample": f"the whole workload ({B * H} sequences of {T} tokens), best of {runs} runs, "
                          f"fp64 token-by-token C loop, OpenMP over batch*head",
            }
        if not args.no_check:
            s = sets[0]
            step(0)
            torch.cuda.synchronize()
            rms = float(np.sqrt(np.mean(ref ** 2)))
            got = s["out"].float().cpu()
            got = got.permute(0, 2, 1, 3) if bthd else got
            err = float(np.abs(got.numpy() - ref).max() / rms)
            result["max_err_over_rms"] = round(err, 6)

    if not args.no_table and args.which == "fwd" and args.config == "dig_xl2_2048" and not bthd:
        for s_ in sets:
            s_.clear()
        sets.clear()
        torch.cuda.empty_cache()
        table = []
        for name, scan in TABLE:
            if name == cfg.name and scan == args.scan and args.out_dtype == "f32":
                row = {"workload": name, "scan": scan, "ms_per_step": round(ms_per_step, 5),
                       "tokens_per_s": round(tokens_per_s, 1), "algorithmic_bytes": alg_bytes,
                       "whole_path_frac": roofline["whole_path_frac"]}
                if "max_err_over_rms" in result:
                    row["max_err_over_rms"] = result["max_err_over_rms"]
            else:
                row = time_forward(name, scan, gla, gi, torch, np, check=not args.no_check)
            table.append(row)
        result["configs"] = table

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
