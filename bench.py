"""Benchmark of the EntropyCache denoising step on one MI355X.

A "step" is one denoising step of the whole hot path (forward in FULL or PARTIAL mode, LM head,
vocabulary reduction, decision).  The timed region runs exactly --steps steps of free-running
generation (EC_AUTO) on the synthetic LLaDA-8B-shaped workload, whose logit scale was calibrated
beforehand so that the fraction of FULL steps is near the paper's recompute ratio; generations
restart (untimed reset) when they finish.  Inputs are resident in HBM before timing starts.

Prints ONE JSON line: whole-job generated tokens/s plus per-mode step rates, the roofline of the
dominant kernel (from HIP events recorded on the library's stream), and the CPU oracle timed on
a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(cfg, T, rows, n_mb):
    """HBM bytes one PARTIAL step must move: every matrix once, the KV cache read once per layer,
    the new K/V rows written.  Activations are left out (< 0.1 %)."""
    import ec_inputs
    es = 2 if cfg.dtype == "bf16" else 4
    kv = cfg.n_layers * 2 * T * cfg.n_kv_heads * cfg.head_dim * es
    kv_w = cfg.n_layers * 2 * rows * cfg.n_kv_heads * cfg.head_dim * es
    return ec_inputs.weight_bytes(cfg) + kv + kv_w


def full_step_flops(cfg, T, n_mb):
    d, f, hq, hkv, hd = cfg.d_model, cfg.d_ffn, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    per_layer = (hq + 2 * hkv) * hd * d + d * hq * hd + 3 * f * d
    gemm = 2.0 * cfg.n_layers * per_layer * T
    attn = 4.0 * T * T * hq * hd * cfg.n_layers
    lm = 2.0 * n_mb * cfg.vocab * d
    return gemm + attn + lm


def gateup_bytes(cfg, rows):
    es = 2 if cfg.dtype == "bf16" else 4
    return 2 * cfg.d_ffn * cfg.d_model * es + rows * cfg.d_model * es + rows * 2 * cfg.d_ffn * 4


def run_generation(g, prompt, mode_fn=None, max_steps=None, timed=False):
    """Runs steps until done (or max_steps); returns (steps, full, tokens, seconds)."""
    import torch
    import paper_2603_18489_amd as ec
    g.reset(prompt)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    steps = full = toks = 0
    while True:
        mode = ec.EC_AUTO if mode_fn is None else mode_fn(steps)
        r = g.step(mode)
        steps += 1
        full += int(r["mode_run"] == ec.EC_FULL)
        toks += r["n_unmasked"]
        if r["done"] or (max_steps is not None and steps >= max_steps):
            break
    torch.cuda.synchronize()
    return steps, full, toks, time.perf_counter() - t0


def calibrate_logit_scale(make_ctx, prompt, target_lo=0.08, target_hi=0.16):
    """Bisection on the LM-head output scale until the FULL-step fraction of a free-running
    generation lies in [target_lo, target_hi] (the paper's recompute ratios imply ~0.11)."""
    lo, hi = 1.0, 64.0
    best = None
    for it in range(12):
        mid = (lo * hi) ** 0.5
        g = make_ctx(mid)
        steps, full, _, _ = run_generation(g, prompt)
        g.close()
        f = full / steps
        log(f"[calibrate] logit_scale={mid:.3f}: FULL fraction {f:.3f} ({full}/{steps})")
        if best is None or abs(f - 0.11) < abs(best[1] - 0.11):
            best = (mid, f)
        if target_lo <= f <= target_hi:
            return mid, f
        if f > target_hi:
            lo = mid          # too uncertain: sharpen the distribution
        else:
            hi = mid
    return best


def bench_batch(args, wl, cfg, dec, dw):
    """Many sequences side by side (decode.batch > 1), every prompt prompt_len ids long (their
    modes still differ from step to step).
    Timed: K free-running steps of the whole batch; then the all-PARTIAL steady state and the
    all-FULL step, forced.  One JSON line like the single-sequence run's, without the CPU leg."""
    import torch
    import ec_inputs
    import paper_2603_18489_amd as ec
    B = dec.batch
    plens = [wl.prompt_len] * B
    prompts = [ec_inputs.make_prompt(cfg.vocab, P, wl.seed + 1000 + b) for b, P in enumerate(plens)]
    scale = args.logit_scale if args.logit_scale > 0 else 8.0
    g = ec.EntropyCache(cfg.replace(logit_scale=scale), dw, dec, prompts)

    def steps_timed(mode_fn, n, reset=True):
        if reset:
            g.reset(prompts)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        toks = full = part = 0
        for i in range(n):
            rs = g.step(mode_fn(i))
            for r in rs:
                if r["n_query_rows"] > 0:
                    toks += r["n_unmasked"]
                    full += int(r["mode_run"] == ec.EC_FULL)
                    part += int(r["mode_run"] == ec.EC_PARTIAL)
            if all(r["done"] for r in rs):
                break
        torch.cuda.synchronize()
        return i + 1, toks, full, part, time.perf_counter() - t0

    steps_timed(lambda i: ec.EC_AUTO, args.warmup)
    steps, toks, full, part, secs = steps_timed(lambda i: ec.EC_AUTO, args.steps)
    _, _, _, _, t_f = steps_timed(lambda i: ec.EC_FULL, 3)
    n_p, tok_p, _, _, t_p = steps_timed(lambda i: ec.EC_FULL if i == 0 else ec.EC_PARTIAL, 25)
    full_ms = t_f / 3 * 1e3
    partial_ms = (t_p - full_ms / 1e3) / (n_p - 1) * 1e3
    g.reset(prompts)
    g.step(ec.EC_FULL)
    g.profile_enable(True)
    for _ in range(8):
        g.step(ec.EC_PARTIAL)
    prof = g.profile_read()
    g.profile_enable(False)
    pp = {k: v / prof["steps"] for k, v in prof["ms"].items()}
    R = sum((34 + 15) // 16 * 16 for _ in range(B))             # rows of the partial step's list
    gu_ms = pp["gateup"] / cfg.n_layers
    gu_flops = 2.0 * R * cfg.d_model * 2 * cfg.d_ffn
    ach = gu_flops / (gu_ms * 1e-3) / 1e12
    T_tot = sum(P + dec.gen_len for P in plens)
    kv_bytes = 2.0 * T_tot * cfg.n_kv_heads * cfg.head_dim * 2 * cfg.n_layers
    step_bytes = ec_inputs.weight_bytes(cfg) + kv_bytes          # weights once + every cache once
    g.close()
    out = {
        "metric": "generated tokens per second, EntropyCache denoising, 16 sequences (LLaDA-8B shape)",
        "value": toks / secs, "unit": "tok/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": secs / steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: L{cfg.n_layers} d{cfg.d_model} {cfg.n_heads}q/"
                               f"{cfg.n_kv_heads}kv x{cfg.head_dim} F{cfg.d_ffn} V{cfg.vocab}, "
                               f"{B} sequences, prompt {plens[0]} each, gen {dec.gen_len}, "
                               f"block {dec.block}, n={dec.tokens_per_step}, k={dec.k_recent}, "
                               f"tau={dec.tau}",
                   "schedule": "free-running EC_AUTO", "logit_scale": scale,
                   "sequence_steps_full": full, "sequence_steps_partial": part},
        "all_partial_step": {"ms": partial_ms, "tok_per_s": B * dec.tokens_per_step / partial_ms * 1e3,
                             "list_rows": R, "algorithmic_GB": step_bytes / 1e9,
                             "hbm_frac": step_bytes / (partial_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "all_full_step": {"ms": full_ms, "rows": T_tot,
                          "tflops": sum(full_step_flops(cfg, P + dec.gen_len, dec.block)
                                        for P in plens) / (full_ms * 1e-3) / 1e12},
        "kernel_ms_partial_step": pp,
        "roofline": {"kernel": "tiled GEMM (gate/up projection, all-partial step of the batch)",
                     "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "launch_ms": gu_ms, "flops_per_launch": gu_flops},
        "cpu_baseline": None,
    }
    print(json.dumps(out))


def cpu_oracle_baseline(cfg, w, dec, prompt, n_full, n_partial, n_tok):
    """Times the fp64 oracle on 2- and 4-layer prefixes of the model (one FULL and one PARTIAL
    step each) and extrapolates linearly in depth to the full model and the same mode schedule."""
    import numpy as np
    from oracle import entropycache as eco
    times = {}
    for L in (2, 4):
        sub = {k: (v[:L] if isinstance(v, list) else v) for k, v in w.items()}
        st = eco.eco_init(eco.OracleModel(cfg.replace(n_layers=L), sub), dec, prompt)
        t0 = time.perf_counter()
        eco.eco_step(st, eco.FULL, keep_logits=False)
        tf = time.perf_counter() - t0
        t0 = time.perf_counter()
        eco.eco_step(st, eco.PARTIAL, keep_logits=False)
        tp = time.perf_counter() - t0
        times[L] = (tf, tp)
        log(f"[cpu oracle] L={L}: FULL {tf:.2f}s PARTIAL {tp:.2f}s")
    per_f = (times[4][0] - times[2][0]) / 2
    per_p = (times[4][1] - times[2][1]) / 2
    tf = times[2][0] + (cfg.n_layers - 2) * per_f
    tp = times[2][1] + (cfg.n_layers - 2) * per_p
    total = n_full * tf + n_partial * tp
    return {"value": n_tok / total, "unit": "tok/s", "cores": os.cpu_count(), "kind": "oracle",
            "sample": f"1 FULL + 1 PARTIAL fp64 step on 2- and 4-layer prefixes of the model "
                      f"(same widths, vocabulary, prompt), extrapolated linearly to "
                      f"{cfg.n_layers} layers and the GPU run's schedule of {n_full} FULL + "
                      f"{n_partial} PARTIAL steps",
            "full_step_s": tf, "partial_step_s": tp}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="llada8b")
    ap.add_argument("--logit-scale", type=float, default=0.0, help="skip calibration")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--threads", type=int, default=16)
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="run one plain device copy of this size first (a known-size dispatch "
                         "that scales rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no collectives, no sharding); "
            "run with --gpus 1")
        sys.exit(2)

    import numpy as np
    import torch
    import ec_inputs
    import paper_2603_18489_amd as ec

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    wl = ec_inputs.WORKLOADS[args.workload]
    cfg, dec = wl.model, wl.decode
    T = wl.prompt_len + dec.gen_len
    t0 = time.perf_counter()
    w = ec_inputs.make_weights(cfg, wl.seed, threads=args.threads)
    prompt = ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed)
    log(f"[bench] weights generated in {time.perf_counter() - t0:.1f}s")
    t0 = time.perf_counter()
    dw = ec.weights_to_device(cfg, w)
    torch.cuda.synchronize()
    log(f"[bench] weights uploaded in {time.perf_counter() - t0:.1f}s")

    if dec.batch > 1:
        del w
        return bench_batch(args, wl, cfg, dec, dw)

    if args.calib_copy_mb > 0:
        src = torch.ones(args.calib_copy_mb << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def make_ctx(scale):
        return ec.EntropyCache(cfg.replace(logit_scale=scale), dw, dec, prompt)

    if args.logit_scale > 0:
        scale, f_cal = args.logit_scale, None
    else:
        scale, f_cal = calibrate_logit_scale(make_ctx, prompt)
    g = make_ctx(scale)

    # ---- timed region: exactly K free-running steps (generations restart untimed) -------------
    def run_k_steps(k):
        done_steps = full = toks = 0
        secs = 0.0
        while done_steps < k:
            s, f, tk, dt = run_generation(g, prompt, max_steps=k - done_steps)
            done_steps += s; full += f; toks += tk; secs += dt
        return done_steps, full, toks, secs

    run_k_steps(args.warmup)
    steps, full, toks, secs = run_k_steps(args.steps)
    partial = steps - full

    # ---- per-mode step rates (forced schedules) ------------------------------------------------
    n_probe = min(64, dec.gen_len)
    s_p, f_p, _, t_p = run_generation(g, prompt, mode_fn=lambda i: ec.EC_FULL if i == 0 else ec.EC_PARTIAL,
                                      max_steps=n_probe)
    # first step is FULL: time it separately below and subtract
    s_f, _, _, t_f = run_generation(g, prompt, mode_fn=lambda i: ec.EC_FULL, max_steps=8)
    full_ms = t_f / s_f * 1e3
    partial_ms = (t_p - full_ms / 1e3) / (s_p - 1) * 1e3

    # ---- kernel-level timing with HIP events on the library's stream ---------------------------
    g.profile_enable(True)
    run_generation(g, prompt, mode_fn=lambda i: ec.EC_FULL if i == 0 else ec.EC_PARTIAL, max_steps=33)
    prof_mixed = g.profile_read()
    g.profile_enable(True)
    run_generation(g, prompt, mode_fn=lambda i: ec.EC_FULL, max_steps=4)
    prof_full = g.profile_read()
    g.profile_enable(False)
    # partial-only numbers: subtract one FULL step's share
    pf = {k: prof_full["ms"][k] / prof_full["steps"] for k in prof_full["ms"]}
    pp = {k: (prof_mixed["ms"][k] - pf[k]) / (prof_mixed["steps"] - 1) for k in pf}
    rows_partial = dec.block + dec.k_recent
    gu_launch_ms = pp["gateup"] / cfg.n_layers
    gu_bytes = gateup_bytes(cfg, rows_partial)
    achieved = gu_bytes / (gu_launch_ms * 1e-3) / 1e9
    roofline = {"kernel": "gemm_bf16_skinny (gate/up projection, partial step)", "bound": "hbm",
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                "launch_ms": gu_launch_ms, "bytes_per_launch": gu_bytes}
    gu_full_ms = pf["gateup"] / cfg.n_layers
    gu_flops = 2.0 * T * cfg.d_model * 2 * cfg.d_ffn
    ach_f = gu_flops / (gu_full_ms * 1e-3) / 1e12
    roofline_full = {"kernel": "gemm_bf16_tiled8 (gate/up projection, full step)", "bound": "mfma",
                     "achieved": ach_f, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": ach_f / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "launch_ms": gu_full_ms, "flops_per_launch": gu_flops}
    # HBM bytes per launch measured with rocprofv3 --pmc (committed summary of the same command)
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_llada8b.json")
    if args.workload == "llada8b" and os.path.exists(tpath):
        tj = json.load(open(tpath))
        for rf, key in ((roofline, "partial_gateup"), (roofline_full, "full_gateup")):
            rf["traffic"] = tj[key]["fetch_bytes"] + (tj[key]["write_bytes"] or 0.0)
            rf["traffic_source"] = "profiles/gemm_kernels_llada8b_hbm_traffic.txt"
    step_bytes = algorithmic_bytes(cfg, T, rows_partial, dec.block)
    step_flops = full_step_flops(cfg, T, dec.block)
    decision_ms = pp["vocab_reduce"] + pp["decide"]

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_oracle_baseline(cfg, w, dec, prompt, full, partial, toks)
    g.close()

    out = {
        "metric": "generated tokens per second, EntropyCache denoising (LLaDA-8B shape)",
        "value": toks / secs, "unit": "tok/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": secs / steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: L{cfg.n_layers} d{cfg.d_model} "
                               f"{cfg.n_heads}q/{cfg.n_kv_heads}kv x{cfg.head_dim} F{cfg.d_ffn} "
                               f"V{cfg.vocab}, prompt {wl.prompt_len}, gen {dec.gen_len}, block "
                               f"{dec.block}, n={dec.tokens_per_step}, k={dec.k_recent}, "
                               f"tau={dec.tau}"
                               + (f", confidence threshold {dec.conf_threshold}" if dec.conf_threshold else "")
                               + (", sliding window" if dec.schedule else ""),
                   "schedule": "free-running EC_AUTO, calibrated logit scale",
                   "logit_scale": scale, "full_fraction": full / steps,
                   "full_steps": full, "partial_steps": partial},
        "steps_per_s": steps / secs,
        "partial_step": {"ms": partial_ms, "steps_per_s": 1e3 / partial_ms,
                         "algorithmic_GB": step_bytes / 1e9,
                         "hbm_GBs": step_bytes / (partial_ms * 1e-3) / 1e9,
                         "hbm_frac": step_bytes / (partial_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "decision_ms": decision_ms,
                         "decision_pct": 100.0 * decision_ms / sum(pp.values())},
        "full_step": {"ms": full_ms, "steps_per_s": 1e3 / full_ms, "flops": step_flops,
                      "tflops": step_flops / (full_ms * 1e-3) / 1e12,
                      "mfma_frac": step_flops / (full_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "kernel_ms_partial_step": pp, "kernel_ms_full_step": pf,
        "roofline": roofline, "roofline_full_step": roofline_full,
        "cpu_baseline": cpu,
        "paper_context": "paper reports 15.2x-26.4x speedup over vanilla on RTX 3090 (trained "
                         "weights, other decoding settings): context, not a target",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
