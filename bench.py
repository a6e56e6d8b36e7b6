"""Benchmark of the EntropyCache denoising step on one MI355X.

A "step" is one denoising step of the whole hot path (forward in FULL or PARTIAL mode, LM head
with the fused vocabulary reduction, decision).  The workload is the synthetic LLaDA-8B-shaped
model (32 layers, prompt 512 + 256 generated tokens, block 32, one token per step, k = 2,
tau = 1.0); its logit scale is calibrated beforehand so that the fraction of FULL steps of a
free-running generation is near the paper's recompute ratio.  Inputs are resident in HBM before
any timing starts.

The timed region runs exactly --steps consecutive free-running (EC_AUTO) steps of that
generation.  The generation is deterministic, so its sequence of modes is known from an earlier
pass: the window starts at the step from which --steps steps hold the same share of FULL steps
as the whole generation does (a window at the very start would hold hardly any), and the steps
before it run untimed.  A complete generation is timed beside it (`whole_generation`).

Prints ONE JSON line: whole-job generated tokens/s, per-mode step rates, the roofline of the
dominant kernel (HIP events recorded on the library's stream), the same step measurements for
the other workloads (Dream-7B shape, long chain-of-thought shape, 16 sequences, and the LLaDA-8B
shape with e4m3-coded matrices), and the CPU oracle timed on a bounded sample of the same workload.
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


def algorithmic_bytes(cfg, T, rows):
    """HBM bytes one PARTIAL step of one sequence must move: every matrix once, the KV cache read
    once per layer, the new K/V rows written.  Activations are left out (< 0.1 %)."""
    import ec_inputs
    es = 4 if cfg.dtype == "f32" else 2
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
    """Algorithmic bytes of one gate/up launch: both matrices once, the rows' operand in, the
    rows' SwiGLU output out (bf16)."""
    es = 4 if cfg.dtype == "f32" else 2
    ws = {"f32": 4, "bf16": 2, "fp8w": 1}[cfg.dtype]
    return 2 * cfg.d_ffn * cfg.d_model * ws + rows * cfg.d_model * es + rows * cfg.d_ffn * es


def run_generation(g, prompt, mode_fn=None, max_steps=None, first_untimed=0):
    """Runs steps until done (or max_steps).  The first `first_untimed` steps run before the
    clock starts (synchronised on both sides).  Returns (modes of all steps, tokens of the timed
    steps, seconds of the timed steps)."""
    import torch
    import paper_2603_18489_amd as ec
    g.reset(prompt)
    modes = []
    toks = 0
    rows = 0
    t0 = None
    while True:
        if len(modes) == first_untimed:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        mode = ec.EC_AUTO if mode_fn is None else mode_fn(len(modes))
        r = g.step(mode)
        modes.append(r["mode_run"])
        rows += r["n_query_rows"]
        if len(modes) > first_untimed:
            toks += r["n_unmasked"]
        if r["done"] or (max_steps is not None and len(modes) >= max_steps):
            break
    torch.cuda.synchronize()
    run_generation.last_rows = rows          # rows recomputed over all steps of this run
    return modes, toks, time.perf_counter() - (t0 if t0 is not None else time.perf_counter())


def calibrate_logit_scale(make_ctx, prompt, target_lo=0.08, target_hi=0.16):
    """Bisection on the LM-head output scale until the FULL-step fraction of a free-running
    generation lies in [target_lo, target_hi] (the paper's recompute ratios imply ~0.11)."""
    lo, hi = 1.0, 64.0
    best = None
    for it in range(12):
        mid = (lo * hi) ** 0.5
        g = make_ctx(mid)
        modes, _, _ = run_generation(g, prompt)
        g.close()
        f = modes.count(0) / len(modes)
        log(f"[calibrate] logit_scale={mid:.3f}: FULL fraction {f:.3f} ({modes.count(0)}/{len(modes)})")
        if best is None or abs(f - 0.11) < abs(best[1] - 0.11):
            best = (mid, f)
        if target_lo <= f <= target_hi:
            return mid, f
        if f > target_hi:
            lo = mid          # too uncertain: sharpen the distribution
        else:
            hi = mid
    return best


def pick_window(modes, k):
    """First step of the k-step window of a generation whose share of FULL steps is closest to the
    whole generation's (earliest on ties).  k >= the generation's length: the whole generation."""
    n = len(modes)
    if k >= n:
        return 0
    full = [1 if m == 0 else 0 for m in modes]
    target = sum(full) / n * k
    best, best_d = 0, None
    cur = sum(full[:k])
    for s in range(0, n - k + 1):
        if s > 0:
            cur += full[s + k - 1] - full[s - 1]
        d = abs(cur - target)
        if best_d is None or d < best_d - 1e-12:
            best, best_d = s, d
    return best


def step_times_forced(g, prompts, B, n_partial=24, n_full=3):
    """Whole-step wall times under forced schedules: (ms per FULL step, ms per PARTIAL step in the
    steady state that follows a FULL step)."""
    import torch
    import paper_2603_18489_amd as ec

    def run(mode_fn, n):
        g.reset(prompts)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            g.step(mode_fn(i))
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    run(lambda i: ec.EC_FULL, 1)                                      # warm-up
    full_ms = run(lambda i: ec.EC_FULL, n_full) / n_full * 1e3
    t = run(lambda i: ec.EC_FULL if i == 0 else ec.EC_PARTIAL, n_partial + 1) * 1e3
    return full_ms, (t - full_ms) / n_partial


def measure_other_workload(name, dw_by_model, threads):
    """Forced-schedule step times of another workload of the configuration list, at logit scale 8
    (uncalibrated: the schedule is forced, so the scale changes nothing measured here)."""
    import ec_inputs
    import paper_2603_18489_amd as ec
    wl = ec_inputs.WORKLOADS[name]
    cfg, dec = wl.model.replace(logit_scale=8.0), wl.decode
    key = (cfg.n_layers, cfg.d_model, cfg.vocab, wl.seed, cfg.dtype)
    if key not in dw_by_model:
        t0 = time.perf_counter()
        dw_by_model[key] = ec.weights_to_device(cfg, ec_inputs.make_weights(cfg, wl.seed, threads=threads))
        log(f"[bench] {name}: weights generated and uploaded in {time.perf_counter() - t0:.1f}s")
    B = dec.batch
    if B == 1:
        prompts = ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed)
    else:
        prompts = [ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed + 1000 + b) for b in range(B)]
    g = ec.EntropyCache(cfg, dw_by_model[key], dec, prompts)
    try:
        full_ms, partial_ms = step_times_forced(g, prompts, B, n_partial=24, n_full=2 if B > 1 else 3)
    finally:
        g.close()
    T = wl.prompt_len + dec.gen_len
    rows = dec.block + dec.k_recent * max(1, dec.tokens_per_step)     # most rows of a partial step
    step_bytes = ec_inputs.weight_bytes(cfg) + B * (algorithmic_bytes(cfg, T, rows) - ec_inputs.weight_bytes(cfg))
    flops = B * full_step_flops(cfg, T, dec.block)
    out = {"workload": f"{name}: L{cfg.n_layers} d{cfg.d_model} {cfg.n_heads}q/{cfg.n_kv_heads}kv "
                       f"F{cfg.d_ffn} V{cfg.vocab}, {B} x (prompt {wl.prompt_len} + gen {dec.gen_len}), "
                       f"n={dec.tokens_per_step}, k={dec.k_recent}, tau={dec.tau}",
           "partial_step": {"ms": partial_ms, "algorithmic_GB": step_bytes / 1e9,
                            "hbm_frac": step_bytes / (partial_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "tok_per_s": B * dec.tokens_per_step / partial_ms * 1e3},
           "full_step": {"ms": full_ms, "flops": flops,
                         "mfma_frac": flops / (full_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}}
    if B > 1:
        # the all-partial step of a batch sits at the ridge: its GEMMs run B x 34 rows
        pflops = 2.0 * B * rows * (ec_inputs.weight_bytes(cfg) / 2)
        out["partial_step"]["mfma_frac"] = pflops / (partial_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS
    log(f"[bench] {name}: partial {partial_ms:.2f} ms, full {full_ms:.2f} ms")
    return out


def blas_threads():
    """Threads numpy's BLAS runs its matmul on (the oracle's only parallel step)."""
    try:
        from threadpoolctl import threadpool_info
        n = [p["num_threads"] for p in threadpool_info() if p.get("user_api") == "blas"]
        if n:
            return max(n)
    except Exception:
        pass
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count()))


def cpu_oracle_baseline(cfg, w, dec, prompt, n_full, n_partial, n_tok):
    """Times the fp64 numpy oracle (oracle/entropycache.py, BLAS matmul as its contraction
    primitive) on 2- and 6-layer prefixes of the model (one FULL and two PARTIAL steps each) and
    extrapolates linearly in depth to the full model and the GPU run's mode schedule."""
    from oracle import entropycache as eco
    times = {}
    for L in (2, 6):
        sub = {k: (v[:L] if isinstance(v, list) else v) for k, v in w.items()}
        st = eco.eco_init(eco.OracleModel(cfg.replace(n_layers=L), sub), dec, prompt)
        t0 = time.perf_counter()
        eco.eco_step(st, eco.FULL, keep_logits=False)
        tf = time.perf_counter() - t0
        t0 = time.perf_counter()
        eco.eco_step(st, eco.PARTIAL, keep_logits=False)
        eco.eco_step(st, eco.PARTIAL, keep_logits=False)
        tp = (time.perf_counter() - t0) / 2
        times[L] = (tf, tp)
        log(f"[cpu oracle] L={L}: FULL {tf:.2f}s PARTIAL {tp:.2f}s")
    per_f = (times[6][0] - times[2][0]) / 4
    per_p = (times[6][1] - times[2][1]) / 4
    tf = times[2][0] + (cfg.n_layers - 2) * per_f
    tp = times[2][1] + (cfg.n_layers - 2) * per_p
    total = n_full * tf + n_partial * tp
    return {"value": n_tok / total, "unit": "tok/s", "cores": blas_threads(), "kind": "oracle",
            "sample": f"1 FULL + 2 PARTIAL fp64 steps on 2- and 6-layer prefixes of the model "
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
    ap.add_argument("--no-other-workloads", action="store_true")
    ap.add_argument("--threads", type=int, default=16)
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="run one plain device copy of this size first (a known-size dispatch "
                         "that scales rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no collectives, no sharding); "
            "run with --gpus 1")
        sys.exit(2)

    import torch
    import ec_inputs
    import paper_2603_18489_amd as ec

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    wl = ec_inputs.WORKLOADS[args.workload]
    cfg, dec = wl.model, wl.decode
    assert dec.batch == 1, "the headline run is a single sequence; batches are measured as other workloads"
    T = wl.prompt_len + dec.gen_len
    t0 = time.perf_counter()
    w = ec_inputs.make_weights(cfg, wl.seed, threads=args.threads)
    prompt = ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed)
    log(f"[bench] weights generated in {time.perf_counter() - t0:.1f}s")
    t0 = time.perf_counter()
    dw = ec.weights_to_device(cfg, w)
    torch.cuda.synchronize()
    log(f"[bench] weights uploaded in {time.perf_counter() - t0:.1f}s")
    dw_by_model = {(cfg.n_layers, cfg.d_model, cfg.vocab, wl.seed, cfg.dtype): dw}

    if args.calib_copy_mb > 0:
        src = torch.ones(args.calib_copy_mb << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def make_ctx(scale):
        return ec.EntropyCache(cfg.replace(logit_scale=scale), dw, dec, prompt)

    if args.logit_scale > 0:
        scale = args.logit_scale
    else:
        scale, _ = calibrate_logit_scale(make_ctx, prompt)
    g = make_ctx(scale)

    # ---- one complete generation: its modes (deterministic) and its time ------------------------
    run_generation(g, prompt)                                           # warm-up
    gen_modes, gen_toks, gen_secs = run_generation(g, prompt)
    gen_steps, gen_full = len(gen_modes), gen_modes.count(ec.EC_FULL)
    whole = {"steps": gen_steps, "full_steps": gen_full, "full_fraction": gen_full / gen_steps,
             "ms_per_step": gen_secs / gen_steps * 1e3, "tok_s": gen_toks / gen_secs,
             "tokens": gen_toks,
             # fraction of KV states recomputed per step (the paper's recompute ratio)
             "recompute_ratio": run_generation.last_rows / (gen_steps * (len(prompt) + dec.gen_len))}

    # ---- timed region: exactly K consecutive free-running steps ---------------------------------
    K = args.steps
    s0 = pick_window(gen_modes, K)
    run_generation(g, prompt, max_steps=max(1, args.warmup))            # W untimed warm-up steps
    steps = full = toks = 0
    secs = 0.0
    while steps < K:                                                    # (K beyond one generation: restart)
        first = s0 if steps == 0 else 0
        modes, tk, dt = run_generation(g, prompt, max_steps=first + (K - steps), first_untimed=first)
        timed = modes[first:]
        steps += len(timed); full += timed.count(ec.EC_FULL); toks += tk; secs += dt
    partial = steps - full

    # ---- per-mode step rates (forced schedules) ------------------------------------------------
    n_probe = min(64, dec.gen_len)
    m_p, _, t_p = run_generation(g, prompt, mode_fn=lambda i: ec.EC_FULL if i == 0 else ec.EC_PARTIAL,
                                 max_steps=n_probe)
    m_f, _, t_f = run_generation(g, prompt, mode_fn=lambda i: ec.EC_FULL, max_steps=8)
    full_ms = t_f / len(m_f) * 1e3
    partial_ms = (t_p * 1e3 - full_ms) / (len(m_p) - 1)

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
                "launch_ms": gu_launch_ms, "bytes_per_launch": gu_bytes,
                "timing": "HIP events around each launch on the library's stream (about 1.5 us "
                          "above the rocprofv3 kernel-trace duration of profiles/)"}
    gu_full_ms = pf["gateup"] / cfg.n_layers
    gu_flops = 2.0 * T * cfg.d_model * 2 * cfg.d_ffn
    ach_f = gu_flops / (gu_full_ms * 1e-3) / 1e12
    roofline_full = {"kernel": "gemm_bf16_tiled8 (gate/up projection, full step)", "bound": "mfma",
                     "achieved": ach_f, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": ach_f / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "launch_ms": gu_full_ms, "flops_per_launch": gu_flops,
                     "timing": roofline["timing"]}
    # HBM bytes per launch measured with rocprofv3 --pmc (committed summary of the same command)
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_llada8b.json")
    if args.workload == "llada8b" and os.path.exists(tpath):
        tj = json.load(open(tpath))
        for rf, key in ((roofline, "partial_gateup"), (roofline_full, "full_gateup")):
            rf["traffic"] = tj[key]["fetch_bytes"] + (tj[key]["write_bytes"] or 0.0)
            rf["traffic_source"] = "committed rocprofv3 --pmc summary profiles/gemm_kernels_llada8b_hbm_traffic.txt"
    step_bytes = algorithmic_bytes(cfg, T, rows_partial)
    step_flops = full_step_flops(cfg, T, dec.block)
    decision_ms = pp["vocab_reduce"] + pp["decide"]
    g.close()

    others = None
    if not args.no_other_workloads and args.workload == "llada8b":
        others = {}
        for name in ("llada8b_cot", "llada8b_b16", "dream7b", "llada8b_fp8"):
            try:
                others[name] = measure_other_workload(name, dw_by_model, args.threads)
            except Exception as e:  # keep the headline line even if a side measurement fails
                others[name] = {"error": repr(e)}
        dw_by_model.clear()

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_oracle_baseline(cfg, w, dec, prompt, full, partial, toks)

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
                   "schedule": f"free-running EC_AUTO, calibrated logit scale; the timed window is "
                               f"steps {s0 + 1}..{s0 + min(K, gen_steps)} of the generation, chosen so "
                               f"that its share of FULL steps matches the whole generation's",
                   "logit_scale": scale, "window_first_step": s0 + 1,
                   "full_fraction": full / steps, "full_steps": full, "partial_steps": partial},
        "steps_per_s": steps / secs,
        "whole_generation": whole,
        "partial_step": {"ms": partial_ms, "steps_per_s": 1e3 / partial_ms,
                         "algorithmic_GB": step_bytes / 1e9,
                         "hbm_GBs": step_bytes / (partial_ms * 1e-3) / 1e9,
                         "hbm_frac": step_bytes / (partial_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "decision_ms": decision_ms,
                         "decision_pct": 100.0 * decision_ms / sum(pp.values()),
                         "decision_note": "decide kernel alone: the vocabulary reduction runs inside "
                                          "the LM-head epilogue"},
        "full_step": {"ms": full_ms, "steps_per_s": 1e3 / full_ms, "flops": step_flops,
                      "tflops": step_flops / (full_ms * 1e-3) / 1e12,
                      "mfma_frac": step_flops / (full_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "kernel_ms_partial_step": pp, "kernel_ms_full_step": pf,
        "roofline": roofline, "roofline_full_step": roofline_full,
        "other_workloads": others,
        "cpu_baseline": cpu,
        "paper_context": "paper reports 15.2x-26.4x speedup over vanilla on RTX 3090 (trained "
                         "weights, other decoding settings): context, not a target",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
