"""Writes the stored oracle traces under tests/golden/: sampled outputs of the fp64 oracle on the
full-size workloads, for short traces of denoising steps that the GPU parity tests replay
(same modes, same committed tokens) and compare sample by sample.  Calls only oracle/ and
ec_inputs/.

  python tests/golden/make_traces.py llada8b       32 layers, prompt 512 + 256 generated
  python tests/golden/make_traces.py dream7b       28 layers, GQA 28/4, 2 tokens per step, T = 1280
  python tests/golden/make_traces.py llada8b_cot   32 layers, prompt 256 + 1024 generated, k = 4
  python tests/golden/make_traces.py llada8b_b16   16 sequences of 1024 + 512 on the 2-layer twin,
                                                   free-running (sequences in different modes)

Each trace is <name>_trace.json (integers, per-row statistics) + <name>_trace.npz (float32
samples: per block row the 16 largest logits and 256 random columns; K and V at sampled
positions, layers and heads over the whole head dimension).  A full-size trace takes 10 - 20
minutes on 8 cores and ~25 GB of host memory.
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import ec_inputs  # noqa: E402
from oracle import entropycache as eco  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
F, P_ = eco.FULL, eco.PARTIAL
TRACES = {
    "llada8b": dict(workload="llada8b", scale=8.0, modes=[F, P_, P_, P_, F, P_]),
    "dream7b": dict(workload="dream7b", scale=8.0, modes=[F, P_, P_, P_, F, P_]),
    "llada8b_cot": dict(workload="llada8b_cot", scale=8.0, modes=[F, P_, P_, P_, F, P_]),
    # batch: the 2-layer twin, every sequence follows its own entropy flag
    "llada8b_b16": dict(workload="llada8b_b16", scale=4.5, n_layers=2, steps=6),
}
N_TOP, N_RAND = 16, 256
N_KV_POS = {1: 64, 16: 8}          # sampled cache positions per step, by batch size
N_KV_HEADS = {1: 4, 16: 2}


def r9(a):
    return [float(f"{v:.9e}") for v in np.asarray(a, dtype=np.float64).ravel()]


def row_sensitivity(z):
    """sum_j p_j |ln p_j + H| for each row: the first-order bound |dH| <= that * max|dz|."""
    out = []
    for row in z:
        m = row.max()
        lse = m + np.log(np.exp(row - m).sum())
        lp = row - lse
        p = np.exp(lp)
        H = -(p * lp).sum()
        out.append(float((p * np.abs(lp + H)).sum()))
    return out


def sample_step(st, r, rng, layers, heads, n_kv_pos, arrays, key):
    """Everything the GPU test compares for one step of one sequence."""
    z = r["logits"]
    nmb, V = z.shape
    rand_cols = np.sort(rng.choice(V, N_RAND, replace=False))
    top = np.argsort(-z, axis=1, kind="stable")[:, :N_TOP]
    cols = np.concatenate([top, np.broadcast_to(rand_cols, (nmb, N_RAND))], axis=1).astype(np.int32)
    arrays[key + "cols"] = cols
    arrays[key + "logits"] = np.take_along_axis(z, cols.astype(np.int64), axis=1).astype(np.float32)
    srt = np.sort(z, axis=1)
    m = z.max(axis=1)
    lse = m + np.log(np.exp(z - m[:, None]).sum(axis=1))
    S = r["S"]
    notS = np.setdiff1d(np.arange(st.T), S)
    n_in = min(len(S), n_kv_pos if len(notS) == 0 else (n_kv_pos * 3) // 4)
    if len(S) <= 40:
        n_in = min(len(S), n_kv_pos - 4)            # a partial step: (nearly) every recomputed row
    n_out = min(len(notS), n_kv_pos - n_in)
    pos = np.sort(np.concatenate([rng.choice(S, n_in, replace=False),
                                  rng.choice(notS, n_out, replace=False)])).astype(np.int32)
    arrays[key + "kv_pos"] = pos
    arrays[key + "K"] = st.Kc[layers][:, pos][:, :, heads, :].astype(np.float32)
    arrays[key + "V"] = st.Vc[layers][:, pos][:, :, heads, :].astype(np.float32)
    return {
        "t": r["t"], "mode": int(r["mode"]), "n_rows": int(len(S)), "Mb": r["Mb"].tolist(),
        "positions": r["positions"], "tokens": r["tokens"],
        "own_positions": r["own_positions"], "own_tokens": r["own_tokens"],
        "E": r["E"], "E_own": r["E_own"], "next_mode": int(r["next_mode"]),
        "R": r["R"], "skip": bool(r["skip"]), "done": bool(r["done"]),
        "tok": r["tok"].tolist(), "conf": r9(r["conf"]), "H": r9(r["H"]), "lse": r9(lse),
        "zmax": r9(m), "top2gap": r9(srt[:, -1] - srt[:, -2]),
        "H_sens": r9(row_sensitivity(z)),
        "logits_absmax": float(np.abs(z).max()),
        "K_absmax": [float(np.abs(st.Kc[l]).max()) for l in layers],
        "V_absmax": [float(np.abs(st.Vc[l]).max()) for l in layers],
    }


def main(name):
    spec = TRACES[name]
    wl = ec_inputs.WORKLOADS[spec["workload"]]
    cfg = wl.model.replace(logit_scale=spec["scale"])
    if "n_layers" in spec:
        cfg = cfg.replace(n_layers=spec["n_layers"])
        eco.enable_f64_cache(True)
    dec = wl.decode
    B = dec.batch
    L = cfg.n_layers
    layers = sorted({0, L // 2 - 1 if L > 2 else L - 1, L - 1})
    nh = N_KV_HEADS[B]
    heads = sorted({(i * cfg.n_kv_heads) // nh + (cfg.n_kv_heads // nh) // 2 for i in range(nh)})
    t0 = time.time()
    w = ec_inputs.make_weights(cfg, wl.seed, threads=8)
    model = eco.OracleModel(cfg, w)
    rng = np.random.default_rng(12345)
    arrays = {}
    out = {"workload": spec["workload"], "logit_scale": spec["scale"], "n_layers": L,
           "layers": layers, "heads": heads, "batch": B, "n_top": N_TOP, "steps": []}
    if B == 1:
        prompt = ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed)
        st = eco.eco_init(model, dec, prompt)
        for i, mode in enumerate(spec["modes"]):
            r = eco.eco_step(st, mode)
            out["steps"].append(sample_step(st, r, rng, layers, heads, N_KV_POS[1], arrays, f"s{i}_"))
            print(f"[{time.time() - t0:6.0f}s] step {r['t']} mode {mode} rows {len(r['S'])} "
                  f"E {r['E']:.4f}", flush=True)
    else:
        prompts = [ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed + 1000 + b)
                   for b in range(B)]
        out["prompt_seeds"] = [wl.seed + 1000 + b for b in range(B)]
        sts = [eco.eco_init(model, dec.replace(batch=1), p) for p in prompts]
        mixed = 0
        for i in range(spec["steps"]):
            per_seq = []
            for b, st in enumerate(sts):
                r = eco.eco_step(st, eco.AUTO)
                per_seq.append(sample_step(st, r, rng, layers, heads, N_KV_POS[16], arrays,
                                           f"s{i}_b{b}_"))
            modes = [s["mode"] for s in per_seq]
            mixed += int(0 < sum(modes) < B)
            out["steps"].append(per_seq)
            print(f"[{time.time() - t0:6.0f}s] step {i + 1} modes {modes}", flush=True)
        assert mixed >= 2, "the trace must hold steps with FULL and PARTIAL sequences side by side"
    with open(os.path.join(HERE, f"{name}_trace.json"), "w") as f:
        json.dump(out, f)
    np.savez(os.path.join(HERE, f"{name}_trace.npz"), **arrays)
    print("wrote", name, "in", int(time.time() - t0), "s")


if __name__ == "__main__":
    main(sys.argv[1])
