"""Writes tests/golden/llada8b_trace.json: sampled outputs of the fp64 oracle on the full
LLaDA-8B-shaped workload (32 layers) for a short teacher-forced trace
FULL, PARTIAL, PARTIAL, PARTIAL, FULL, PARTIAL.  Calls only oracle/ and ec_inputs/.
The GPU parity test replays the same modes and committed tokens and compares these samples.
Takes a few minutes and ~25 GB of host memory:  python tests/golden/make_llada8b_trace.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import ec_inputs  # noqa: E402
from oracle import entropycache as eco  # noqa: E402

WORKLOAD = "llada8b"
LOGIT_SCALE = 8.0
MODES = [eco.FULL, eco.PARTIAL, eco.PARTIAL, eco.PARTIAL, eco.FULL, eco.PARTIAL]
LAYERS = [0, 15, 31]
HEADS = [0, 17]
NCOLS = 24


def r9(a):
    return [float(f"{v:.9e}") for v in np.asarray(a, dtype=np.float64).ravel()]


def main():
    wl = ec_inputs.WORKLOADS[WORKLOAD]
    cfg = wl.model.replace(logit_scale=LOGIT_SCALE)
    w = ec_inputs.make_weights(cfg, wl.seed, threads=8)
    prompt = ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed)
    st = eco.eco_init(eco.OracleModel(cfg, w), wl.decode, prompt)
    rng = np.random.default_rng(12345)
    cols = np.sort(rng.choice(cfg.vocab, NCOLS, replace=False))
    out = {"workload": WORKLOAD, "logit_scale": LOGIT_SCALE, "cols": cols.tolist(),
           "layers": LAYERS, "heads": HEADS, "steps": []}
    for mode in MODES:
        r = eco.eco_step(st, mode)
        S = r["S"]
        notS = np.setdiff1d(np.arange(st.T), S)
        pos = np.sort(np.concatenate([rng.choice(S, min(12, len(S)), replace=False),
                                      rng.choice(notS, 4, replace=False) if len(notS) >= 4
                                      else rng.choice(S, 4, replace=False)]))
        srt = np.sort(r["logits"], axis=1)
        step = {
            "t": r["t"], "mode": int(mode), "n_rows": int(len(S)),
            "S_head": S[:40].tolist(), "Mb": r["Mb"].tolist(),
            "positions": r["positions"], "tokens": r["tokens"], "E": r["E"],
            "R": r["R"], "skip": bool(r["skip"]),
            "tok": r["tok"].tolist(), "conf": r9(r["conf"]), "H": r9(r["H"]),
            "logits_cols": r9(r["logits"][:, cols]), "logits_absmax": float(np.abs(r["logits"]).max()),
            "logits_range": float(np.ptp(r["logits"])),
            "top2gap": r9(srt[:, -1] - srt[:, -2]),
            "kv_pos": pos.tolist(),
            "K": {str(l): r9(st.Kc[l][pos][:, HEADS, :8]) for l in LAYERS},
            "V": {str(l): r9(st.Vc[l][pos][:, HEADS, :8]) for l in LAYERS},
            "K_absmax": {str(l): float(np.abs(st.Kc[l]).max()) for l in LAYERS},
            "V_absmax": {str(l): float(np.abs(st.Vc[l]).max()) for l in LAYERS},
        }
        out["steps"].append(step)
        print("step", r["t"], "mode", mode, "rows", len(S), "E", r["E"], flush=True)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "llada8b_trace.json")
    with open(path, "w") as f:
        json.dump(out, f)
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
