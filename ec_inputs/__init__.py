"""Seeded synthetic inputs for the EntropyCache step: model shapes, random weights, prompts.

This module serves both the CPU oracle and the HIP path and therefore holds none of the
method's arithmetic: it only describes shapes and draws random numbers.  The one numeric
transform it owns is the storage encoding of a weight (float32 -> bfloat16 bit pattern with
round-to-nearest-even), which is a property of the input, not of the method.

Weights follow the synthetic-model recipe: every matrix is N(0, 0.02) drawn from a
counter-based generator (Philox) whose key is derived from (seed, tensor id, chunk id), so the
values do not depend on how many threads draw them.  Norm gains are 1.0 unless `gain_jitter`
is given (tests use a jitter so that a dropped gain multiply cannot hide).
"""
from __future__ import annotations

import dataclasses
import hashlib
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Tuple

import numpy as np

_CHUNK = 1 << 20  # elements drawn per Philox key


@dataclasses.dataclass(frozen=True)
class ModelCfg:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    mask_id: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    logit_scale: float = 1.0
    # storage type of the weights: "f32", "bf16", or "fp8w" = matrices as 8-bit e4m3 codes with one
    # float32 scale per output row (QuantMatrix), everything else (embedding, norm gains) bfloat16.
    # The GPU's activations and KV cache are float32 for "f32" and bfloat16 otherwise.
    dtype: str = "f32"

    def replace(self, **kw) -> "ModelCfg":
        return dataclasses.replace(self, **kw)


@dataclasses.dataclass(frozen=True)
class DecodeCfg:
    gen_len: int
    block: int = 32
    k_recent: int = 2
    tokens_per_step: int = 1
    tau: float = 1.0
    batch: int = 1
    conf_threshold: float = 0.0   # > 0: unmask every block row whose confidence exceeds it
    gate_metric: int = 0          # 0 max entropy, 1 entropy sum, 2 max confidence
    schedule: int = 0             # 0 fixed blocks, 1 sliding window of `block` masked slots

    def replace(self, **kw) -> "DecodeCfg":
        return dataclasses.replace(self, **kw)


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    model: ModelCfg
    decode: DecodeCfg
    prompt_len: int
    seed: int


def _llada(dtype="bf16", n_layers=32) -> ModelCfg:
    return ModelCfg(n_layers=n_layers, d_model=4096, n_heads=32, n_kv_heads=32, head_dim=128,
                    d_ffn=12288, vocab=126464, mask_id=126463, rms_eps=1e-5, rope_base=500000.0,
                    dtype=dtype)


def _dream(dtype="bf16", n_layers=28) -> ModelCfg:
    return ModelCfg(n_layers=n_layers, d_model=3584, n_heads=28, n_kv_heads=4, head_dim=128,
                    d_ffn=18944, vocab=152064, mask_id=152063, rms_eps=1e-5, rope_base=1e6,
                    dtype=dtype)


WORKLOADS: Dict[str, Workload] = {
    # tiny fp32 model the oracle runs end to end in seconds
    "tiny_f32": Workload(
        "tiny_f32",
        ModelCfg(n_layers=2, d_model=256, n_heads=4, n_kv_heads=4, head_dim=64, d_ffn=768,
                 vocab=4096, mask_id=4095, rms_eps=1e-5, rope_base=10000.0, dtype="f32"),
        DecodeCfg(gen_len=64, block=32, k_recent=2, tokens_per_step=1, tau=2.0), 64, 1),
    # LLaDA-8B shape, prompt 512 + generation 256: partial step = 34 rows against 768 keys
    "llada8b": Workload("llada8b", _llada(),
                        DecodeCfg(gen_len=256, block=32, k_recent=2, tokens_per_step=1, tau=1.0),
                        512, 2),
    # Dream-7B / Qwen2.5-7B shape (GQA 28/4), 2 tokens per step
    "dream7b": Workload("dream7b", _dream(),
                        DecodeCfg(gen_len=256, block=32, k_recent=2, tokens_per_step=2, tau=1.0),
                        1024, 3),
    # long chain-of-thought shape on the LLaDA-8B model
    "llada8b_cot": Workload("llada8b_cot", _llada(),
                            DecodeCfg(gen_len=1024, block=32, k_recent=4, tokens_per_step=1,
                                      tau=0.5), 256, 2),
    # the paper's own decoding settings on the LLaDA-8B shape: sliding window of 32, confidence-
    # based parallel decoding at 0.9, tau = 1.5, k = 64 (partial steps of up to 96 rows)
    "llada8b_paper": Workload("llada8b_paper", _llada(),
                              DecodeCfg(gen_len=256, block=32, k_recent=64, tokens_per_step=1,
                                        tau=1.5, conf_threshold=0.9, schedule=1), 512, 2),
    # 16 sequences side by side on the LLaDA-8B model, prompts of 1024, 512 generated tokens each:
    # partial steps of 16 x (<= 34) rows, full steps of up to 24 576 rows, mixed within a step
    "llada8b_b16": Workload("llada8b_b16", _llada(),
                            DecodeCfg(gen_len=512, block=32, k_recent=2, tokens_per_step=1,
                                      tau=1.0, batch=16), 1024, 2),
    # the LLaDA-8B shape with its matrices stored as e4m3 codes + per-row scales: half the bytes
    # to stream per partial step (beyond the paper: its method is orthogonal to the weight format)
    "llada8b_fp8": Workload("llada8b_fp8", _llada(dtype="fp8w"),
                            DecodeCfg(gen_len=256, block=32, k_recent=2, tokens_per_step=1, tau=1.0),
                            512, 2),
    "llada8b_fp8_l2": Workload("llada8b_fp8_l2", _llada(dtype="fp8w", n_layers=2),
                               DecodeCfg(gen_len=256, block=32, k_recent=2, tokens_per_step=1,
                                         tau=1.0), 512, 2),
    # reduced-depth twins (same widths and vocabulary, 2 layers) for whole-generation parity
    "llada8b_l2": Workload("llada8b_l2", _llada(n_layers=2),
                           DecodeCfg(gen_len=256, block=32, k_recent=2, tokens_per_step=1,
                                     tau=1.0), 512, 2),
    "dream7b_l2": Workload("dream7b_l2", _dream(n_layers=2),
                           DecodeCfg(gen_len=256, block=32, k_recent=2, tokens_per_step=2,
                                     tau=1.0), 1024, 3),
}


# ----------------------------------------------------------------------------------------------
# storage encoding
# ----------------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit pattern (uint16), round to nearest, ties to even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def f32_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> 8-bit e4m3 code (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no
    infinities, S.1111.111 = NaN), round to nearest with ties to even, saturating at +-448."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    sign = ((u >> np.uint32(24)) & np.uint32(0x80)).astype(np.uint8)
    a = u & np.uint32(0x7FFFFFFF)
    # normal range (|x| >= 2^-6): round the float32 mantissa to 3 bits, ties to even
    r = a + np.uint32(0x7FFFF) + ((a >> np.uint32(20)) & np.uint32(1))
    e = (r >> np.uint32(23)).astype(np.int32) - 127 + 7
    m = ((r >> np.uint32(20)) & np.uint32(7)).astype(np.int32)
    code = (e << 3) | m
    # below the smallest normal the grid is uniform with step 2^-9 (8 steps reach 2^-6 = code 8)
    sub = np.rint(np.minimum(np.abs(x), np.float32(1.0)) * np.float32(512.0)).astype(np.int32)
    code = np.where(np.abs(x) < np.float32(2.0 ** -6), sub, code)
    code = np.minimum(code, 0x7E)                       # saturate (also infinities)
    return (code.astype(np.uint8) | sign)


class QuantMatrix:
    """A matrix stored as e4m3 codes [out, in] with one float32 scale per output row: its value
    is scale[row] * e4m3(codes[row, col])."""
    __slots__ = ("codes", "scale")

    def __init__(self, codes: np.ndarray, scale: np.ndarray):
        self.codes, self.scale = codes, scale

    ndim = 2

    @property
    def shape(self):
        return self.codes.shape


def quantize_rows_e4m3(w: np.ndarray) -> QuantMatrix:
    """Per-row scale = max |w| / 448 (the largest e4m3 magnitude), codes = e4m3(w / scale)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    amax = np.abs(w).max(axis=1)
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    return QuantMatrix(f32_to_e4m3_bits(w / scale[:, None]), scale)


# ----------------------------------------------------------------------------------------------
# random draws
# ----------------------------------------------------------------------------------------------
def _key(seed: int, tensor_id: str, chunk: int) -> int:
    h = hashlib.blake2b(f"{seed}/{tensor_id}/{chunk}".encode(), digest_size=16).digest()
    return int.from_bytes(h, "little")


def _draw_chunk(seed: int, tensor_id: str, chunk: int, n: int, std: float, bf16: bool):
    g = np.random.Generator(np.random.Philox(key=_key(seed, tensor_id, chunk)))
    x = g.standard_normal(n, dtype=np.float32)
    x *= np.float32(std)
    return f32_to_bf16_bits(x) if bf16 else x


def normal_tensor(seed: int, tensor_id: str, shape: Tuple[int, ...], std: float, dtype: str,
                  pool: ThreadPoolExecutor | None = None) -> np.ndarray:
    """N(0, std) tensor of `shape`; float32, or uint16 bfloat16 bit patterns when dtype=="bf16"."""
    n = int(np.prod(shape))
    bf16 = dtype == "bf16"
    out = np.empty(n, dtype=np.uint16 if bf16 else np.float32)
    jobs = []
    for c, lo in enumerate(range(0, n, _CHUNK)):
        hi = min(n, lo + _CHUNK)
        jobs.append((c, lo, hi))

    def run(job):
        c, lo, hi = job
        out[lo:hi] = _draw_chunk(seed, tensor_id, c, hi - lo, std, bf16)

    if pool is None or len(jobs) == 1:
        for j in jobs:
            run(j)
    else:
        list(pool.map(run, jobs))
    return out.reshape(shape)


def _gain(seed: int, tensor_id: str, d: int, jitter: float, dtype: str) -> np.ndarray:
    g = np.ones(d, dtype=np.float32)
    if jitter:
        r = np.random.Generator(np.random.Philox(key=_key(seed, tensor_id, 0)))
        g += np.float32(jitter) * r.standard_normal(d, dtype=np.float32)
    return f32_to_bf16_bits(g) if dtype == "bf16" else g


def make_weights(cfg: ModelCfg, seed: int, std: float = 0.02, gain_jitter: float = 0.0,
                 threads: int = 8) -> Dict[str, object]:
    """All tensors of the model, row-major [out, in].

    Returns {"tok_emb": [V,d], "lm_head": [V,d], "final_norm": [d], and lists of length L:
    "attn_norm" [d], "wq" [Hq*hd,d], "wk"/"wv" [Hkv*hd,d], "wo" [d,Hq*hd], "mlp_norm" [d],
    "w_gate"/"w_up" [F,d], "w_down" [d,F]}.
    """
    d, hq, hkv, hd, f, v = (cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn,
                            cfg.vocab)
    quant = cfg.dtype == "fp8w"
    dt = "bf16" if quant else cfg.dtype
    w: Dict[str, object] = {}
    with ThreadPoolExecutor(max_workers=max(1, threads)) as pool:
        def nt(name, shape):
            if not quant:
                return normal_tensor(seed, name, shape, std, dt, pool)
            # the same float32 draws, then e4m3 codes with per-row scales (row blocks in parallel)
            x = normal_tensor(seed, name, shape, std, "f32", pool)
            step = max(1, (1 << 22) // shape[1])
            parts = list(pool.map(lambda lo: quantize_rows_e4m3(x[lo:lo + step]),
                                  range(0, shape[0], step)))
            return QuantMatrix(np.concatenate([p.codes for p in parts]),
                               np.concatenate([p.scale for p in parts]))
        w["tok_emb"] = normal_tensor(seed, "tok_emb", (v, d), std, dt, pool)
        w["lm_head"] = nt("lm_head", (v, d))
        w["final_norm"] = _gain(seed, "final_norm", d, gain_jitter, dt)
        per_layer: Dict[str, List[np.ndarray]] = {k: [] for k in (
            "attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")}
        for l in range(cfg.n_layers):
            per_layer["attn_norm"].append(_gain(seed, f"attn_norm.{l}", d, gain_jitter, dt))
            per_layer["wq"].append(nt(f"wq.{l}", (hq * hd, d)))
            per_layer["wk"].append(nt(f"wk.{l}", (hkv * hd, d)))
            per_layer["wv"].append(nt(f"wv.{l}", (hkv * hd, d)))
            per_layer["wo"].append(nt(f"wo.{l}", (d, hq * hd)))
            per_layer["mlp_norm"].append(_gain(seed, f"mlp_norm.{l}", d, gain_jitter, dt))
            per_layer["w_gate"].append(nt(f"w_gate.{l}", (f, d)))
            per_layer["w_up"].append(nt(f"w_up.{l}", (f, d)))
            per_layer["w_down"].append(nt(f"w_down.{l}", (d, f)))
        w.update(per_layer)
    return w


def make_prompt(vocab: int, prompt_len: int, seed: int) -> np.ndarray:
    """`prompt_len` token ids uniform in [0, vocab-96): the prompt never holds the mask id."""
    g = np.random.Generator(np.random.Philox(key=_key(seed + 1000, "prompt", 0)))
    return g.integers(0, vocab - 96, size=prompt_len, dtype=np.int64).astype(np.int32)


def weight_bytes(cfg: ModelCfg) -> int:
    """Bytes of all matrices streamed by one step (layers + LM head; not the embedding)."""
    d, hq, hkv, hd, f, v = (cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn,
                            cfg.vocab)
    per_layer = (hq + 2 * hkv) * hd * d + d * hq * hd + 3 * f * d
    esz = {"bf16": 2, "fp8w": 1}.get(cfg.dtype, 4)
    return (cfg.n_layers * per_layer + v * d) * esz
