"""A dense, cache-free forward of the bidirectional Llama-style model, written independently of
the oracle for use as its pin: torch float64, explicit T x T score matrix per head, RoPE through
complex multiplication, library softmax / silu.  No KV cache, no row subsets: every position is
recomputed from the current token ids, which is what a full step must equal."""
import math

import numpy as np
import torch


def _t64(w):
    if w.dtype == np.uint16:
        w = (w.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return torch.from_numpy(np.ascontiguousarray(w)).to(torch.float64)


def _norm(h, g, eps):
    return h * torch.rsqrt((h * h).mean(-1, keepdim=True) + eps) * g


def _rope_complex(v, base):
    """v: [T, nh, hd]; position = row index.  (v_j + i v_{j+hd/2}) * exp(i * pos * theta_j)."""
    T, nh, hd = v.shape
    half = hd // 2
    theta = torch.tensor([base ** (-(2.0 * j) / hd) for j in range(half)], dtype=torch.float64)
    pos = torch.arange(T, dtype=torch.float64)
    rot = torch.polar(torch.ones(T, half, dtype=torch.float64), pos[:, None] * theta[None, :])
    z = torch.complex(v[..., :half], v[..., half:]) * rot[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def dense_forward(cfg, w, x):
    """Returns (final-normed hidden [T,d], logits [T,V], K [L,T,Hkv,hd] post-RoPE, V [L,T,Hkv,hd])."""
    hq, hkv, hd = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    T = len(x)
    h = _t64(w["tok_emb"])[torch.as_tensor(np.asarray(x), dtype=torch.long)]
    Ks, Vs = [], []
    for l in range(cfg.n_layers):
        u = _norm(h, _t64(w["attn_norm"][l]), cfg.rms_eps)
        q = torch.nn.functional.linear(u, _t64(w["wq"][l])).view(T, hq, hd)
        k = torch.nn.functional.linear(u, _t64(w["wk"][l])).view(T, hkv, hd)
        v = torch.nn.functional.linear(u, _t64(w["wv"][l])).view(T, hkv, hd)
        q, k = _rope_complex(q, cfg.rope_base), _rope_complex(k, cfg.rope_base)
        Ks.append(k.clone())
        Vs.append(v.clone())
        o = torch.zeros(T, hq, hd, dtype=torch.float64)
        for a in range(hq):
            kv = a // (hq // hkv)
            scores = torch.zeros(T, T, dtype=torch.float64)
            for i in range(T):
                for j in range(T):
                    scores[i, j] = torch.dot(q[i, a], k[j, kv]) / math.sqrt(hd)
            p = torch.softmax(scores, dim=-1)
            o[:, a] = p @ v[:, kv]
        h = h + torch.nn.functional.linear(o.reshape(T, hq * hd), _t64(w["wo"][l]))
        u = _norm(h, _t64(w["mlp_norm"][l]), cfg.rms_eps)
        g = torch.nn.functional.silu(torch.nn.functional.linear(u, _t64(w["w_gate"][l])))
        up = torch.nn.functional.linear(u, _t64(w["w_up"][l]))
        h = h + torch.nn.functional.linear(g * up, _t64(w["w_down"][l]))
    hf = _norm(h, _t64(w["final_norm"]), cfg.rms_eps)
    logits = cfg.logit_scale * torch.nn.functional.linear(hf, _t64(w["lm_head"]))
    return hf.numpy(), logits.numpy(), torch.stack(Ks).numpy(), torch.stack(Vs).numpy()
