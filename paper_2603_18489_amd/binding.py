"""Thin ctypes binding of libec.so (include/ec.h).  Argument marshalling only: every step of the
denoising path runs in the library's HIP kernels.  PyTorch supplies device memory and the stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libec.so")

EC_MAX_N = 32
EC_MAX_BLOCK = 128
EC_MAX_BATCH = 64
EC_F32, EC_BF16, EC_FP8W = 0, 1, 2
EC_FULL, EC_PARTIAL, EC_AUTO = 0, 1, 2
EC_GATE_MAX_ENTROPY, EC_GATE_ENTROPY_SUM, EC_GATE_MAX_CONFIDENCE = 0, 1, 2
EC_SCHED_BLOCKS, EC_SCHED_SLIDING = 0, 1
EC_OK, EC_ERR_ARG, EC_ERR_CONFIG, EC_ERR_WORKSPACE, EC_ERR_STATE, EC_ERR_HIP = 0, -1, -2, -3, -4, -5
EC_ERR_HOST_MEMORY = -6
EC_ERR_NONFINITE = -7
(EC_K_EMBED, EC_K_NORM, EC_K_QKV, EC_K_ROPE_KV, EC_K_ATTN, EC_K_OPROJ, EC_K_GATEUP, EC_K_SWIGLU,
 EC_K_DOWN, EC_K_LMHEAD, EC_K_VOCAB_REDUCE, EC_K_DECIDE, EC_K_COUNT) = range(13)
KERNEL_CLASS_NAMES = ["embed", "norm", "qkv", "rope_kv", "attn", "oproj", "gateup", "swiglu",
                      "down", "lmhead", "vocab_reduce", "decide"]
(EC_DBG_LOGITS, EC_DBG_KCACHE, EC_DBG_VCACHE, EC_DBG_X, EC_DBG_MASKED, EC_DBG_HIST, EC_DBG_ROWS,
 EC_DBG_ROW_STATS) = range(8)

EXPORTS = ["ec_workspace_bytes", "ec_init", "ec_reset", "ec_step", "ec_step_forced", "ec_debug_keep_logits",
           "ec_step_forced_batch", "ec_generate", "ec_profile_enable", "ec_profile_read",
           "ec_debug_read", "ec_debug_read_seq", "ec_destroy", "ec_strerror", "ec_last_error",
           "ec_row_entropy_workspace_bytes", "ec_row_entropy", "ec_row_entropy_noalloc"]


class ec_model_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads",
                                         "head_dim", "d_ffn", "vocab", "mask_id")] + \
               [(n, C.c_float) for n in ("rms_eps", "rope_base", "logit_scale")] + \
               [("dtype", C.c_int32)]


QUANT_MATRICES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


class ec_weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "wq", "wk", "wv", "wo",
                                                      "mlp_norm", "w_gate", "w_up", "w_down")] + \
               [("lm_head_scale", C.c_void_p)] + \
               [(n + "_scale", C.POINTER(C.c_void_p)) for n in QUANT_MATRICES]


class ec_decode_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "gen_len", "block", "k_recent",
                                         "tokens_per_step")] + \
               [("tau", C.c_float), ("conf_threshold", C.c_float), ("gate_metric", C.c_int32),
                ("schedule", C.c_int32)]


class ec_step_result(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_unmasked", "done", "mode_run", "next_mode",
                                         "n_query_rows", "step_index", "n_block_rows",
                                         "n_recent_next")] + \
               [("max_entropy", C.c_float),
                ("positions", C.c_int32 * EC_MAX_N), ("tokens", C.c_int32 * EC_MAX_N),
                ("entropy", C.c_float * EC_MAX_N), ("confidence", C.c_float * EC_MAX_N)]

    def as_dict(self) -> dict:
        n = self.n_unmasked
        return {"n_unmasked": n, "done": bool(self.done), "mode_run": self.mode_run,
                "next_mode": self.next_mode, "n_query_rows": self.n_query_rows,
                "step_index": self.step_index, "n_block_rows": self.n_block_rows,
                "n_recent_next": self.n_recent_next, "max_entropy": float(self.max_entropy),
                "positions": list(self.positions[:n]), "tokens": list(self.tokens[:n]),
                "entropy": list(self.entropy[:n]), "confidence": list(self.confidence[:n])}


class ec_gen_stats(C.Structure):
    _fields_ = [("steps", C.c_int32), ("full_steps", C.c_int32), ("partial_steps", C.c_int32),
                ("tokens", C.c_int32), ("rows_recomputed", C.c_int64), ("ms_total", C.c_double)]


class ec_profile(C.Structure):
    _fields_ = [("ms", C.c_double * EC_K_COUNT), ("launches", C.c_int64 * EC_K_COUNT),
                ("steps", C.c_int64)]


_lib = None


def load_library() -> C.CDLL:
    """Loads libec.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2603_18489_amd.build` "
                           "(or __graft_entry__.build()) first")
    lib = C.CDLL(LIB_PATH)
    vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
    lib.ec_workspace_bytes.restype = C.c_size_t
    lib.ec_workspace_bytes.argtypes = [C.POINTER(ec_model_cfg), C.POINTER(ec_decode_cfg), i32p]
    lib.ec_init.restype = C.c_int
    lib.ec_init.argtypes = [C.POINTER(vp), C.POINTER(ec_model_cfg), C.POINTER(ec_weights),
                            C.POINTER(ec_decode_cfg), i32p, i32p, vp, C.c_size_t, vp]
    lib.ec_reset.restype = C.c_int
    lib.ec_reset.argtypes = [vp, i32p]
    lib.ec_step.restype = C.c_int
    lib.ec_step.argtypes = [vp, C.c_int, C.POINTER(ec_step_result)]
    lib.ec_step_forced.restype = C.c_int
    lib.ec_step_forced.argtypes = [vp, C.c_int, C.c_int32, i32p, i32p, C.POINTER(ec_step_result)]
    lib.ec_step_forced_batch.restype = C.c_int
    lib.ec_step_forced_batch.argtypes = [vp, i32p, i32p, i32p, i32p, C.POINTER(ec_step_result)]
    lib.ec_generate.restype = C.c_int
    lib.ec_generate.argtypes = [vp, i32p, C.POINTER(ec_gen_stats)]
    lib.ec_profile_enable.restype = C.c_int
    lib.ec_profile_enable.argtypes = [vp, C.c_int]
    lib.ec_profile_read.restype = C.c_int
    lib.ec_profile_read.argtypes = [vp, C.POINTER(ec_profile)]
    lib.ec_debug_keep_logits.restype = C.c_int
    lib.ec_debug_keep_logits.argtypes = [vp, C.c_int]
    lib.ec_debug_read.restype = C.c_int
    lib.ec_debug_read.argtypes = [vp, C.c_int, C.c_int, vp, C.c_size_t]
    lib.ec_debug_read_seq.restype = C.c_int
    lib.ec_debug_read_seq.argtypes = [vp, C.c_int, C.c_int, C.c_int, vp, C.c_size_t]
    lib.ec_row_entropy_workspace_bytes.restype = C.c_size_t
    lib.ec_row_entropy_workspace_bytes.argtypes = [C.c_int32, C.c_int32]
    lib.ec_row_entropy.restype = C.c_int
    lib.ec_row_entropy.argtypes = [vp, C.c_int32, C.c_int32, C.c_size_t, vp, vp, C.c_size_t, vp]
    lib.ec_row_entropy_noalloc.restype = C.c_int
    lib.ec_row_entropy_noalloc.argtypes = [vp, C.c_int32, C.c_int32, C.c_size_t, vp, vp]
    lib.ec_destroy.restype = None
    lib.ec_destroy.argtypes = [vp]
    lib.ec_strerror.restype = C.c_char_p
    lib.ec_strerror.argtypes = [C.c_int]
    lib.ec_last_error.restype = C.c_char_p
    lib.ec_last_error.argtypes = [vp]
    _lib = lib
    return lib


class EcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ec error {code} ({load_library().ec_strerror(code).decode()}): {msg}")
        self.code = code


def model_cfg_struct(cfg) -> ec_model_cfg:
    return ec_model_cfg(cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim,
                        cfg.d_ffn, cfg.vocab, cfg.mask_id, cfg.rms_eps, cfg.rope_base,
                        cfg.logit_scale, {"f32": EC_F32, "bf16": EC_BF16, "fp8w": EC_FP8W}[cfg.dtype])


def decode_cfg_struct(dec) -> ec_decode_cfg:
    return ec_decode_cfg(dec.batch, dec.gen_len, dec.block, dec.k_recent, dec.tokens_per_step,
                         dec.tau, getattr(dec, "conf_threshold", 0.0),
                         getattr(dec, "gate_metric", 0), getattr(dec, "schedule", 0))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _i32p(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def weights_to_device(cfg, w: Dict[str, object], device="cuda:0") -> Dict[str, object]:
    """Uploads host weights (float32, uint16 bfloat16 bit patterns, or matrices as e4m3 codes +
    float32 row scales) as torch device tensors; a quantised matrix `name` becomes the uint8 tensor
    `name` and the float32 tensor `name_scale`."""
    import torch

    def up(a: np.ndarray):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
        return torch.from_numpy(a).to(device)

    out: Dict[str, object] = {}
    for k, v in w.items():
        items = v if isinstance(v, list) else [v]
        if hasattr(items[0], "codes"):
            codes, scales = [up(x.codes) for x in items], [up(x.scale) for x in items]
            out[k] = codes if isinstance(v, list) else codes[0]
            out[k + "_scale"] = scales if isinstance(v, list) else scales[0]
        else:
            out[k] = [up(x) for x in v] if isinstance(v, list) else up(v)
    return out


def row_entropy(logits, stream=None):
    """ec_row_entropy on a float32 CUDA tensor [rows, vocab] (row stride = logits.stride(0)):
    returns a float32 CUDA tensor [rows, 4] (token, confidence, entropy, max logit).  The
    workspace is a torch allocation; the call is enqueued on `stream` (default: current)."""
    import torch
    lib = load_library()
    rows, vocab = logits.shape
    assert logits.dtype == torch.float32 and logits.stride(1) == 1
    stats = torch.empty((rows, 4), dtype=torch.float32, device=logits.device)
    if rows == 0:
        return stats         # (an empty tensor has no address to hand over)
    need = lib.ec_row_entropy_workspace_bytes(rows, vocab)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=logits.device)
    st = stream if stream is not None else torch.cuda.current_stream()
    rc = lib.ec_row_entropy(C.c_void_p(logits.data_ptr()), rows, vocab,
                            logits.stride(0) if rows > 1 else vocab, C.c_void_p(stats.data_ptr()),
                            C.c_void_p(ws.data_ptr()), need, C.c_void_p(st.cuda_stream))
    if rc != EC_OK:
        raise EcError(rc, lib.ec_last_error(None).decode())
    st.synchronize()     # the workspace is released on return
    return stats


def row_entropy_noalloc(logits, stats, stream=None):
    """ec_row_entropy_noalloc: `stats` is a caller-provided float32 CUDA tensor [rows, 4]; the
    call itself allocates nothing.  Enqueued on `stream` (default: current), not synchronised."""
    import torch
    lib = load_library()
    rows, vocab = logits.shape
    assert logits.dtype == torch.float32 and logits.stride(1) == 1
    assert stats.dtype == torch.float32 and stats.is_contiguous() and stats.shape == (rows, 4)
    st = stream if stream is not None else torch.cuda.current_stream()
    rc = lib.ec_row_entropy_noalloc(C.c_void_p(logits.data_ptr()), rows, vocab,
                                    logits.stride(0) if rows > 1 else vocab,
                                    C.c_void_p(stats.data_ptr()), C.c_void_p(st.cuda_stream))
    if rc != EC_OK:
        raise EcError(rc, lib.ec_last_error(None).decode())


class EntropyCache:
    """One context: holds the torch tensors the library borrows (weights, workspace).
    With dec.batch > 1, `prompt` is a list of dec.batch prompts and the per-sequence results
    come back as lists in sequence order."""

    def __init__(self, cfg, dev_weights: Dict[str, object], dec, prompt, stream=None):
        import torch
        self.lib = load_library()
        self.cfg, self.dec = cfg, dec
        self.B = dec.batch
        prompts = [list(prompt)] if self.B == 1 else [list(p) for p in prompt]
        assert len(prompts) == self.B
        self.Ps = [len(p) for p in prompts]
        self.N = dec.gen_len
        self.Ts = [p + self.N for p in self.Ps]
        self.P, self.T = self.Ps[0], self.Ts[0]
        self._w = dev_weights  # keep alive
        self._mc, self._dc = model_cfg_struct(cfg), decode_cfg_struct(dec)
        L = cfg.n_layers
        ws = ec_weights()
        ws.tok_emb = dev_weights["tok_emb"].data_ptr()
        ws.lm_head = dev_weights["lm_head"].data_ptr()
        ws.final_norm = dev_weights["final_norm"].data_ptr()
        self._ptr_arrays = {}
        for name in ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down"):
            arr = (C.c_void_p * L)(*[t.data_ptr() for t in dev_weights[name]])
            self._ptr_arrays[name] = arr
            setattr(ws, name, C.cast(arr, C.POINTER(C.c_void_p)))
        if cfg.dtype == "fp8w":
            ws.lm_head_scale = dev_weights["lm_head_scale"].data_ptr()
            for name in QUANT_MATRICES:
                arr = (C.c_void_p * L)(*[t.data_ptr() for t in dev_weights[name + "_scale"]])
                self._ptr_arrays[name + "_scale"] = arr
                setattr(ws, name + "_scale", C.cast(arr, C.POINTER(C.c_void_p)))
        self._ws = ws
        plen = _i32(self.Ps)
        need = self.lib.ec_workspace_bytes(C.byref(self._mc), C.byref(self._dc), _i32p(plen))
        if need == 0:
            # let ec_init produce the message
            need = 256
        self.workspace_bytes = need
        self._workspace = torch.empty(need, dtype=torch.uint8, device=dev_weights["tok_emb"].device)
        self._stream = stream if stream is not None else torch.cuda.current_stream()
        ctx = C.c_void_p()
        pr = _i32([t for p in prompts for t in p])
        rc = self.lib.ec_init(C.byref(ctx), C.byref(self._mc), C.byref(self._ws),
                              C.byref(self._dc), _i32p(pr), _i32p(plen),
                              C.c_void_p(self._workspace.data_ptr()), need,
                              C.c_void_p(self._stream.cuda_stream))
        if rc != EC_OK:
            raise EcError(rc, self.lib.ec_last_error(None).decode())
        self.ctx = ctx

    def _check(self, rc: int):
        if rc != EC_OK:
            raise EcError(rc, self.lib.ec_last_error(self.ctx).decode())

    def reset(self, prompt):
        prompts = [list(prompt)] if self.B == 1 else [list(p) for p in prompt]
        assert [len(p) for p in prompts] == self.Ps
        pr = _i32([t for p in prompts for t in p])
        self._check(self.lib.ec_reset(self.ctx, _i32p(pr)))

    def step(self, mode: int = EC_AUTO):
        r = (ec_step_result * self.B)()
        self._check(self.lib.ec_step(self.ctx, mode, r))
        return r[0].as_dict() if self.B == 1 else [x.as_dict() for x in r]

    def step_forced_batch(self, modes: Sequence[int], positions, tokens) -> List[dict]:
        """positions / tokens: one list per sequence (ignored for finished sequences)."""
        r = (ec_step_result * self.B)()
        n = _i32([len(p) for p in positions])
        p = _i32([v for q in positions for v in q] or [0])
        t = _i32([v for q in tokens for v in q] or [0])
        self._check(self.lib.ec_step_forced_batch(self.ctx, _i32p(_i32(modes)), _i32p(n), _i32p(p),
                                                  _i32p(t), r))
        return [x.as_dict() for x in r]

    def step_forced(self, mode: int, positions: Sequence[int], tokens: Sequence[int]) -> dict:
        r = ec_step_result()
        p, t = _i32(positions), _i32(tokens)
        self._check(self.lib.ec_step_forced(self.ctx, mode, len(p), _i32p(p), _i32p(t), C.byref(r)))
        return r.as_dict()

    def generate(self):
        out = np.zeros(self.B * self.N, dtype=np.int32)
        st = ec_gen_stats()
        self._check(self.lib.ec_generate(self.ctx, _i32p(out), C.byref(st)))
        stats = {k: getattr(st, k) for k, _ in ec_gen_stats._fields_}
        return (out if self.B == 1 else out.reshape(self.B, self.N)), stats

    def keep_logits(self, on: bool = True):
        """Makes the following steps store their logits so that EC_DBG_LOGITS can read them."""
        self._check(self.lib.ec_debug_keep_logits(self.ctx, int(on)))

    def profile_enable(self, on: bool):
        self._check(self.lib.ec_profile_enable(self.ctx, int(on)))

    def profile_read(self) -> dict:
        p = ec_profile()
        self._check(self.lib.ec_profile_read(self.ctx, C.byref(p)))
        return {"steps": p.steps,
                "ms": {n: p.ms[i] for i, n in enumerate(KERNEL_CLASS_NAMES)},
                "launches": {n: p.launches[i] for i, n in enumerate(KERNEL_CLASS_NAMES)}}

    def debug_read(self, what: int, layer: int = 0, count: Optional[int] = None,
                   seq: int = 0) -> np.ndarray:
        cfg = self.cfg
        T = self.Ts[seq]
        kvw = cfg.n_kv_heads * cfg.head_dim
        if what == EC_DBG_LOGITS:
            n = self.dec.block if count is None else count
            out = np.empty((n, cfg.vocab), dtype=np.float32)
        elif what in (EC_DBG_KCACHE, EC_DBG_VCACHE):
            out = np.empty((T, cfg.n_kv_heads, cfg.head_dim),
                           dtype=np.float32 if cfg.dtype == "f32" else np.uint16)
        elif what == EC_DBG_X:
            out = np.empty(T, dtype=np.int32)
        elif what == EC_DBG_MASKED:
            out = np.empty(T, dtype=np.uint8)
        elif what == EC_DBG_HIST:
            out = np.empty(self.N, dtype=np.int32)
        elif what == EC_DBG_ROWS:
            out = np.empty(int(count), dtype=np.int32)
        elif what == EC_DBG_ROW_STATS:
            n = self.dec.block if count is None else count
            out = np.empty((n, 4), dtype=np.float32)
        else:
            raise ValueError("unknown debug item")
        self._check(self.lib.ec_debug_read_seq(self.ctx, seq, what, layer,
                                               out.ctypes.data_as(C.c_void_p), out.nbytes))
        return out

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.ec_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
