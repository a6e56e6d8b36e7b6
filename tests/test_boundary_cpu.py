"""The C-ABI library without a GPU: it loads, exports every symbol include/ec.h declares, its
structs have the layout the binding assumes, and argument validation (which runs before any HIP
call) returns the documented error codes."""
import ctypes as C
import os
import re
import subprocess
import tempfile

import numpy as np
import pytest

import ec_inputs
import paper_2603_18489_amd as ec

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ec.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ec.LIB_PATH):
        from paper_2603_18489_amd import build
        build.build()
    return ec.load_library()


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ec_[a-z_]+)\s*\(", src)))


def test_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert sorted(names) == sorted(ec.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layout_matches_header():
    prog = r'''
    #include <stdio.h>
    #include "ec.h"
    int main(void) {
      printf("%zu %zu %zu %zu %zu %zu %d %d %d\n", sizeof(ec_model_cfg), sizeof(ec_weights),
             sizeof(ec_decode_cfg), sizeof(ec_step_result), sizeof(ec_gen_stats),
             sizeof(ec_profile), EC_MAX_N, EC_MAX_BLOCK, EC_K_COUNT);
      return 0;
    }'''
    with tempfile.TemporaryDirectory() as td:
        cfile = os.path.join(td, "s.c")
        open(cfile, "w").write(prog)
        exe = os.path.join(td, "s")
        subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), cfile, "-o", exe])
        vals = [int(v) for v in subprocess.check_output([exe]).split()]
    assert vals == [C.sizeof(ec.ec_model_cfg), C.sizeof(ec.ec_weights), C.sizeof(ec.ec_decode_cfg),
                    C.sizeof(ec.ec_step_result), C.sizeof(ec.ec_gen_stats),
                    C.sizeof(ec.ec_profile), ec.EC_MAX_N, ec.EC_MAX_BLOCK, ec.EC_K_COUNT]


def _cfgs(name="tiny_f32"):
    wl = ec_inputs.WORKLOADS[name]
    return ec.model_cfg_struct(wl.model), ec.decode_cfg_struct(wl.decode), wl


def test_workspace_bytes_and_config_checks(lib):
    mc, dc, wl = _cfgs()
    plen = np.array([wl.prompt_len], dtype=np.int32)
    p = plen.ctypes.data_as(C.POINTER(C.c_int32))
    n = lib.ec_workspace_bytes(C.byref(mc), C.byref(dc), p)
    T = wl.prompt_len + wl.decode.gen_len
    kv = wl.model.n_layers * 2 * T * wl.model.n_kv_heads * wl.model.head_dim * 4
    assert n > kv and n % 256 == 0
    assert lib.ec_workspace_bytes(None, C.byref(dc), p) == 0
    # LLaDA-8B shape: KV cache + re-tiled bf16 matrices dominate
    mc8, dc8, wl8 = _cfgs("llada8b")
    plen8 = np.array([wl8.prompt_len], dtype=np.int32)
    n8 = lib.ec_workspace_bytes(C.byref(mc8), C.byref(dc8), plen8.ctypes.data_as(C.POINTER(C.c_int32)))
    assert n8 > ec_inputs.weight_bytes(wl8.model) + 32 * 2 * 768 * 4096 * 2
    assert n8 < 20e9
    bad = ec.model_cfg_struct(wl.model.replace(head_dim=48))
    assert lib.ec_workspace_bytes(C.byref(bad), C.byref(dc), p) == 0


def test_init_argument_errors_without_gpu(lib):
    mc, dc, wl = _cfgs()
    ctx = C.c_void_p()
    plen = np.array([wl.prompt_len], dtype=np.int32)
    pl = plen.ctypes.data_as(C.POINTER(C.c_int32))
    prompt = ec_inputs.make_prompt(wl.model.vocab, wl.prompt_len, 1)
    pp = prompt.ctypes.data_as(C.POINTER(C.c_int32))
    ws = ec.ec_weights()
    assert lib.ec_init(None, C.byref(mc), C.byref(ws), C.byref(dc), pp, pl, None, 0, None) == ec.EC_ERR_ARG
    assert lib.ec_init(C.byref(ctx), None, C.byref(ws), C.byref(dc), pp, pl, None, 0, None) == ec.EC_ERR_ARG
    assert b"NULL" in lib.ec_last_error(None)
    for field, val in (("head_dim", 48), ("n_kv_heads", 3), ("mask_id", 4096), ("dtype", "x")):
        if field == "dtype":
            bad = ec.model_cfg_struct(wl.model); bad.dtype = 7
        else:
            bad = ec.model_cfg_struct(wl.model.replace(**{field: val}))
        assert lib.ec_init(C.byref(ctx), C.byref(bad), C.byref(ws), C.byref(dc), pp, pl, None, 0,
                           None) == ec.EC_ERR_CONFIG, field
    for field, val in (("batch", 2), ("block", 0), ("block", 129), ("tokens_per_step", 33),
                       ("gen_len", 0), ("k_recent", -1)):
        badd = ec.decode_cfg_struct(wl.decode.replace(**{field: val}))
        assert lib.ec_init(C.byref(ctx), C.byref(mc), C.byref(ws), C.byref(badd), pp, pl, None, 0,
                           None) == ec.EC_ERR_CONFIG, field
    # weights all NULL
    assert lib.ec_init(C.byref(ctx), C.byref(mc), C.byref(ws), C.byref(dc), pp, pl, None, 0, None) == ec.EC_ERR_ARG
    # prompt id outside the vocabulary
    badp = prompt.copy(); badp[3] = wl.model.vocab
    assert lib.ec_init(C.byref(ctx), C.byref(mc), C.byref(ws), C.byref(dc),
                       badp.ctypes.data_as(C.POINTER(C.c_int32)), pl, None, 0, None) == ec.EC_ERR_ARG
    # non-NULL weights but no / short / misaligned workspace
    L = wl.model.n_layers
    arr = (C.c_void_p * L)(*([0x1000] * L))
    for n in ("tok_emb", "lm_head", "final_norm"):
        setattr(ws, n, 0x1000)
    for n in ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down"):
        setattr(ws, n, C.cast(arr, C.POINTER(C.c_void_p)))
    assert lib.ec_init(C.byref(ctx), C.byref(mc), C.byref(ws), C.byref(dc), pp, pl, None, 0, None) == ec.EC_ERR_WORKSPACE
    assert lib.ec_init(C.byref(ctx), C.byref(mc), C.byref(ws), C.byref(dc), pp, pl, C.c_void_p(0x100000), 1024, None) == ec.EC_ERR_WORKSPACE
    assert b"too small" in lib.ec_last_error(None)
    assert lib.ec_init(C.byref(ctx), C.byref(mc), C.byref(ws), C.byref(dc), pp, pl, C.c_void_p(0x100010), 1 << 40, None) == ec.EC_ERR_WORKSPACE
    assert not ctx.value


def test_batch_and_decode_option_checks(lib):
    mc, dc, wl = _cfgs("llada8b_l2")
    ctx = C.c_void_p()
    ws = ec.ec_weights()
    i32p = C.POINTER(C.c_int32)
    plens = np.array([40, 7, 100], dtype=np.int32)
    prompt = ec_inputs.make_prompt(wl.model.vocab, int(plens.sum()), 1)
    pp, pl = prompt.ctypes.data_as(i32p), plens.ctypes.data_as(i32p)
    one = ec.decode_cfg_struct(wl.decode.replace(batch=1))
    three = ec.decode_cfg_struct(wl.decode.replace(batch=3))
    # a batch needs room for every sequence's cache and rows
    n1 = lib.ec_workspace_bytes(C.byref(mc), C.byref(one), pl)
    n3 = lib.ec_workspace_bytes(C.byref(mc), C.byref(three), pl)
    assert n1 > 0 and n3 > n1
    # a valid batch configuration gets past the configuration check (and fails on the weights)
    assert lib.ec_init(C.byref(ctx), C.byref(mc), C.byref(ws), C.byref(three), pp, pl, None, 0,
                       None) == ec.EC_ERR_ARG
    for field, val in (("batch", 0), ("batch", ec.EC_MAX_BATCH + 1), ("conf_threshold", 1.0),
                       ("conf_threshold", -0.1), ("gate_metric", 3), ("schedule", 2)):
        bad = ec.decode_cfg_struct(wl.decode.replace(**{field: val}))
        assert lib.ec_workspace_bytes(C.byref(mc), C.byref(bad), pl) == 0, field
        assert lib.ec_init(C.byref(ctx), C.byref(mc), C.byref(ws), C.byref(bad), pp, pl, None, 0,
                           None) == ec.EC_ERR_CONFIG, field
    # batches run on the bfloat16 path only
    mcf, _, wlf = _cfgs("tiny_f32")
    two = ec.decode_cfg_struct(wlf.decode.replace(batch=2))
    assert lib.ec_init(C.byref(ctx), C.byref(mcf), C.byref(ws), C.byref(two), pp, pl, None, 0,
                       None) == ec.EC_ERR_CONFIG
    assert b"bfloat16" in lib.ec_last_error(None)
    r = ec.ec_step_result()
    assert lib.ec_step_forced_batch(None, pl, pl, pl, pl, C.byref(r)) == ec.EC_ERR_ARG
    assert lib.ec_debug_read_seq(None, 0, 0, 0, None, 0) == ec.EC_ERR_ARG


def test_null_context_calls(lib):
    r = ec.ec_step_result()
    assert lib.ec_step(None, ec.EC_AUTO, C.byref(r)) == ec.EC_ERR_ARG
    assert lib.ec_generate(None, None, None) == ec.EC_ERR_ARG
    assert lib.ec_reset(None, None) == ec.EC_ERR_ARG
    assert lib.ec_profile_enable(None, 1) == ec.EC_ERR_ARG
    assert lib.ec_debug_read(None, 0, 0, None, 0) == ec.EC_ERR_ARG
    lib.ec_destroy(None)
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert len(lib.ec_strerror(code)) > 0


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU program: any other --gpus value ends with a message, before any GPU
    or library work."""
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode == 2
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_row_entropy_argument_errors_without_gpu(lib):
    """The context-free reduction call validates before any HIP work."""
    vp = C.c_void_p
    z, st, ws = vp(0x100000), vp(0x200000), vp(0x300000)
    need = lib.ec_row_entropy_workspace_bytes(32, 126464)
    assert need == 32 * 62 * 16 and need % 256 == 0
    assert lib.ec_row_entropy_workspace_bytes(ec.EC_MAX_BLOCK + 1, 4096) == 0
    assert lib.ec_row_entropy_workspace_bytes(4, 1) == 0
    assert lib.ec_row_entropy_workspace_bytes(4, 163841) == 0
    call = lib.ec_row_entropy
    assert call(None, 4, 4096, 4096, st, ws, need, None) == ec.EC_ERR_ARG
    assert call(z, 4, 4096, 4096, None, ws, need, None) == ec.EC_ERR_ARG
    assert call(z, -1, 4096, 4096, st, ws, need, None) == ec.EC_ERR_ARG
    assert call(z, ec.EC_MAX_BLOCK + 1, 4096, 4096, st, ws, need, None) == ec.EC_ERR_ARG
    assert call(z, 4, 4096, 4095, st, ws, need, None) == ec.EC_ERR_ARG
    assert b"stride" in lib.ec_last_error(None)
    assert call(z, 4, 4096, 4096, vp(0x200004), ws, need, None) == ec.EC_ERR_ARG
    assert call(z, 4, 4096, 4096, st, None, need, None) == ec.EC_ERR_WORKSPACE
    assert call(z, 4, 4096, 4096, st, vp(0x300010), need, None) == ec.EC_ERR_WORKSPACE
    assert call(z, 32, 126464, 126464, st, ws, need - 256, None) == ec.EC_ERR_WORKSPACE
    assert len(lib.ec_strerror(ec.EC_ERR_HOST_MEMORY)) > 0
    assert len(lib.ec_strerror(ec.EC_ERR_NONFINITE)) > 0
