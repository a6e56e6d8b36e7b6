"""The decision costs O(V) and nothing else (Method section, "Entropy-based skipping": the
decision is independent of context length, model depth and hidden dimension; complexity table
of the paper): device time of the vocabulary reduction + decision kernels, from the library's
own HIP events, is flat in T, L and d at a fixed vocabulary and grows linearly with V."""
import numpy as np
import pytest

import ec_inputs
import paper_2603_18489_amd as ec

pytestmark = pytest.mark.gpu


def decision_us(dtype, V, d, L, P, N=64, steps=24):
    """Mean device time per step (microseconds) of the kernel classes vocab_reduce + decide over
    `steps` PARTIAL steps (32 block rows at first), and of the whole step."""
    cfg = ec_inputs.ModelCfg(n_layers=L, d_model=d, n_heads=d // 64, n_kv_heads=d // 64,
                             head_dim=64, d_ffn=2 * d, vocab=V, mask_id=V - 1, rms_eps=1e-5,
                             rope_base=10000.0, logit_scale=12.0, dtype=dtype)
    w = ec_inputs.make_weights(cfg, 3)
    dec = ec_inputs.DecodeCfg(gen_len=N, block=32, k_recent=2, tokens_per_step=1, tau=1e9)
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, w), dec, ec_inputs.make_prompt(V, P, 1))
    try:
        g.step(ec.EC_FULL)
        for _ in range(3):
            g.step(ec.EC_PARTIAL)          # warm-up
        g.profile_enable(True)
        for _ in range(steps):
            g.step(ec.EC_PARTIAL)
        p = g.profile_read()
        g.profile_enable(False)
    finally:
        g.close()
    dec_us = (p["ms"]["vocab_reduce"] + p["ms"]["decide"]) / p["steps"] * 1e3
    return dec_us, sum(p["ms"].values()) / p["steps"] * 1e3


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_decision_time_does_not_depend_on_context_depth_or_width(dtype):
    V = 4096
    base, step_base = decision_us(dtype, V, d=256, L=2, P=192)
    seen = {"base": (base, step_base)}
    for name, kw in (("T x16", dict(d=256, L=2, P=4032)), ("L x4", dict(d=256, L=8, P=192)),
                     ("d x4", dict(d=1024, L=2, P=192))):
        t, step = decision_us(dtype, V, **kw)
        seen[name] = (t, step)
    print(dtype, {k: (round(a, 2), round(b, 1)) for k, (a, b) in seen.items()})
    for name, (t, step) in seen.items():
        assert abs(t - base) <= 0.25 * base, f"{name}: decision {t:.2f} us vs {base:.2f} us"
    # ... while the step around it grows (four times the layers: more than twice the time)
    assert seen["L x4"][1] > 2.0 * step_base


def test_decision_time_is_linear_in_the_vocabulary():
    """float32 path (logits materialised, reduced by vocab_reduce): t(V) = a + b V."""
    Vs = [4096, 32768, 126464]
    ts = [decision_us("f32", V, d=256, L=2, P=192)[0] for V in Vs]
    print(dict(zip(Vs, [round(t, 2) for t in ts])))
    assert ts[0] < ts[1] < ts[2]
    b = (ts[2] - ts[0]) / (Vs[2] - Vs[0])
    predicted_mid = ts[0] + b * (Vs[1] - Vs[0])
    assert abs(predicted_mid - ts[1]) <= 0.25 * ts[1], (predicted_mid, ts[1])
    # the O(V) term is visible above the launch and event overhead, with about the right ratio
    ideal = (Vs[2] - Vs[0]) / (Vs[1] - Vs[0])
    assert ts[2] - ts[0] > 2.0 and 0.5 * ideal <= (ts[2] - ts[0]) / (ts[1] - ts[0]) <= 2.0 * ideal


def test_row_entropy_call_is_linear_in_the_vocabulary():
    import torch
    lib_times = []
    Vs = [8192, 65536, 163840]
    for V in Vs:
        z = torch.randn((32, V), dtype=torch.float32, device="cuda") * 5.0
        out = torch.empty((32, 4), dtype=torch.float32, device="cuda")
        for _ in range(5):
            ec.row_entropy_noalloc(z, out)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(50):
            ec.row_entropy_noalloc(z, out)
        b.record()
        torch.cuda.synchronize()
        lib_times.append(a.elapsed_time(b) / 50 * 1e3)
    print(dict(zip(Vs, [round(t, 2) for t in lib_times])))
    slope = (lib_times[2] - lib_times[0]) / (Vs[2] - Vs[0])
    mid = lib_times[0] + slope * (Vs[1] - Vs[0])
    assert lib_times[0] < lib_times[1] < lib_times[2]
    assert abs(mid - lib_times[1]) <= 0.3 * lib_times[1]
