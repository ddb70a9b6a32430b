"""GPU parity tests of the fixed layer steps against the oracle: feed-forward, attention and
whole-layer shards, forward and backward, at small ragged sizes and at the full sizes of the
named workloads (the launch configuration the benchmark times).

Backward calls receive the ORACLE's saved forward tensors as inputs on both sides, so that the
ReLU mask (an integer decision taken from the saved activation) is identical by construction."""
import numpy as np
import pytest
import torch

import mtf_inputs
import paper_1811_02084_amd as mtf
from oracle import layer as OL
from oracle import layout as OLY
from oracle.einsum import NT
from oracle.metrics import m2, rel_l2
from helpers import f64, named, to_dev, on_device, BF16_TOL, F32_TOL, WEIGHT_DIMS
from oracle.layer import B, L, D, F, H, K, V

pytestmark = pytest.mark.gpu


def _check(tag, got, ref, tol=BF16_TOL):
    err = m2(f64(got), ref.data if isinstance(ref, NT) else ref)
    print(f"    {tag}: max rel err {err:.3e}", flush=True)
    assert err <= tol, (tag, err)


def _check_exact(tag, got, stored, exact, tol=BF16_TOL):
    """`got` against exact mathematics (`exact`: the oracle with no storage rounding anywhere), so
    that parity does not rest on the oracle's choice of rounding points alone.  Storing the
    intermediate activations in bf16 is part of the method's precision contract and by itself moves
    a result away from exact mathematics: `stored` is the oracle WITH that rounding, and its own
    distance from `exact` (a pure-oracle number) is the floor no bf16-storing path can beat - at
    2 M outputs behind five stored tensors it exceeds the element-wise bound on its own.  Gates:
    element-wise maximum within floor + bound / 2 (half of what the triangle inequality would allow
    a path that meets the bound against `stored`), and relative l2 error <= bound / 4."""
    floor = m2(stored.data, exact.data)
    err, l2 = m2(f64(got), exact.data), rel_l2(f64(got), exact.data)
    print(f"    {tag} vs exact mathematics: max rel err {err:.3e} (storage-rounding floor {floor:.3e}), "
          f"relative l2 {l2:.3e}", flush=True)
    assert err <= floor + tol / 2, (tag, err, floor)
    assert l2 <= tol / 4, (tag, l2)


def _ffn_case(cfg, label):
    print(f"FFN {label}", flush=True)
    g = on_device(cfg)
    x, w_in, w_out, dy = (named(cfg["x"], (B, L, D)), named(cfg["w_in"], (D, F)), named(cfg["w_out"], (F, D)),
                          named(cfg["dy"], (B, L, D)))
    ref = OL.ffn_fwd(x, w_in, w_out)
    a, y = mtf.ffn_fwd(g["x"], g["w_in"], g["w_out"])
    _check("a", a, ref["a"])
    _check("y_partial", y, ref["y"])
    refb = OL.ffn_bwd(x, ref["a"], w_in, w_out, dy)
    got = mtf.ffn_bwd(g["x"], to_dev(ref["a"], torch.bfloat16), g["w_in"], g["w_out"], g["dy"])
    for k in ("dw_in", "dw_out", "dx"):
        _check(k, got[k], refb[k])


def test_ffn_small_ragged():
    _ffn_case(mtf_inputs.ffn_inputs(21, 3, 100, 264, 520, 4096), "x[3,100,264] d_ff 520")


def test_ffn_config2_full_size():
    _ffn_case(mtf_inputs.config2(), "config 2")


LSE_TOL = 1e-3       # lse is an fp32 statistic of logits built from bf16 q, k (see _mha_case)


def _mha_case(cfg, causal, label, exact_gate=False):
    print(f"MHA {label} causal={causal}", flush=True)
    g = on_device(cfg)
    x = named(cfg["x"], (B, L, D))
    w = {k: named(cfg[k], WEIGHT_DIMS[k]) for k in ("w_q", "w_k", "w_v", "w_o")}
    dy = named(cfg["dy"], (B, L, D))
    ref = OL.mha_fwd(x, w["w_q"], w["w_k"], w["w_v"], w["w_o"], cfg["scale"], causal)
    got = mtf.mha_fwd(g["x"], g["w_q"], g["w_k"], g["w_v"], g["w_o"], cfg["scale"], causal)
    for k in ("q", "k", "v", "ctx", "y"):
        _check(k, got[k], ref[k])
    # lse = max + log(sum exp): fp32 on the device from fp32-accumulated logits of magnitude <= ~10,
    # i.e. absolute errors of a few 1e-6 x |logit| plus exp2/log2 approximations (~1e-6 relative);
    # gated two orders of magnitude below the bf16 bound and well above that arithmetic
    _check("lse", got["lse"], ref["lse"], LSE_TOL)
    if exact_gate:
        # parity must not rest on the oracle's choice of rounding points alone: the same outputs
        # against exact mathematics (no storage rounding anywhere in the oracle), same bound
        exact = OL.mha_fwd(x, w["w_q"], w["w_k"], w["w_v"], w["w_o"], cfg["scale"], causal, OL.identity)
        for k in ("ctx", "y"):
            _check_exact(k, got[k], ref[k], exact[k])
        _check_exact("lse", got["lse"], ref["lse"], exact["lse"], LSE_TOL)
    refb = OL.mha_bwd(x, w["w_q"], w["w_k"], w["w_v"], w["w_o"], ref["q"], ref["k"], ref["v"], ref["ctx"],
                      ref["lse"], dy, cfg["scale"], causal)
    sv = {k: to_dev(ref[k], torch.bfloat16) for k in ("q", "k", "v", "ctx")}
    gotb = mtf.mha_bwd(g["x"], g["w_q"], g["w_k"], g["w_v"], g["w_o"], sv["q"], sv["k"], sv["v"], sv["ctx"],
                       to_dev(ref["lse"], torch.float32), g["dy"], cfg["scale"], causal)
    for k in ("dw_q", "dw_k", "dw_v", "dw_o", "dx"):
        _check(k, gotb[k], refb[k])


@pytest.mark.parametrize("causal", [False, True])
def test_mha_small_ragged(causal):
    _mha_case(mtf_inputs.mha_inputs(22, 2, 200, 264, 3, 128, 24), causal, "x[2,200,264] 3 heads")


def test_mha_single_position_and_one_tile_edge():
    _mha_case(mtf_inputs.mha_inputs(23, 1, 1, 64, 1, 128, 1), True, "length 1")
    _mha_case(mtf_inputs.mha_inputs(24, 1, 65, 64, 1, 128, 1), True, "length 65")


def test_mha_head_width_256():
    """The head width of the paper's language models through the same entry point: ragged, both masks."""
    for causal in (False, True):
        _mha_case(mtf_inputs.mha_inputs(27, 2, 168, 264, 3, 256, 24), causal, "x[2,168,264] 3 heads of width 256")


def test_mha_config3_full_size():
    cfg = mtf_inputs.config3()
    _mha_case(cfg, cfg["causal"], "config 3", exact_gate=True)


def test_attention_closed_forms_on_device():
    """scale = 0 makes every visible logit equal: ctx is the (running, if causal) mean of v."""
    cfg = mtf_inputs.mha_inputs(25, 1, 130, 64, 2, 128, 2)
    g = on_device(cfg)
    for causal in (False, True):
        got = mtf.mha_fwd(g["x"], g["w_q"], g["w_k"], g["w_v"], g["w_o"], 0.0, causal)
        v = f64(got["v"])
        want = np.cumsum(v, axis=1) / np.arange(1, 131)[None, :, None, None] if causal else \
            np.broadcast_to(v.mean(axis=1, keepdims=True), v.shape)
        assert m2(f64(got["ctx"]), want) <= BF16_TOL
        lse = f64(got["lse"])
        want_lse = np.log(np.arange(1, 131)) if causal else np.full(130, np.log(130.0))
        assert np.max(np.abs(lse - want_lse[None, None, :])) <= 1e-4


def _layer_case(cfg, causal, label, exact_gate=False):
    print(f"LAYER {label}", flush=True)
    g = on_device(cfg)
    w = {k: g[k] for k in WEIGHT_DIMS}
    wn = {k: named(cfg[k], WEIGHT_DIMS[k]) for k in WEIGHT_DIMS}
    x, dz = named(cfg["x"], (B, L, D)), named(cfg["dz"], (B, L, D))
    bufs = mtf.layer_alloc(g["x"], w)
    z = mtf.layer_fwd(g["x"], w, cfg["scale"], causal, bufs)
    ref = OL.layer_fwd(x, wn, cfg["scale"], causal)
    _check("z", z, ref["z"])
    for k in ("q", "k", "v", "ctx", "u", "a"):
        _check("saved " + k, bufs["saved"][k], ref["saved"][k])
    _check("saved lse", bufs["saved"]["lse"], ref["saved"]["lse"], LSE_TOL)
    if exact_gate:
        # the same outputs against exact mathematics (oracle without any storage rounding)
        exact = OL.layer_fwd(x, wn, cfg["scale"], causal, OL.identity)
        _check_exact("z", z, ref["z"], exact["z"])
        _check_exact("ctx", bufs["saved"]["ctx"], ref["saved"]["ctx"], exact["saved"]["ctx"])
        _check_exact("u", bufs["saved"]["u"], ref["saved"]["u"], exact["saved"]["u"])
    saved = {k: to_dev(v, torch.float32 if k == "lse" else torch.bfloat16) for k, v in ref["saved"].items()}
    dx = mtf.layer_bwd(g["x"], w, saved, g["dz"], cfg["scale"], causal, bufs)
    refb = OL.layer_bwd(x, wn, ref["saved"], dz, cfg["scale"], causal)
    _check("dx", dx, refb["dx"])
    for k in ("dw_q", "dw_k", "dw_v", "dw_o", "dw_in", "dw_out"):
        _check(k, bufs["grads"][k], refb[k])
    # One step with the device's own saved tensors (what the benchmark runs), all eight outputs.
    # Here the ReLU mask is decided by the device's own `a`, which differs from the oracle's at the
    # few positions whose pre-activation is within rounding of 0.  There a whole term da[t, f] *
    # w_in[:, f] (in du, and through du in everything the attention backward produces) or
    # u[t, :] * da[t, f] (in dw_in) appears or disappears - an isolated deviation that is not small
    # next to sums of a few hundred to a few thousand terms - so the element-wise maximum is not
    # the measure for this pass; the relative l2 error is held to the same bound.  dw_out does not
    # depend on the mask and keeps the element-wise gate.  (With the oracle's saved tensors on both
    # sides, above, every output meets the element-wise bound.)
    mtf.layer_fwd(g["x"], w, cfg["scale"], causal, bufs)
    dx = mtf.layer_bwd(g["x"], w, bufs["saved"], g["dz"], cfg["scale"], causal, bufs)
    outs = dict(dx=dx, **{k: bufs["grads"][k] for k in ("dw_q", "dw_k", "dw_v", "dw_o", "dw_in", "dw_out")})
    for k, t in outs.items():
        err = rel_l2(f64(t), refb[k].data)
        print(f"    {k} (device-saved): relative l2 err {err:.3e}, max rel err {m2(f64(t), refb[k].data):.3e}",
              flush=True)
        assert err <= BF16_TOL, (k, err)
    _check("dw_out (device-saved)", outs["dw_out"], refb["dw_out"])


def test_layer_small_ragged():
    _layer_case(mtf_inputs.layer_inputs(26, 2, 136, 256, 2, 128, 520, 64, 16384), True, "x[2,136,256]")


def test_layer_head_width_256():
    _layer_case(mtf_inputs.layer_inputs(28, 2, 200, 256, 2, 256, 520, 32, 16384), True, "x[2,200,256] 2 heads of width 256")


def test_layer_config5_full_size():
    cfg = mtf_inputs.config5()
    _layer_case(cfg, cfg["causal"], "config 5", exact_gate=True)


def test_rejected_shapes():
    x = torch.zeros(1, 8, 64, dtype=torch.bfloat16, device="cuda")
    wq = torch.zeros(64, 2, 64, dtype=torch.bfloat16, device="cuda")           # d_k = 64: no fused kernel
    wo = torch.zeros(2, 64, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(mtf.MtfError) as e:
        mtf.mha_fwd(x, wq, wq, wq, wo, 1.0, False)
    assert e.value.name == "MTF_ERR_UNSUPPORTED"
