"""Layer normalisation over d_model on the device against the oracle: forward, the form that first
adds a sublayer's partial sums to the residual, and backward."""
import numpy as np
import pytest
import torch

import mtf_inputs
from helpers import named as to_nt
from oracle import norm as ON
from oracle.metrics import m2

pytestmark = pytest.mark.gpu

B, L, D = "batch", "length", "d_model"
TOL = 2e-2          # bf16-stored outputs (y, u, dx)
STAT_TOL = 1e-5     # fp32 statistics and fp32 parameter gradients from identical bf16 inputs
EPS = 1e-6


@pytest.fixture(scope="module")
def mtf():
    import paper_1811_02084_amd as m
    return m


def f64(t):
    return t.detach().double().cpu().numpy()


def _inputs(seed, b, l, d, shift=0.0, spread=1.0):
    x = (mtf_inputs.normal(61, seed, (b, l, d), 1.0, torch.float32) * spread + shift).to(torch.bfloat16)
    gain = (mtf_inputs.normal(61, seed + 1, (d,), 0.25, torch.float32) + 1.0).to(torch.bfloat16)
    bias = mtf_inputs.normal(61, seed + 2, (d,), 0.5)
    dy = mtf_inputs.normal(61, seed + 3, (b, l, d))
    return x, gain, bias, dy


CASES = [  # batch, length, d_model, shift, spread
    (8, 512, 1024, 0.0, 1.0),       # the layer shard's activations (config 5 token count)
    (2, 37, 1024, 3.0, 0.5),        # rows not a multiple of the waves per workgroup; a large mean
    (3, 5, 8, 0.0, 1.0),            # the smallest row the kernels accept
    (2, 9, 520, -1.0, 2.0),         # a ragged second chunk
    (1, 7, 1536, 0.0, 1.0),         # three of four chunks
    (2, 3, 4096, 0.5, 1.0),         # the widest row
    (1, 1, 256, 0.0, 1.0),
]


@pytest.mark.parametrize("case", CASES, ids=[f"b{c[0]}-l{c[1]}-d{c[2]}" for c in CASES])
def test_layer_norm_forward_backward(mtf, case):
    b, l, d, shift, spread = case
    x, gain, bias, dy = _inputs(10 * d + l, b, l, d, shift, spread)
    xn, gn, bn, dyn = to_nt(x, (B, L, D)), to_nt(gain, (D,)), to_nt(bias, (D,)), to_nt(dy, (B, L, D))
    ref = ON.layer_norm_fwd(xn, gn, bn, EPS)
    y, mean, rstd = mtf.layer_norm_fwd(x.cuda(), gain.cuda(), bias.cuda(), EPS)
    assert m2(f64(y), ref["y"].data) <= TOL
    assert np.max(np.abs(f64(mean) - ref["mean"].data)) <= STAT_TOL * max(1.0, np.max(np.abs(ref["mean"].data)))
    assert np.max(np.abs(f64(rstd) / ref["rstd"].data - 1.0)) <= STAT_TOL
    # backward from the oracle's statistics on both sides
    refb = ON.layer_norm_bwd(xn, gn, ref["mean"], ref["rstd"], dyn)
    mean_s = torch.from_numpy(ref["mean"].data).float().cuda()
    rstd_s = torch.from_numpy(ref["rstd"].data).float().cuda()
    dx, dgain, dbias = mtf.layer_norm_bwd(x.cuda(), gain.cuda(), mean_s, rstd_s, dy.cuda())
    assert m2(f64(dx), refb["dx"].data) <= TOL
    # sums of rows * d products of bf16 inputs in fp32: the bound scales with the sum of magnitudes
    xhat = (f64(x) - ref["mean"].data[..., None]) * ref["rstd"].data[..., None]
    bound_g = np.abs(f64(dy) * xhat).reshape(-1, d).sum(axis=0)
    bound_b = np.abs(f64(dy)).reshape(-1, d).sum(axis=0)
    assert np.max(np.abs(f64(dgain) - refb["dgain"].data) / np.maximum(bound_g, 1e-30)) <= STAT_TOL
    assert np.max(np.abs(f64(dbias) - refb["dbias"].data) / np.maximum(bound_b, 1e-30)) <= STAT_TOL


@pytest.mark.parametrize("n", [1, 2, 3, 4])
def test_residual_form(mtf, n):
    b, l, d = 4, 129, 1024
    x, gain, bias, _ = _inputs(200 + n, b, l, d)
    parts = [mtf_inputs.normal(61, 300 + 10 * n + i, (b, l, d), 0.7, torch.float32) for i in range(n)]
    ref = ON.residual_layer_norm_fwd([to_nt(p, (B, L, D)) for p in parts], to_nt(x, (B, L, D)), to_nt(gain, (D,)),
                                     to_nt(bias, (D,)), EPS)
    dev_parts = [p.cuda() for p in parts]
    u, y, mean, rstd = mtf.residual_layer_norm_fwd(dev_parts, x.cuda(), gain.cuda(), bias.cuda(), EPS)
    assert m2(f64(u), ref["u"].data) <= TOL
    assert m2(f64(y), ref["y"].data) <= TOL
    # the one-pass form is the two-pass composition bit for bit
    u2 = mtf.reduce_partials(dev_parts, residual=x.cuda(), out_dtype=torch.bfloat16)
    y2, mean2, rstd2 = mtf.layer_norm_fwd(u2, gain.cuda(), bias.cuda(), EPS)
    assert torch.equal(u, u2) and torch.equal(y, y2) and torch.equal(mean, mean2) and torch.equal(rstd, rstd2)
    # statistics are those of the stored sum: compare with the oracle run on the device's u
    ref_u = ON.layer_norm_fwd(to_nt(u.cpu(), (B, L, D)), to_nt(gain, (D,)), to_nt(bias, (D,)), EPS)
    assert np.max(np.abs(f64(mean) - ref_u["mean"].data)) <= STAT_TOL
    assert np.max(np.abs(f64(rstd) / ref_u["rstd"].data - 1.0)) <= STAT_TOL


def test_closed_forms_on_device(mtf):
    d = 1024
    gain = (mtf_inputs.normal(61, 400, (d,), 0.25, torch.float32) + 1.0).to(torch.bfloat16).cuda()
    bias = mtf_inputs.normal(61, 401, (d,), 0.5).cuda()
    # constant rows: no deviation, y = bias exactly, rstd = 1/sqrt(eps)
    x = torch.full((3, 4, d), 2.5, dtype=torch.bfloat16, device="cuda")
    y, mean, rstd = mtf.layer_norm_fwd(x, gain, bias, 1e-4)
    assert torch.equal(y, bias.expand(3, 4, d))
    assert torch.all(mean == 2.5) and torch.allclose(rstd, torch.full_like(rstd, 100.0), rtol=1e-6)
    # +-1 alternating with eps = 0: mean 0, variance 1, y = gain * x + bias
    x = torch.tensor([1.0, -1.0], device="cuda").repeat(d // 2).to(torch.bfloat16).reshape(1, 1, d)
    y, mean, rstd = mtf.layer_norm_fwd(x, gain, bias, 0.0)
    want = (gain.float() * x.float() + bias.float()).to(torch.bfloat16)
    assert torch.equal(y, want) and float(mean) == 0.0 and float(rstd) == 1.0
    # no rows: nothing to do, dgain = dbias = 0
    e = torch.empty((0, 4, d), dtype=torch.bfloat16, device="cuda")
    y, mean, rstd = mtf.layer_norm_fwd(e, gain, bias, 1e-6)
    dx, dgain, dbias = mtf.layer_norm_bwd(e, gain, mean, rstd, e)
    assert dx.numel() == 0 and float(dgain.abs().max()) == 0.0 and float(dbias.abs().max()) == 0.0


def test_backward_is_reproducible(mtf):
    x, gain, bias, dy = (t.cuda() for t in _inputs(500, 8, 300, 1024))
    _, mean, rstd = mtf.layer_norm_fwd(x, gain, bias, EPS)
    a = mtf.layer_norm_bwd(x, gain, mean, rstd, dy)
    b = mtf.layer_norm_bwd(x, gain, mean, rstd, dy)
    assert all(torch.equal(p, q) for p, q in zip(a, b))


def test_rejected_shapes(mtf):
    gain = torch.ones(4100, dtype=torch.bfloat16, device="cuda")
    for d in (12, 4104):          # not a multiple of 8; wider than the kernels keep in registers
        x = torch.zeros((2, d), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(mtf.MtfError) as e:
            mtf.layer_norm_fwd(x, gain, gain, 1e-6)
        assert e.value.name == "MTF_ERR_UNSUPPORTED"
    x = torch.zeros((2, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(mtf.MtfError) as e:
        mtf.layer_norm_fwd(x, gain, gain, -1.0)
    assert e.value.name == "MTF_ERR_UNSUPPORTED"
    with pytest.raises(mtf.MtfError) as e:
        mtf.residual_layer_norm_fwd([torch.zeros((2, 64), device="cuda")] * 5, x, gain, gain, 1e-6)
    assert e.value.name == "MTF_ERR_UNSUPPORTED"
