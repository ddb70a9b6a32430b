"""The data-parallel training step (Algorithm 1, steps 2 and 3) on the device against the oracle:
the sum of the virtual processors' gradients and the parameter update; and one whole step of the
feed-forward layer in the data-parallel layout on a virtual mesh."""
import numpy as np
import pytest
import torch

import mtf_inputs
from helpers import named as to_nt
from oracle import layer as OL
from oracle import optim as OO
from oracle.layer import B, L, D, F
from oracle.metrics import m2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mtf():
    import paper_1811_02084_amd as m
    return m


def f64(t):
    return t.detach().double().cpu().numpy()


@pytest.mark.parametrize("n,count", [(1, 4096), (2, 1 << 20), (3, 1000003), (4, 8 * 1024 * 1024), (7, 12345), (64, 777)])
def test_sgd_step_against_the_oracle(mtf, n, count):
    master = mtf_inputs.normal(81, 0, (count,), 0.05, torch.float32)
    grads = [mtf_inputs.normal(81, 1 + i, (count,), 2.0, torch.float32) for i in range(n)]
    lr = 0.0123
    want_master, want_weights = OO.sgd_step(f64(master), [f64(g) for g in grads], lr)
    dm = master.clone().cuda()
    dw = torch.empty(count, dtype=torch.bfloat16, device="cuda")
    mtf.sgd_step([g.cuda() for g in grads], lr, dm, dw)
    # fp32 arithmetic on identical fp32 inputs: n additions, one multiply-add
    bound = np.abs(f64(master)) + lr * np.sum([np.abs(f64(g)) for g in grads], axis=0)
    assert np.max(np.abs(f64(dm) - want_master) / bound) <= (n + 2) * 2.0 ** -24
    # the copy for the einsums is the device's master rounded to nearest even, and within bf16 of the oracle's
    assert torch.equal(dw, dm.to(torch.bfloat16))
    assert m2(f64(dw), want_weights) <= 2e-2
    # without the bf16 copy
    dm2 = master.clone().cuda()
    mtf.sgd_step([g.cuda() for g in grads], lr, dm2)
    assert torch.equal(dm, dm2)


def test_zero_learning_rate_and_empty(mtf):
    master = mtf_inputs.normal(81, 20, (1000,), 1.0, torch.float32).cuda()
    g = mtf_inputs.normal(81, 21, (1000,), 1.0, torch.float32).cuda()
    before = master.clone()
    mtf.sgd_step([g, g], 0.0, master)
    assert torch.equal(master, before)
    e = torch.empty(0, device="cuda")
    mtf.sgd_step([e], 1.0, e)
    with pytest.raises(mtf.MtfError) as err:
        mtf.sgd_step([g] * 65, 1.0, master)
    assert err.value.name == "MTF_ERR_UNSUPPORTED"


def test_data_parallel_step_of_the_feed_forward_layer(mtf):
    """Batch split over 4 virtual processors, parameters replicated (the data-parallel layout of
    the worked example): every processor runs forward and backward on its sub-batch, the step sums
    the four gradients and updates.  Compared with the oracle's step on the whole batch."""
    cfg = mtf_inputs.ffn_inputs(82, 8, 96, 256, 520, 520)
    lr = 0.05
    xn, dyn = to_nt(cfg["x"], (B, L, D)), to_nt(cfg["dy"], (B, L, D))
    w_in, w_out = to_nt(cfg["w_in"], (D, F)), to_nt(cfg["w_out"], (F, D))
    a_ref = OL.ffn_fwd(xn, w_in, w_out)["a"]
    g_ref = OL.ffn_bwd(xn, a_ref, w_in, w_out, dyn)
    grads = {"dw_in": [], "dw_out": []}
    for p in range(4):
        xs, dys = cfg["x"][2 * p:2 * p + 2].cuda(), cfg["dy"][2 * p:2 * p + 2].cuda()
        a, _ = mtf.ffn_fwd(xs, cfg["w_in"].cuda(), cfg["w_out"].cuda())
        g = mtf.ffn_bwd(xs, a, cfg["w_in"].cuda(), cfg["w_out"].cuda(), dys)
        for k in grads:
            grads[k].append(g[k])
    for k, w in (("dw_in", cfg["w_in"]), ("dw_out", cfg["w_out"])):
        master = w.float().cuda()
        shadow = torch.empty_like(w, device="cuda")
        mtf.sgd_step(grads[k], lr, master, shadow)
        want_master, _ = OO.sgd_step(f64(w), [g_ref[k].data], lr)
        # the update itself against the oracle's full-batch gradient
        step = (f64(w) - f64(master)) / lr
        assert m2(step, g_ref[k].data) <= 2e-2, k
        assert m2(f64(master), want_master) <= 2e-2
        assert torch.equal(shadow, master.to(torch.bfloat16))
