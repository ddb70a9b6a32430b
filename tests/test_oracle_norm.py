"""Pins for the oracle's layer normalisation: values worked by hand, closed forms, the invariances
the definition implies, plain loops, and finite differences / adjoint identities of the backward."""
import math

import numpy as np

from oracle.einsum import nt
from oracle import norm as ON
from oracle.layer import identity

RNG = np.random.default_rng(181102084 + 7)
B, L, D = "batch", "length", "d_model"


def test_forward_values_worked_by_hand():
    # x = [1, 2, 3, 4]: mean 2.5, squared deviations 2.25, 0.25, 0.25, 2.25 -> variance 1.25;
    # deviations / sqrt(1.25) = -3/sqrt(5), -1/sqrt(5), 1/sqrt(5), 3/sqrt(5)
    x = nt(np.array([[1.0, 2.0, 3.0, 4.0]]), (B, D))
    gain, bias = nt(np.array([1.0, 2.0, 3.0, 4.0]), (D,)), nt(np.array([0.5, 0.0, -0.5, 1.0]), (D,))
    r = ON.layer_norm_fwd(x, gain, bias, 0.0, identity)
    s5 = math.sqrt(5.0)
    want = [1.0 * -3 / s5 + 0.5, 2.0 * -1 / s5, 3.0 * 1 / s5 - 0.5, 4.0 * 3 / s5 + 1.0]
    assert np.allclose(r["y"].data[0], want, rtol=0, atol=1e-15)
    assert r["mean"].data[0] == 2.5 and r["mean"].dims == (B,)
    assert abs(r["rstd"].data[0] - 1.0 / math.sqrt(1.25)) < 1e-15
    # with eps: variance 1.25 + 0.75 = 2 under the root
    r = ON.layer_norm_fwd(x, gain, bias, 0.75, identity)
    assert abs(r["rstd"].data[0] - 1.0 / math.sqrt(2.0)) < 1e-15
    assert abs(r["y"].data[0, 3] - (4.0 * 1.5 / math.sqrt(2.0) + 1.0)) < 1e-15


def test_closed_forms():
    gain, bias = nt(RNG.standard_normal(6), (D,)), nt(RNG.standard_normal(6), (D,))
    # a constant row has no deviation: y = bias whatever the gain (eps keeps the root finite)
    x = nt(np.full((2, 3, 6), 7.25), (B, L, D))
    r = ON.layer_norm_fwd(x, gain, bias, 1e-6, identity)
    assert np.array_equal(r["y"].data, np.broadcast_to(bias.data, (2, 3, 6)))
    assert np.array_equal(r["rstd"].data, np.full((2, 3), 1e3))
    # +-1 alternating: mean 0, variance 1, y = gain * x + bias
    x = nt(np.tile([1.0, -1.0], 3)[None, :], (B, D))
    r = ON.layer_norm_fwd(x, gain, bias, 0.0, identity)
    assert np.allclose(r["y"].data[0], gain.data * x.data[0] + bias.data, rtol=0, atol=1e-15)
    # unit gain, zero bias: every row of y has mean 0 and mean square var / (var + eps)
    x = nt(RNG.standard_normal((4, 5, 16)) * 3 + 2, (B, L, D))
    one, zero = nt(np.ones(16), (D,)), nt(np.zeros(16), (D,))
    r = ON.layer_norm_fwd(x, one, zero, 0.0, identity)
    assert np.max(np.abs(r["y"].data.mean(axis=2))) < 1e-14
    assert np.max(np.abs((r["y"].data ** 2).mean(axis=2) - 1.0)) < 1e-13


def test_forward_against_plain_loops_any_position_of_d_model():
    x = nt(RNG.standard_normal((3, 5, 4)), (B, D, L))          # d_model in the middle
    gain, bias = nt(RNG.standard_normal(5), (D,)), nt(RNG.standard_normal(5), (D,))
    eps = 1e-3
    r = ON.layer_norm_fwd(x, gain, bias, eps, identity)
    assert r["mean"].dims == (B, L)
    for b in range(3):
        for l in range(4):
            row = [x.data[b, d, l] for d in range(5)]
            mean = sum(row) / 5
            var = sum((v - mean) ** 2 for v in row) / 5
            for d in range(5):
                want = gain.data[d] * (row[d] - mean) / math.sqrt(var + eps) + bias.data[d]
                assert abs(r["y"].data[b, d, l] - want) < 1e-14
            assert abs(r["mean"].data[b, l] - mean) < 1e-15


def test_invariance_to_shift_and_positive_scale():
    x = nt(RNG.standard_normal((2, 7, 12)), (B, L, D))
    gain, bias = nt(RNG.standard_normal(12), (D,)), nt(RNG.standard_normal(12), (D,))
    y = ON.layer_norm_fwd(x, gain, bias, 0.0, identity)["y"].data
    y2 = ON.layer_norm_fwd(nt(x.data * 3.5 + 11.0, x.dims), gain, bias, 0.0, identity)["y"].data
    assert np.max(np.abs(y - y2)) < 1e-12
    # a negative scale flips the normalised deviations
    y3 = ON.layer_norm_fwd(nt(-x.data, x.dims), gain, nt(np.zeros(12), (D,)), 0.0, identity)["y"].data
    assert np.max(np.abs(y3 + (y - bias.data))) < 1e-12


def _loss(x, gain, bias, dy, eps):
    return float(np.sum(ON.layer_norm_fwd(x, gain, bias, eps, identity)["y"].data * dy.data))


def test_backward_finite_differences():
    eps = 1e-5
    x = nt(RNG.standard_normal((2, 3, 8)), (B, L, D))
    gain, bias = nt(RNG.standard_normal(8) + 1.0, (D,)), nt(RNG.standard_normal(8), (D,))
    dy = nt(RNG.standard_normal((2, 3, 8)), (B, L, D))
    f = ON.layer_norm_fwd(x, gain, bias, eps, identity)
    g = ON.layer_norm_bwd(x, gain, f["mean"], f["rstd"], dy, identity)
    h = 1e-6
    for name, t in (("dx", x), ("dgain", gain), ("dbias", bias)):
        num = np.zeros_like(t.data)
        it = np.nditer(t.data, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            keep = t.data[i]
            t.data[i] = keep + h
            up = _loss(x, gain, bias, dy, eps)
            t.data[i] = keep - h
            dn = _loss(x, gain, bias, dy, eps)
            t.data[i] = keep
            num[i] = (up - dn) / (2 * h)
        assert np.max(np.abs(num - g[name].data)) < 1e-7, name


def test_backward_identities():
    x = nt(RNG.standard_normal((3, 4, 10)), (B, L, D))
    gain = nt(RNG.standard_normal(10), (D,))
    dy = nt(RNG.standard_normal((3, 4, 10)), (B, L, D))
    f = ON.layer_norm_fwd(x, gain, nt(np.zeros(10), (D,)), 0.0, identity)
    g = ON.layer_norm_bwd(x, gain, f["mean"], f["rstd"], dy, identity)
    # y does not change when a row of x is shifted or (eps = 0) scaled: dx is orthogonal to the
    # constant row and to the row's deviations
    assert np.max(np.abs(g["dx"].data.sum(axis=2))) < 1e-13
    dev = x.data - x.data.mean(axis=2, keepdims=True)
    assert np.max(np.abs((g["dx"].data * dev).sum(axis=2))) < 1e-13
    # two positions: the normalised row is always (+-1, -+1), so no gradient reaches x
    x2 = nt(RNG.standard_normal((5, 2)), (B, D))
    f2 = ON.layer_norm_fwd(x2, nt(np.array([2.0, -3.0]), (D,)), nt(np.zeros(2), (D,)), 0.0, identity)
    g2 = ON.layer_norm_bwd(x2, nt(np.array([2.0, -3.0]), (D,)), f2["mean"], f2["rstd"],
                           nt(RNG.standard_normal((5, 2)), (B, D)), identity)
    assert np.max(np.abs(g2["dx"].data)) < 1e-13
    # dbias is the plain sum of dy over the rows; dgain the sum of dy * normalised deviation
    assert np.allclose(g["dbias"].data, dy.data.reshape(-1, 10).sum(axis=0), rtol=0, atol=1e-13)
    xhat = dev / np.sqrt((dev ** 2).mean(axis=2, keepdims=True))
    assert np.allclose(g["dgain"].data, (dy.data * xhat).reshape(-1, 10).sum(axis=0), rtol=0, atol=1e-12)


def test_residual_form_is_the_sum_then_the_normalisation():
    res = nt(RNG.standard_normal((2, 3, 8)), (B, L, D))
    parts = [nt(RNG.standard_normal((2, 3, 8)), (B, L, D)) for _ in range(3)]
    gain, bias = nt(RNG.standard_normal(8), (D,)), nt(RNG.standard_normal(8), (D,))
    r = ON.residual_layer_norm_fwd(parts, res, gain, bias, 1e-6, identity)
    u = res.data + parts[0].data + parts[1].data + parts[2].data
    assert np.allclose(r["u"].data, u, rtol=0, atol=1e-15)
    want = ON.layer_norm_fwd(nt(u, (B, L, D)), gain, bias, 1e-6, identity)
    assert np.allclose(r["y"].data, want["y"].data, rtol=0, atol=1e-14)
    # with storage rounding the statistics are those of the *stored* sum
    from oracle.bf16 import round_to_bf16
    r = ON.residual_layer_norm_fwd(parts, res, gain, bias, 1e-6)
    assert np.array_equal(r["u"].data, round_to_bf16(u))
    assert np.allclose(r["mean"].data, round_to_bf16(u).mean(axis=2), rtol=0, atol=1e-15)
