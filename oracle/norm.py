"""Layer normalisation over d_model, forward and backward (test infrastructure only).

The paper does not define it: its Transformer is "as in" the original Transformer paper, where
every sublayer's output is LayerNorm(x + Sublayer(x)).  In the paper's own vocabulary (section
"Operation Implementation") it is two reductions over d_model (paragraph "Reduction": reduce_mean
of x and of the squared deviations) and component-wise operations with implicit broadcasting
(paragraph "Component-wise Operations"; section "Mesh-TensorFlow syntax").  With d_model unsplit -
the data-parallel and the model-parallel layouts of the Transformer - both reductions are local.

Reading taken: y = gain * (x - mean) / sqrt(var + eps) + bias with mean and the *biased* variance
(mean of squared deviations) over d_model, gain[d_model] and bias[d_model] parameters like the
worked example's bias (stored bf16 on the device, their gradients fp32).  `store` marks what the
device keeps in bfloat16: the normalised output y, the incoming gradient dy and the gradient dx.
The statistics (mean, 1/sqrt(var + eps)) stay unrounded (the device keeps them in fp32).

Pins: tests/test_oracle_norm.py (values worked by hand, closed forms, invariances, finite
differences of the backward).
"""
import numpy as np

from .bf16 import round_to_bf16
from .einsum import NT, add_broadcast, reduce

D = "d_model"


def _rows(t):
    return tuple(d for d in t.dims if d != D)


def _mean_over_d(t):
    """reduce_mean over d_model, result broadcastable back against t (d_model kept as size 1)."""
    m = reduce(t, _rows(t), "sum").data / t.data.shape[t.dims.index(D)]
    return np.expand_dims(m, t.dims.index(D))


def _along_d(p, like):
    """A [d_model] parameter shaped to broadcast against `like`."""
    shape = [1] * len(like.dims)
    shape[like.dims.index(D)] = p.data.shape[0]
    return p.data.reshape(shape)


def layer_norm_fwd(x, gain, bias, eps, store=round_to_bf16):
    """x[..., d_model, ...], gain[d_model], bias[d_model] -> dict(y, mean, rstd).
    mean and rstd = 1/sqrt(var + eps) have x's dims without d_model."""
    mean = _mean_over_d(x)
    dev = x.data - mean
    var = _mean_over_d(NT(dev * dev, x.dims))
    rstd = 1.0 / np.sqrt(var + eps)
    y = dev * rstd * _along_d(gain, x) + _along_d(bias, x)
    ax = x.dims.index(D)
    return dict(y=NT(store(y), x.dims), mean=NT(np.squeeze(mean, ax), _rows(x)),
                rstd=NT(np.squeeze(rstd, ax), _rows(x)))


def layer_norm_bwd(x, gain, mean, rstd, dy, store=round_to_bf16):
    """Gradients of sum(y * dy) w.r.t. x, gain and bias, from the saved statistics.
    With xhat = (x - mean) * rstd and g = gain * dy:
      dgain = reduce_sum(dy * xhat -> [d_model]),  dbias = reduce_sum(dy -> [d_model]),
      dx = rstd * (g - mean_d(g) - xhat * mean_d(g * xhat))."""
    ax = x.dims.index(D)
    dy = NT(store(dy.data), dy.dims)
    xhat = (x.data - np.expand_dims(mean.data, ax)) * np.expand_dims(rstd.data, ax)
    dgain = reduce(NT(dy.data * xhat, x.dims), (D,), "sum")
    dbias = reduce(dy, (D,), "sum")
    g = dy.data * _along_d(gain, x)
    c1 = _mean_over_d(NT(g, x.dims))
    c2 = _mean_over_d(NT(g * xhat, x.dims))
    dx = np.expand_dims(rstd.data, ax) * (g - c1 - xhat * c2)
    return dict(dx=NT(store(dx), x.dims), dgain=dgain, dbias=dbias)


def residual_layer_norm_fwd(parts, residual, gain, bias, eps, store=round_to_bf16):
    """The point where a sublayer's partial sums meet again, followed by the normalisation:
    u = residual + sum of `parts` (what the Allreduce and the residual add deliver; stored), then
    layer_norm_fwd(u).  Returns dict(u, y, mean, rstd); the statistics are those of the stored u."""
    u = residual
    for p in parts:
        u = add_broadcast(u, p)
    u = NT(store(u.data), residual.dims)
    out = layer_norm_fwd(u, gain, bias, eps, store)
    out["u"] = u
    return out
