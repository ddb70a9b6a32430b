"""Feed-forward and multi-head-attention sublayers, forward and backward (test infrastructure only).

Every contraction is the named einsum of oracle.einsum, in fp64.  The sublayers are the
two of the model-parallel Transformer (section 'Model-Parallel "Transformer"'): with the
layout ("d_ff" -> mesh, "heads" -> mesh) a processor holds W_in[d_model, d_ff/n],
W_out[d_ff/n, d_model], W_{q,k,v}[d_model, heads/n, d_k] and W_o[heads/n, d_v, d_model];
its outputs y (and dx in backward) contract the split dim and are therefore PARTIAL sums
that the lowering would Allreduce ("Operation Implementation", einsum paragraph; worked
example, "Model-Parallel Layout").  The feed-forward sublayer is the worked example
y = Relu(x w) v without its bias; ffn_bias_* are the example as printed, with it.  Gradients of einsums are einsums ("Data-Parallel
Layout" remarks that parameter gradients are einsums that reduce out batch).

`store` is applied to exactly those tensors the device path keeps in bfloat16 between
einsums (activations); parameter gradients and partial sums stay unrounded (the device
keeps them in fp32).  Pass store=identity for exact mathematics.

Readings (the paper defers the sublayer details to the original Transformer paper):
scaled dot-product attention with an explicit `scale` applied to the logits; softmax over
memory_length with the row maximum subtracted; causal mask = position (l, m) visible iff
m <= l, masked positions get probability exactly 0; relu(0) = 0 with gradient 0 at 0; no
bias, layer norm or dropout; the residual is added after the Allreduce.
"""
import numpy as np

from .bf16 import round_to_bf16
from .einsum import NT, add_broadcast, einsum, reduce

B, L, M, D, F, H, K, V = ("batch", "length", "memory_length", "d_model", "d_ff",
                          "heads", "d_k", "d_v")


def identity(x):
    return x


def _st(t, store):
    return NT(store(t.data), t.dims)


def _rename(t, old, new):
    return NT(t.data, tuple(new if d == old else d for d in t.dims))


# ----------------------------------------------------------------------------- feed-forward

def ffn_fwd(x, w_in, w_out, store=round_to_bf16):
    """x[B,L,D], w_in[D,F], w_out[F,D] -> dict(a=relu(x w_in) [B,L,F], y=a w_out [B,L,D])."""
    h = einsum([x, w_in], (B, L, F))
    a = _st(NT(np.maximum(h.data, 0.0), h.dims), store)
    y = einsum([a, w_out], (B, L, D))
    return dict(a=a, y=y)


def ffn_bwd(x, a, w_in, w_out, dy, store=round_to_bf16):
    """Gradients of sum(y * dy) w.r.t. w_in, w_out and x; `a` is the saved activation and
    carries the ReLU mask (a > 0 exactly where the pre-activation was > 0)."""
    dy = _st(dy, store)
    dw_out = einsum([a, dy], (F, D))
    da = einsum([dy, w_out], (B, L, F))
    dh = _st(NT(np.where(a.data > 0.0, da.data, 0.0), da.dims), store)
    dw_in = einsum([x, dh], (D, F))
    dx = einsum([dh, w_in], (B, L, D))
    return dict(dw_in=dw_in, dw_out=dw_out, dx=dx, dh=dh)


def ffn_bias_fwd(x, w_in, bias, w_out, store=round_to_bf16):
    """The worked example as printed: y = Relu(x w + bias) v, bias[F] broadcast over the token
    dims (section "Example: Two Fully-Connected Layers").  Returns dict(a, y)."""
    h = add_broadcast(einsum([x, w_in], (B, L, F)), bias)
    a = _st(NT(np.maximum(h.data, 0.0), h.dims), store)
    y = einsum([a, w_out], (B, L, D))
    return dict(a=a, y=y)


def ffn_bias_bwd(x, a, w_in, w_out, dy, store=round_to_bf16):
    """ffn_bwd plus dbias: the bias was broadcast over batch and length, so its gradient is the
    reduce_sum of dh over those dims (a reduction that reduces out `batch`, hence an Allreduce
    in the data-parallel layout like the other parameter gradients)."""
    g = ffn_bwd(x, a, w_in, w_out, dy, store)
    g["dbias"] = reduce(g["dh"], (F,), "sum")
    return g


# ----------------------------------------------------------------------------- attention

def _visible(n_l, n_m, causal):
    if not causal:
        return np.ones((n_l, n_m), dtype=bool)
    return np.arange(n_m)[None, :] <= np.arange(n_l)[:, None]


def _softmax_parts(q, k_, scale, causal):
    """e = exp(logits - rowmax) with masked positions 0, tot = row sums, mx = row maxima."""
    s = einsum([q, k_], (B, H, L, M))
    vis = _visible(s.data.shape[2], s.data.shape[3], causal)
    logits = np.where(vis, scale * s.data, -np.inf)
    mx = logits.max(axis=-1, keepdims=True)
    e = np.where(vis, np.exp(logits - mx), 0.0)
    tot = e.sum(axis=-1, keepdims=True)
    return e, tot, mx


def attention_probs(q, k_, scale, causal):
    """logits = scale * einsum(q, k_) [B,H,L,M]; softmax over M.  Returns (p, lse)."""
    e, tot, mx = _softmax_parts(q, k_, scale, causal)
    return NT(e / tot, (B, H, L, M)), NT((mx + np.log(tot))[..., 0], (B, H, L))


def attention_core_fwd(q, k_, v_, scale, causal, store=round_to_bf16):
    """ctx = einsum(softmax(scale * einsum(q, k_)), v_) and lse, from stored q, k_, v_."""
    e, tot, mx = _softmax_parts(q, k_, scale, causal)
    # ctx = einsum(p, v_) with p = e / tot.  The exponentials enter the contraction in
    # storage precision; the row sum that normalises them is taken before rounding.
    ctx_un = einsum([NT(store(e), (B, H, L, M)), v_], (B, L, H, V))
    inv = NT(1.0 / tot[..., 0], (B, H, L))
    ctx = _st(einsum([ctx_un, inv], (B, L, H, V)), store)
    lse = NT((mx + np.log(tot))[..., 0], (B, H, L))
    return ctx, lse


def attention_core_bwd(q, k_, v_, ctx, lse, dctx, scale, causal, store=round_to_bf16):
    """Gradients w.r.t. q, k_, v_ given the (stored) dctx; probabilities are recomputed from the
    logits and lse."""
    s = einsum([q, k_], (B, H, L, M))
    vis = _visible(s.data.shape[2], s.data.shape[3], causal)
    p = NT(np.where(vis, np.exp(scale * s.data - lse.data[..., None]), 0.0), s.dims)
    dp = einsum([dctx, v_], (B, H, L, M))
    # softmax Jacobian: ds = p * (dp - sum_m p*dp); sum_m p*dp = sum_v dctx*ctx
    delta = einsum([dctx, ctx], (B, H, L))
    ds = _st(NT(scale * p.data * (dp.data - delta.data[..., None]), s.dims), store)
    dv_ = _st(einsum([_st(p, store), dctx], (B, M, H, V)), store)
    dq = _st(einsum([ds, k_], (B, L, H, K)), store)
    dk_ = _st(einsum([ds, q], (B, M, H, K)), store)
    return dq, dk_, dv_


def mha_fwd(x, w_q, w_k, w_v, w_o, scale, causal, store=round_to_bf16):
    """Self-attention: memory = x.  Returns q, k, v, ctx, lse (saved) and y [B,L,D]."""
    x_m = _rename(x, L, M)
    q = _st(einsum([x, w_q], (B, L, H, K)), store)
    k_ = _st(einsum([x_m, w_k], (B, M, H, K)), store)
    v_ = _st(einsum([x_m, w_v], (B, M, H, V)), store)
    ctx, lse = attention_core_fwd(q, k_, v_, scale, causal, store)
    y = einsum([ctx, w_o], (B, L, D))
    return dict(q=q, k=k_, v=v_, ctx=ctx, lse=lse, y=y)


def mha_bwd(x, w_q, w_k, w_v, w_o, q, k_, v_, ctx, lse, dy, scale, causal,
            store=round_to_bf16):
    """Gradients of sum(y * dy).  q, k_, v_, ctx, lse are the saved forward tensors; the
    probabilities are recomputed from the logits and lse."""
    x_m = _rename(x, L, M)
    dy = _st(dy, store)
    dw_o = einsum([ctx, dy], (H, V, D))
    dctx = _st(einsum([dy, w_o], (B, L, H, V)), store)
    dq, dk_, dv_ = attention_core_bwd(q, k_, v_, ctx, lse, dctx, scale, causal, store)
    dw_q = einsum([x, dq], (D, H, K))
    dw_k = einsum([x_m, dk_], (D, H, K))
    dw_v = einsum([x_m, dv_], (D, H, V))
    dx = (einsum([dq, w_q], (B, L, D)).data
          + einsum([dk_, w_k], (B, M, D)).data
          + einsum([dv_, w_v], (B, M, D)).data)
    return dict(dw_q=dw_q, dw_k=dw_k, dw_v=dw_v, dw_o=dw_o, dx=NT(dx, (B, L, D)),
                dq=dq, dk=dk_, dv=dv_, dctx=dctx)


# ----------------------------------------------------------------------------- whole layer

def layer_fwd(x, w, scale, causal, store=round_to_bf16):
    """u = x + R(MHA(x)); z = u + R(FFN(u)).  R is the Allreduce point; for the single
    slice computed here it is the identity, so u and z are this processor's partial view.
    w: dict with w_q, w_k, w_v, w_o, w_in, w_out."""
    att = mha_fwd(x, w["w_q"], w["w_k"], w["w_v"], w["w_o"], scale, causal, store)
    u = _st(NT(x.data + att["y"].data, x.dims), store)
    ff = ffn_fwd(u, w["w_in"], w["w_out"], store)
    z = _st(NT(u.data + ff["y"].data, x.dims), store)
    saved = dict(q=att["q"], k=att["k"], v=att["v"], ctx=att["ctx"], lse=att["lse"],
                 u=u, a=ff["a"])
    return dict(z=z, saved=saved, y_mha=att["y"], y_ffn=ff["y"])


def layer_bwd(x, w, saved, dz, scale, causal, store=round_to_bf16):
    dz = _st(dz, store)
    ff = ffn_bwd(saved["u"], saved["a"], w["w_in"], w["w_out"], dz, store)
    du = _st(NT(dz.data + ff["dx"].data, dz.dims), store)
    att = mha_bwd(x, w["w_q"], w["w_k"], w["w_v"], w["w_o"], saved["q"], saved["k"],
                  saved["v"], saved["ctx"], saved["lse"], du, scale, causal, store)
    dx = _st(NT(du.data + att["dx"].data, dz.dims), store)
    return dict(dx=dx, du=du, dw_in=ff["dw_in"], dw_out=ff["dw_out"], dw_q=att["dw_q"],
                dw_k=att["dw_k"], dw_v=att["dw_v"], dw_o=att["dw_o"])
