"""Vocabulary-split operations of the model-parallel Transformer (test infrastructure only).

Section 'Model-Parallel "Transformer"' splits three dims across the mesh: d_ff, heads and
vocab.  The operations that carry `vocab` are the token embedding and the output layer with its
softmax cross-entropy.  The paper gives no formulas for them (it defers to the original
Transformer); they are written here with the paper's own operations only, so that their lowering
follows from "Operation Implementation":

  embedding   e[b,l,D] = einsum(onehot(ids)[b,l,vocab], E[vocab,D])       vocab reduced out
  logits      z[b,l,vocab] = einsum(x[b,l,D], W[D,vocab])                 vocab kept (split)
  loss        m = reduce_max(z -> [b,l]);  s = reduce_sum(exp(z - m) -> [b,l]);
              t = einsum(onehot(targets)[b,l,vocab], z -> [b,l]);  loss = m + log(s) - t

Every reduction / einsum that reduces out the split `vocab` is followed by an Allreduce (max for
reduce_max, sum otherwise) over the mesh dims vocab maps to.  Gradients are einsums and
component-wise operations again: dz = (exp(z - m) / s - onehot(targets)) * dloss (dloss broadcast
over vocab), dW = einsum(x, dz), dx = einsum(dz, W) (vocab reduced out: partial sums),
dE = einsum(onehot(ids), de).

Readings: ids outside [0, vocab) are an error; logits, the statistics m, s, t and the loss are
kept in fp32 on the device (no rounding here), dz is stored in bf16 (`store`).
"""
import numpy as np

from .bf16 import round_to_bf16
from .einsum import NT, add_broadcast, einsum, reduce

B, L, D, VOCAB = "batch", "length", "d_model", "vocab"


def identity(x):
    return x


def onehot(ids, vocab):
    """ids: integer array [b, l] -> NT [b, l, vocab] with a single 1 per position."""
    ids = np.asarray(ids)
    if ids.size and (ids.min() < 0 or ids.max() >= vocab):
        raise ValueError("id outside the vocabulary")
    out = np.zeros(ids.shape + (vocab,), dtype=np.float64)
    np.put_along_axis(out, ids[..., None], 1.0, axis=-1)
    return NT(out, (B, L, VOCAB))


def embedding_fwd(ids, table):
    """table: NT [vocab, D] -> e [b, l, D]."""
    return einsum([onehot(ids, table.data.shape[0]), table], (B, L, D))


def embedding_bwd(ids, de, vocab):
    """de: NT [b, l, D] -> dE [vocab, D] (rows of tokens that never occur are 0)."""
    return einsum([onehot(ids, vocab), de], (VOCAB, D))


def xent_fwd(x, w, targets):
    """x [b,l,D], w [D,vocab], integer targets [b,l] -> dict(logits, m, s, t, loss)."""
    z = einsum([x, w], (B, L, VOCAB))
    m = reduce(z, (B, L), "max")
    shifted = add_broadcast(z, NT(-m.data, m.dims))
    s = reduce(NT(np.exp(shifted.data), z.dims), (B, L), "sum")
    t = einsum([onehot(targets, w.data.shape[1]), z], (B, L))
    loss = NT(m.data + np.log(s.data) - t.data, (B, L))
    return dict(logits=z, m=m, s=s, t=t, loss=loss)


def xent_bwd(x, w, targets, logits, m, s, dloss, store=round_to_bf16):
    """Gradients of sum(loss * dloss) w.r.t. w and x; logits, m, s are the saved forward tensors."""
    p = np.exp(logits.data - m.data[..., None]) / s.data[..., None]
    dz = NT(store((p - onehot(targets, w.data.shape[1]).data) * dloss.data[..., None]), logits.dims)
    dw = einsum([x, dz], (D, VOCAB))
    dx = einsum([dz, w], (B, L, D))
    return dict(dz=dz, dw=dw, dx=dx)


# ----------------------------------------------------------------------------- on a mesh

def lowered_xent_fwd(x, w, targets, mesh, layout):
    """The loss computed the way the mesh would: every processor's local einsums / reductions on
    its slices, each reduction over the split vocab followed by its Allreduce.  Returns
    dict coord -> NT loss slice [b_local, l]."""
    from .layout import all_coords, lowered_einsum, lowered_reduce, slice_tensor
    vocab = w.data.shape[1]
    _, z = lowered_einsum([x, w], (B, L, VOCAB), mesh, layout)          # vocab kept: local slices
    z_full = einsum([x, w], (B, L, VOCAB))
    for c in all_coords(mesh):                                           # lowered_* work from full tensors
        assert np.allclose(z[c].data, slice_tensor(z_full, mesh, layout, c).data, rtol=0, atol=1e-12)
    _, m = lowered_reduce(z_full, (B, L), "max", mesh, layout)
    m_full = reduce(z_full, (B, L), "max")
    e_full = NT(np.exp(add_broadcast(z_full, NT(-m_full.data, m_full.dims)).data), z_full.dims)
    _, s = lowered_reduce(e_full, (B, L), "sum", mesh, layout)
    _, t = lowered_einsum([onehot(targets, vocab), z_full], (B, L), mesh, layout)
    return {c: NT(m[c].data + np.log(s[c].data) - t[c].data, (B, L)) for c in all_coords(mesh)}
