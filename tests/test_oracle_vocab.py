"""Pins for the oracle's vocabulary-split operations: embedding as an einsum with a one-hot
tensor, logits + softmax cross-entropy written with reduce_max / reduce_sum / einsum."""
import itertools

import numpy as np
import pytest
from scipy.special import log_softmax

from oracle.einsum import nt
from oracle.layout import all_coords, einsum_plan, lowered_einsum, slice_tensor
from oracle import vocab as OV
from oracle.vocab import B, L, D, VOCAB, identity

RNG = np.random.default_rng(20841811)


def _case(b=3, l=4, d=5, v=12):
    x = nt(RNG.standard_normal((b, l, d)), (B, L, D))
    w = nt(RNG.standard_normal((d, v)), (D, VOCAB))
    table = nt(RNG.standard_normal((v, d)), (VOCAB, D))
    ids = RNG.integers(0, v, size=(b, l))
    targets = RNG.integers(0, v, size=(b, l))
    dloss = nt(RNG.standard_normal((b, l)), (B, L))
    return x, w, table, ids, targets, dloss


def test_embedding_is_a_row_gather_and_its_gradient_a_scatter_add():
    x, w, table, ids, _, _ = _case()
    e = OV.embedding_fwd(ids, table)
    np.testing.assert_array_equal(e.data, np.take(table.data, ids, axis=0))       # library routine
    de = nt(RNG.standard_normal(e.data.shape), (B, L, D))
    want = np.zeros_like(table.data)
    np.add.at(want, ids.reshape(-1), de.data.reshape(-1, de.data.shape[-1]))
    np.testing.assert_allclose(OV.embedding_bwd(ids, de, table.data.shape[0]).data, want, atol=1e-13)
    with pytest.raises(ValueError):
        OV.embedding_fwd(np.array([[12]]), table)


def test_loss_matches_library_log_softmax_and_closed_forms():
    x, w, _, _, targets, _ = _case()
    f = OV.xent_fwd(x, w, targets)
    ls = log_softmax(x.data @ w.data, axis=-1)
    want = -np.take_along_axis(ls, targets[..., None], axis=-1)[..., 0]
    np.testing.assert_allclose(f["loss"].data, want, atol=1e-12)
    # equal logits: loss = log(vocab); one dominant logit on the target: loss -> 0
    zero = OV.xent_fwd(x, nt(np.zeros_like(w.data), w.dims), targets)
    np.testing.assert_allclose(zero["loss"].data, np.log(w.data.shape[1]), atol=1e-13)
    xb = nt(np.ones((1, 1, 1)), (B, L, D))
    wb = nt(np.array([[0.0, 50.0, 0.0]]), (D, VOCAB))
    assert OV.xent_fwd(xb, wb, np.array([[1]]))["loss"].data[0, 0] < 1e-20
    # large logits do not overflow (the maximum is subtracted)
    big = OV.xent_fwd(xb, nt(np.array([[1000.0, 999.0]]), (D, VOCAB)), np.array([[0]]))
    assert abs(big["loss"].data[0, 0] - np.log1p(np.exp(-1.0))) < 1e-12


def test_loss_backward_finite_differences():
    x, w, _, _, targets, dloss = _case()
    f = OV.xent_fwd(x, w, targets)
    g = OV.xent_bwd(x, w, targets, f["logits"], f["m"], f["s"], dloss, identity)
    loss = lambda x, w: float((OV.xent_fwd(x, w, targets)["loss"].data * dloss.data).sum())
    eps = 1e-6
    for name, t, grad in (("x", x, g["dx"]), ("w", w, g["dw"])):
        for idx in itertools.islice(np.ndindex(t.data.shape), 0, None, max(1, t.data.size // 9)):
            hi, lo = t.data.copy(), t.data.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args = dict(x=x, w=w)
            fd = (loss(**{**args, name: nt(hi, t.dims)}) - loss(**{**args, name: nt(lo, t.dims)})) / (2 * eps)
            assert abs(fd - grad.data[idx]) < 1e-6 * max(1.0, abs(fd)), (name, idx)
    # each row of dz sums to 0 (softmax minus one-hot), scaled by dloss
    np.testing.assert_allclose(g["dz"].data.sum(axis=-1), 0.0, atol=1e-12)


LAYOUTS = {
    "transformer-model-parallel": ([("all", 4)], [("vocab", "all"), ("d_ff", "all"), ("heads", "all")]),
    "batch-rows-vocab-cols": ([("rows", 3), ("cols", 2)], [("batch", "rows"), ("vocab", "cols")]),
    "replicated": ([("all", 2)], []),
}


@pytest.mark.parametrize("name", sorted(LAYOUTS))
def test_vocab_split_loss_and_embedding_are_layout_independent(name):
    mesh, layout = LAYOUTS[name]
    x, w, table, ids, targets, dloss = _case()
    full = OV.xent_fwd(x, w, targets)
    lowered = OV.lowered_xent_fwd(x, w, targets, mesh, layout)
    for c in all_coords(mesh):
        np.testing.assert_allclose(lowered[c].data, slice_tensor(full["loss"], mesh, layout, c).data, atol=1e-12)
    # embedding: vocab is reduced out, so the local results are partial sums
    e_full = OV.embedding_fwd(ids, table)
    _, e = lowered_einsum([OV.onehot(ids, table.data.shape[0]), table], (B, L, D), mesh, layout)
    for c in all_coords(mesh):
        np.testing.assert_array_equal(e[c].data, slice_tensor(e_full, mesh, layout, c).data)


def test_which_vocab_operations_need_an_allreduce():
    """Model-parallel Transformer layout: logits keep vocab (no Allreduce); the three
    reductions of the loss, the embedding and dx reduce it out (Allreduce over vocab's mesh dim);
    dW reduces out batch (no Allreduce unless batch is split too)."""
    b, l, d, v = 4, 6, 8, 12
    mp = ([("all", 4)], [("vocab", "all"), ("d_ff", "all"), ("heads", "all")])
    two = ([("rows", 2), ("cols", 2)], [("batch", "rows"), ("vocab", "cols")])
    ops = {
        "logits": ([(B, L, D), (D, VOCAB)], [(b, l, d), (d, v)], (B, L, VOCAB)),
        "row statistics": ([(B, L, VOCAB)], [(b, l, v)], (B, L)),
        "embedding": ([(B, L, VOCAB), (VOCAB, D)], [(b, l, v), (v, d)], (B, L, D)),
        "dx": ([(B, L, VOCAB), (D, VOCAB)], [(b, l, v), (d, v)], (B, L, D)),
        "dW": ([(B, L, D), (B, L, VOCAB)], [(b, l, d), (b, l, v)], (D, VOCAB)),
    }
    want = {"logits": ([], []), "row statistics": ([0], [1]), "embedding": ([0], [1]), "dx": ([0], [1]),
            "dW": ([], [0])}
    for name, (ins, sizes, out) in ops.items():
        assert einsum_plan(ins, sizes, out, *mp)["reduce_axes"] == want[name][0], name
        assert einsum_plan(ins, sizes, out, *two)["reduce_axes"] == want[name][1], name
