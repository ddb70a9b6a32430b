"""Pins for the oracle's data-parallel training step (Algorithm 1): hand-worked values, and the
statement the algorithm rests on - the processors' gradients of their sub-batches add up to the
gradient of the whole batch - checked with the feed-forward layer's own backward."""
import numpy as np

from oracle import layer as OL
from oracle import optim as OO
from oracle.einsum import nt
from oracle.layer import B, L, D, F, identity
from oracle.layout import all_coords, slice_tensor

RNG = np.random.default_rng(181102084 + 11)


def test_step_worked_by_hand():
    master = np.array([1.0, -2.0, 0.5])
    grads = [np.array([0.5, 1.0, -1.0]), np.array([1.5, -1.0, 3.0])]          # sum: 2, 0, 2
    new, shadow = OO.sgd_step(master, grads, 0.25, identity)
    assert new.tolist() == [0.5, -2.0, 0.0] and shadow.tolist() == new.tolist()
    assert OO.allreduce_sum(grads).tolist() == [2.0, 0.0, 2.0]
    # a zero learning rate changes nothing; one processor is plain gradient descent
    assert OO.sgd_step(master, grads, 0.0, identity)[0].tolist() == master.tolist()
    assert OO.sgd_step(master, grads[:1], 2.0, identity)[0].tolist() == [0.0, -4.0, 2.5]
    # the copy the einsums read is the rounded master: 1 + 2^-9 is not a bfloat16 value
    new, shadow = OO.sgd_step(np.array([1.0]), [np.array([-(2.0 ** -9)])], 1.0)
    assert new[0] == 1.0 + 2.0 ** -9 and shadow[0] == 1.0


def test_sub_batch_gradients_add_up_to_the_batch_gradient():
    """Data-parallel layout of the worked example: batch split over 4 processors, parameters
    replicated.  Sum over processors of the local parameter gradients = gradient of the full batch,
    hence the same step as on one processor."""
    mesh, layout = [("all", 4)], [("batch", "all")]
    x = nt(RNG.standard_normal((8, 3, 6)), (B, L, D))
    dy = nt(RNG.standard_normal((8, 3, 6)), (B, L, D))
    w_in, w_out = nt(RNG.standard_normal((6, 10)), (D, F)), nt(RNG.standard_normal((10, 6)), (F, D))
    full = OL.ffn_bwd(x, OL.ffn_fwd(x, w_in, w_out, identity)["a"], w_in, w_out, dy, identity)
    parts = {"dw_in": [], "dw_out": []}
    for c in all_coords(mesh):
        xs, dys = slice_tensor(x, mesh, layout, c), slice_tensor(dy, mesh, layout, c)
        g = OL.ffn_bwd(xs, OL.ffn_fwd(xs, w_in, w_out, identity)["a"], w_in, w_out, dys, identity)
        for k in parts:
            parts[k].append(g[k].data)
    for k, w in (("dw_in", w_in), ("dw_out", w_out)):
        assert np.allclose(OO.allreduce_sum(parts[k]), full[k].data, rtol=0, atol=1e-12)
        stepped, _ = OO.sgd_step(w.data, parts[k], 0.1, identity)
        assert np.allclose(stepped, w.data - 0.1 * full[k].data, rtol=0, atol=1e-12)


def test_allreduce_point_with_a_componentwise_operation_worked_by_hand():
    parts = [np.array([1.0, -2.0, 0.5, -0.25]), np.array([0.5, 1.0, -0.5, -0.25])]      # sum: 1.5, -1, 0, -0.5
    assert OO.allreduce_then(parts, store=identity).tolist() == [1.5, -1.0, 0.0, -0.5]
    assert OO.allreduce_then(parts, op="relu", store=identity).tolist() == [1.5, 0.0, 0.0, 0.0]
    # the ReLU gradient: the sum passes where the saved activation is > 0 (0 and -0 block it)
    aux = np.array([2.0, 3.0, 0.0, -0.0])
    assert OO.allreduce_then(parts, op="mask", aux=aux, store=identity).tolist() == [1.5, -1.0, 0.0, 0.0]
    res = np.array([-2.0, 2.0, 1.0, 1.0])
    assert OO.allreduce_then(parts, residual=res, op="relu", store=identity).tolist() == [0.0, 1.0, 1.0, 0.5]
    # relu(sum) is not the sum of relus: the operation follows the Allreduce
    assert OO.allreduce_then(parts, op="relu", store=identity).tolist() != \
        (np.maximum(parts[0], 0) + np.maximum(parts[1], 0)).tolist()
    # storage rounding applies to the result: 1 + 2^-9 rounds to 1 in bfloat16
    assert OO.allreduce_then([np.array([1.0]), np.array([2.0 ** -9])])[0] == 1.0
    # the worked example on the 3-D layout: relu of the Allreduce over the d_model split equals the
    # unsplit hidden layer
    mesh, layout = [("planes", 2)], [("d_model", "planes")]
    x = nt(RNG.standard_normal((2, 3, 8)), (B, L, D))
    w_in = nt(RNG.standard_normal((8, 5)), (D, F))
    from oracle.einsum import einsum
    hs = [einsum([slice_tensor(x, mesh, layout, c), slice_tensor(w_in, mesh, layout, c)], (B, L, F)).data
          for c in all_coords(mesh)]
    want = np.maximum(einsum([x, w_in], (B, L, F)).data, 0.0)
    assert np.allclose(OO.allreduce_then(hs, op="relu", store=identity), want, rtol=0, atol=1e-13)

