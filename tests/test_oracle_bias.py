"""Pins for the oracle's reduction, broadcasting addition and the worked example with its bias
(y = Relu(x w + bias) v): plain loops, special cases that fall back on other routines, finite
differences, the example's printed slice shapes and Allreduce volumes with the bias counted."""
import itertools

import numpy as np
import pytest

from oracle.einsum import EinsumError, add_broadcast, einsum, einsum_definition, nt, reduce
from oracle.layout import (all_coords, einsum_plan, lowered_add_broadcast, lowered_einsum,
                           lowered_reduce, slice_spec, slice_tensor)
from oracle import layer as OL
from oracle.layer import B, L, D, F, identity

RNG = np.random.default_rng(181102084)


# ------------------------------------------------------------------ add_broadcast
def test_add_broadcast_plain_loops_any_position():
    big = nt(RNG.standard_normal((2, 3, 4)), ("p", "q", "r"))
    for dims in [("r",), ("q",), ("p",), ("q", "r"), ("r", "p"), ("p", "q", "r"), ()]:
        small = nt(RNG.standard_normal([dict(p=2, q=3, r=4)[d] for d in dims]), dims)
        for got in (add_broadcast(big, small), add_broadcast(small, big)):
            assert got.dims == big.dims
            for i, j, k in itertools.product(range(2), range(3), range(4)):
                at = dict(p=i, q=j, r=k)
                want = big.data[i, j, k] + small.data[tuple(at[d] for d in dims)]
                assert got.data[i, j, k] == want


def test_add_broadcast_rejects_non_subset_and_size_mismatch():
    a = nt(np.zeros((2, 3)), ("p", "q"))
    with pytest.raises(EinsumError) as e:
        add_broadcast(a, nt(np.zeros((2, 4)), ("p", "r")))
    assert e.value.code == "NOT_BROADCASTABLE"
    with pytest.raises(EinsumError) as e:
        add_broadcast(a, nt(np.zeros(4), ("q",)))
    assert e.value.code == "SIZE_MISMATCH"


# ------------------------------------------------------------------ reduce
def test_reduce_plain_loops_and_einsum_special_case():
    t = nt(RNG.standard_normal((3, 4, 5)), ("p", "q", "r"))
    for out in [("q",), ("r", "p"), ("p", "q", "r"), (), ("q", "p")]:
        s, m = reduce(t, out, "sum"), reduce(t, out, "max")
        assert s.dims == tuple(out) and m.dims == tuple(out)
        for idx in itertools.product(*[range(dict(p=3, q=4, r=5)[d]) for d in out]):
            fixed = dict(zip(out, idx))
            vals = [t.data[i, j, k] for i, j, k in itertools.product(range(3), range(4), range(5))
                    if all(dict(p=i, q=j, r=k)[d] == v for d, v in fixed.items())]
            assert abs(s.data[idx] - sum(vals)) < 1e-12
            assert m.data[idx] == max(vals)
        # a sum-reduction is the one-operand einsum
        np.testing.assert_allclose(s.data, einsum_definition([t], out).data, atol=1e-12)


def test_reduce_rejects_new_dims():
    with pytest.raises(EinsumError) as e:
        reduce(nt(np.zeros((2, 3)), ("p", "q")), ("z",))
    assert e.value.code == "OUT_NOT_SUBSET"


def test_lowered_reduce_is_layout_independent():
    """Local reduction + Allreduce over the mesh dims of reduced-out split dims gives every
    processor its slice of the unsplit result, for sum and for max."""
    t = nt(RNG.integers(-9, 10, size=(4, 6, 8)).astype(np.float64), ("batch", "hidden", "io"))
    mesh = [("rows", 2), ("cols", 2)]
    for layout in ([("batch", "rows"), ("hidden", "cols")], [("io", "cols")], [("batch", "cols"), ("io", "rows")], []):
        for out in (("hidden",), ("io", "batch"), ()):
            for op in ("sum", "max"):
                full = reduce(t, out, op)
                _, red = lowered_reduce(t, out, op, mesh, layout)
                for c in all_coords(mesh):
                    want = slice_tensor(full, mesh, layout, c)
                    assert np.array_equal(red[c].data, want.data), (layout, out, op, c)


# ------------------------------------------------------------------ the worked example with bias
def _example(b=4, d_io=3, d_h=6, ints=False):
    draw = (lambda *s: RNG.integers(-2, 3, size=s).astype(np.float64)) if ints else (lambda *s: RNG.standard_normal(s))
    x = nt(draw(b, 1, d_io), (B, L, D))
    w = nt(draw(d_io, d_h), (D, F))
    bias = nt(draw(d_h), (F,))
    v = nt(draw(d_h, d_io), (F, D))
    dy = nt(draw(b, 1, d_io), (B, L, D))
    return x, w, bias, v, dy


def test_ffn_bias_forward_plain_loops_and_zero_bias_special_case():
    x, w, bias, v, _ = _example()
    got = OL.ffn_bias_fwd(x, w, bias, v, identity)
    b, _, d = x.data.shape
    f = w.data.shape[1]
    for i in range(b):
        hid = [max(sum(x.data[i, 0, t] * w.data[t, u] for t in range(d)) + bias.data[u], 0.0) for u in range(f)]
        np.testing.assert_allclose(got["a"].data[i, 0], hid, atol=1e-13)
        for t in range(d):
            assert abs(got["y"].data[i, 0, t] - sum(hid[u] * v.data[u, t] for u in range(f))) < 1e-12
    zero = nt(np.zeros(f), (F,))
    np.testing.assert_array_equal(OL.ffn_bias_fwd(x, w, zero, v, identity)["y"].data,
                                  OL.ffn_fwd(x, w, v, identity)["y"].data)


def test_ffn_bias_backward_finite_differences():
    x, w, bias, v, dy = _example()
    fwd = OL.ffn_bias_fwd(x, w, bias, v, identity)
    g = OL.ffn_bias_bwd(x, fwd["a"], w, v, dy, identity)
    loss = lambda x, w, bias, v: float((OL.ffn_bias_fwd(x, w, bias, v, identity)["y"].data * dy.data).sum())
    eps = 1e-6
    for name, t, grad in (("x", x, g["dx"]), ("w", w, g["dw_in"]), ("bias", bias, g["dbias"]), ("v", v, g["dw_out"])):
        for idx in itertools.islice(np.ndindex(t.data.shape), 0, None, max(1, t.data.size // 7)):
            hi, lo = t.data.copy(), t.data.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args = dict(x=x, w=w, bias=bias, v=v)
            fd = (loss(**{**args, name: nt(hi, t.dims)}) - loss(**{**args, name: nt(lo, t.dims)})) / (2 * eps)
            assert abs(fd - grad.data[idx]) < 1e-6 * max(1.0, abs(fd)), (name, idx)
    # dbias is the column sum of dh
    np.testing.assert_allclose(g["dbias"].data, g["dh"].data.sum(axis=(0, 1)), atol=1e-12)


EXAMPLE_LAYOUTS = {
    "data-parallel": ([("all", 4)], [("batch", "all")]),
    "model-parallel": ([("all", 2)], [("d_ff", "all")]),
    "data+model": ([("rows", 2), ("cols", 2)], [("batch", "rows"), ("d_ff", "cols")]),
    "three-dimensional": ([("rows", 2), ("cols", 2), ("planes", 3)],
                          [("batch", "rows"), ("d_ff", "cols"), ("d_model", "planes")]),
    "replicated": ([("all", 3)], []),
}


@pytest.mark.parametrize("name", sorted(EXAMPLE_LAYOUTS))
def test_example_with_bias_gives_identical_results_in_every_layout(name):
    """The section's claim for its layouts ("Each will produce identical results"), with the bias:
    forward and every gradient, integers so that equality is exact."""
    mesh, layout = EXAMPLE_LAYOUTS[name]
    x, w, bias, v, dy = _example(b=4, d_io=3, d_h=6, ints=True)
    full = OL.ffn_bias_fwd(x, w, bias, v, identity)
    gfull = OL.ffn_bias_bwd(x, full["a"], w, v, dy, identity)
    _, xw = lowered_einsum([x, w], (B, L, F), mesh, layout)
    a_loc = {}
    for c in all_coords(mesh):
        h = add_broadcast(xw[c], slice_tensor(bias, mesh, layout, c))
        a_loc[c] = nt(np.maximum(h.data, 0.0), h.dims)
        assert np.array_equal(a_loc[c].data, slice_tensor(full["a"], mesh, layout, c).data)
    # lowered_* take full tensors; re-assemble `a` from the slices just checked
    a_full = full["a"]
    _, y = lowered_einsum([a_full, v], (B, L, D), mesh, layout)
    _, dbias = lowered_reduce(gfull["dh"], (F,), "sum", mesh, layout)
    _, dw = lowered_einsum([x, gfull["dh"]], (D, F), mesh, layout)
    for c in all_coords(mesh):
        assert np.array_equal(y[c].data, slice_tensor(full["y"], mesh, layout, c).data)
        assert np.array_equal(dbias[c].data, slice_tensor(gfull["dbias"], mesh, layout, c).data)
        assert np.array_equal(dw[c].data, slice_tensor(gfull["dw_in"], mesh, layout, c).data)
    # the addition itself, lowered: every processor adds its slices and holds its slice of h
    h_full = add_broadcast(einsum([x, w], (B, L, F)), bias)
    h_loc = lowered_add_broadcast(einsum([x, w], (B, L, F)), bias, mesh, layout)
    for c in all_coords(mesh):
        assert np.array_equal(h_loc[c].data, slice_tensor(h_full, mesh, layout, c).data)


def test_example_slices_and_allreduce_volumes_with_bias():
    """Model-parallel layout: w, v and bias are split across the hidden dim (bias slice
    [d_h/n]).  Data-parallel layout: every parameter gradient reduces out batch, so the values
    allreduced per processor are the parameters: 2 d_io d_h for w and v plus d_h for the bias -
    the text's "approximately 2 d_io d_h"."""
    b, d_io, d_h, n = 8, 5, 12, 4
    mp_mesh, mp = [("all", n)], [("d_ff", "all")]
    assert slice_spec((F,), (d_h,), mp_mesh, mp, (1,)) == ((d_h // n,), (d_h // n,))
    assert slice_spec((D, F), (d_io, d_h), mp_mesh, mp, (2,))[1] == (d_io, d_h // n)
    dp_mesh, dp = [("all", n)], [("batch", "all")]
    grads = {  # gradient -> (operand dims, operand sizes, output dims)
        "dw": ([(B, D), (B, F)], [(b, d_io), (b, d_h)], (D, F)),
        "dv": ([(B, F), (B, D)], [(b, d_h), (b, d_io)], (F, D)),
        "dbias": ([(B, F)], [(b, d_h)], (F,)),
    }
    volume = 0
    for ins, sizes, out in grads.values():
        plan = einsum_plan(ins, sizes, out, dp_mesh, dp)
        assert plan["reduce_axes"] == [0]
        volume += int(np.prod(plan["local_out"]))
    assert volume == 2 * d_io * d_h + d_h
    # model-parallel: the bias gradient is split, nothing to allreduce
    assert einsum_plan([(B, F)], [(b, d_h)], (F,), mp_mesh, mp)["reduce_axes"] == []
