"""Pins for the oracle's named einsum (section "Operation Implementation", einsum paragraph):
pure-Python loops over the whole iteration space, textbook special cases, the all-ones
closed form, exact integer evaluation, linearity, and the error cases."""
import itertools
import random

import numpy as np
import pytest

import oracle.einsum as E
from oracle.einsum import nt, einsum, einsum_definition, einsum_abs, EinsumError, flops


def loops_einsum(inputs, out_dims):
    """Every point of the iteration space visited once; exact Python arithmetic on the
    values given (ints stay ints)."""
    sizes = {}
    for data, dims in inputs:
        for d, n in zip(dims, np.shape(data)):
            sizes[d] = n
    names = list(sizes)
    out = {}
    for point in itertools.product(*[range(sizes[d]) for d in names]):
        at = dict(zip(names, point))
        term = 1
        for data, dims in inputs:
            term = term * data[tuple(at[d] for d in dims)]
        key = tuple(at[d] for d in out_dims)
        out[key] = out.get(key, 0) + term
    res = np.zeros([sizes[d] for d in out_dims], dtype=object)
    for key, v in out.items():
        res[key] = v
    return res


def both_paths(inputs, out_dims):
    """Result of the written-out definition and of the large-size path (numpy.einsum)."""
    a = einsum_definition(inputs, out_dims)
    old = E._DEFINITION_LIMIT
    E._DEFINITION_LIMIT = 0
    try:
        b = einsum(inputs, out_dims)
    finally:
        E._DEFINITION_LIMIT = old
    assert a.dims == b.dims == tuple(out_dims)
    return a.data, b.data


def test_matmul_triple_loop():
    rng = np.random.default_rng(0)
    a, b = rng.standard_normal((5, 7)), rng.standard_normal((7, 3))
    want = np.zeros((5, 3))
    for i in range(5):
        for j in range(3):
            for k in range(7):
                want[i, j] += a[i, k] * b[k, j]
    for got in both_paths([nt(a, "ik"), nt(b, "kj")], "ij"):
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)
    # transposed output must be the transposed matrix, not a reinterpretation
    for got in both_paths([nt(a, "ik"), nt(b, "kj")], "ji"):
        np.testing.assert_allclose(got, want.T, rtol=1e-13, atol=1e-13)


def test_special_cases():
    rng = np.random.default_rng(1)
    a, b = rng.standard_normal((2, 3, 4)), rng.standard_normal((2, 4, 5))
    want = np.stack([a[i] @ b[i] for i in range(2)])
    for got in both_paths([nt(a, "bik"), nt(b, "bkj")], "bij"):          # batched matmul
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)
    u, v = rng.standard_normal(4), rng.standard_normal(6)
    for got in both_paths([nt(u, "i"), nt(v, "j")], "ij"):                # outer product
        np.testing.assert_allclose(got, np.outer(u, v), rtol=1e-14)
    for got in both_paths([nt(a, "bik")], "i"):                           # reduce_sum
        np.testing.assert_allclose(got, a.sum(axis=(0, 2)), rtol=1e-13)
    for got in both_paths([nt(a, "bik")], "kbi"):                         # pure transpose
        assert np.array_equal(got, a.transpose(2, 0, 1))
    for got in both_paths([nt(u, "i"), nt(u, "i")], ""):                  # dot product
        np.testing.assert_allclose(got, np.dot(u, u), rtol=1e-14)
    c = rng.standard_normal(5)
    for got in both_paths([nt(a, "bik"), nt(c, "j")], "bj"):              # broadcast + reduce
        np.testing.assert_allclose(got, np.outer(a.sum(axis=(1, 2)), c), rtol=1e-13)


def test_random_named_shapes_against_loops_exact_integers():
    rnd = random.Random(3)
    names = ["batch", "length", "d_model", "d_ff", "heads", "d_k"]
    for trial in range(40):
        sizes = {d: rnd.randint(1, 4) for d in names}
        da = rnd.sample(names, rnd.randint(1, 4))
        db = rnd.sample(names, rnd.randint(1, 4))
        pool = list(dict.fromkeys(da + db))
        out = rnd.sample(pool, rnd.randint(0, len(pool)))
        rng = np.random.default_rng(trial)
        a = rng.integers(-3, 4, [sizes[d] for d in da])
        b = rng.integers(-3, 4, [sizes[d] for d in db])
        want = loops_einsum([(a, da), (b, db)], out).astype(np.int64)
        for got in both_paths([nt(a, da), nt(b, db)], out):
            assert got.shape == want.shape
            assert np.array_equal(got, want.astype(np.float64)), (da, db, out)


def test_all_ones_closed_form():
    a = nt(np.ones((3, 4, 5)), ("batch", "length", "d_model"))
    b = nt(np.ones((5, 6)), ("d_model", "d_ff"))
    for got in both_paths([a, b], ("batch", "d_ff")):
        assert np.array_equal(got, np.full((3, 6), 4 * 5.0))
    for got in both_paths([a, b], ()):
        assert got == 3 * 4 * 5 * 6
    assert flops([a, b]) == 2 * 3 * 4 * 5 * 6


def test_three_operands_and_linearity():
    rng = np.random.default_rng(5)
    a, a2 = rng.standard_normal((3, 4)), rng.standard_normal((3, 4))
    b, c = rng.standard_normal((4, 5)), rng.standard_normal((5, 2))
    got = einsum_definition([nt(a, "ij"), nt(b, "jk"), nt(c, "kl")], "il").data
    np.testing.assert_allclose(got, a @ b @ c, rtol=1e-12)
    f = lambda m: einsum([nt(m, "ij"), nt(b, "jk")], "ik").data
    np.testing.assert_allclose(f(2 * a - 3 * a2), 2 * f(a) - 3 * f(a2), rtol=1e-12, atol=1e-12)
    swapped = einsum([nt(b, "jk"), nt(a, "ij")], "ik").data
    np.testing.assert_allclose(swapped, f(a), rtol=1e-13)
    ab = einsum_abs([nt(a, "ij"), nt(b, "jk")], "ik").data
    np.testing.assert_allclose(ab, np.abs(a) @ np.abs(b), rtol=1e-13)
    assert np.all(ab >= np.abs(f(a)) - 1e-12)


def test_library_path_at_mid_size_against_the_definition():
    """The large-size path hands the contraction to numpy.einsum(optimize=True), which at these
    extents re-orders the operands, merges dims and calls the matrix-multiply routine: the result
    must still be the definition's, to fp64 summation-order accuracy.  Shapes of the layer's
    einsums (a projection with a batch dim, its weight gradient with two reduced dims and a
    transposed output, the two attention products with two batch dims), extents 48..80."""
    rng = np.random.default_rng(11)
    cases = [
        ([((3, 48, 80), ("batch", "length", "d_model")), ((80, 64), ("d_model", "d_ff"))], ("batch", "length", "d_ff")),
        ([((3, 48, 80), ("batch", "length", "d_model")), ((3, 48, 64), ("batch", "length", "d_ff"))], ("d_ff", "d_model")),
        ([((2, 48, 3, 16), ("batch", "length", "heads", "d_k")), ((2, 56, 3, 16), ("batch", "memory_length", "heads", "d_k"))],
         ("batch", "heads", "length", "memory_length")),
        ([((2, 3, 48, 56), ("batch", "heads", "length", "memory_length")), ((2, 56, 3, 16), ("batch", "memory_length", "heads", "d_v"))],
         ("batch", "length", "heads", "d_v")),
        ([((2, 48, 3, 16), ("batch", "length", "heads", "d_v")), ((3, 16, 80), ("heads", "d_v", "d_model"))],
         ("batch", "length", "d_model")),
    ]
    for operands, out in cases:
        inputs = [nt(rng.standard_normal(shape), dims) for shape, dims in operands]
        want, got = both_paths(inputs, out)
        scale = einsum_abs(inputs, out).data                              # |x|.|y| of every output
        assert got.shape == want.shape
        assert np.max(np.abs(got - want) / scale) <= 1e-12, (operands, out)
        # and an independent statement of the same contraction: plain loops over the batch dims
        # around numpy's matrix product for the first case
    a, b = rng.standard_normal((3, 48, 80)), rng.standard_normal((80, 64))
    want = np.stack([a[i] @ b for i in range(3)])
    for got in both_paths([nt(a, ("batch", "length", "d_model")), nt(b, ("d_model", "d_ff"))], ("batch", "length", "d_ff")):
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_errors():
    a = nt(np.zeros((2, 2)), ("d_model", "d_ff"))
    with pytest.raises(EinsumError) as e:
        einsum([E.NT(np.zeros((2, 2)), ("d_ff", "d_ff"))], ("d_ff",))
    assert e.value.code == "DUP_DIM"
    with pytest.raises(EinsumError) as e:
        einsum([a, nt(np.zeros((3, 2)), ("d_ff", "batch"))], ("batch",))
    assert e.value.code == "SIZE_MISMATCH"
    with pytest.raises(EinsumError) as e:
        einsum([a], ("heads",))
    assert e.value.code == "OUT_NOT_SUBSET"
