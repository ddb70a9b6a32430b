"""Named-dimension einsum (test infrastructure only).

Section "Operation Implementation", paragraph "Einstein Summation": every input is
broadcast to the shape made of the union of all input dimensions, the broadcast inputs
are multiplied component-wise, and every dimension that is not in the requested output
shape is summed out.  Dimensions are identified by NAME; a tensor is a pair
(fp64 ndarray, tuple of distinct names), row-major in the order the names are listed.

  einsum_definition   that sentence written out with numpy broadcasting (memory grows
                      with the full iteration space, so small inputs only)
  einsum              same result; above a size threshold the contraction is handed to
                      numpy's own einsum in fp64 (a library primitive as one step)
  einsum_abs          the same contraction of absolute values (denominator of the
                      forward-error measure M1)
  reduce              reduce_sum / reduce_max: the output dims are a subset of the input
                      dims ("Operation Implementation", paragraph "Reduction")
  add_broadcast       component-wise addition with implicit broadcasting of the operand
                      whose shape is a subset of the other's ("Mesh-TensorFlow syntax")
"""
from collections import namedtuple
import string
import numpy as np

NT = namedtuple("NT", ["data", "dims"])       # named tensor: ndarray + tuple of names


class EinsumError(ValueError):
    """code is one of DUP_DIM, SIZE_MISMATCH, OUT_NOT_SUBSET, NOT_BROADCASTABLE."""

    def __init__(self, code, msg=""):
        super().__init__(f"{code}: {msg}")
        self.code = code


def nt(data, dims):
    data = np.asarray(data, dtype=np.float64)
    dims = tuple(dims)
    if data.ndim != len(dims):
        raise ValueError(f"rank {data.ndim} array given {len(dims)} names")
    return NT(data, dims)


def union_dims(inputs):
    """Ordered union (by first appearance) of the inputs' dims -> dict name -> size.

    A name may appear once per tensor ("Mesh-TensorFlow: Beyond Batch Splitting": two
    identically named dims in one tensor are illegal) and must have one size everywhere.
    """
    sizes = {}
    for t in inputs:
        if len(set(t.dims)) != len(t.dims):
            raise EinsumError("DUP_DIM", str(t.dims))
        for name, n in zip(t.dims, t.data.shape):
            if sizes.setdefault(name, n) != n:
                raise EinsumError("SIZE_MISMATCH", f"{name}: {sizes[name]} vs {n}")
    return sizes


def _check_out(sizes, out_dims):
    out_dims = tuple(out_dims)
    if len(set(out_dims)) != len(out_dims):
        raise EinsumError("DUP_DIM", str(out_dims))
    for d in out_dims:
        if d not in sizes:
            raise EinsumError("OUT_NOT_SUBSET", d)
    return out_dims


def einsum_definition(inputs, out_dims):
    """Broadcast to the union shape, multiply component-wise, reduce out the rest."""
    sizes = union_dims(inputs)
    out_dims = _check_out(sizes, out_dims)
    union = list(sizes)
    prod = np.ones([1] * len(union), dtype=np.float64)
    for t in inputs:
        # move this tensor's axes into union order, size-1 axes where it lacks a dim
        order = sorted(range(len(t.dims)), key=lambda ax: union.index(t.dims[ax]))
        arr = np.transpose(t.data, order)
        shape = [sizes[d] if d in t.dims else 1 for d in union]
        prod = prod * arr.reshape(shape)                  # implicit broadcast
    prod = np.broadcast_to(prod, [sizes[d] for d in union])
    reduced = tuple(i for i, d in enumerate(union) if d not in out_dims)
    res = prod.sum(axis=reduced) if reduced else np.array(prod)
    kept = [d for d in union if d in out_dims]
    res = np.transpose(res, [kept.index(d) for d in out_dims])
    return NT(np.array(res, dtype=np.float64, order="C"), out_dims)


_DEFINITION_LIMIT = 1 << 22        # elements of the iteration space


def einsum(inputs, out_dims):
    """Named einsum in fp64; large iteration spaces go through numpy.einsum."""
    sizes = union_dims(inputs)
    out_dims = _check_out(sizes, out_dims)
    space = 1
    for n in sizes.values():
        space *= n
    if space <= _DEFINITION_LIMIT:
        return einsum_definition(inputs, out_dims)
    letter = {d: string.ascii_letters[i] for i, d in enumerate(sizes)}
    spec = ",".join("".join(letter[d] for d in t.dims) for t in inputs)
    spec += "->" + "".join(letter[d] for d in out_dims)
    res = np.einsum(spec, *[t.data for t in inputs], optimize=True)
    return NT(np.array(res, dtype=np.float64, order="C"), out_dims)


def einsum_abs(inputs, out_dims):
    """einsum of |inputs|: sum over the reduced dims of |prod of inputs|."""
    return einsum([NT(np.abs(t.data), t.dims) for t in inputs], out_dims)


def flops(inputs):
    """One multiply-add per point of the iteration space (Appendix B, 'Iteration Space')."""
    space = 1
    for n in union_dims(inputs).values():
        space *= n
    return 2 * space


def reduce(t, out_dims, op="sum"):
    """Reduction whose output dims are a subset of the input dims: every other dim is summed
    (op="sum") or maximised (op="max") out; the result is laid out in out_dims order."""
    sizes = union_dims([t])
    out_dims = _check_out(sizes, out_dims)
    gone = tuple(i for i, d in enumerate(t.dims) if d not in out_dims)
    if op == "sum":
        res = t.data.sum(axis=gone) if gone else np.array(t.data)
    elif op == "max":
        res = t.data.max(axis=gone) if gone else np.array(t.data)
    else:
        raise ValueError(op)
    kept = [d for d in t.dims if d in out_dims]
    res = np.transpose(res, [kept.index(d) for d in out_dims])
    return NT(np.array(res, dtype=np.float64, order="C"), out_dims)


def add_broadcast(a, b):
    """a + b where the dims of one operand are a subset of the other's: the smaller operand is
    repeated along the dims it lacks.  The result has the larger operand's dims, in its order."""
    sizes = union_dims([a, b])
    big, small = (a, b) if len(a.dims) >= len(b.dims) else (b, a)
    if not set(small.dims) <= set(big.dims):
        raise EinsumError("NOT_BROADCASTABLE", f"{a.dims} + {b.dims}")
    # the small operand's axes in the order they occur in the big one, size 1 elsewhere
    order = sorted(range(len(small.dims)), key=lambda ax: big.dims.index(small.dims[ax]))
    arr = np.transpose(small.data, order)
    shape = [sizes[d] if d in small.dims else 1 for d in big.dims]
    return NT(np.array(big.data + arr.reshape(shape), dtype=np.float64, order="C"), big.dims)
