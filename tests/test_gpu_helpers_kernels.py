"""GPU parity tests of the HBM-bound helpers: slice gather/scatter (bit-exact), partial-sum
reduce and dtype cast, each against the oracle through the C ABI."""
import numpy as np
import pytest
import torch

import paper_1811_02084_amd as mtf
from oracle import layout as OLY
from oracle import optim as OO
from oracle.layer import identity
from oracle.bf16 import f64_to_bf16_bits
from oracle.einsum import NT
from oracle.metrics import m2
from helpers import f64, F32_TOL

pytestmark = pytest.mark.gpu

CASES = [
    # dims, sizes, mesh, layout
    (("batch", "io", "hidden"), (4, 5, 6), [("rows", 2), ("cols", 3)], [("batch", "rows"), ("hidden", "cols")]),
    (("batch", "length", "d_model"), (64, 16, 128), [("rows", 4), ("cols", 4)], [("batch", "rows"), ("d_ff", "cols")]),
    (("d_model", "d_ff"), (128, 1024), [("rows", 4), ("cols", 4)], [("batch", "rows"), ("d_ff", "cols")]),
    (("d_ff", "d_model"), (1024, 128), [("rows", 4), ("cols", 4)], [("batch", "rows"), ("d_ff", "cols")]),
    (("d_model", "heads", "d_k"), (40, 8, 24), [("all", 4)], [("heads", "all")]),
    (("vocab",), (30,), [("all", 5)], [("vocab", "all")]),
    (("batch", "io"), (6, 7), [("all", 3)], []),                       # replicated: whole tensor
    (("a", "b", "c", "d"), (4, 6, 4, 10), [("x", 2), ("y", 2), ("z", 2)], [("a", "x"), ("c", "y"), ("d", "z")]),
]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_slice_copy_bit_exact(case, dtype):
    dims, sizes, mesh, layout = CASES[case]
    print(f"slice_copy case {case} {dtype}", flush=True)
    n = int(np.prod(sizes))
    # distinct bit patterns per element: iota for fp32, iota over the 16-bit patterns for bf16
    if dtype == torch.float32:
        full = torch.arange(n, dtype=torch.float32).reshape(sizes)
    else:
        full = (torch.arange(n, dtype=torch.int32) % 30000).to(torch.int16).view(torch.bfloat16).reshape(sizes)
    raw = lambda t: t.cpu().contiguous().view(torch.int32 if dtype == torch.float32 else torch.int16).numpy()
    dfull = full.cuda()
    for coord in OLY.all_coords(mesh):
        got = mtf.slice_copy(dfull, dims, mesh, layout, coord)
        offs, locs = OLY.slice_spec(dims, sizes, mesh, layout, coord)
        want = raw(full)[tuple(slice(o, o + s) for o, s in zip(offs, locs))]
        assert tuple(got.shape) == locs
        assert np.array_equal(raw(got), want), coord
    # scatter every slice of a fresh tensor back: must reproduce the original exactly
    rebuilt = torch.zeros_like(dfull)
    for coord in OLY.all_coords(mesh):
        piece = mtf.slice_copy(dfull, dims, mesh, layout, coord)
        mtf.slice_copy(rebuilt, dims, mesh, layout, coord, slice_buf=piece, scatter=True)
    assert np.array_equal(raw(rebuilt), raw(full))


@pytest.mark.parametrize("count", [0, 1, 3, 4, 1027, 1 << 20])
@pytest.mark.parametrize("n", [1, 4, 16])
def test_reduce_partials(n, count):
    print(f"reduce_partials n={n} count={count}", flush=True)
    rng = np.random.default_rng(n * 1000 + count % 997)
    parts = [rng.standard_normal(count).astype(np.float32) for _ in range(n)]
    res = rng.standard_normal(count).astype(np.float32)
    dparts = [torch.from_numpy(p).cuda() for p in parts]
    want = sum(p.astype(np.float64) for p in parts)
    got = mtf.reduce_partials(dparts)
    assert m2(f64(got), want) <= F32_TOL
    res_bf = torch.from_numpy(res).to(torch.bfloat16)
    got = mtf.reduce_partials(dparts, residual=res_bf.cuda(), out_dtype=torch.float32)
    assert m2(f64(got), want + res_bf.double().numpy()) <= F32_TOL
    got = mtf.reduce_partials(dparts, residual=torch.from_numpy(res).cuda(), out_dtype=torch.bfloat16)
    assert m2(f64(got), want + res.astype(np.float64)) <= 2.0 ** -8        # one bf16 rounding
    # integer-valued partials: every order of summation is exact, so the result is bit-exact
    ints = [rng.integers(-8, 9, count).astype(np.float32) for _ in range(n)]
    got = mtf.reduce_partials([torch.from_numpy(p).cuda() for p in ints])
    assert np.array_equal(got.cpu().numpy(), sum(ints))


@pytest.mark.parametrize("count", [5, 1027, 1 << 18])
@pytest.mark.parametrize("n", [2, 4, 7])
def test_reduce_partials_with_a_componentwise_epilogue(n, count):
    """ReLU, and the ReLU gradient's mask, applied to the complete sum by the reduce itself
    (mtf_reduce_partials_epi): against the definition in fp64, bit-exact on integer-valued partials,
    and bit-identical to the reduce followed by the component-wise pass."""
    print(f"reduce_partials_epi n={n} count={count}", flush=True)
    rng = np.random.default_rng(n * 7919 + count)
    parts = [rng.standard_normal(count).astype(np.float32) for _ in range(n)]
    dparts = [torch.from_numpy(p).cuda() for p in parts]
    aux = rng.standard_normal(count).astype(np.float32)
    aux[::5] = 0.0                                   # exactly zero: gradient 0 there
    aux[1::11] = -0.0
    daux = torch.from_numpy(aux).to(torch.bfloat16).cuda()
    aux_stored = daux.float().cpu().numpy()
    visible = aux_stored > 0.0
    for dt, tol in ((torch.float32, F32_TOL), (torch.bfloat16, 2.0 ** -8)):
        got = mtf.reduce_partials(dparts, out_dtype=dt, epi=mtf.EPI_RELU)
        assert m2(f64(got), OO.allreduce_then(parts, op="relu", store=identity)) <= tol
        assert not bool((got.float() < 0).any())
        got = mtf.reduce_partials(dparts, out_dtype=dt, epi=mtf.EPI_MASK_GT0, aux=daux)
        assert m2(f64(got), OO.allreduce_then(parts, op="mask", aux=aux_stored, store=identity)) <= tol
        assert not bool(got.float()[torch.from_numpy(~visible).cuda()].any())
    if count % 8 == 0:                               # the component-wise path of the einsum call takes whole vectors
        plain = mtf.reduce_partials(dparts, out_dtype=torch.bfloat16)
        two_pass = mtf.einsum_local(plain, ("i",), None, None, ("i",), epi=mtf.EPI_RELU)
        assert torch.equal(mtf.reduce_partials(dparts, out_dtype=torch.bfloat16, epi=mtf.EPI_RELU), two_pass)
        two_pass = mtf.einsum_local(plain, ("i",), None, None, ("i",), epi=mtf.EPI_MASK_GT0, aux=daux)
        assert torch.equal(mtf.reduce_partials(dparts, out_dtype=torch.bfloat16, epi=mtf.EPI_MASK_GT0, aux=daux),
                           two_pass)
    ints = [rng.integers(-8, 9, count).astype(np.float32) for _ in range(n)]
    got = mtf.reduce_partials([torch.from_numpy(p).cuda() for p in ints], epi=mtf.EPI_RELU)
    assert np.array_equal(got.cpu().numpy(), OO.allreduce_then(ints, op="relu", store=identity))
    res = torch.from_numpy(rng.integers(-8, 9, count).astype(np.float32)).to(torch.bfloat16)
    got = mtf.reduce_partials([torch.from_numpy(p).cuda() for p in ints], residual=res.cuda(), out_dtype=torch.float32,
                              epi=mtf.EPI_MASK_GT0, aux=daux)
    assert np.array_equal(got.cpu().numpy(), OO.allreduce_then(ints, residual=res.float().numpy(), op="mask",
                                                              aux=aux_stored, store=identity))


def test_cast_rounds_to_nearest_even_bit_exact():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(1 << 18) * np.exp(rng.uniform(-30, 30, 1 << 18))).astype(np.float32)
    x[:4] = [1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -0.0, 3.0e38]             # ties and extremes
    got = mtf.cast(torch.from_numpy(x).cuda(), torch.bfloat16)
    bits = got.cpu().view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, f64_to_bf16_bits(x.astype(np.float64)))
    back = mtf.cast(got, torch.float32)
    assert np.array_equal(back.cpu().numpy(), got.float().cpu().numpy())
