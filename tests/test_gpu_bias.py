"""Parity of the worked example with its bias (y = Relu(x w + bias) v), of component-wise addition
with implicit broadcasting and of local reductions against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import mtf_inputs
from helpers import named as to_nt
from oracle import layer as OL
from oracle.einsum import add_broadcast as o_add, einsum as o_einsum, nt, reduce as o_reduce
from oracle.metrics import m2
from oracle.layer import B, L, D, F
from oracle.layout import all_coords, slice_spec

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2     # bf16 inputs, fp32 accumulation
TOL_F32 = 1e-5


@pytest.fixture(scope="module")
def mtf():
    import paper_1811_02084_amd as m
    return m


def _dev(t):
    return t.cuda()


def _ffn_bias_case(cfg_id, b, l, d, f):
    x = mtf_inputs.normal(cfg_id, 0, (b, l, d))
    w_in = mtf_inputs.normal(cfg_id, 1, (d, f), std=d ** -0.5)
    w_out = mtf_inputs.normal(cfg_id, 2, (f, d), std=f ** -0.5)
    dy = mtf_inputs.normal(cfg_id, 3, (b, l, d))
    bias = mtf_inputs.normal(cfg_id, 4, (f,), std=0.5)
    return x, w_in, bias, w_out, dy


@pytest.mark.parametrize("shape", [(2, 37, 72, 200), (3, 50, 264, 328), (16, 256, 1024, 4096)],
                         ids=["ragged-small", "ragged-tiles", "config2-size"])
def test_ffn_bias_forward_backward(mtf, shape):
    b, l, d, f = shape
    x, w_in, bias, w_out, dy = _ffn_bias_case(21, b, l, d, f)
    f64 = lambda t, dims: nt(t.double().numpy(), dims)
    ref = OL.ffn_bias_fwd(f64(x, (B, L, D)), f64(w_in, (D, F)), f64(bias, (F,)), f64(w_out, (F, D)))
    a, y = mtf.ffn_bias_fwd(_dev(x), _dev(w_in), _dev(bias), _dev(w_out))
    assert m2(a.float().cpu().numpy(), ref["a"].data) <= TOL_BF16
    assert m2(y.cpu().numpy(), ref["y"].data) <= TOL_BF16
    # backward on the oracle's saved activation: both sides take the ReLU decision from the same bits
    a_ref = torch.from_numpy(ref["a"].data).to(torch.bfloat16)
    gref = OL.ffn_bias_bwd(f64(x, (B, L, D)), nt(a_ref.double().numpy(), (B, L, F)), f64(w_in, (D, F)),
                           f64(w_out, (F, D)), f64(dy, (B, L, D)))
    got = mtf.ffn_bias_bwd(_dev(x), _dev(a_ref), _dev(w_in), _dev(w_out), _dev(dy))
    for name in ("dw_in", "dw_out", "dbias", "dx"):
        err = m2(got[name].cpu().numpy(), gref[name].data)
        assert err <= TOL_BF16, (name, err)


def test_bias_epilogues_of_einsum_local(mtf):
    """MTF_EPI_BIAS / MTF_EPI_BIAS_RELU on the MFMA path (bf16) and on the generic path (fp32,
    and a bias over an innermost dim that is not the whole n extent)."""
    rng = np.random.Generator(np.random.Philox(key=[mtf_inputs.BASE_SEED, 31]))
    m, n, k = 304, 264, 200
    for dtype, tol in ((torch.bfloat16, TOL_BF16), (torch.float32, TOL_F32)):
        a = torch.from_numpy(rng.standard_normal((m, k), dtype=np.float32)).to(dtype)
        bmat = torch.from_numpy(rng.standard_normal((k, n), dtype=np.float32)).to(dtype)
        bias = torch.from_numpy(rng.standard_normal(n, dtype=np.float32)).to(dtype)
        h = o_add(o_einsum([to_nt(a, ("m", "k")), to_nt(bmat, ("k", "n"))], ("m", "n")), to_nt(bias, ("n",)))
        for epi, want in ((mtf.EPI_BIAS, h.data), (mtf.EPI_BIAS_RELU, np.maximum(h.data, 0.0))):
            got = mtf.einsum_local(_dev(a), ("m", "k"), _dev(bmat), ("k", "n"), ("m", "n"),
                                   out_dtype=torch.float32, epi=epi, aux=_dev(bias))
            assert m2(got.cpu().numpy(), want) <= tol, (dtype, epi)
    # out [m, h, c] with n = (h, c) merged: the bias runs over c only
    a = torch.from_numpy(rng.standard_normal((64, 48), dtype=np.float32)).to(torch.bfloat16)
    w = torch.from_numpy(rng.standard_normal((48, 4, 16), dtype=np.float32)).to(torch.bfloat16)
    bias = torch.from_numpy(rng.standard_normal(16, dtype=np.float32)).to(torch.bfloat16)
    h = o_add(o_einsum([to_nt(a, ("m", "k")), to_nt(w, ("k", "h", "c"))], ("m", "h", "c")), to_nt(bias, ("c",)))
    got = mtf.einsum_local(_dev(a), ("m", "k"), _dev(w), ("k", "h", "c"), ("m", "h", "c"),
                           out_dtype=torch.float32, epi=mtf.EPI_BIAS, aux=_dev(bias))
    assert m2(got.cpu().numpy(), h.data) <= TOL_BF16


@pytest.mark.parametrize("b_dims", [("r",), ("q",), ("p",), ("q", "r"), ("r", "p"), ("p", "q", "r")])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_add_broadcast(mtf, b_dims, dtype):
    sizes = dict(p=5, q=36, r=24)
    a = mtf_inputs.small_ints(22, 0, (5, 36, 24), dtype=dtype)
    b = mtf_inputs.small_ints(22, 1 + len(b_dims), tuple(sizes[d] for d in b_dims), dtype=dtype)
    want = o_add(to_nt(a, ("p", "q", "r")), to_nt(b, b_dims)).data
    got = mtf.add_broadcast(_dev(a), ("p", "q", "r"), _dev(b), b_dims)
    assert np.array_equal(got.double().cpu().numpy(), want)       # small integers: exact in both dtypes


def test_add_broadcast_errors(mtf):
    a = torch.zeros((4, 8), device="cuda")
    with pytest.raises(mtf.MtfError) as e:
        mtf.add_broadcast(a, ("p", "q"), torch.zeros(8, device="cuda"), ("z",))
    assert e.value.name == "MTF_ERR_OUT_NOT_SUBSET"
    with pytest.raises(mtf.MtfError) as e:
        mtf.add_broadcast(a, ("p", "q"), torch.zeros(4, device="cuda"), ("q",))
    assert e.value.name == "MTF_ERR_SIZE_MISMATCH"


REDUCE_CASES = [
    (("p", "q", "r"), (37, 50, 264), ("r",)),          # columns: trailing dim kept
    (("p", "q", "r"), (37, 50, 264), ("q", "r")),      # columns, two kept dims
    (("p", "q", "r"), (37, 50, 264), ("p",)),          # rows: leading dim kept
    (("p", "q", "r"), (37, 50, 264), ("p", "q")),
    (("p", "q", "r"), (37, 50, 264), ("q",)),          # middle dim kept: generic
    (("p", "q", "r"), (37, 50, 264), ("r", "p")),      # transposed output: generic
    (("p", "q", "r"), (37, 50, 263), ("r",)),          # odd columns: generic
    (("p", "q"), (4096, 4096), ("q",)),                # the dbias shape of config 2
]


@pytest.mark.parametrize("case", REDUCE_CASES, ids=[f"{c[1]}->{','.join(c[2])}" for c in REDUCE_CASES])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_reduce_local(mtf, case, dtype):
    dims, shape, out = case
    x = mtf_inputs.normal(23, len(out) + 7 * len(shape), shape, dtype=dtype)
    ref = to_nt(x, dims)
    got_sum = mtf.reduce_local(_dev(x), dims, out, mtf.REDUCE_SUM)
    got_max = mtf.reduce_local(_dev(x), dims, out, mtf.REDUCE_MAX)
    want_sum, want_max = o_reduce(ref, out, "sum").data, o_reduce(ref, out, "max").data
    # forward-error bound of a sum: relative to the sum of absolute values
    denom = o_reduce(nt(np.abs(ref.data), dims), out, "sum").data
    assert np.max(np.abs(got_sum.cpu().numpy() - want_sum) / denom) <= TOL_F32
    assert np.array_equal(got_max.double().cpu().numpy(), want_max)   # a maximum is one of the inputs


def test_reduce_local_small_ints_exact_and_errors(mtf):
    x = mtf_inputs.small_ints(23, 99, (64, 48, 40), dtype=torch.bfloat16)
    for out in (("r",), ("p",), ("q", "p"), ()):
        if not out:
            continue
        want = o_reduce(to_nt(x, ("p", "q", "r")), out, "sum").data
        got = mtf.reduce_local(_dev(x), ("p", "q", "r"), out)
        assert np.array_equal(got.double().cpu().numpy(), want)
    with pytest.raises(mtf.MtfError) as e:
        mtf.reduce_local(_dev(x), ("p", "q", "r"), ("z",))
    assert e.value.name == "MTF_ERR_OUT_NOT_SUBSET"


def test_example_with_bias_on_virtual_meshes(mtf):
    """The example's layouts on one GPU: every processor's slice computed by the library, the
    Allreduce groups summed by mtf_reduce_partials; integers, so every layout must reproduce the
    unsplit result bit for bit (forward y and the bias gradient)."""
    b, d_io, d_h = 8, 16, 32
    x = mtf_inputs.small_ints(24, 0, (b, 1, d_io), dtype=torch.float32)
    w = mtf_inputs.small_ints(24, 1, (d_io, d_h), dtype=torch.float32)
    bias = mtf_inputs.small_ints(24, 2, (d_h,), dtype=torch.float32)
    v = mtf_inputs.small_ints(24, 3, (d_h, d_io), dtype=torch.float32)
    dy = mtf_inputs.small_ints(24, 4, (b, 1, d_io), dtype=torch.float32)
    f64 = lambda t, dims: nt(t.double().numpy(), dims)
    full = OL.ffn_bias_fwd(f64(x, (B, L, D)), f64(w, (D, F)), f64(bias, (F,)), f64(v, (F, D)), OL.identity)
    gfull = OL.ffn_bias_bwd(f64(x, (B, L, D)), full["a"], f64(w, (D, F)), f64(v, (F, D)), f64(dy, (B, L, D)),
                            OL.identity)
    layouts = {
        "data-parallel": ([("all", 4)], [("batch", "all")]),
        "model-parallel": ([("all", 4)], [("d_ff", "all")]),
        "data+model": ([("rows", 2), ("cols", 2)], [("batch", "rows"), ("d_ff", "cols")]),
    }
    dh_full = torch.from_numpy(gfull["dh"].data).float()
    for name, (mesh, layout) in layouts.items():
        y_parts, db_parts = {}, {}
        for c in all_coords(mesh):
            sl = lambda t, dims: mtf.slice_copy(_dev(t), dims, mesh, layout, c)
            h = mtf.einsum_local(sl(x, (B, L, D)), (B, L, D), sl(w, (D, F)), (D, F), (B, L, F),
                                 epi=mtf.EPI_BIAS_RELU, aux=sl(bias, (F,)))
            y_parts[c] = mtf.einsum_local(h, (B, L, F), sl(v, (F, D)), (F, D), (B, L, D))
            db_parts[c] = mtf.reduce_local(sl(dh_full, (B, L, F)), (B, L, F), (F,))
        for out_dims, parts, want in (((B, L, D), y_parts, full["y"]), ((F,), db_parts, gfull["dbias"])):
            if out_dims == (F,):
                plan = mtf.einsum_plan([(B, b), (L, 1), (F, d_h)], None, [(F, d_h)], mesh, layout)
            else:
                plan = mtf.einsum_plan([(B, b), (L, 1), (F, d_h)], [(F, d_h), (D, d_io)],
                                       [(B, b), (L, 1), (D, d_io)], mesh, layout)
            axes = plan["reduce_axes"]
            for c in all_coords(mesh):
                group = [c2 for c2 in all_coords(mesh) if all(c2[i] == c[i] for i in range(len(mesh)) if i not in axes)]
                total = mtf.reduce_partials([parts[g].contiguous() for g in group])
                offs, locs = slice_spec(out_dims, want.data.shape, mesh, layout, c)
                idx = tuple(slice(o, o + n) for o, n in zip(offs, locs))
                assert np.array_equal(total.double().cpu().numpy(), want.data[idx]), (name, out_dims, c)


def test_example_on_the_three_dimensional_layout(mtf):
    """batch -> rows, hidden -> cols, io -> planes: every matrix is tiled across two mesh dims and
    replicated in the third, and every einsum needs an Allreduce across one mesh dim ("Data-
    Parallel, Model-Parallel Layouts", last layout).  The hidden layer's sum must be complete
    before the bias and the ReLU, so these run as component-wise operations after the reduce."""
    b, d_io, d_h = 8, 16, 32
    x = mtf_inputs.small_ints(25, 0, (b, 1, d_io), dtype=torch.float32)
    w = mtf_inputs.small_ints(25, 1, (d_io, d_h), dtype=torch.float32)
    bias = mtf_inputs.small_ints(25, 2, (d_h,), dtype=torch.float32)
    v = mtf_inputs.small_ints(25, 3, (d_h, d_io), dtype=torch.float32)
    f64 = lambda t, dims: nt(t.double().numpy(), dims)
    full = OL.ffn_bias_fwd(f64(x, (B, L, D)), f64(w, (D, F)), f64(bias, (F,)), f64(v, (F, D)), OL.identity)
    mesh = [("rows", 2), ("cols", 2), ("planes", 2)]
    layout = [("batch", "rows"), ("d_ff", "cols"), ("d_model", "planes")]
    coords = all_coords(mesh)
    shp = lambda dims, sizes: list(zip(dims, sizes))
    p1 = mtf.einsum_plan(shp((B, L, D), (b, 1, d_io)), shp((D, F), (d_io, d_h)), shp((B, L, F), (b, 1, d_h)), mesh, layout)
    p2 = mtf.einsum_plan(shp((B, L, F), (b, 1, d_h)), shp((F, D), (d_h, d_io)), shp((B, L, D), (b, 1, d_io)), mesh, layout)
    assert p1["reduce_axes"] == [2] and p2["reduce_axes"] == [1]           # planes, then cols
    group = lambda c, axes: [c2 for c2 in coords if all(c2[i] == c[i] for i in range(3) if i not in axes)]
    sl = lambda t, dims, c: mtf.slice_copy(_dev(t), dims, mesh, layout, c)
    h_part = {c: mtf.einsum_local(sl(x, (B, L, D), c), (B, L, D), sl(w, (D, F), c), (D, F), (B, L, F)) for c in coords}
    a = {}
    for c in coords:
        h = mtf.reduce_partials([h_part[g] for g in group(c, [2])])
        h = mtf.add_broadcast(h, (B, L, F), sl(bias, (F,), c), (F,))
        a[c] = mtf.einsum_local(h, (B, L, F), None, None, (B, L, F), epi=mtf.EPI_RELU)      # component-wise
        offs, locs = slice_spec((B, L, F), full["a"].data.shape, mesh, layout, c)
        idx = tuple(slice(o, o + n) for o, n in zip(offs, locs))
        assert np.array_equal(a[c].double().cpu().numpy(), full["a"].data[idx]), c
    y_part = {c: mtf.einsum_local(a[c], (B, L, F), sl(v, (F, D), c), (F, D), (B, L, D)) for c in coords}
    for c in coords:
        y = mtf.reduce_partials([y_part[g] for g in group(c, [1])])
        offs, locs = slice_spec((B, L, D), full["y"].data.shape, mesh, layout, c)
        idx = tuple(slice(o, o + n) for o, n in zip(offs, locs))
        assert np.array_equal(y.double().cpu().numpy(), full["y"].data[idx]), c


def test_seeded_sweep_of_reductions_and_broadcasts(mtf):
    """Random ranks, sizes, kept dims and output orders: every kernel pattern (columns, rows,
    generic; vector and scalar runs) against the oracle."""
    rng = np.random.Generator(np.random.Philox(key=[mtf_inputs.BASE_SEED, 61]))
    names = ["p", "q", "r", "s"]
    for case in range(30):
        rank = int(rng.integers(1, 5))
        dims = tuple(names[:rank])
        shape = tuple(int(rng.choice([1, 3, 8, 24, 40, 130])) for _ in dims)
        keep = [d for d in dims if rng.random() < 0.5]
        rng.shuffle(keep)
        dtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
        print(f"sweep {case}: {dict(zip(dims, shape))} keep {keep} {dtype}", flush=True)
        x = mtf_inputs.small_ints(26, case, shape, dtype=dtype)
        ref = to_nt(x, dims)
        for op, name in ((mtf.REDUCE_SUM, "sum"), (mtf.REDUCE_MAX, "max")):
            got = mtf.reduce_local(_dev(x), dims, tuple(keep), op)
            want = o_reduce(ref, tuple(keep), name).data
            assert np.array_equal(got.double().cpu().numpy().reshape(want.shape), want), (case, name)
        if keep:
            b = mtf_inputs.small_ints(27, case, tuple(dict(zip(dims, shape))[d] for d in keep), dtype=dtype)
            got = mtf.add_broadcast(_dev(x), dims, _dev(b), tuple(keep))
            assert np.array_equal(got.double().cpu().numpy(), o_add(ref, to_nt(b, tuple(keep))).data), case
