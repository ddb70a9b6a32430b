"""The paper's central invariant on the device: every layout gives the identical result.
A virtual mesh of slices is held on one GPU; each coordinate's slices are gathered with
mtf_slice_copy, its share of the layer is computed, and the partial sums are reduced along the
mesh dims the einsum plan names (the stand-in for the Allreduce)."""
import numpy as np
import pytest
import torch

import mtf_inputs
import paper_1811_02084_amd as mtf
from oracle import layer as OL
from oracle import layout as OLY
from oracle.einsum import NT
from oracle.metrics import m2
from helpers import f64, named, on_device, BF16_TOL, F32_TOL
from oracle.layer import B, L, D, F

pytestmark = pytest.mark.gpu

X, WI, WO, HID = (B, L, D), (D, F), (F, D), (B, L, F)


def _virtual_mesh_ffn(g, mesh, layout, fp32, kranges=0):
    """Returns {coord: y after the grouped reduce} computed slice by slice on the device.
    kranges > 0: the second einsum of every slice as that many ranges of d_ff; their sums all go
    into the group's reduce."""
    shp = lambda t, dims: list(zip(dims, t.shape))
    plan = mtf.einsum_plan(shp(g["x"], X)[:2] + [(F, g["w_in"].shape[1])], shp(g["w_out"], WO),
                           shp(g["x"], X), mesh, layout)
    axes = plan["reduce_axes"]
    partial = {}
    for c in OLY.all_coords(mesh):
        xs = mtf.slice_copy(g["x"], X, mesh, layout, c)
        wi = mtf.slice_copy(g["w_in"], WI, mesh, layout, c)
        wo = mtf.slice_copy(g["w_out"], WO, mesh, layout, c)
        if fp32:
            h = mtf.einsum_local(xs, X, wi, WI, HID, epi=mtf.EPI_RELU)
            partial[c] = [mtf.einsum_local(h, HID, wo, WO, X)]
        elif kranges:
            h = mtf.einsum_local(xs, X, wi, WI, HID, epi=mtf.EPI_RELU)
            partial[c] = mtf.einsum_local_kranges(h, HID, wo, WO, X, kranges)
        else:
            partial[c] = [mtf.ffn_fwd(xs, wi, wo)[1]]
    out = {}
    for c in OLY.all_coords(mesh):
        group = [c2 for c2 in OLY.all_coords(mesh)
                 if all(c2[i] == c[i] for i in range(len(mesh)) if i not in axes)]
        out[c] = mtf.reduce_partials([t for c2 in group for t in partial[c2]])
    return out, axes


def test_config1_tiny_fp32_mesh_of_4():
    cfg = mtf_inputs.config1()
    g = on_device(cfg)
    mesh, layout = cfg["mesh"], cfg["layout"]
    out, axes = _virtual_mesh_ffn(g, mesh, layout, fp32=True)
    assert axes == [0]                                        # d_ff is reduced out and split
    ref = OL.ffn_fwd(named(cfg["x"], X), named(cfg["w_in"], WI), named(cfg["w_out"], WO), OL.identity)["y"]
    for c, y in out.items():
        assert m2(f64(y), ref.data) <= F32_TOL, c             # every processor ends with the full y
    # unsplit computation on the device agrees as well
    h = mtf.einsum_local(g["x"], X, g["w_in"], WI, HID, epi=mtf.EPI_RELU)
    y = mtf.einsum_local(h, HID, g["w_out"], WO, X)
    assert m2(f64(y), ref.data) <= F32_TOL


@pytest.mark.parametrize("mesh,layout", [
    ([("all", 4)], [("batch", "all")]),
    ([("all", 4)], [("d_ff", "all")]),
    ([("rows", 2), ("cols", 2)], [("batch", "rows"), ("d_ff", "cols")]),
    ([("rows", 2), ("cols", 2), ("planes", 2)], [("batch", "rows"), ("d_ff", "cols"), ("d_model", "planes")]),
    ([("all", 3)], []),
])
def test_layouts_of_the_worked_example_bit_exact_on_integers(mesh, layout):
    """Integer-valued inputs: all partial sums are exact, so every layout must agree bit for bit."""
    print(f"layout {layout} on {mesh}", flush=True)
    x = mtf_inputs.small_ints(31, 0, (4, 6, 16), dtype=torch.float32).cuda()
    w_in = mtf_inputs.small_ints(31, 1, (16, 24), dtype=torch.float32).cuda()
    hidden_full = mtf.einsum_local(x, X, w_in, WI, HID)
    for c in OLY.all_coords(mesh):
        plan = mtf.einsum_plan(list(zip(X, x.shape)), list(zip(WI, w_in.shape)),
                               list(zip(HID, hidden_full.shape)), mesh, layout)
        group = [c2 for c2 in OLY.all_coords(mesh)
                 if all(c2[i] == c[i] for i in range(len(mesh)) if i not in plan["reduce_axes"])]
        parts = [mtf.einsum_local(mtf.slice_copy(x, X, mesh, layout, c2), X,
                                  mtf.slice_copy(w_in, WI, mesh, layout, c2), WI, HID) for c2 in group]
        got = mtf.reduce_partials(parts)
        want = mtf.slice_copy(hidden_full, HID, mesh, layout, c)
        assert torch.equal(got, want), c


def test_config4_virtual_4x4_mesh_full_size():
    cfg = mtf_inputs.config4()
    g = on_device(cfg)
    mesh, layout = cfg["mesh"], cfg["layout"]
    print("config 4: 16 slices", flush=True)
    out, axes = _virtual_mesh_ffn(g, mesh, layout, fp32=False)
    assert axes == [1]                                        # summed by processor-column index
    print("config 4: unsplit layer on the device", flush=True)
    _, y_full = mtf.ffn_fwd(g["x"], g["w_in"], g["w_out"])
    for c, y in out.items():
        want = mtf.slice_copy(y_full, X, mesh, layout, c)
        # identical bf16 products, fp32 sums taken in a different order
        assert m2(f64(y), f64(want)) <= 1e-4, c
    # against the oracle on sampled tokens (a feed-forward output row depends on its own input row
    # only): after the reduce every processor of a mesh row holds that row's complete y, so each
    # sampled token is checked on all four processors (mesh columns) of its row
    # the second einsum of every slice as two ranges of d_ff (mtf_einsum_local_kranges), eight range
    # sums per group: same products, another summation order
    print("config 4: 16 slices, second einsum in two ranges", flush=True)
    out2, _ = _virtual_mesh_ffn(g, mesh, layout, fp32=False, kranges=2)
    for c, y in out2.items():
        assert m2(f64(y), f64(out[c])) <= 1e-4, c
    print("config 4: oracle on sampled tokens, every mesh column", flush=True)
    rng = np.random.default_rng(4)
    w_in, w_out = named(cfg["w_in"], WI), named(cfg["w_out"], WO)
    n_tok = 96
    bis, lis = rng.integers(0, 64, n_tok), rng.integers(0, 256, n_tok)
    bis[:4] = [0, 15, 16, 63]                                 # first / last batch element of a mesh row
    lis[:4] = [0, 255, 0, 255]
    xr = NT(np.stack([f64(cfg["x"][b, l]) for b, l in zip(bis, lis)])[:, None, :], X)   # [n_tok, 1, D]
    ref = OL.ffn_fwd(xr, w_in, w_out)["y"].data[:, 0]
    host = {c: f64(y) for c, y in out.items()}
    assert {r for r, _ in host} == {0, 1, 2, 3} and {c for _, c in host} == {0, 1, 2, 3}
    for col in range(4):
        got = np.stack([host[(b // 16, col)][b % 16, l] for b, l in zip(bis, lis)])
        err = m2(got, ref)
        print(f"    column {col}: max rel err {err:.3e} over {n_tok} tokens", flush=True)
        assert err <= BF16_TOL, col


def _mesh3d_tools(g, mesh, layout, coords):
    """Helpers for running the feed-forward sublayer on the 3-D layout, processor by processor
    through the library: slices of the inputs, the Allreduce mesh dims of an einsum from its
    plan, and the grouped reduce of per-processor partial sums."""
    sizes = dict(zip(X, g["x"].shape))
    sizes[F] = g["w_in"].shape[1]
    shp = lambda dims: [(d, sizes[d]) for d in dims]
    axes = lambda p, q, out: mtf.einsum_plan(shp(p), shp(q), shp(out), mesh, layout)["reduce_axes"]
    group = lambda c, ax: [c2 for c2 in coords if all(c2[i] == c[i] for i in range(len(mesh)) if i not in ax)]
    sl = lambda name, dims: {c: mtf.slice_copy(g[name], dims, mesh, layout, c) for c in coords}
    # epi / aux: a component-wise operation riding on the reduce (aux per processor)
    reduced = lambda parts, ax, dtype, epi=mtf.EPI_NONE, aux=None: {
        c: mtf.reduce_partials([t for c2 in group(c, ax) for t in (parts[c2] if isinstance(parts[c2], list)
                                                                      else [parts[c2]])],
                               out_dtype=dtype, epi=epi, aux=None if aux is None else aux[c]) for c in coords}
    return axes, sl, reduced


def _mesh3d_forward(g, mesh, layout, coords, fused=False):
    """Every einsum leaves partial sums (section "Data-Parallel, Model-Parallel Layouts", last
    layout), each summed over the mesh dim its plan names; the ReLU is a component-wise operation
    applied once the hidden layer's sum is complete - as a pass of its own, or (fused) by the pass
    that completes the sum.  Returns per-processor a and y."""
    axes, sl, reduced = _mesh3d_tools(g, mesh, layout, coords)
    xs, wi, wo = sl("x", X), sl("w_in", WI), sl("w_out", WO)
    ax_h, ax_y = axes(X, WI, HID), axes(HID, WO, X)
    assert ax_h == [2] and ax_y == [1]                          # over planes, then over cols
    h_parts = {c: mtf.einsum_local(xs[c], X, wi[c], WI, HID, out_dtype=torch.float32) for c in coords}
    if fused:
        a = reduced(h_parts, ax_h, torch.bfloat16, mtf.EPI_RELU)
    else:
        h = reduced(h_parts, ax_h, torch.bfloat16)
        a = {c: mtf.einsum_local(h[c], HID, None, None, HID, epi=mtf.EPI_RELU) for c in coords}
    # fused: the narrow einsums also run as two ranges of their contracted dim (mtf_einsum_local_kranges)
    es = (lambda p, pd, q, qd, od: mtf.einsum_local_kranges(p, pd, q, qd, od, 2)) if fused else \
        (lambda p, pd, q, qd, od: mtf.einsum_local(p, pd, q, qd, od, out_dtype=torch.float32))
    y = reduced({c: es(a[c], HID, wo[c], WO, X) for c in coords}, ax_y, torch.float32)
    return dict(a=a, y=y)


def _mesh3d_backward(g, mesh, layout, coords, a, fused=False):
    """Backward from given per-processor activations `a`: four more einsums, each a partial sum."""
    axes, sl, reduced = _mesh3d_tools(g, mesh, layout, coords)
    xs, wi, wo, dys = sl("x", X), sl("w_in", WI), sl("w_out", WO), sl("dy", X)
    ax_dwo, ax_da, ax_dwi, ax_dx = axes(HID, X, WO), axes(X, WO, HID), axes(X, HID, WI), axes(HID, WI, X)
    assert ax_dwo == [0] and ax_da == [2] and ax_dwi == [0] and ax_dx == [1]   # rows, planes, rows, cols
    out = {}
    es = (lambda p, pd, q, qd, od: mtf.einsum_local_kranges(p, pd, q, qd, od, 2)) if fused else \
        (lambda p, pd, q, qd, od: mtf.einsum_local(p, pd, q, qd, od, out_dtype=torch.float32))
    out["dw_out"] = reduced({c: es(a[c], HID, dys[c], X, WO) for c in coords}, ax_dwo, torch.float32)
    da_parts = {c: mtf.einsum_local(dys[c], X, wo[c], WO, HID, out_dtype=torch.float32) for c in coords}
    if fused:
        dh = reduced(da_parts, ax_da, torch.bfloat16, mtf.EPI_MASK_GT0, a)
    else:
        da = reduced(da_parts, ax_da, torch.bfloat16)
        dh = {c: mtf.einsum_local(da[c], HID, None, None, HID, epi=mtf.EPI_MASK_GT0, aux=a[c]) for c in coords}
    out["dh"] = dh
    out["dw_in"] = reduced({c: es(xs[c], X, dh[c], HID, WI) for c in coords}, ax_dwi, torch.float32)
    out["dx"] = reduced({c: es(dh[c], HID, wi[c], WI, X) for c in coords}, ax_dx, torch.float32)
    return out


def test_three_dimensional_layout_at_shard_size_bf16():
    """The last layout of the worked example (batch -> rows, hidden -> cols, io -> planes) at shard
    size in bf16: every processor's einsums run on the matrix-core kernel on its slices
    (x[16,256,512], w[512,4096], v[4096,512]), every einsum's partial sums are reduced over the
    mesh dim its plan names, and the assembled result is compared with the oracle's unsplit layer."""
    cfg = mtf_inputs.config7()
    g = on_device(cfg)
    mesh, layout = cfg["mesh"], cfg["layout"]
    coords = OLY.all_coords(mesh)
    # each local einsum of this layout takes the matrix-core path
    for a_d, b_d, o_d, a_s, b_s, o_s in (
            (X, WI, HID, (16, 256, 512), (512, 4096), (16, 256, 4096)),
            (HID, WO, X, (16, 256, 4096), (4096, 512), (16, 256, 512)),
            (HID, X, WO, (16, 256, 4096), (16, 256, 512), (4096, 512)),
            (X, HID, WI, (16, 256, 512), (16, 256, 4096), (512, 4096))):
        assert mtf.einsum_local_path(list(zip(a_d, a_s)), list(zip(b_d, b_s)), list(zip(o_d, o_s))) == mtf.PATH_MFMA
    print("3-D layout: 8 processors, forward", flush=True)
    fwd = _mesh3d_forward(g, mesh, layout, coords)
    x, w_in, w_out, dy = (named(cfg["x"], X), named(cfg["w_in"], WI), named(cfg["w_out"], WO), named(cfg["dy"], X))
    print("3-D layout: oracle, unsplit", flush=True)
    ref = OL.ffn_fwd(x, w_in, w_out)
    for c in coords:
        for k, dims in (("a", HID), ("y", X)):
            want = OLY.slice_tensor(ref[k], mesh, layout, c)
            err = m2(f64(fwd[k][c]), want.data)
            assert err <= BF16_TOL, (k, c, err)
    # processors that differ only along the reduced mesh dim end with identical sums
    assert torch.equal(fwd["y"][(0, 0, 0)], fwd["y"][(0, 1, 0)])
    # backward from the oracle's activation (the ReLU mask is then the same bits on both sides)
    print("3-D layout: backward", flush=True)
    a_ref = {c: to_dev_bf16(OLY.slice_tensor(ref["a"], mesh, layout, c).data) for c in coords}
    refb = OL.ffn_bwd(x, ref["a"], w_in, w_out, dy)
    got = _mesh3d_backward(g, mesh, layout, coords, a_ref)
    for c in coords:
        for k, dims in (("dw_in", WI), ("dw_out", WO), ("dx", X)):
            want = OLY.slice_tensor(refb[k], mesh, layout, c)
            err = m2(f64(got[k][c]), want.data)
            assert err <= BF16_TOL, (k, c, err)
    print("3-D layout: all slices within tolerance", flush=True)
    # the ReLU and its gradient mask applied by the reduce that completes the sum: the same bits;
    # the narrow einsums as two ranges of their contracted dim: another summation order, same bound
    print("3-D layout: component-wise operations fused into the reduces, narrow einsums in ranges", flush=True)
    fwd2 = _mesh3d_forward(g, mesh, layout, coords, fused=True)
    got2 = _mesh3d_backward(g, mesh, layout, coords, a_ref, fused=True)
    for c in coords:
        assert torch.equal(fwd2["a"][c], fwd["a"][c]) and torch.equal(got2["dh"][c], got["dh"][c]), c
        err = m2(f64(fwd2["y"][c]), OLY.slice_tensor(ref["y"], mesh, layout, c).data)
        assert err <= BF16_TOL, ("y", c, err)
        for k in ("dw_in", "dw_out", "dx"):
            err = m2(f64(got2[k][c]), OLY.slice_tensor(refb[k], mesh, layout, c).data)
            assert err <= BF16_TOL, (k, c, err)


def to_dev_bf16(arr):
    return torch.from_numpy(np.ascontiguousarray(arr)).to(torch.bfloat16).cuda()
