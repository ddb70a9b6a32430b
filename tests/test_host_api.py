"""CPU-only tests of the C-ABI library: it loads, exports every declared symbol, and its
host-side integer logic (mesh numbering, slices, einsum lowering plan, error codes) agrees
bit-for-bit with the oracle.  No kernel is launched here."""
import ctypes as C
import os
import random
import re

import pytest

import paper_1811_02084_amd as mtf
from oracle import layout as OLY
from oracle.einsum import EinsumError

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "mtf.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(mtf_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 20
    for name in sorted(declared):
        assert hasattr(mtf.lib, name), f"{name} declared in mtf.h but not exported by libmtf.so"


def test_status_strings():
    for code, name in mtf.STATUS.items():
        assert mtf.status_string(code) == name


def _code(exc):
    """Oracle error code -> library status name."""
    return "MTF_ERR_" + exc.code


def _random_case(rnd):
    mesh_names = ["rows", "cols", "planes", "all"]
    mesh = [(n, rnd.choice([1, 2, 3, 4])) for n in rnd.sample(mesh_names, rnd.randint(1, 3))]
    tdims = ["batch", "length", "d_model", "d_ff", "heads", "d_k", "vocab"]
    dims = rnd.sample(tdims, rnd.randint(0, 5))
    shape = [(d, rnd.choice([1, 2, 3, 4, 6, 8, 12, 24])) for d in dims]
    layout = []
    for d in rnd.sample(tdims, rnd.randint(0, 4)):
        layout.append((d, rnd.choice([m for m, _ in mesh] + (["nowhere"] if rnd.random() < 0.05 else []))))
    if layout and rnd.random() < 0.05:
        layout.append(layout[0])                       # duplicate rule
    coord = [rnd.randrange(s) for _, s in mesh]
    if rnd.random() < 0.05:
        coord[0] = mesh[0][1]                          # out of range
    return mesh, shape, layout, coord


def test_slice_matches_oracle_on_random_cases():
    rnd = random.Random(1811)
    n_ok = n_err = 0
    for _ in range(3000):
        mesh, shape, layout, coord = _random_case(rnd)
        dims, sizes = [d for d, _ in shape], [s for _, s in shape]
        try:
            want = OLY.slice_spec(dims, sizes, mesh, layout, tuple(coord))
        except OLY.LayoutError as e:
            with pytest.raises(mtf.MtfError) as got:
                mtf.slice(shape, mesh, layout, coord)
            assert got.value.name == _code(e), (mesh, shape, layout, coord)
            n_err += 1
            continue
        assert mtf.slice(shape, mesh, layout, coord) == want, (mesh, shape, layout, coord)
        n_ok += 1
    assert n_ok > 500 and n_err > 200


def test_rank_coord_round_trip_and_three_views():
    for mesh in ([("a", 16), ("b", 16), ("c", 2)], [("a", 32), ("b", 16)], [("a", 512)]):
        for rank in (0, 1, 31, 37, 255, 511):
            c = mtf.rank_to_coord(mesh, rank)
            assert c == OLY.rank_to_coord(mesh, rank)
            assert mtf.coord_to_rank(mesh, c) == rank
        with pytest.raises(mtf.MtfError) as e:
            mtf.rank_to_coord(mesh, 512)
        assert e.value.name == "MTF_ERR_COORD_RANGE"
    with pytest.raises(mtf.MtfError):
        mtf.coord_to_rank([("a", 4)], (4,))


def test_einsum_plan_matches_oracle():
    rnd = random.Random(2084)
    tdims = ["batch", "length", "d_model", "d_ff", "heads", "d_k"]
    n_ok = n_err = 0
    for _ in range(2000):
        mesh, _, layout, _ = _random_case(rnd)
        size = {d: rnd.choice([2, 4, 6, 8, 12]) for d in tdims}
        da, db = rnd.sample(tdims, rnd.randint(1, 4)), rnd.sample(tdims, rnd.randint(1, 4))
        pool = list(dict.fromkeys(da + db))
        do = rnd.sample(pool, rnd.randint(0, len(pool)))
        if rnd.random() < 0.05:
            do = do + ["vocab"]
        a, b = [(d, size[d]) for d in da], [(d, size[d]) for d in db]
        o = [(d, size.get(d, 3)) for d in do]
        try:
            want = OLY.einsum_plan([da, db], [[s for _, s in a], [s for _, s in b]], do, mesh, layout)
        except (OLY.LayoutError, EinsumError) as e:
            with pytest.raises(mtf.MtfError) as got:
                mtf.einsum_plan(a, b, o, mesh, layout)
            assert got.value.name == _code(e), (a, b, o, mesh, layout)
            n_err += 1
            continue
        got = mtf.einsum_plan(a, b, o, mesh, layout)
        assert got["local_in"] == want["local_in"] and got["local_out"] == want["local_out"]
        assert got["reduce_axes"] == want["reduce_axes"] and got["flops_local"] == want["flops_local"]
        n_ok += 1
    assert n_ok > 300 and n_err > 100


def test_paper_layouts_through_the_library():
    b, d_io, d_h, n = 48, 12, 24, 4
    assert mtf.slice([("batch", b), ("io", d_io)], [("all", n)], [("batch", "all")], (3,)) == ((36, 0), (12, 12))
    assert mtf.slice([("io", d_io), ("hidden", d_h)], [("all", n)], [("hidden", "all")], (1,)) == ((0, 6), (12, 6))
    with pytest.raises(mtf.MtfError) as e:      # the illegal layout of the worked example
        mtf.slice([("batch", b), ("hidden", d_h)], [("all", n)], [("batch", "all"), ("hidden", "all")], (0,))
    assert e.value.name == "MTF_ERR_LAYOUT_CONFLICT"
    plan = mtf.einsum_plan([("batch", b), ("hidden", d_h)], [("hidden", d_h), ("io", d_io)],
                           [("batch", b), ("io", d_io)], [("rows", 2), ("cols", 2)],
                           [("batch", "rows"), ("hidden", "cols")])
    assert plan["reduce_axes"] == [1] and plan["local_out"] == (24, 12)     # summed by processor-column


def test_argument_validation_needs_no_gpu():
    """Entry points reject bad arguments before touching the device."""
    lib = mtf.lib
    d = mtf.mtf_ffn_dims(2, 8, 16, 64)
    assert lib.mtf_ffn_fwd(C.byref(d), None, None, None, None, None, None) == -1          # NULL
    bad = mtf.mtf_ffn_dims(2, 8, 15, 64)
    p = C.c_void_p(4096)
    assert lib.mtf_ffn_fwd(C.byref(bad), p, p, p, p, p, None) == -10                      # UNSUPPORTED
    assert lib.mtf_ffn_bwd(C.byref(d), p, p, p, p, p, p, p, p, None, C.c_size_t(0), None) == -11   # WORKSPACE
    m = mtf.mtf_mha_dims(2, 8, 16, 2, 64)
    assert lib.mtf_mha_fwd(C.byref(m), p, p, p, p, p, C.c_float(1.0), 0, p, p, p, p, p, p, None) == -10
    assert lib.mtf_ffn_fwd(C.byref(d), C.c_void_p(4097), p, p, p, p, None) == -14         # ALIGN
    assert lib.mtf_ffn_bwd_workspace_bytes(C.byref(d)) == 2 * 8 * 64 * 2
    assert lib.mtf_reduce_partials(None, 1, None, 0, p, 0, C.c_int64(4), None) == -1
    arr = (C.c_void_p * 1)(None)
    assert lib.mtf_reduce_partials(arr, 1, None, 0, None, 0, C.c_int64(0), None) == 0        # empty: nothing to do
    assert b"MTF_ERR" in lib.mtf_last_error()
    one = (C.c_void_p * 1)(4096)
    assert lib.mtf_reduce_partials_epi(one, 1, None, 0, p, 0, C.c_int64(8), 3, None, None) == -10   # no such epilogue here
    assert lib.mtf_reduce_partials_epi(one, 1, None, 0, p, 0, C.c_int64(8), 2, None, None) == -1    # mask without aux
    assert lib.mtf_reduce_partials_epi(one, 1, None, 0, p, 0, C.c_int64(8), 2, C.c_void_p(4098), None) == -14
    assert lib.mtf_einsum_local_kranges(p, None, p, None, None, 2, None, None) == -1                 # outs NULL
    assert lib.mtf_einsum_local_kranges(p, None, p, None, one, 5, None, None) == -10                # at most 4 ranges
    # the worked example with its bias, broadcasting addition, local reduction
    assert lib.mtf_ffn_bias_fwd(C.byref(d), p, p, None, p, p, p, None) == -1                     # bias NULL
    assert lib.mtf_ffn_bias_bwd(C.byref(d), p, p, p, p, p, p, p, p, p, None, C.c_size_t(0), None) == -11
    assert lib.mtf_ffn_bias_bwd_workspace_bytes(C.byref(d)) >= lib.mtf_ffn_bwd_workspace_bytes(C.byref(d))
    k = mtf.binding._Keep()
    big, small, other = k.shape([("p", 4), ("q", 8)]), k.shape([("q", 8)]), k.shape([("z", 8)])
    wrong = k.shape([("q", 4)])
    assert lib.mtf_add_broadcast(p, C.byref(big), p, C.byref(other), p, 0, 0, None) == -9        # OUT_NOT_SUBSET
    assert lib.mtf_add_broadcast(p, C.byref(big), p, C.byref(wrong), p, 0, 0, None) == -3        # SIZE_MISMATCH
    assert lib.mtf_add_broadcast(None, C.byref(big), p, C.byref(small), p, 0, 0, None) == -1
    assert lib.mtf_reduce_local(p, C.byref(big), p, C.byref(other), 0, 0, 0, None, C.c_size_t(0), None) == -9
    assert lib.mtf_reduce_local(p, C.byref(big), p, C.byref(small), 0, 0, 7, None, C.c_size_t(0), None) == -10
    assert lib.mtf_reduce_local(p, C.byref(big), p, C.byref(small), 0, 0, 0, None, C.c_size_t(0), None) == -11
    assert lib.mtf_reduce_local_workspace_bytes(C.byref(big), C.byref(small)) > 0
    # attention core at any head width
    m64 = mtf.mtf_mha_dims(2, 16, 128, 2, 64)                                 # no fused kernel at this width
    assert lib.mtf_attention_fwd_workspace_bytes(C.byref(m64)) > 0
    for fused in (128, 256):
        mf = mtf.mtf_mha_dims(2, 16, 2 * fused, 2, fused)
        assert lib.mtf_attention_fwd_workspace_bytes(C.byref(mf)) == 0
        assert lib.mtf_attention_bwd_workspace_bytes(C.byref(mf)) == 2 * 2 * 16 * 4   # delta[batch, heads, length] fp32
    assert lib.mtf_attention_fwd(C.byref(m64), p, p, p, C.c_float(1.0), 0, p, p, None, C.c_size_t(0), None) == -11
    assert lib.mtf_attention_fwd(C.byref(mtf.mtf_mha_dims(2, 12, 128, 2, 64)), p, p, p, C.c_float(1.0), 0, p, p,
                                 p, C.c_size_t(1 << 30), None) == -10                                  # length % 8
    assert lib.mtf_attention_bwd(C.byref(m64), p, p, p, p, p, None, C.c_float(1.0), 0, p, p, p, p,
                                 C.c_size_t(1 << 30), None) == -1
    # the data-parallel training step
    arr1 = (C.c_void_p * 1)(4096)
    assert lib.mtf_sgd_step(None, 1, C.c_float(0.1), p, p, C.c_int64(8), None) == -1
    assert lib.mtf_sgd_step(arr1, 0, C.c_float(0.1), p, p, C.c_int64(8), None) == -10
    assert lib.mtf_sgd_step(arr1, 1, C.c_float(0.1), None, p, C.c_int64(8), None) == -1
    assert lib.mtf_sgd_step(arr1, 1, C.c_float(0.1), C.c_void_p(4100), p, C.c_int64(8), None) == -14
    assert lib.mtf_sgd_step(arr1, 1, C.c_float(0.1), None, None, C.c_int64(0), None) == 0       # nothing to update
    # layer normalisation
    i64 = C.c_int64
    lib.mtf_layer_norm_bwd_workspace_bytes.restype = C.c_size_t
    assert lib.mtf_layer_norm_fwd(None, p, p, C.c_float(1e-6), i64(4), i64(64), p, p, p, None) == -1
    assert lib.mtf_layer_norm_fwd(p, p, p, C.c_float(1e-6), i64(4), i64(60), p, p, p, None) == -10      # d_model % 8
    assert lib.mtf_layer_norm_fwd(p, p, p, C.c_float(1e-6), i64(4), i64(8192), p, p, p, None) == -10    # too wide
    assert lib.mtf_layer_norm_fwd(p, p, p, C.c_float(1e-6), i64(-1), i64(64), p, p, p, None) == -3
    assert lib.mtf_layer_norm_fwd(p, p, p, C.c_float(1e-6), i64(0), i64(64), p, p, p, None) == 0        # no rows
    assert lib.mtf_layer_norm_fwd(C.c_void_p(4100), p, p, C.c_float(1e-6), i64(4), i64(64), p, p, p, None) == -14
    assert lib.mtf_residual_layer_norm_fwd(None, 0, p, p, p, C.c_float(1e-6), i64(4), i64(64), p, p, p, p, None) == -10
    assert lib.mtf_residual_layer_norm_fwd(None, 2, p, p, p, C.c_float(1e-6), i64(4), i64(64), p, p, p, p, None) == -1
    assert lib.mtf_layer_norm_bwd_workspace_bytes(i64(4096), i64(1024)) == 512 * 2 * 1024 * 4
    assert lib.mtf_layer_norm_bwd_workspace_bytes(i64(6), i64(64)) == 2 * 2 * 64 * 4
    assert lib.mtf_layer_norm_bwd(p, p, p, p, p, i64(8), i64(64), p, p, p, None, C.c_size_t(0), None) == -11
    assert lib.mtf_layer_norm_bwd(p, p, p, p, p, i64(8), i64(64), p, None, p, p, C.c_size_t(1 << 20), None) == -1
    # vocabulary-split operations
    assert lib.mtf_embedding_local(None, i64(4), p, i64(8), i64(16), i64(0), p, 0, None) == -1
    assert lib.mtf_embedding_local(p, i64(4), p, i64(8), i64(12), i64(0), p, 0, None) == -10          # d_model % 8
    assert lib.mtf_embedding_local(p, i64(0), None, i64(8), i64(16), i64(0), None, 0, None) == 0      # no tokens
    assert lib.mtf_embedding_grad_local(p, i64(4), p, i64(0), i64(16), i64(0), p, None) == -3
    assert lib.mtf_max_partials(None, 1, p, i64(4), None) == -1
    assert lib.mtf_xent_stats_local(p, i64(4), i64(8), None, p, i64(0), p, p, None) == -1
    assert lib.mtf_xent_loss(p, p, None, p, i64(4), None) == -1
    assert lib.mtf_xent_grad_local(p, i64(4), i64(6), p, p, p, i64(0), p, p, None) == -10             # vocab % 4


def test_reshape_plan_matches_oracle_and_the_papers_three_cases():
    from oracle.layout import reshape_plan as o_plan
    mesh, layout = [("all", 4)], [("batch", "all"), ("hidden", "all")]
    shp = lambda dims, sizes=(8, 12): list(zip(dims, sizes))
    assert mtf.reshape_plan(shp(("batch", "io")), shp(("rows", "io")), mesh, layout) == ["allgather"]
    assert mtf.reshape_plan(shp(("rows", "io")), shp(("batch", "io")), mesh, layout) == ["slice"]
    assert mtf.reshape_plan(shp(("batch", "units")), shp(("examples", "hidden")), mesh, layout) == ["alltoall"]
    two = [("rows", 2), ("cols", 2)]
    lay2 = [("batch", "rows"), ("hidden", "cols"), ("vocab", "cols"), ("z", "rows")]
    names = ["batch", "hidden", "vocab", "z", "p", "q"]
    import itertools
    for a in itertools.permutations(names, 2):
        for b in itertools.permutations(names, 2):
            try:
                want = o_plan(a, b, (8, 12), two, lay2)
            except Exception as e:              # both must refuse, with the same code
                with pytest.raises(mtf.MtfError) as got:
                    mtf.reshape_plan(shp(a), shp(b), two, lay2)
                assert got.value.name == "MTF_ERR_" + e.code, (a, b)
                continue
            assert mtf.reshape_plan(shp(a), shp(b), two, lay2) == want, (a, b)


def test_einsum_local_path_reports_the_kernel_that_would_run():
    """Host-only query: which of the two kernels a local einsum would get.  Includes the bound on
    the leading dims that the matrix-core kernel's 32-bit per-lane byte offsets impose."""
    import torch
    P = mtf.einsum_local_path
    X, W, Hd = ("batch", "length", "d_model"), ("d_model", "d_ff"), ("batch", "length", "d_ff")
    shp = lambda dims, sizes: list(zip(dims, sizes))
    # the feed-forward einsum of config 2: bf16, everything divisible by 8
    assert P(shp(X, (16, 256, 1024)), shp(W, (1024, 4096)), shp(Hd, (16, 256, 4096))) == mtf.PATH_MFMA
    # its weight gradient (both operands token-major) and the transposed-weight product
    assert P(shp(X, (16, 256, 1024)), shp(Hd, (16, 256, 4096)), shp(W, (1024, 4096))) == mtf.PATH_MFMA
    assert P(shp(Hd, (16, 256, 4096)), shp(W, (1024, 4096)), shp(X, (16, 256, 1024))) == mtf.PATH_MFMA
    # fp32 inputs, an odd contraction size, a one-operand einsum: the generic kernel
    assert P(shp(X, (2, 8, 16)), shp(W, (16, 64)), shp(Hd, (2, 8, 64)), in_dtype=torch.float32) == mtf.PATH_GENERIC
    assert P(shp(X, (2, 8, 20)), shp(W, (20, 64)), shp(Hd, (2, 8, 64))) == mtf.PATH_GENERIC
    assert P(shp(X, (2, 8, 16)), None, [("d_model", 16)]) == mtf.PATH_GENERIC
    # one operand, dims kept in place: the component-wise pass (whole 16-byte vectors only)
    assert P(shp(X, (2, 8, 16)), None, shp(X, (2, 8, 16)), epi=mtf.EPI_RELU) == mtf.PATH_COMPONENTWISE
    assert P(shp(X, (2, 8, 16)), None, shp(("length", "batch", "d_model"), (8, 2, 16))) == mtf.PATH_GENERIC
    assert P(shp(X, (3, 1, 5)), None, shp(X, (3, 1, 5))) == mtf.PATH_GENERIC
    # misaligned operand address: reported as the error the einsum itself would give
    with pytest.raises(mtf.MtfError) as e:
        P(shp(X, (2, 8, 16)), shp(W, (16, 64)), shp(Hd, (2, 8, 64)), a_ptr=0x1004)
    assert e.value.name == "MTF_ERR_ALIGN"
    # leading dims: a k-contiguous operand's per-lane offset reaches 255 * ld * 2 + 128 bytes, an
    # mn-contiguous one's 63 * ld * 2 + 512; both must fit in 32 bits
    k_ok = ((2 ** 32 - 1 - 128) // (255 * 2)) // 8 * 8            # largest ld (multiple of 8) that fits
    assert P([("length", 8), ("d_model", k_ok)], [("d_model", k_ok), ("d_ff", 8)],
             [("length", 8), ("d_ff", 8)]) == mtf.PATH_MFMA
    assert P([("length", 8), ("d_model", k_ok + 8)], [("d_model", k_ok + 8), ("d_ff", 8)],
             [("length", 8), ("d_ff", 8)]) == mtf.PATH_GENERIC
    n_ok = ((2 ** 32 - 1 - 512) // (63 * 2)) // 8 * 8
    assert P([("length", 8), ("d_model", 64)], [("d_model", 64), ("d_ff", n_ok)],
             [("length", 8), ("d_ff", n_ok)]) == mtf.PATH_MFMA
    assert P([("length", 8), ("d_model", 64)], [("d_model", 64), ("d_ff", n_ok + 8)],
             [("length", 8), ("d_ff", n_ok + 8)]) == mtf.PATH_GENERIC


def test_reshape_of_a_rank_0_tensor_is_refused():
    from paper_1811_02084_amd import binding
    k = binding._Keep()
    empty = k.shape([])
    place = k.place([("all", 2)], [], [0])
    ptrs = (C.c_void_p * 2)(0x1000, 0x2000)
    rc = binding.lib.mtf_reshape_virtual(ptrs, C.byref(empty), C.byref(empty), C.byref(place), C.c_void_p(0x3000),
                                         0, None)
    assert mtf.status_string(rc) == "MTF_ERR_RANK"
