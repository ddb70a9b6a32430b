"""Pins for the oracle's layout / slice / lowering code against what the paper prints:
slice shapes of the worked example, Table 1, the Allreduce volumes, the replication
statements, the illegal and inefficient layouts, the three views of 512 processors,
Appendix B's two ratios, and the layout-independence statement (bit-exact with integers)."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle.einsum import nt, einsum, EinsumError
from oracle.layout import (LayoutError, all_coords, coord_to_rank, einsum_plan, lowered_einsum,
                           mesh_size, rank_to_coord, slice_spec, slice_tensor)

GOLD = os.path.join(os.path.dirname(__file__), "golden")
SYM = dict(b=48, d_io=12, d_h=24, n=4, r=2, c=4, p=3)

# the einsums of the worked example, forward then backward (gradients of einsums are einsums)
EXAMPLE = [
    ("h", ("batch", "io"), ("io", "hidden"), ("batch", "hidden")),
    ("y", ("batch", "hidden"), ("hidden", "io"), ("batch", "io")),
    ("dv", ("batch", "hidden"), ("batch", "io"), ("hidden", "io")),
    ("dh", ("batch", "io"), ("hidden", "io"), ("batch", "hidden")),
    ("dw", ("batch", "io"), ("batch", "hidden"), ("io", "hidden")),
    ("dx", ("batch", "hidden"), ("io", "hidden"), ("batch", "io")),
]
SIZE = dict(batch=SYM["b"], io=SYM["d_io"], hidden=SYM["d_h"])


def _rows(fname):
    for line in open(os.path.join(GOLD, fname)):
        line = line.strip()
        if line and not line.startswith("#"):
            yield [f.strip() for f in line.split(";")]


def _mesh(text):
    return [(kv.split("=")[0], SYM[kv.split("=")[1]]) for kv in text.split(",")]


def _layout(text):
    return [tuple(kv.split(">")) for kv in text.split(",")] if text else []


def _val(expr):
    return Fraction(eval(expr, {}, {k: Fraction(v) for k, v in SYM.items()}))


def _plan(e, mesh, layout):
    _, da, db, do = e
    return einsum_plan([da, db], [[SIZE[d] for d in da], [SIZE[d] for d in db]], do, mesh, layout)


def test_slice_shapes_printed_in_the_worked_example():
    n_checked = 0
    for row in _rows("example_slices.txt"):
        if row[2] == "ALLREDUCED":
            continue
        mesh_t, lay_t, tensor, dims_t, shape_t = row
        mesh, layout, dims = _mesh(mesh_t), _layout(lay_t), tuple(dims_t.split(","))
        want = tuple(int(_val(s)) for s in shape_t.split(","))
        for coord in all_coords(mesh):
            offs, locs = slice_spec(dims, [SIZE[d] for d in dims], mesh, layout, coord)
            assert locs == want, (tensor, coord)
        n_checked += 1
    assert n_checked == 5


def test_allreduced_values_per_processor():
    for row in _rows("example_slices.txt"):
        if row[2] != "ALLREDUCED":
            continue
        mesh_t, lay_t, tag, expr = row
        mesh, layout = _mesh(mesh_t), _layout(lay_t)
        total = 0
        for e in EXAMPLE:
            plan = _plan(e, mesh, layout)
            if plan["reduce_axes"]:
                total += int(np.prod(plan["local_out"]))
        assert total == _val(expr), (lay_t, total)


def test_table1_comp_comm_memory():
    rows = list(_rows("table1_costs.txt"))
    assert len(rows) == 5
    for mesh_t, lay_t, comp, comm, mem in rows:
        mesh, layout = _mesh(mesh_t), _layout(lay_t)
        plans = {e[0]: _plan(e, mesh, layout) for e in EXAMPLE}
        # computation: one multiply-add per local iteration-space point, every einsum alike
        for pl in plans.values():
            assert Fraction(pl["flops_local"], 2) == _val(comp)
        # communication: the table drops the constant 2 (forward + backward)
        allred = sum(int(np.prod(pl["local_out"])) for pl in plans.values() if pl["reduce_axes"])
        assert allred == 2 * _val(comm)
        # memory: slices of x, h and w (v has the size of w)
        coord = (0,) * len(mesh)
        elems = 0
        for dims in (("batch", "io"), ("batch", "hidden"), ("io", "hidden")):
            _, locs = slice_spec(dims, [SIZE[d] for d in dims], mesh, layout, coord)
            elems += int(np.prod(locs))
        assert elems == _val(mem)


def test_which_einsums_allreduce_where():
    dp = ([("all", 4)], [("batch", "all")])
    mp = ([("all", 4)], [("hidden", "all")])
    two = ([("rows", 2), ("cols", 4)], [("batch", "rows"), ("hidden", "cols")])
    three = ([("rows", 2), ("cols", 4), ("planes", 3)],
             [("batch", "rows"), ("hidden", "cols"), ("io", "planes")])
    red = lambda ml: {e[0]: _plan(e, *ml)["reduce_axes"] for e in EXAMPLE}
    assert red(dp) == dict(h=[], y=[], dv=[0], dh=[], dw=[0], dx=[])        # only parameter grads
    assert red(mp) == dict(h=[], y=[0], dv=[], dh=[], dw=[], dx=[0])        # y and dx
    assert red(two) == dict(h=[], y=[1], dv=[0], dh=[], dw=[0], dx=[1])     # by column / by row
    r3 = red(three)
    assert all(len(axes) == 1 for axes in r3.values())                      # exactly one mesh dim
    assert r3 == dict(h=[2], y=[1], dv=[0], dh=[2], dw=[0], dx=[1])
    # 3-D: every matrix tiled over two mesh dims and replicated over the third
    mesh3, lay3 = three
    for dims in (("batch", "io"), ("batch", "hidden"), ("io", "hidden")):
        holders = {}
        for c in all_coords(mesh3):
            holders.setdefault(slice_spec(dims, [SIZE[d] for d in dims], mesh3, lay3, c), []).append(c)
        used = [m for t, m in lay3 if t in dims]
        assert len(used) == 2
        (free_size,) = [s for nm, s in mesh3 if nm not in used]
        assert len(holders) == mesh_size(mesh3) // free_size
        assert all(len(v) == free_size for v in holders.values())


def test_replication_statements():
    mesh = [("all", 4)]
    for dims in (("io", "hidden"), ("hidden", "io"), ("hidden",)):           # w, v, bias under DP
        specs = {slice_spec(dims, [SIZE[d] for d in dims], mesh, [("batch", "all")], c)
                 for c in all_coords(mesh)}
        assert specs == {(tuple(0 for _ in dims), tuple(SIZE[d] for d in dims))}
    for dims in (("batch", "io"),):                                          # x, y under MP
        specs = {slice_spec(dims, [SIZE[d] for d in dims], mesh, [("hidden", "all")], c)
                 for c in all_coords(mesh)}
        assert len(specs) == 1
    mesh2, lay2 = [("rows", 2), ("cols", 4)], [("batch", "rows"), ("hidden", "cols")]
    for r in range(2):                                                       # same row, same x slice
        specs = {slice_spec(("batch", "io"), (48, 12), mesh2, lay2, (r, c)) for c in range(4)}
        assert specs == {((r * 24, 0), (24, 12))}


def test_empty_layout_is_full_replication_and_still_correct():
    rng = np.random.default_rng(0)
    x = nt(rng.integers(-2, 3, (6, 4)), ("batch", "io"))
    w = nt(rng.integers(-2, 3, (4, 8)), ("io", "hidden"))
    loc, red = lowered_einsum([x, w], ("batch", "hidden"), [("all", 3)], [])
    full = einsum([x, w], ("batch", "hidden"))
    for c in all_coords([("all", 3)]):
        assert np.array_equal(loc[c].data, full.data) and np.array_equal(red[c].data, full.data)


def test_illegal_and_rejected_layouts():
    mesh = [("all", 4)]
    bad = [("batch", "all"), ("hidden", "all")]
    with pytest.raises(LayoutError) as e:                  # the paper's illegal layout: tensor h
        slice_spec(("batch", "hidden"), (48, 24), mesh, bad, (0,))
    assert e.value.code == "LAYOUT_CONFLICT"
    slice_spec(("batch", "io"), (48, 12), mesh, bad, (0,))      # x alone is fine under it
    with pytest.raises(LayoutError) as e:
        slice_spec(("batch",), (50,), mesh, [("batch", "all")], (0,))
    assert e.value.code == "INDIVISIBLE"
    with pytest.raises(LayoutError) as e:
        slice_spec(("batch", "batch"), (4, 4), mesh, [], (0,))
    assert e.value.code == "DUP_DIM"
    with pytest.raises(LayoutError) as e:
        slice_spec(("batch",), (4,), mesh, [("batch", "nowhere")], (0,))
    assert e.value.code == "UNKNOWN_MESH_DIM"
    with pytest.raises(LayoutError) as e:
        slice_spec(("batch",), (4,), [("a", 2), ("b", 2)], [("batch", "a"), ("batch", "b")], (0, 0))
    assert e.value.code == "DUP_RULE"
    with pytest.raises(LayoutError) as e:
        slice_spec(("batch",), (4,), mesh, [("batch", "all")], (4,))
    assert e.value.code == "COORD_RANGE"
    # two different dims of ONE einsum on one mesh dim (each tensor alone is legal)
    with pytest.raises(LayoutError) as e:
        einsum_plan([("batch",), ("hidden",)], [(4,), (4,)], (), mesh, bad)
    assert e.value.code == "LAYOUT_CONFLICT"
    with pytest.raises(EinsumError) as e:
        einsum_plan([("batch",)], [(4,)], ("hidden",), mesh, [])
    assert e.value.code == "OUT_NOT_SUBSET"


def test_same_processors_three_mesh_views():
    views = [[("a", 16), ("b", 16), ("c", 2)], [("a", 32), ("b", 16)], [("a", 512)]]
    for mesh in views:
        grid = np.arange(512).reshape([s for _, s in mesh])
        for rank in (0, 1, 31, 32, 255, 511):
            coord = rank_to_coord(mesh, rank)
            assert grid[coord] == rank and coord_to_rank(mesh, coord) == rank
    assert rank_to_coord(views[0], 37) == (1, 2, 1) and rank_to_coord(views[1], 37) == (2, 5)
    with pytest.raises(LayoutError):
        rank_to_coord(views[2], 512)


def test_iota_slices_and_exact_tiling():
    mesh = [("rows", 2), ("cols", 3), ("planes", 2)]
    layout = [("batch", "rows"), ("hidden", "cols")]
    t = nt(np.arange(4 * 5 * 6).reshape(4, 5, 6), ("batch", "io", "hidden"))
    cover = np.zeros(t.data.shape, dtype=int)
    for c in all_coords(mesh):
        s = slice_tensor(t, mesh, layout, c)
        offs, locs = slice_spec(t.dims, t.data.shape, mesh, layout, c)
        assert locs == (2, 5, 2) and offs == (2 * c[0], 0, 2 * c[1])
        # the value of an iota tensor IS its global linear index
        assert s.data[0, 0, 0] == offs[0] * 30 + offs[2]
        assert s.data[1, 4, 1] == (offs[0] + 1) * 30 + 4 * 6 + offs[2] + 1
        cover[tuple(slice(o, o + n) for o, n in zip(offs, locs))] += 1
    assert np.all(cover == 2)                 # once per replica; replicas = size of unused "planes"


def test_appendix_b_ratios():
    u = 64
    sz = [(u, u), (u, u)]
    dims = [("i", "k"), ("k", "j")]
    def ratio(mesh, layout):
        pl = einsum_plan(dims, sz, ("i", "j"), mesh, layout)
        elems = sum(int(np.prod(s)) for s in pl["local_in"]) + int(np.prod(pl["local_out"]))
        return Fraction(pl["flops_local"], elems)
    assert ratio([("r", 8), ("c", 8)], [("i", "r"), ("j", "c")]) == Fraction(2 * u, 17)
    assert ratio([("x", 4), ("y", 4), ("z", 4)], [("i", "x"), ("j", "y"), ("k", "z")]) == Fraction(u, 6)


LAYOUTS = [
    ([("all", 4)], [("batch", "all")]),
    ([("all", 4)], [("hidden", "all")]),
    ([("rows", 2), ("cols", 2)], [("batch", "rows"), ("hidden", "cols")]),
    ([("rows", 2), ("cols", 2), ("planes", 2)],
     [("batch", "rows"), ("hidden", "cols"), ("io", "planes")]),
    ([("all", 4)], []),
]


@pytest.mark.parametrize("mesh,layout", LAYOUTS)
def test_layout_independence_bit_exact_on_integers(mesh, layout):
    """Every layout of the worked example gives the identical result: the reduced partial
    sums each processor ends up with are exactly its slice of the unsplit einsum."""
    rng = np.random.default_rng(11)
    sizes = dict(batch=8, io=4, hidden=12)
    for name, da, db, do in EXAMPLE:
        a = nt(rng.integers(-2, 3, [sizes[d] for d in da]), da)
        b = nt(rng.integers(-2, 3, [sizes[d] for d in db]), db)
        full = einsum([a, b], do)
        local, reduced = lowered_einsum([a, b], do, mesh, layout)
        for c in all_coords(mesh):
            assert np.array_equal(reduced[c].data, slice_tensor(full, mesh, layout, c).data), name
