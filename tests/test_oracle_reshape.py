"""Pins for the oracle's reshape lowering: the three communication patterns the paper names, and
the collectives written out against the plain definition (the slice of the renamed tensor)."""
import numpy as np
import pytest

from oracle.einsum import nt
from oracle.layout import (LayoutError, all_coords, alltoall_exchange, lowered_reshape, reshape_plan,
                           slice_tensor)

RNG = np.random.default_rng(1811)


def test_the_three_patterns_of_the_reshape_subsection():
    mesh, layout = [("all", 4)], [("batch", "all"), ("hidden", "all")]
    sizes = (8, 12)
    # split in the input, not in the output: allgather
    assert reshape_plan(("batch", "io"), ("rows", "io"), sizes, mesh, layout) == ["allgather"]
    # split in the output, not in the input: slicing only
    assert reshape_plan(("rows", "io"), ("batch", "io"), sizes, mesh, layout) == ["slice"]
    # different dims split across the same mesh dim before and after (data- to model-parallel): alltoall
    assert reshape_plan(("batch", "units"), ("examples", "hidden"), sizes, mesh, layout) == ["alltoall"]
    # same position split before and after, or nothing split: no communication
    assert reshape_plan(("batch", "io"), ("batch", "d"), sizes, mesh, layout) == ["none"]
    assert reshape_plan(("p", "q"), ("r", "s"), sizes, mesh, layout) == ["none"]
    two = [("rows", 2), ("cols", 2)]
    lay2 = [("batch", "rows"), ("hidden", "cols"), ("vocab", "cols")]
    assert reshape_plan(("batch", "hidden"), ("tokens", "vocab"), sizes, two, lay2) == ["allgather", "none"]
    assert reshape_plan(("hidden", "x"), ("batch", "hidden"), sizes, two, lay2) == ["slice", "alltoall"]
    with pytest.raises(LayoutError) as e:
        reshape_plan(("batch", "io"), ("io",), sizes, mesh, layout)
    assert e.value.code == "SIZE_MISMATCH"
    with pytest.raises(LayoutError) as e:
        reshape_plan(("batch", "io"), ("io", "hidden"), (8, 10), mesh, layout)
    assert e.value.code == "INDIVISIBLE"


CASES = [
    ([("all", 4)], [("batch", "all"), ("hidden", "all")], ("batch", "io"), ("rows", "io")),
    ([("all", 4)], [("batch", "all"), ("hidden", "all")], ("rows", "io"), ("batch", "io")),
    ([("all", 4)], [("batch", "all"), ("hidden", "all")], ("batch", "units"), ("examples", "hidden")),
    ([("rows", 2), ("cols", 3)], [("batch", "rows"), ("hidden", "cols"), ("vocab", "cols"), ("z", "rows")],
     ("batch", "hidden", "k"), ("tokens", "x", "vocab")),
    ([("rows", 2), ("cols", 3)], [("batch", "rows"), ("hidden", "cols"), ("vocab", "cols"), ("z", "rows")],
     ("hidden", "batch", "k"), ("z", "m", "vocab")),
    ([("rows", 2), ("cols", 3)], [], ("a", "b", "c"), ("d", "e", "f")),
]


@pytest.mark.parametrize("case", CASES, ids=[f"{c[2]}->{c[3]}" for c in CASES])
def test_collectives_give_every_processor_the_slice_of_the_renamed_tensor(case):
    mesh, layout, in_dims, out_dims = case
    t = nt(RNG.integers(0, 1000, size=(12,) * len(in_dims)).astype(np.float64), in_dims)
    got = lowered_reshape(t, out_dims, mesh, layout)
    renamed = nt(t.data, out_dims)
    for c in all_coords(mesh):
        want = slice_tensor(renamed, mesh, layout, c)
        assert got[c].dims == tuple(out_dims)
        assert np.array_equal(got[c].data, want.data), c


def test_alltoall_exchange_delivers_what_gather_then_slice_delivers():
    """Switching from data- to model-parallelism: batch split before, hidden split after."""
    mesh, layout = [("all", 4)], [("batch", "all"), ("hidden", "all")]
    t = nt(RNG.integers(0, 1000, size=(8, 12)).astype(np.float64), ("batch", "units"))
    slices = [slice_tensor(t, mesh, layout, (j,)).data for j in range(4)]
    moved = alltoall_exchange(slices, 0, 1)
    want = lowered_reshape(t, ("examples", "hidden"), mesh, layout)
    for j in range(4):
        assert np.array_equal(moved[j], want[(j,)].data)
        assert moved[j].shape == (8, 3)
    # every member sends (n-1)/n of its slice, an allgather would receive (n-1) whole slices
    sent = sum(a.size for a in slices) * 3 // 4
    assert sent == 8 * 12 * 3 // 4


# ------------------------------------------------------------------ reshape that changes sizes
from oracle.layout import lowered_reshape_general, reshape_general  # noqa: E402


def test_size_changing_reshape_worked_by_hand():
    # [4, 3] holding 0..11, rows split over 2 processors: processor 0 has 0..5, processor 1 has 6..11.
    # As [2, 6] with the second dim split: the full output is [[0..5], [6..11]], so processor 0
    # holds columns 0..2 of both rows and processor 1 columns 3..5.
    t = nt(np.arange(12.0).reshape(4, 3), ("a", "b"))
    mesh, layout = [("x", 2)], [("a", "x"), ("d", "x")]
    for fn in (reshape_general, lowered_reshape_general):
        got = fn(t, ("c", "d"), (2, 6), mesh, layout)
        assert got[(0,)].dims == ("c", "d")
        assert got[(0,)].data.tolist() == [[0.0, 1.0, 2.0], [6.0, 7.0, 8.0]]
        assert got[(1,)].data.tolist() == [[3.0, 4.0, 5.0], [9.0, 10.0, 11.0]]
    # merging both dims into one unsplit dim: everybody holds everything, in order
    got = lowered_reshape_general(t, ("flat",), (12,), mesh, layout)
    assert got[(0,)].data.tolist() == list(range(12)) and got[(1,)].data.tolist() == list(range(12))
    # splitting heads out of a merged dim: [2, 6] -> [2, 3, 2] with the new middle dim split
    t2 = nt(np.arange(12.0).reshape(2, 6), ("tokens", "merged"))
    got = lowered_reshape_general(t2, ("tokens", "heads", "k"), (2, 3, 2), [("x", 3)], [("heads", "x")])
    assert got[(1,)].data.tolist() == [[[2.0, 3.0]], [[8.0, 9.0]]]


GENERAL_CASES = [  # mesh, layout, in dims, in sizes, out dims, out sizes
    ([("x", 2)], [("a", "x"), ("d", "x")], ("a", "b"), (4, 6), ("c", "d"), (3, 8)),
    ([("x", 2), ("y", 3)], [("batch", "x"), ("heads", "y")], ("batch", "length", "hidden"), (4, 5, 12),
     ("tokens", "heads", "k"), (20, 6, 2)),
    ([("x", 2), ("y", 2)], [("tokens", "x"), ("hidden", "y")], ("tokens", "heads", "k"), (8, 4, 3),
     ("batch", "length", "hidden"), (2, 4, 12)),
    ([("x", 4)], [("p", "x"), ("s", "x")], ("p", "q", "r"), (4, 2, 6), ("s", "t"), (8, 6)),
    ([("x", 2), ("y", 2)], [("a", "x"), ("b", "y"), ("c", "y"), ("d", "x")], ("a", "b"), (6, 4), ("c", "d"), (4, 6)),
    ([("x", 3)], [("nothing", "x")], ("a", "b"), (5, 7), ("c",), (35,)),
]


@pytest.mark.parametrize("case", GENERAL_CASES, ids=[str(c[3]) + "->" + str(c[5]) for c in GENERAL_CASES])
def test_size_changing_reshape_from_slices_equals_the_definition(case):
    mesh, layout, in_dims, in_sizes, out_dims, out_sizes = case
    t = nt(RNG.standard_normal(in_sizes), in_dims)
    want = reshape_general(t, out_dims, out_sizes, mesh, layout)
    got = lowered_reshape_general(t, out_dims, out_sizes, mesh, layout)
    for c in all_coords(mesh):
        assert got[c].dims == want[c].dims and np.array_equal(got[c].data, want[c].data)
    # assembling the output slices and reshaping back gives the input again
    full = np.empty(out_sizes)
    from oracle.layout import slice_spec
    for c in all_coords(mesh):
        offs, locs = slice_spec(out_dims, out_sizes, mesh, layout, c)
        full[tuple(slice(o, o + n) for o, n in zip(offs, locs))] = got[c].data
    assert np.array_equal(full.reshape(in_sizes), t.data)


def test_size_changing_reshape_with_equal_sizes_is_the_renaming_reshape():
    mesh, layout = [("all", 4)], [("batch", "all"), ("hidden", "all")]
    t = nt(RNG.standard_normal((8, 12)), ("batch", "units"))
    a = lowered_reshape(t, ("examples", "hidden"), mesh, layout)
    b = lowered_reshape_general(t, ("examples", "hidden"), (8, 12), mesh, layout)
    for c in all_coords(mesh):
        assert np.array_equal(a[c].data, b[c].data)


def test_size_changing_reshape_errors():
    t = nt(np.zeros((4, 6)), ("a", "b"))
    with pytest.raises(LayoutError) as e:
        reshape_general(t, ("c", "d"), (5, 5), [("x", 2)], [("a", "x")])
    assert e.value.code == "SIZE_MISMATCH"
    with pytest.raises(LayoutError) as e:
        reshape_general(t, ("c", "d"), (8, 3), [("x", 2)], [("d", "x")])
    assert e.value.code == "INDIVISIBLE"
