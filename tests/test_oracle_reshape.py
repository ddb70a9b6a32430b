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
