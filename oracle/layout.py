"""Mesh, computation layout, per-processor slices and einsum lowering (test infrastructure only).

Sections "Hardware Assumptions" (mesh = n-dimensional array of processors, a naming
abstraction), "Mesh-TensorFlow: Beyond Batch Splitting" (named dims; the computation
layout is a partial map tensor-dim -> mesh-dim), "Tensor Representations" (a tensor's
layout is the restriction of that map to its dims and must be injective; each mapped
dim is cut down to the stripe of the processor's coordinate; sizes must divide evenly)
and "Operation Implementation" (an einsum runs locally on the slices and is followed by
an Allreduce over the mesh dims that reduced-out split dims map to).

Readings taken where the text leaves a choice:
  * a stripe is the contiguous block [c*n, (c+1)*n) for coordinate c;
  * processors are numbered row-major over the mesh shape (last mesh dim fastest), which
    is what makes one processor set viewable as [16,16,2], [32,16] or [512] by reshape;
  * layout rules naming dims a tensor does not have are simply dropped (restriction);
  * for an einsum, the union of its operands' dims is held to the same injectivity rule
    as a single tensor: two different dims of one einsum on one mesh dim would make the
    processors cover only diagonal blocks of the iteration space.

A mesh is a list of (name, size); a layout is a list of (tensor_dim, mesh_dim).
"""
import itertools
import numpy as np

from .einsum import NT, add_broadcast, einsum, reduce, union_dims, EinsumError


class LayoutError(ValueError):
    """code: DUP_DIM, DUP_RULE, UNKNOWN_MESH_DIM, LAYOUT_CONFLICT, INDIVISIBLE, COORD_RANGE."""

    def __init__(self, code, msg=""):
        super().__init__(f"{code}: {msg}")
        self.code = code


def mesh_size(mesh):
    n = 1
    for _, s in mesh:
        n *= s
    return n


def rank_to_coord(mesh, rank):
    if not 0 <= rank < mesh_size(mesh):
        raise LayoutError("COORD_RANGE", f"rank {rank}")
    coord = []
    for _, s in reversed(mesh):
        coord.append(rank % s)
        rank //= s
    return tuple(reversed(coord))


def coord_to_rank(mesh, coord):
    check_coord(mesh, coord)
    rank = 0
    for (_, s), c in zip(mesh, coord):
        rank = rank * s + c
    return rank


def check_coord(mesh, coord):
    if len(coord) != len(mesh):
        raise LayoutError("COORD_RANGE", "length")
    for (_, s), c in zip(mesh, coord):
        if not 0 <= c < s:
            raise LayoutError("COORD_RANGE", f"{c} not in [0,{s})")


def check_mesh_and_layout(mesh, layout):
    names = [n for n, _ in mesh]
    if len(set(names)) != len(names):
        raise LayoutError("DUP_DIM", "mesh dim names")
    seen = set()
    for tdim, mdim in layout:
        if tdim in seen:                      # the layout is a map: one image per tensor dim
            raise LayoutError("DUP_RULE", tdim)
        seen.add(tdim)
        if mdim not in names:
            raise LayoutError("UNKNOWN_MESH_DIM", mdim)


def tensor_layout(dims, mesh, layout):
    """Restriction of the computation layout to `dims`: dict tensor_dim -> mesh axis index."""
    check_mesh_and_layout(mesh, layout)
    if len(set(dims)) != len(dims):
        raise LayoutError("DUP_DIM", str(dims))
    axis = {n: i for i, (n, _) in enumerate(mesh)}
    restr, used = {}, {}
    for tdim, mdim in layout:
        if tdim in dims:
            if mdim in used:
                raise LayoutError("LAYOUT_CONFLICT", f"{used[mdim]} and {tdim} both on {mdim}")
            used[mdim] = tdim
            restr[tdim] = axis[mdim]
    return restr


def slice_spec(dims, sizes, mesh, layout, coord):
    """(offsets, local sizes) of the slice the processor at `coord` holds."""
    restr = tensor_layout(dims, mesh, layout)
    check_coord(mesh, coord)
    offs, locs = [], []
    for d, n in zip(dims, sizes):
        if d in restr:
            parts = mesh[restr[d]][1]
            if n % parts:
                raise LayoutError("INDIVISIBLE", f"{d}={n} over {parts}")
            loc = n // parts
            offs.append(coord[restr[d]] * loc)
            locs.append(loc)
        else:
            offs.append(0)
            locs.append(n)
    return tuple(offs), tuple(locs)


def slice_tensor(t, mesh, layout, coord):
    offs, locs = slice_spec(t.dims, t.data.shape, mesh, layout, coord)
    idx = tuple(slice(o, o + n) for o, n in zip(offs, locs))
    return NT(np.array(t.data[idx], order="C"), t.dims)


def einsum_plan(in_dims, in_sizes, out_dims, mesh, layout):
    """What the lowering of one einsum needs to know, from names and sizes alone.

    Returns dict: union (name->size), reduced (names summed out), reduce_axes (sorted mesh
    axes the partial results must be summed over), local sizes of every operand and of the
    output, flops_global and flops_local.
    """
    sizes = {}
    for dims, shp in zip(in_dims, in_sizes):
        if len(set(dims)) != len(dims):
            raise LayoutError("DUP_DIM", str(dims))
        for d, n in zip(dims, shp):
            if sizes.setdefault(d, n) != n:
                raise EinsumError("SIZE_MISMATCH", d)
    if len(set(out_dims)) != len(out_dims):
        raise LayoutError("DUP_DIM", str(out_dims))
    for d in out_dims:
        if d not in sizes:
            raise EinsumError("OUT_NOT_SUBSET", d)
    union = tuple(sizes)
    restr = tensor_layout(union, mesh, layout)        # injectivity over the whole einsum
    origin = (0,) * len(mesh)
    loc = {}
    for d in union:
        _, (n,) = slice_spec((d,), (sizes[d],), mesh, layout, origin)
        loc[d] = n
    reduced = tuple(d for d in union if d not in out_dims)
    reduce_axes = sorted({restr[d] for d in reduced if d in restr})
    space_g = space_l = 1
    for d in union:
        space_g *= sizes[d]
        space_l *= loc[d]
    return dict(union=sizes, reduced=reduced, reduce_axes=reduce_axes,
                local_in=[tuple(loc[d] for d in dims) for dims in in_dims],
                local_out=tuple(loc[d] for d in out_dims),
                flops_global=2 * space_g, flops_local=2 * space_l)


def all_coords(mesh):
    return list(itertools.product(*[range(s) for _, s in mesh]))


def lowered_einsum(inputs, out_dims, mesh, layout):
    """Run the einsum the way the mesh would: per-processor local einsum on slices, then
    the grouped Allreduce.  Returns (local, reduced): dicts coord -> NT, `local` holding
    every processor's partial result and `reduced` what it holds after the Allreduce."""
    plan = einsum_plan([t.dims for t in inputs], [t.data.shape for t in inputs],
                       out_dims, mesh, layout)
    local = {}
    for c in all_coords(mesh):
        local[c] = einsum([slice_tensor(t, mesh, layout, c) for t in inputs], out_dims)
    reduced = {}
    axes = plan["reduce_axes"]
    for c in all_coords(mesh):
        acc = np.zeros_like(local[c].data)
        for c2 in all_coords(mesh):            # processors that differ from c only along `axes`
            if all(c2[i] == c[i] for i in range(len(mesh)) if i not in axes):
                acc = acc + local[c2].data
        reduced[c] = NT(acc, tuple(out_dims))
    return local, reduced


def lowered_reduce(t, out_dims, op, mesh, layout):
    """A reduction the way the mesh would run it ("Operation Implementation", paragraph
    "Reduction"): local reduction of each slice, then an Allreduce (with the same operator)
    over the mesh dims that reduced-out split dims map to.  Returns (local, reduced) like
    lowered_einsum."""
    plan = einsum_plan([t.dims], [t.data.shape], out_dims, mesh, layout)
    combine = np.add if op == "sum" else np.maximum
    local = {c: reduce(slice_tensor(t, mesh, layout, c), out_dims, op) for c in all_coords(mesh)}
    reduced = {}
    axes = plan["reduce_axes"]
    for c in all_coords(mesh):
        acc = None
        for c2 in all_coords(mesh):            # processors that differ from c only along `axes`
            if all(c2[i] == c[i] for i in range(len(mesh)) if i not in axes):
                acc = local[c2].data if acc is None else combine(acc, local[c2].data)
        reduced[c] = NT(acc, tuple(out_dims))
    return local, reduced


def lowered_add_broadcast(a, b, mesh, layout):
    """Component-wise addition with implicit broadcasting, per processor: the layouts of the
    operands and of the result are restrictions of one computation layout, so each processor
    adds its slices and holds its slice of the result; no communication."""
    return {c: add_broadcast(slice_tensor(a, mesh, layout, c), slice_tensor(b, mesh, layout, c))
            for c in all_coords(mesh)}


# ----------------------------------------------------------------------------- reshape

def reshape_plan(in_dims, out_dims, sizes, mesh, layout):
    """Communication of a reshape that keeps the dim sizes and changes (some of) the names
    (subsection "Reshape").  Returns one entry per mesh axis:
      'none'       the axis splits the same position before and after (or neither);
      'slice'      a dim is split in the output but not in the input: slicing only;
      'allgather'  a dim is split in the input but not in the output;
      'alltoall'   different positions are split across this mesh axis before and after."""
    if len(in_dims) != len(out_dims) or len(in_dims) != len(sizes):
        raise LayoutError("SIZE_MISMATCH", "reshape must keep rank and sizes")
    lin, lout = tensor_layout(in_dims, mesh, layout), tensor_layout(out_dims, mesh, layout)
    origin = (0,) * len(mesh)
    slice_spec(in_dims, sizes, mesh, layout, origin)       # divisibility of both views
    slice_spec(out_dims, sizes, mesh, layout, origin)
    plan = []
    for axis in range(len(mesh)):
        pin = [i for i, d in enumerate(in_dims) if lin.get(d) == axis]
        pout = [i for i, d in enumerate(out_dims) if lout.get(d) == axis]
        if not pin and not pout:
            plan.append("none")
        elif pin and not pout:
            plan.append("allgather")
        elif pout and not pin:
            plan.append("slice")
        else:
            plan.append("none" if pin == pout else "alltoall")
    return plan


def alltoall_exchange(group_slices, pos_was_split, pos_becomes_split):
    """MPI-alltoall among the n members of one group: member i cuts its slice into n stripes
    along `pos_becomes_split`, sends stripe j to member j, and concatenates what it receives (in
    member order) along `pos_was_split`.  Returns the members' new slices."""
    n = len(group_slices)
    cut = [np.array_split(a, n, axis=pos_becomes_split) for a in group_slices]
    return [np.concatenate([cut[src][me] for src in range(n)], axis=pos_was_split) for me in range(n)]


def lowered_reshape(t, out_dims, mesh, layout):
    """The reshape the way the mesh would run it, starting from every processor's input slice.
    Per mesh axis, among the processors that differ only along that axis: an axis that splits
    position p in the input gathers along p (allgather: the group's slices concatenated in
    coordinate order); an axis that splits position q in the output keeps the own stripe along q.
    An alltoall axis does both - it delivers exactly what its gather followed by its slicing
    delivers, while moving 1/n of the data (alltoall_exchange; see the tests).  All gathers are
    done before all slicings, so that an axis may take over a position another axis gives up.
    Returns dict coord -> NT with the output names."""
    plan = reshape_plan(t.dims, out_dims, t.data.shape, mesh, layout)
    lin, lout = tensor_layout(t.dims, mesh, layout), tensor_layout(tuple(out_dims), mesh, layout)
    cur = {c: slice_tensor(t, mesh, layout, c).data for c in all_coords(mesh)}
    pos_in = {axis: [i for i, d in enumerate(t.dims) if lin.get(d) == axis] for axis in range(len(mesh))}
    pos_out = {axis: [i for i, d in enumerate(out_dims) if lout.get(d) == axis] for axis in range(len(mesh))}
    for axis, kind in enumerate(plan):                       # gathers
        if kind in ("allgather", "alltoall"):
            n = mesh[axis][1]
            cur = {c: np.concatenate([cur[c[:axis] + (j,) + c[axis + 1:]] for j in range(n)], axis=pos_in[axis][0])
                   for c in all_coords(mesh)}
    for axis, kind in enumerate(plan):                       # slicings
        if kind in ("slice", "alltoall"):
            n = mesh[axis][1]
            cur = {c: np.array_split(cur[c], n, axis=pos_out[axis][0])[c[axis]] for c in all_coords(mesh)}
    return {c: NT(np.array(a, order="C"), tuple(out_dims)) for c, a in cur.items()}


# ----------------------------------------------------------------------------- reshape that changes sizes

def reshape_general(t, out_dims, out_sizes, mesh, layout):
    """A reshape that may change rank and dim sizes (subsection "Reshape": "simple in the
    non-distributed case"): the elements keep their row-major order, the output gets its own
    names and is laid out by them.  This is the definition: reshape the full tensor, then slice.
    Returns dict coord -> NT."""
    total = 1
    for n in out_sizes:
        total *= n
    if len(out_dims) != len(out_sizes) or total != t.data.size:
        raise LayoutError("SIZE_MISMATCH", f"{t.data.shape} -> {tuple(out_sizes)}")
    # both views must be legal under the layout (names first, then divisibility, as reshape_plan)
    tensor_layout(t.dims, mesh, layout)
    tensor_layout(tuple(out_dims), mesh, layout)
    origin = (0,) * len(mesh)
    slice_spec(t.dims, t.data.shape, mesh, layout, origin)
    slice_spec(out_dims, out_sizes, mesh, layout, origin)
    full = NT(np.array(t.data, order="C").reshape(tuple(out_sizes)), tuple(out_dims))
    return {c: slice_tensor(full, mesh, layout, c) for c in all_coords(mesh)}


def lowered_reshape_general(t, out_dims, out_sizes, mesh, layout):
    """The same from the processors' INPUT slices, one element at a time: an element of a
    processor's output slice has a position in the full output, hence a row-major rank among all
    elements, hence a position in the full input; the input slice that holds that position belongs
    to the processor whose coordinate on every mesh axis that splits an input dim is the stripe
    the position falls in (on the other axes: the reader's own coordinate - those processors hold
    copies).  Plain loops; for small cases.  Returns dict coord -> NT."""
    in_dims, in_sizes = t.dims, t.data.shape
    lin = tensor_layout(in_dims, mesh, layout)
    slices = {c: slice_tensor(t, mesh, layout, c) for c in all_coords(mesh)}
    total = 1
    for n in out_sizes:
        total *= n
    if len(out_dims) != len(out_sizes) or total != t.data.size:
        raise LayoutError("SIZE_MISMATCH", f"{in_sizes} -> {tuple(out_sizes)}")
    result = {}
    for c in all_coords(mesh):
        offs, locs = slice_spec(out_dims, out_sizes, mesh, layout, c)
        out = np.empty(locs, dtype=np.float64)
        for idx in np.ndindex(*locs):
            rank = 0                                    # row-major rank of the element in the full tensor
            for i, n in enumerate(out_sizes):
                rank = rank * n + offs[i] + idx[i]
            pos = [0] * len(in_sizes)                   # its position in the full input
            for i in range(len(in_sizes) - 1, -1, -1):
                pos[i] = rank % in_sizes[i]
                rank //= in_sizes[i]
            owner, local = list(c), []
            for i, d in enumerate(in_dims):
                if d in lin:
                    stripe = in_sizes[i] // mesh[lin[d]][1]
                    owner[lin[d]] = pos[i] // stripe
                    local.append(pos[i] % stripe)
                else:
                    local.append(pos[i])
            out[idx] = slices[tuple(owner)].data[tuple(local)]
        result[c] = NT(out, tuple(out_dims))
    return result
