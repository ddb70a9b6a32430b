"""ctypes binding of include/mtf.h — same names, argument marshalling only."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmtf.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1811_02084_amd.build` "
                      "(there is no CPU or PyTorch fallback)")
lib = C.CDLL(LIB_PATH)

MAX_RANK = 8
F32, BF16 = 0, 1
EPI_NONE, EPI_RELU, EPI_MASK_GT0, EPI_BIAS, EPI_BIAS_RELU = 0, 1, 2, 3, 4
REDUCE_SUM, REDUCE_MAX = 0, 1

STATUS = {0: "MTF_OK", -1: "MTF_ERR_NULL", -2: "MTF_ERR_DUP_DIM", -3: "MTF_ERR_SIZE_MISMATCH",
          -4: "MTF_ERR_INDIVISIBLE", -5: "MTF_ERR_LAYOUT_CONFLICT", -6: "MTF_ERR_DUP_RULE",
          -7: "MTF_ERR_UNKNOWN_MESH_DIM", -8: "MTF_ERR_COORD_RANGE", -9: "MTF_ERR_OUT_NOT_SUBSET",
          -10: "MTF_ERR_UNSUPPORTED", -11: "MTF_ERR_WORKSPACE", -12: "MTF_ERR_HIP",
          -13: "MTF_ERR_RANK", -14: "MTF_ERR_ALIGN"}


class mtf_dim(C.Structure):
    _fields_ = [("name", C.c_char_p), ("size", C.c_int64)]


class mtf_shape(C.Structure):
    _fields_ = [("dims", C.POINTER(mtf_dim)), ("rank", C.c_int32)]


class mtf_rule(C.Structure):
    _fields_ = [("tensor_dim", C.c_char_p), ("mesh_dim", C.c_char_p)]


class mtf_place(C.Structure):
    _fields_ = [("mesh", mtf_shape), ("rules", C.POINTER(mtf_rule)), ("n_rules", C.c_int32),
                ("coord", C.POINTER(C.c_int64))]


class mtf_ffn_dims(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("batch", "length", "d_model", "d_ff")]


class mtf_mha_dims(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("batch", "length", "d_model", "heads", "d_k")]


class mtf_layer_dims(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("batch", "length", "d_model", "heads", "d_k", "d_ff")]


class mtf_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_q", "w_k", "w_v", "w_o", "w_in", "w_out")]


class mtf_layer_saved(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("q", "k", "v", "ctx", "lse", "u", "a")]


class mtf_layer_grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dw_q", "dw_k", "dw_v", "dw_o", "dw_in", "dw_out")]


class MtfError(RuntimeError):
    def __init__(self, code):
        self.code = code
        self.name = STATUS.get(code, str(code))
        super().__init__(lib.mtf_last_error().decode() or self.name)


lib.mtf_status_string.restype = C.c_char_p
lib.mtf_last_error.restype = C.c_char_p
for _f in ("mtf_attention_fwd_workspace_bytes", "mtf_attention_bwd_workspace_bytes", "mtf_ffn_bwd_workspace_bytes", "mtf_ffn_bias_bwd_workspace_bytes", "mtf_mha_bwd_workspace_bytes",
           "mtf_layer_fwd_workspace_bytes", "mtf_layer_bwd_workspace_bytes",
           "mtf_reduce_local_workspace_bytes"):
    if hasattr(lib, _f):
        getattr(lib, _f).restype = C.c_size_t


def _check(rc):
    if rc != 0:
        raise MtfError(rc)


def status_string(code):
    return lib.mtf_status_string(int(code)).decode()


# ------------------------------------------------------------------ marshalling helpers
class _Keep:
    """Holds the ctypes objects a struct points to for the duration of a call."""

    def __init__(self):
        self.refs = []

    def shape(self, dims):
        """dims: sequence of (name, size)."""
        dims = list(dims)
        arr = (mtf_dim * max(len(dims), 1))()
        for i, (n, s) in enumerate(dims):
            arr[i].name = n.encode() if isinstance(n, str) else n
            arr[i].size = int(s)
        self.refs.append(arr)
        return mtf_shape(C.cast(arr, C.POINTER(mtf_dim)), len(dims))

    def place(self, mesh, layout, coord):
        layout = list(layout)
        rules = (mtf_rule * max(len(layout), 1))()
        for i, (t, m) in enumerate(layout):
            rules[i].tensor_dim = t.encode()
            rules[i].mesh_dim = m.encode()
        self.refs.append(rules)
        p = mtf_place()
        p.mesh = self.shape(mesh)
        p.rules = C.cast(rules, C.POINTER(mtf_rule)) if layout else None
        p.n_rules = len(layout)
        if coord is not None:
            carr = (C.c_int64 * max(len(coord), 1))(*[int(c) for c in coord])
            self.refs.append(carr)
            p.coord = C.cast(carr, C.POINTER(C.c_int64))
        else:
            p.coord = None
        return p


def _dt(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _torch_dt(code):
    return torch.float32 if code == F32 else torch.bfloat16


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _named(t, dims):
    dims = list(dims)
    if len(dims) != t.dim():
        raise ValueError(f"{t.dim()}-d tensor given {len(dims)} dim names")
    return [(n, s) for n, s in zip(dims, t.shape)]


# ------------------------------------------------------------------ host-only calls
def rank_to_coord(mesh, rank):
    k = _Keep()
    m = k.shape(mesh)
    out = (C.c_int64 * max(len(mesh), 1))()
    _check(lib.mtf_rank_to_coord(C.byref(m), C.c_int64(rank), out))
    return tuple(out[i] for i in range(len(mesh)))


def coord_to_rank(mesh, coord):
    k = _Keep()
    m = k.shape(mesh)
    carr = (C.c_int64 * max(len(mesh), 1))(*[int(c) for c in coord])
    out = C.c_int64()
    _check(lib.mtf_coord_to_rank(C.byref(m), carr, C.byref(out)))
    return out.value


def slice(shape, mesh, layout, coord):
    """shape: [(name, size)...] -> (offsets, sizes) of the slice held at `coord`."""
    k = _Keep()
    s = k.shape(shape)
    p = k.place(mesh, layout, coord)
    n = max(len(shape), 1)
    off, sz = (C.c_int64 * n)(), (C.c_int64 * n)()
    _check(lib.mtf_slice(C.byref(s), C.byref(p), off, sz))
    return tuple(off[i] for i in range(len(shape))), tuple(sz[i] for i in range(len(shape)))


def einsum_plan(a, b, out, mesh, layout):
    """a, b, out: global shapes [(name, size)...] (b may be None).  Returns dict with local
    sizes, reduce_axes (mesh dim indices needing an Allreduce) and flops_local."""
    k = _Keep()
    sa, so = k.shape(a), k.shape(out)
    sb = k.shape(b) if b is not None else None
    p = k.place(mesh, layout, None)
    la = (C.c_int64 * max(len(a), 1))()
    lb = (C.c_int64 * max(len(b) if b is not None else 0, 1))()
    lo = (C.c_int64 * max(len(out), 1))()
    mask, fl = C.c_uint32(), C.c_int64()
    _check(lib.mtf_einsum_plan(C.byref(sa), C.byref(sb) if sb is not None else None, C.byref(so),
                               C.byref(p), la, lb, lo, C.byref(mask), C.byref(fl)))
    return dict(local_in=[tuple(la[i] for i in range(len(a)))] +
                ([tuple(lb[i] for i in range(len(b)))] if b is not None else []),
                local_out=tuple(lo[i] for i in range(len(out))),
                reduce_axes=[i for i in range(len(mesh)) if mask.value >> i & 1],
                flops_local=fl.value)


COMM = {0: "none", 1: "slice", 2: "allgather", 3: "alltoall"}


def reshape_plan(in_shape, out_shape, mesh, layout):
    """in_shape / out_shape: global shapes [(name, size)...] of equal sizes.  Returns, per mesh dim,
    'none' | 'slice' | 'allgather' | 'alltoall'."""
    k = _Keep()
    si, so = k.shape(in_shape), k.shape(out_shape)
    p = k.place(mesh, layout, None)
    comm = (C.c_int32 * max(len(mesh), 1))()
    _check(lib.mtf_reshape_plan(C.byref(si), C.byref(so), C.byref(p), comm))
    return [COMM[comm[i]] for i in range(len(mesh))]


def reshape_virtual(in_slices, in_shape, out_shape, mesh, layout, coord, out=None):
    """in_slices: every processor's slice of the input (by rank); returns the output slice of the
    processor at `coord` (written into `out` if given)."""
    k = _Keep()
    si, so = k.shape(in_shape), k.shape(out_shape)
    p = k.place(mesh, layout, coord)
    if out is None:
        _, sz = slice(out_shape, mesh, layout, coord)
        out = torch.empty(sz, dtype=in_slices[0].dtype, device=in_slices[0].device)
    arr = (C.c_void_p * len(in_slices))(*[t.data_ptr() for t in in_slices])
    for t in in_slices:
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("slices must be contiguous device tensors")
    _check(lib.mtf_reshape_virtual(arr, C.byref(si), C.byref(so), C.byref(p), _ptr(out), _dt(out), _stream()))
    return out


def reshape_general_virtual(in_slices, in_shape, out_shape, mesh, layout, coord, out=None):
    """reshape_virtual for a reshape that changes rank or sizes (row-major element order kept)."""
    k = _Keep()
    si, so = k.shape(in_shape), k.shape(out_shape)
    p = k.place(mesh, layout, coord)
    if out is None:
        _, sz = slice(out_shape, mesh, layout, coord)
        out = torch.empty(sz, dtype=in_slices[0].dtype, device=in_slices[0].device)
    arr = (C.c_void_p * len(in_slices))(*[t.data_ptr() for t in in_slices])
    for t in in_slices:
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("slices must be contiguous device tensors")
    _check(lib.mtf_reshape_general_virtual(arr, C.byref(si), C.byref(so), C.byref(p), _ptr(out), _dt(out),
                                           _stream()))
    return out


# ------------------------------------------------------------------ device calls
def slice_copy(full, dims, mesh, layout, coord, slice_buf=None, scatter=False):
    """Gathers the slice of `full` (scatter=False) or writes slice_buf back into it."""
    k = _Keep()
    shp = _named(full, dims)
    s = k.shape(shp)
    p = k.place(mesh, layout, coord)
    if slice_buf is None:
        _, sz = slice(shp, mesh, layout, coord)
        slice_buf = torch.empty(sz, dtype=full.dtype, device=full.device)
    _check(lib.mtf_slice_copy(_ptr(full), _ptr(slice_buf), C.byref(s), C.byref(p), _dt(full),
                              1 if scatter else 0, _stream()))
    return slice_buf


def einsum_local(a, a_dims, b, b_dims, out_dims, out_dtype=None, epi=EPI_NONE, aux=None,
                 alpha=1.0, accumulate=False, out=None):
    k = _Keep()
    sa = k.shape(_named(a, a_dims))
    sb = k.shape(_named(b, b_dims)) if b is not None else None
    sizes = dict(_named(a, a_dims))
    if b is not None:
        sizes.update(_named(b, b_dims))
    missing = [d for d in out_dims if d not in sizes]
    out_shape = [(d, sizes.get(d, 1)) for d in out_dims]
    if out is None:
        if missing:      # let the library report it; no buffer is needed for that
            out = torch.empty(1, dtype=out_dtype or a.dtype, device=a.device)
        else:
            out = torch.empty([s for _, s in out_shape], dtype=out_dtype or a.dtype, device=a.device)
    so = k.shape(out_shape)
    _check(lib.mtf_einsum_local(_ptr(a), C.byref(sa), _ptr(b), C.byref(sb) if sb is not None else None,
                                _ptr(out), C.byref(so), _dt(a), _dt(out), int(epi), _ptr(aux),
                                C.c_float(alpha), 1 if accumulate else 0, _stream()))
    return out


def einsum_local_kranges(a, a_dims, b, b_dims, out_dims, n, outs=None):
    """The einsum with its contracted dim cut into n ranges: a list of n fp32 partial sums."""
    k = _Keep()
    sa, sb = k.shape(_named(a, a_dims)), k.shape(_named(b, b_dims))
    sizes = dict(_named(a, a_dims))
    sizes.update(_named(b, b_dims))
    out_shape = [(d, sizes.get(d, 1)) for d in out_dims]
    if outs is None:
        outs = [torch.empty([s for _, s in out_shape], dtype=torch.float32, device=a.device) for _ in range(n)]
    so = k.shape(out_shape)
    arr = (C.c_void_p * n)(*[o.data_ptr() for o in outs])
    _check(lib.mtf_einsum_local_kranges(_ptr(a), C.byref(sa), _ptr(b), C.byref(sb), arr, n, C.byref(so), _stream()))
    return outs


PATH_GENERIC, PATH_MFMA, PATH_COMPONENTWISE = 0, 1, 2


def einsum_local_path(a_dims, b_dims, out_dims, in_dtype=torch.bfloat16, out_dtype=torch.float32, epi=EPI_NONE,
                      a_ptr=0x1000, b_ptr=0x2000, out_ptr=0x3000, aux_ptr=0x4000):
    """Which kernel einsum_local would run (PATH_MFMA / PATH_GENERIC) for operands of these named
    shapes ([(name, size)] lists) and addresses.  Host only: nothing is dereferenced or launched."""
    k = _Keep()
    sa, so = k.shape(a_dims), k.shape(out_dims)
    sb = k.shape(b_dims) if b_dims is not None else None
    code = lambda dt: F32 if dt == torch.float32 else BF16
    needs_aux = epi in (EPI_MASK_GT0, EPI_BIAS, EPI_BIAS_RELU)
    rc = lib.mtf_einsum_local_path(C.c_void_p(a_ptr), C.byref(sa), C.c_void_p(b_ptr) if sb is not None else None,
                                   C.byref(sb) if sb is not None else None, C.c_void_p(out_ptr), C.byref(so),
                                   code(in_dtype), code(out_dtype), int(epi),
                                   C.c_void_p(aux_ptr) if needs_aux else None, C.c_float(1.0), 0)
    if rc < 0:
        raise MtfError(rc)
    return rc


def reduce_partials(partials, residual=None, out_dtype=torch.float32, out=None, epi=EPI_NONE, aux=None):
    """epi / aux: component-wise operation on the complete sum (mtf_reduce_partials_epi)."""
    n = len(partials)
    count = partials[0].numel()
    arr = (C.c_void_p * n)(*[p.data_ptr() for p in partials])
    for p in partials:
        if p.dtype != torch.float32 or p.numel() != count or not p.is_contiguous():
            raise ValueError("partials must be contiguous fp32 tensors of one size")
    if out is None:
        out = torch.empty(partials[0].shape, dtype=out_dtype, device=partials[0].device)
    if aux is not None and (aux.dtype != torch.bfloat16 or aux.numel() != count or not aux.is_contiguous()):
        raise ValueError("aux must be a contiguous bf16 tensor of the partials' size")
    _check(lib.mtf_reduce_partials_epi(arr, n, _ptr(residual), _dt(residual) if residual is not None else F32,
                                       _ptr(out), _dt(out), C.c_int64(count), int(epi), _ptr(aux), _stream()))
    return out


def sgd_step(grads, lr, master, weights=None):
    """master (fp32, in place) -= lr * sum(grads); weights (bf16, optional) <- rounded master."""
    n, count = len(grads), master.numel()
    for g_ in grads:
        if g_.dtype != torch.float32 or g_.numel() != count or not g_.is_contiguous():
            raise ValueError("gradients must be contiguous fp32 tensors of the parameter's size")
    if master.dtype != torch.float32 or (weights is not None and (weights.dtype != torch.bfloat16 or weights.numel() != count)):
        raise ValueError("master must be fp32, weights bf16 of the same size")
    arr = (C.c_void_p * n)(*[g_.data_ptr() for g_ in grads])
    lib.mtf_sgd_step.argtypes = [C.c_void_p, C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    _check(lib.mtf_sgd_step(arr, n, lr, _ptr(master), _ptr(weights), count, _stream()))
    return master, weights


def add_broadcast(a, a_dims, b, b_dims, out_dtype=None):
    """a + b with b's dims a subset of a's (b repeated along the dims it lacks)."""
    k = _Keep()
    sa = k.shape(_named(a, a_dims))
    sb = k.shape(_named(b, b_dims))
    out = torch.empty(a.shape, dtype=out_dtype or a.dtype, device=a.device)
    _check(lib.mtf_add_broadcast(_ptr(a), C.byref(sa), _ptr(b), C.byref(sb), _ptr(out), _dt(a), _dt(out),
                                 _stream()))
    return out


def reduce_local(x, x_dims, out_dims, op=REDUCE_SUM, out_dtype=torch.float32):
    """reduce_sum / reduce_max of one slice: dims of x not named in out_dims are reduced out."""
    k = _Keep()
    named = _named(x, x_dims)
    sizes = dict(named)
    sx = k.shape(named)
    missing = [d for d in out_dims if d not in sizes]
    out_shape = [(d, sizes.get(d, 1)) for d in out_dims]
    out = torch.empty([1] if missing else [n for _, n in out_shape], dtype=out_dtype, device=x.device)
    so = k.shape(out_shape)
    need = lib.mtf_reduce_local_workspace_bytes(C.byref(sx), C.byref(so))
    ws = _ws(need, x.device)
    _check(lib.mtf_reduce_local(_ptr(x), C.byref(sx), _ptr(out), C.byref(so), _dt(x), _dt(out), int(op),
                                _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return out


REDUCE_STATIC_MAX_SCRATCH = 4 << 20


def reduce_local_static(x, x_dims, out_dims, op=REDUCE_SUM, out=None, out_dtype=torch.float32):
    """reduce_local through the entry point that allocates nothing inside the library (its scratch
    is a static device array); `out` may be passed in so that the call allocates nothing at all."""
    k = _Keep()
    named = _named(x, x_dims)
    sizes = dict(named)
    sx = k.shape(named)
    missing = [d for d in out_dims if d not in sizes]
    out_shape = [(d, sizes.get(d, 1)) for d in out_dims]
    if out is None:
        out = torch.empty([1] if missing else [n for _, n in out_shape], dtype=out_dtype, device=x.device)
    so = k.shape(out_shape)
    _check(lib.mtf_reduce_local_static(_ptr(x), C.byref(sx), _ptr(out), C.byref(so), _dt(x), _dt(out), int(op),
                                       _stream()))
    return out


# ------------------------------------------------------------------ vocabulary-split operations
def embedding_local(ids, table_local, vocab_offset, out_dtype=torch.float32):
    """ids int32 [...]; table_local bf16 [vocab_local, d_model] -> partial sum [..., d_model]."""
    out = torch.empty(tuple(ids.shape) + (table_local.shape[1],), dtype=out_dtype, device=table_local.device)
    _check(lib.mtf_embedding_local(_ptr(ids), C.c_int64(ids.numel()), _ptr(table_local),
                                   C.c_int64(table_local.shape[0]), C.c_int64(table_local.shape[1]),
                                   C.c_int64(vocab_offset), _ptr(out), _dt(out), _stream()))
    return out


def embedding_grad_local(ids, de, vocab_local, vocab_offset):
    dt = torch.empty((vocab_local, de.shape[-1]), dtype=torch.float32, device=de.device)
    _check(lib.mtf_embedding_grad_local(_ptr(ids), C.c_int64(ids.numel()), _ptr(de), C.c_int64(vocab_local),
                                        C.c_int64(de.shape[-1]), C.c_int64(vocab_offset), _ptr(dt), _stream()))
    return dt


def max_partials(partials, out=None):
    n, count = len(partials), partials[0].numel()
    for p in partials:
        if p.dtype != torch.float32 or p.numel() != count or not p.is_contiguous():
            raise ValueError("partials must be contiguous fp32 tensors of one size")
    arr = (C.c_void_p * n)(*[p.data_ptr() for p in partials])
    if out is None:
        out = torch.empty(partials[0].shape, dtype=torch.float32, device=partials[0].device)
    _check(lib.mtf_max_partials(arr, n, _ptr(out), C.c_int64(count), _stream()))
    return out


def xent_stats_local(logits_local, row_max, targets, vocab_offset):
    """logits_local fp32 [..., vocab_local] -> (sumexp, picked), fp32 [...]."""
    rows, vl = logits_local.numel() // logits_local.shape[-1], logits_local.shape[-1]
    sumexp = torch.empty(logits_local.shape[:-1], dtype=torch.float32, device=logits_local.device)
    picked = torch.empty_like(sumexp)
    _check(lib.mtf_xent_stats_local(_ptr(logits_local), C.c_int64(rows), C.c_int64(vl), _ptr(row_max),
                                    _ptr(targets), C.c_int64(vocab_offset), _ptr(sumexp), _ptr(picked), _stream()))
    return sumexp, picked


def xent_loss(row_max, sumexp, picked):
    loss = torch.empty_like(row_max)
    _check(lib.mtf_xent_loss(_ptr(row_max), _ptr(sumexp), _ptr(picked), _ptr(loss), C.c_int64(row_max.numel()),
                             _stream()))
    return loss


def xent_grad_local(logits_local, row_max, sumexp, targets, vocab_offset, dloss):
    rows, vl = logits_local.numel() // logits_local.shape[-1], logits_local.shape[-1]
    dz = torch.empty(logits_local.shape, dtype=torch.bfloat16, device=logits_local.device)
    _check(lib.mtf_xent_grad_local(_ptr(logits_local), C.c_int64(rows), C.c_int64(vl), _ptr(row_max), _ptr(sumexp),
                                   _ptr(targets), C.c_int64(vocab_offset), _ptr(dloss), _ptr(dz), _stream()))
    return dz


def cast(x, dtype):
    out = torch.empty(x.shape, dtype=dtype, device=x.device)
    _check(lib.mtf_cast(_ptr(x), _dt(x), _ptr(out), _dt(out), C.c_int64(x.numel()), _stream()))
    return out


# ------------------------------------------------------------------ fixed layer steps
def _ws(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def ffn_fwd(x, w_in, w_out):
    """x[batch,length,d_model], w_in[d_model,d_ff], w_out[d_ff,d_model] (bf16) ->
    (a bf16 [batch,length,d_ff], y_partial fp32 [batch,length,d_model])."""
    b, l, dm = x.shape
    d = mtf_ffn_dims(b, l, dm, w_in.shape[1])
    a = torch.empty((b, l, w_in.shape[1]), dtype=torch.bfloat16, device=x.device)
    y = torch.empty((b, l, dm), dtype=torch.float32, device=x.device)
    _check(lib.mtf_ffn_fwd(C.byref(d), _ptr(x), _ptr(w_in), _ptr(w_out), _ptr(a), _ptr(y), _stream()))
    return a, y


def ffn_bwd(x, a, w_in, w_out, dy, workspace=None):
    b, l, dm = x.shape
    d = mtf_ffn_dims(b, l, dm, w_in.shape[1])
    need = lib.mtf_ffn_bwd_workspace_bytes(C.byref(d))
    ws = workspace if workspace is not None else _ws(need, x.device)
    dw_in = torch.empty(w_in.shape, dtype=torch.float32, device=x.device)
    dw_out = torch.empty(w_out.shape, dtype=torch.float32, device=x.device)
    dx = torch.empty(x.shape, dtype=torch.float32, device=x.device)
    _check(lib.mtf_ffn_bwd(C.byref(d), _ptr(x), _ptr(a), _ptr(w_in), _ptr(w_out), _ptr(dy), _ptr(dw_in),
                           _ptr(dw_out), _ptr(dx), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return dict(dw_in=dw_in, dw_out=dw_out, dx=dx)


def ffn_bias_fwd(x, w_in, bias, w_out):
    """The worked example with its bias: a = relu(x w_in + bias), y_partial = a w_out."""
    b, l, dm = x.shape
    d = mtf_ffn_dims(b, l, dm, w_in.shape[1])
    a = torch.empty((b, l, w_in.shape[1]), dtype=torch.bfloat16, device=x.device)
    y = torch.empty((b, l, dm), dtype=torch.float32, device=x.device)
    _check(lib.mtf_ffn_bias_fwd(C.byref(d), _ptr(x), _ptr(w_in), _ptr(bias), _ptr(w_out), _ptr(a), _ptr(y),
                                _stream()))
    return a, y


def ffn_bias_bwd(x, a, w_in, w_out, dy, workspace=None):
    b, l, dm = x.shape
    d = mtf_ffn_dims(b, l, dm, w_in.shape[1])
    need = lib.mtf_ffn_bias_bwd_workspace_bytes(C.byref(d))
    ws = workspace if workspace is not None else _ws(need, x.device)
    dw_in = torch.empty(w_in.shape, dtype=torch.float32, device=x.device)
    dw_out = torch.empty(w_out.shape, dtype=torch.float32, device=x.device)
    dbias = torch.empty(w_in.shape[1], dtype=torch.float32, device=x.device)
    dx = torch.empty(x.shape, dtype=torch.float32, device=x.device)
    _check(lib.mtf_ffn_bias_bwd(C.byref(d), _ptr(x), _ptr(a), _ptr(w_in), _ptr(w_out), _ptr(dy), _ptr(dw_in),
                                _ptr(dbias), _ptr(dw_out), _ptr(dx), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return dict(dw_in=dw_in, dw_out=dw_out, dbias=dbias, dx=dx)


def mha_fwd(x, w_q, w_k, w_v, w_o, scale, causal):
    b, l, dm = x.shape
    h, dk = w_q.shape[1], w_q.shape[2]
    d = mtf_mha_dims(b, l, dm, h, dk)
    mk = lambda: torch.empty((b, l, h, dk), dtype=torch.bfloat16, device=x.device)
    q, k, v, ctx = mk(), mk(), mk(), mk()
    lse = torch.empty((b, h, l), dtype=torch.float32, device=x.device)
    y = torch.empty((b, l, dm), dtype=torch.float32, device=x.device)
    _check(lib.mtf_mha_fwd(C.byref(d), _ptr(x), _ptr(w_q), _ptr(w_k), _ptr(w_v), _ptr(w_o),
                           C.c_float(scale), int(bool(causal)), _ptr(q), _ptr(k), _ptr(v), _ptr(ctx),
                           _ptr(lse), _ptr(y), _stream()))
    return dict(q=q, k=k, v=v, ctx=ctx, lse=lse, y=y)


def mha_bwd(x, w_q, w_k, w_v, w_o, q, k, v, ctx, lse, dy, scale, causal, workspace=None):
    b, l, dm = x.shape
    h, dk = w_q.shape[1], w_q.shape[2]
    d = mtf_mha_dims(b, l, dm, h, dk)
    need = lib.mtf_mha_bwd_workspace_bytes(C.byref(d))
    ws = workspace if workspace is not None else _ws(need, x.device)
    f32 = lambda t: torch.empty(t.shape, dtype=torch.float32, device=x.device)
    out = dict(dw_q=f32(w_q), dw_k=f32(w_k), dw_v=f32(w_v), dw_o=f32(w_o), dx=f32(x))
    _check(lib.mtf_mha_bwd(C.byref(d), _ptr(x), _ptr(w_q), _ptr(w_k), _ptr(w_v), _ptr(w_o), _ptr(q),
                           _ptr(k), _ptr(v), _ptr(ctx), _ptr(lse), _ptr(dy), C.c_float(scale),
                           int(bool(causal)), _ptr(out["dw_q"]), _ptr(out["dw_k"]), _ptr(out["dw_v"]),
                           _ptr(out["dw_o"]), _ptr(out["dx"]), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return out


def attention_fwd(q, k, v, scale, causal):
    """The attention core for any head width: q, k, v bf16 [batch, length, heads, d_k] -> (ctx, lse)."""
    b, l, h, dk = q.shape
    d = mtf_mha_dims(b, l, h * dk, h, dk)
    ctx = torch.empty_like(q)
    lse = torch.empty((b, h, l), dtype=torch.float32, device=q.device)
    ws = _ws(lib.mtf_attention_fwd_workspace_bytes(C.byref(d)), q.device)
    _check(lib.mtf_attention_fwd(C.byref(d), _ptr(q), _ptr(k), _ptr(v), C.c_float(scale), int(bool(causal)),
                                 _ptr(ctx), _ptr(lse), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return ctx, lse


def attention_bwd(q, k, v, ctx, lse, dctx, scale, causal):
    b, l, h, dk = q.shape
    d = mtf_mha_dims(b, l, h * dk, h, dk)
    dq, dk_, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    ws = _ws(lib.mtf_attention_bwd_workspace_bytes(C.byref(d)), q.device)
    _check(lib.mtf_attention_bwd(C.byref(d), _ptr(q), _ptr(k), _ptr(v), _ptr(ctx), _ptr(lse), _ptr(dctx),
                                 C.c_float(scale), int(bool(causal)), _ptr(dq), _ptr(dk_), _ptr(dv), _ptr(ws),
                                 C.c_size_t(ws.numel()), _stream()))
    return dq, dk_, dv


def _layer_dims(x, w):
    b, l, dm = x.shape
    return mtf_layer_dims(b, l, dm, w["w_q"].shape[1], w["w_q"].shape[2], w["w_in"].shape[1])


def _weights(w):
    return mtf_layer_weights(*[w[n].data_ptr() for n in ("w_q", "w_k", "w_v", "w_o", "w_in", "w_out")])


def layer_alloc(x, w):
    """Buffers a layer step needs, allocated once (saved activations, grads, workspaces)."""
    b, l, dm = x.shape
    h, dk, f = w["w_q"].shape[1], w["w_q"].shape[2], w["w_in"].shape[1]
    dev = x.device
    d = _layer_dims(x, w)
    bf = lambda *s: torch.empty(s, dtype=torch.bfloat16, device=dev)
    saved = dict(q=bf(b, l, h, dk), k=bf(b, l, h, dk), v=bf(b, l, h, dk), ctx=bf(b, l, h, dk),
                 lse=torch.empty((b, h, l), dtype=torch.float32, device=dev), u=bf(b, l, dm), a=bf(b, l, f))
    grads = {"d" + n: torch.empty(w[n].shape, dtype=torch.float32, device=dev)
             for n in ("w_q", "w_k", "w_v", "w_o", "w_in", "w_out")}
    return dict(saved=saved, grads=grads, z=bf(b, l, dm), dx=bf(b, l, dm),
                ws_fwd=_ws(lib.mtf_layer_fwd_workspace_bytes(C.byref(d)), dev),
                ws_bwd=_ws(lib.mtf_layer_bwd_workspace_bytes(C.byref(d)), dev))


def _saved(s):
    return mtf_layer_saved(*[s[n].data_ptr() for n in ("q", "k", "v", "ctx", "lse", "u", "a")])


def layer_fwd(x, w, scale, causal, bufs):
    d = _layer_dims(x, w)
    ww, sv = _weights(w), _saved(bufs["saved"])
    _check(lib.mtf_layer_fwd(C.byref(d), _ptr(x), C.byref(ww), C.c_float(scale), int(bool(causal)),
                             C.byref(sv), _ptr(bufs["z"]), _ptr(bufs["ws_fwd"]),
                             C.c_size_t(bufs["ws_fwd"].numel()), _stream()))
    return bufs["z"]


def layer_bwd(x, w, saved, dz, scale, causal, bufs):
    d = _layer_dims(x, w)
    ww, sv = _weights(w), _saved(saved)
    g = mtf_layer_grads(*[bufs["grads"][n].data_ptr() for n in ("dw_q", "dw_k", "dw_v", "dw_o", "dw_in", "dw_out")])
    _check(lib.mtf_layer_bwd(C.byref(d), _ptr(x), C.byref(ww), C.byref(sv), _ptr(dz), C.c_float(scale),
                             int(bool(causal)), C.byref(g), _ptr(bufs["dx"]), _ptr(bufs["ws_bwd"]),
                             C.c_size_t(bufs["ws_bwd"].numel()), _stream()))
    return bufs["dx"]


# ------------------------------------------------------------------ layer normalisation
def _bf16_rows(t, what):
    if t.dtype != torch.bfloat16:
        raise ValueError(f"{what} must be bf16")
    d = t.shape[-1]
    return t.numel() // d if d else 0, d


def layer_norm_fwd(x, gain, bias, eps):
    """x bf16 [..., d_model], gain / bias bf16 [d_model] -> (y bf16, mean fp32 [...], rstd fp32 [...])."""
    rows, d = _bf16_rows(x, "x")
    y = torch.empty_like(x)
    mean = torch.empty(x.shape[:-1], dtype=torch.float32, device=x.device)
    rstd = torch.empty_like(mean)
    lib.mtf_layer_norm_fwd.argtypes = [C.c_void_p] * 3 + [C.c_float, C.c_int64, C.c_int64] + [C.c_void_p] * 4
    _check(lib.mtf_layer_norm_fwd(_ptr(x), _ptr(gain), _ptr(bias), eps, rows, d, _ptr(y), _ptr(mean), _ptr(rstd),
                                  _stream()))
    return y, mean, rstd


def residual_layer_norm_fwd(partials, residual, gain, bias, eps):
    """u = residual + sum(partials) stored bf16, then the normalisation of u -> (u, y, mean, rstd)."""
    rows, d = _bf16_rows(residual, "residual")
    n = len(partials)
    for p_ in partials:
        if p_.dtype != torch.float32 or p_.shape != residual.shape or not p_.is_contiguous():
            raise ValueError("partials must be contiguous fp32 tensors of the residual's shape")
    arr = (C.c_void_p * max(n, 1))(*[p_.data_ptr() for p_ in partials])
    u, y = torch.empty_like(residual), torch.empty_like(residual)
    mean = torch.empty(residual.shape[:-1], dtype=torch.float32, device=residual.device)
    rstd = torch.empty_like(mean)
    lib.mtf_residual_layer_norm_fwd.argtypes = ([C.c_void_p, C.c_int32] + [C.c_void_p] * 3 +
                                                [C.c_float, C.c_int64, C.c_int64] + [C.c_void_p] * 5)
    _check(lib.mtf_residual_layer_norm_fwd(arr, n, _ptr(residual), _ptr(gain), _ptr(bias), eps, rows, d,
                                           _ptr(u), _ptr(y), _ptr(mean), _ptr(rstd), _stream()))
    return u, y, mean, rstd


def layer_norm_bwd(x, gain, mean, rstd, dy):
    """-> (dx bf16, dgain fp32 [d_model], dbias fp32 [d_model])."""
    rows, d = _bf16_rows(x, "x")
    dx = torch.empty_like(x)
    dgain = torch.empty(d, dtype=torch.float32, device=x.device)
    dbias = torch.empty_like(dgain)
    lib.mtf_layer_norm_bwd_workspace_bytes.restype = C.c_size_t
    lib.mtf_layer_norm_bwd_workspace_bytes.argtypes = [C.c_int64, C.c_int64]
    ws = _ws(lib.mtf_layer_norm_bwd_workspace_bytes(rows, d), x.device)
    lib.mtf_layer_norm_bwd.argtypes = [C.c_void_p] * 5 + [C.c_int64, C.c_int64] + [C.c_void_p] * 4 + [C.c_size_t, C.c_void_p]
    _check(lib.mtf_layer_norm_bwd(_ptr(x), _ptr(gain), _ptr(mean), _ptr(rstd), _ptr(dy), rows, d, _ptr(dx),
                                  _ptr(dgain), _ptr(dbias), _ptr(ws), ws.numel(), _stream()))
    return dx, dgain, dbias


# ------------------------------------------------------------------ measurement aid
class mtf_kernel_time(C.Structure):
    _fields_ = [("kernel", C.c_char * 96), ("launches", C.c_int64), ("total_ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double)]


def mfma_ceiling(operands, iters, sink):
    """One launch of the MFMA-only kernel; returns the FLOP it performs.  sink: >= 66 floats
    (sink[64], sink[65]: the loop's span in shader cycles and in 100 MHz ticks)."""
    if operands.numel() < 4096 or sink.numel() < 66:
        raise ValueError("mfma_ceiling: operands needs 4096 bf16 elements, sink 66 floats")
    flops = C.c_double()
    _check(lib.mtf_mfma_ceiling(_ptr(operands), C.c_int32(iters), _ptr(sink), C.byref(flops), _stream()))
    return flops.value


def timing_enable(on):
    _check(lib.mtf_timing_enable(1 if on else 0))


def timing_collect(max_kinds=64):
    """Per-kernel totals of the launches made while timing was enabled (synchronises)."""
    arr = (mtf_kernel_time * max_kinds)()
    n = C.c_int32()
    _check(lib.mtf_timing_collect(arr, max_kinds, C.byref(n)))
    return [dict(kernel=arr[i].kernel.decode(), launches=arr[i].launches, total_ms=arr[i].total_ms,
                 flops=arr[i].flops, bytes=arr[i].bytes) for i in range(n.value)]
