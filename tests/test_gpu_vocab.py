"""Parity of the vocabulary-split operations (embedding, logits + softmax cross-entropy, their
gradients) against the oracle, through the C ABI: one processor's stripe at its real shape, and a
virtual mesh on which the Allreduce groups (max and sum) are combined on the GPU."""
import numpy as np
import pytest
import torch

import mtf_inputs
from helpers import named as to_nt
from oracle import vocab as OV
from oracle.einsum import NT, nt
from oracle.einsum import add_broadcast as o_add, einsum as o_einsum, reduce as o_reduce
from oracle.layout import all_coords, slice_spec, slice_tensor
from oracle.metrics import m2
from oracle.vocab import B, L, D, VOCAB

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
TOL_F32 = 1e-5


@pytest.fixture(scope="module")
def mtf():
    import paper_1811_02084_amd as m
    return m


def _dev(t):
    return t.cuda()


CASES = {
    "ragged-small": dict(batch=3, length=37, d_model=72, vocab_local=200, vocab_total=600, offset=200),
    "whole-vocab": dict(batch=2, length=50, d_model=264, vocab_local=328, vocab_total=328, offset=0),
    # the stripe of config 6 at its real shape (16 x 256 tokens, d_model 1024, ids 2048 .. 4095); the
    # oracle needs the whole vocabulary, so the group here is 2 processors instead of 16 (nothing the
    # processor computes depends on how many others there are)
    "config6-size": dict(batch=16, length=256, d_model=1024, vocab_local=2048, vocab_total=4096, offset=2048),
}


def _local_oracle_tables(cfg, offset):
    """The stripe of the vocabulary this processor holds, as rows / columns of full-size tensors
    that are zero elsewhere (what the processor's partial sums correspond to)."""
    vt, vl = cfg["vocab_total"], cfg["table"].shape[0]
    table = np.zeros((vt, cfg["table"].shape[1]))
    table[offset:offset + vl] = cfg["table"].double().numpy()
    return nt(table, (VOCAB, D))


@pytest.mark.parametrize("case", sorted(CASES))
def test_embedding_stripe(mtf, case):
    p = CASES[case]
    cfg = mtf_inputs.vocab_inputs(31, p["batch"], p["length"], p["d_model"], p["vocab_local"], p["vocab_total"])
    off, vl = p["offset"], p["vocab_local"]
    ids = cfg["ids"]
    want = OV.embedding_fwd(ids.numpy(), _local_oracle_tables(cfg, off))
    for dtype in (torch.float32, torch.bfloat16):
        got = mtf.embedding_local(_dev(ids), _dev(cfg["table"]), off, out_dtype=dtype)
        assert np.array_equal(got.double().cpu().numpy(), want.data)          # a copy: bit-exact
    # gradient: rows of the stripe only, summed in token order
    de = to_nt(cfg["de"], (B, L, D))
    want_dt = OV.embedding_bwd(ids.numpy(), de, p["vocab_total"]).data[off:off + vl]
    got_dt = mtf.embedding_grad_local(_dev(ids), _dev(cfg["de"]), vl, off)
    assert m2(got_dt.cpu().numpy(), want_dt) <= TOL_F32


def test_embedding_gradient_with_repeated_tokens_is_exact_on_integers(mtf):
    ids = mtf_inputs.token_ids(32, 0, (4, 300), 7)                      # every row is hit ~170 times
    de = mtf_inputs.small_ints(32, 1, (4, 300, 40))
    want = OV.embedding_bwd(ids.numpy(), to_nt(de, (B, L, D)), 7).data
    got = mtf.embedding_grad_local(_dev(ids), _dev(de), 5, 1)           # stripe = ids 1..5
    assert np.array_equal(got.double().cpu().numpy(), want[1:6])


def _stripe_problem(cfg, p):
    """The full-vocabulary problem whose processor `c` holds this stripe: the output-layer weight
    is the stripe's columns and zero elsewhere, laid out over a mesh of vocab_total / vocab_local
    processors with vocab split across it.  Zero columns elsewhere make this processor's partial
    sum of dx the whole dx, so every gradient the device produces has an oracle counterpart."""
    vt, vl, off = p["vocab_total"], p["vocab_local"], p["offset"]
    w_full = np.zeros((cfg["w_vocab"].shape[0], vt))
    w_full[:, off:off + vl] = cfg["w_vocab"].double().numpy()
    mesh, layout = [("all", vt // vl)], [("vocab", "all")]
    return nt(w_full, (D, VOCAB)), mesh, layout, (off // vl,)


@pytest.mark.parametrize("case", sorted(CASES))
def test_loss_stripe_forward_backward(mtf, case):
    """One processor's stripe of the output layer.  Every expected value is produced by the oracle
    (oracle.vocab.xent_fwd / xent_bwd on the full vocabulary, the stripe taken with the oracle's
    own slicing; the per-stripe statistics with the oracle's reduce / add_broadcast / einsum)."""
    p = CASES[case]
    print(f"vocab stripe {case}", flush=True)
    cfg = mtf_inputs.vocab_inputs(33, p["batch"], p["length"], p["d_model"], p["vocab_local"], p["vocab_total"])
    off, vl, vt = p["offset"], p["vocab_local"], p["vocab_total"]
    x = to_nt(cfg["x"], (B, L, D))
    w_full, mesh, layout, c = _stripe_problem(cfg, p)
    targets = cfg["targets"].numpy()
    full = OV.xent_fwd(x, w_full, targets)
    z_ref = slice_tensor(full["logits"], mesh, layout, c)                # [b, l, vocab_local]
    z = mtf.einsum_local(_dev(cfg["x"]), (B, L, D), _dev(cfg["w_vocab"]), (D, VOCAB), (B, L, VOCAB),
                         out_dtype=torch.float32)
    assert m2(z.cpu().numpy(), z_ref.data) <= TOL_BF16
    # the statistics kernels are fed the ORACLE's logits (stored fp32) and the oracle's group-wide
    # row maximum, so that every expected value below comes from the oracle side alone
    z = _dev(torch.from_numpy(z_ref.data).float())
    z_st = NT(z.double().cpu().numpy(), z_ref.dims)                       # what the device reads
    m_loc = mtf.reduce_local(z, (B, L, VOCAB), (B, L), mtf.REDUCE_MAX)
    assert np.array_equal(m_loc.double().cpu().numpy(), o_reduce(z_st, (B, L), "max").data)
    m_grp = _dev(torch.from_numpy(full["m"].data).float())
    m_st = NT(m_grp.double().cpu().numpy(), (B, L))
    sumexp, picked = mtf.xent_stats_local(z, m_grp, _dev(cfg["targets"]), off)
    want_s = o_reduce(NT(np.exp(o_add(z_st, NT(-m_st.data, m_st.dims)).data), z_st.dims), (B, L), "sum")
    want_t = o_einsum([slice_tensor(OV.onehot(targets, vt), mesh, layout, c), z_st], (B, L))
    assert m2(sumexp.cpu().numpy(), want_s.data) <= TOL_F32
    assert np.array_equal(picked.double().cpu().numpy(), want_t.data)
    if vt == vl:                                                         # the group is this one processor
        loss = mtf.xent_loss(m_grp, sumexp, picked)
        assert m2(loss.cpu().numpy(), full["loss"].data) <= TOL_F32
        assert m2(sumexp.cpu().numpy(), full["s"].data) <= TOL_F32
    # backward from the oracle's group-wide statistics
    dloss = to_nt(cfg["dloss"], (B, L))
    ref = OV.xent_bwd(x, w_full, targets, full["logits"], full["m"], full["s"], dloss)
    s_grp = _dev(torch.from_numpy(full["s"].data).float())
    dz = mtf.xent_grad_local(z, m_grp, s_grp, _dev(cfg["targets"]), off, _dev(cfg["dloss"]))
    dz_ref = slice_tensor(ref["dz"], mesh, layout, c)
    assert m2(dz.float().cpu().numpy(), dz_ref.data) <= TOL_BF16
    # the two gradient einsums from the oracle's stored dz (already on the bf16 grid) on both sides
    dz_dev = _dev(torch.from_numpy(dz_ref.data).to(torch.bfloat16))
    assert np.array_equal(dz_dev.double().cpu().numpy(), dz_ref.data)
    dw = mtf.einsum_local(_dev(cfg["x"]), (B, L, D), dz_dev, (B, L, VOCAB), (D, VOCAB), out_dtype=torch.float32)
    dx = mtf.einsum_local(dz_dev, (B, L, VOCAB), _dev(cfg["w_vocab"]), (D, VOCAB), (B, L, D),
                          out_dtype=torch.float32)
    assert m2(dw.cpu().numpy(), slice_tensor(ref["dw"], mesh, layout, c).data) <= TOL_BF16
    assert m2(dx.cpu().numpy(), ref["dx"].data) <= TOL_BF16


def test_vocab_split_on_virtual_meshes(mtf):
    """The Transformer's model-parallel layout (vocab over the whole mesh) and the 2-D layout
    (batch over rows, vocab over cols): every processor's stripe computed by the library, the
    max / sum Allreduce groups combined on the GPU; loss and embedding must equal the unsplit
    oracle on every processor."""
    b, l, d, v = 4, 6, 32, 48
    cfg = mtf_inputs.vocab_inputs(34, b, l, d, v, v, dtype=torch.float32)
    x, w, table = cfg["x"], cfg["w_vocab"], cfg["table"].to(torch.bfloat16)
    ids, targets = cfg["ids"], cfg["targets"]
    full = OV.xent_fwd(to_nt(x, (B, L, D)), to_nt(w, (D, VOCAB)), targets.numpy())
    e_full = OV.embedding_fwd(ids.numpy(), to_nt(table, (VOCAB, D)))
    layouts = {
        "model-parallel": ([("all", 4)], [("vocab", "all"), ("d_ff", "all"), ("heads", "all")]),
        "batch-rows-vocab-cols": ([("rows", 2), ("cols", 2)], [("batch", "rows"), ("vocab", "cols")]),
    }
    for name, (mesh, layout) in layouts.items():
        coords = all_coords(mesh)
        plan = mtf.einsum_plan([(B, b), (L, l), (VOCAB, v)], None, [(B, b), (L, l)], mesh, layout)
        axes = plan["reduce_axes"]
        group_of = lambda c: [c2 for c2 in coords if all(c2[i] == c[i] for i in range(len(mesh)) if i not in axes)]
        z, m_loc, ids_loc, tgt_loc, voff, emb = {}, {}, {}, {}, {}, {}
        for c in coords:
            sl = lambda t, dims: mtf.slice_copy(_dev(t), dims, mesh, layout, c)
            z[c] = mtf.einsum_local(sl(x, (B, L, D)), (B, L, D), sl(w, (D, VOCAB)), (D, VOCAB), (B, L, VOCAB))
            m_loc[c] = mtf.reduce_local(z[c], (B, L, VOCAB), (B, L), mtf.REDUCE_MAX)
            (voff[c],), _ = slice_spec((VOCAB,), (v,), mesh, layout, c)
            bo, bn = slice_spec((B,), (b,), mesh, layout, c)
            ids_loc[c] = _dev(ids[bo[0]:bo[0] + bn[0]].contiguous())
            tgt_loc[c] = _dev(targets[bo[0]:bo[0] + bn[0]].contiguous())
            emb[c] = mtf.embedding_local(ids_loc[c], sl(table, (VOCAB, D)), voff[c])
        for c in coords:
            g = group_of(c)
            gmax = mtf.max_partials([m_loc[k] for k in g])
            stats = {k: mtf.xent_stats_local(z[k], gmax, tgt_loc[k], voff[k]) for k in g}
            gsum = mtf.reduce_partials([stats[k][0] for k in g])
            gpick = mtf.reduce_partials([stats[k][1] for k in g])
            loss = mtf.xent_loss(gmax, gsum, gpick)
            offs, locs = slice_spec((B, L), (b, l), mesh, layout, c)
            idx = tuple(slice(o, o + n) for o, n in zip(offs, locs))
            assert m2(loss.cpu().numpy(), full["loss"].data[idx]) <= 1e-5, (name, c)
            e = mtf.reduce_partials([emb[k] for k in g])
            offs, locs = slice_spec((B, L, D), (b, l, d), mesh, layout, c)
            idx = tuple(slice(o, o + n) for o, n in zip(offs, locs))
            assert np.array_equal(e.double().cpu().numpy(), e_full.data[idx]), (name, c)


def test_vocab_entry_point_errors(mtf):
    ids = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(mtf.MtfError) as e:
        mtf.embedding_local(ids, torch.zeros((4, 12), dtype=torch.bfloat16, device="cuda"), 0)
    assert e.value.name == "MTF_ERR_UNSUPPORTED"                        # d_model % 8
    z = torch.zeros((8, 6), dtype=torch.float32, device="cuda")
    r = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(mtf.MtfError) as e:
        mtf.xent_grad_local(z, r, r, ids, 0, r)
    assert e.value.name == "MTF_ERR_UNSUPPORTED"                        # vocab_local % 4
