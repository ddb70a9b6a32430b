"""Parity of the vocabulary-split operations (embedding, logits + softmax cross-entropy, their
gradients) against the oracle, through the C ABI: one processor's stripe at its real shape, and a
virtual mesh on which the Allreduce groups (max and sum) are combined on the GPU."""
import numpy as np
import pytest
import torch

import mtf_inputs
from helpers import named as to_nt
from oracle import vocab as OV
from oracle.einsum import nt
from oracle.layout import all_coords, slice_spec
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
    "config6-size": dict(batch=16, length=256, d_model=1024, vocab_local=2048, vocab_total=32768, offset=2048),
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


@pytest.mark.parametrize("case", sorted(CASES))
def test_loss_stripe_forward_backward(mtf, case):
    """One processor's stripe: its local statistics against the oracle's on the same stripe, then
    (whole-vocab case) the loss itself, then the logits gradient and the two gradient einsums."""
    p = CASES[case]
    cfg = mtf_inputs.vocab_inputs(33, p["batch"], p["length"], p["d_model"], p["vocab_local"], p["vocab_total"])
    off, vl = p["offset"], p["vocab_local"]
    x, w = to_nt(cfg["x"], (B, L, D)), to_nt(cfg["w_vocab"], (D, VOCAB))
    z_ref = x.data @ w.data                                              # [b, l, vocab_local], fp64
    z = mtf.einsum_local(_dev(cfg["x"]), (B, L, D), _dev(cfg["w_vocab"]), (D, VOCAB), (B, L, VOCAB),
                         out_dtype=torch.float32)
    assert m2(z.cpu().numpy(), z_ref) <= TOL_BF16
    # the statistics kernels are fed the ORACLE's logits (stored fp32), so that every expected
    # value below comes from the oracle side alone
    z = _dev(torch.from_numpy(z_ref).float())
    zd = z.double().cpu().numpy()
    m_loc = mtf.reduce_local(z, (B, L, VOCAB), (B, L), mtf.REDUCE_MAX)
    assert np.array_equal(m_loc.double().cpu().numpy(), zd.max(axis=-1))
    targets = cfg["targets"]
    sumexp, picked = mtf.xent_stats_local(z, m_loc, _dev(targets), off)
    want_s = np.exp(zd - zd.max(axis=-1, keepdims=True)).sum(axis=-1)
    tl = targets.numpy().astype(np.int64) - off
    local = (tl >= 0) & (tl < vl)
    want_t = np.where(local, np.take_along_axis(zd, np.clip(tl, 0, vl - 1)[..., None], axis=-1)[..., 0], 0.0)
    assert m2(sumexp.cpu().numpy(), want_s) <= TOL_F32
    assert np.array_equal(picked.double().cpu().numpy(), want_t)
    if p["vocab_total"] == vl:                                           # the group is this one processor
        loss = mtf.xent_loss(m_loc, sumexp, picked)
        want = zd.max(axis=-1) + np.log(want_s) - want_t
        assert m2(loss.cpu().numpy(), want) <= TOL_F32
        full = OV.xent_fwd(x, w, targets.numpy())                        # and against the oracle end to end
        assert m2(loss.cpu().numpy(), full["loss"].data) <= TOL_F32
    # backward from given (group-wide) statistics
    dloss = cfg["dloss"]
    dz = mtf.xent_grad_local(z, m_loc, sumexp, _dev(targets), off, _dev(dloss))
    onehot = np.zeros_like(zd)
    np.put_along_axis(onehot, np.clip(tl, 0, vl - 1)[..., None], local[..., None].astype(np.float64), axis=-1)
    want_dz = (np.exp(zd - zd.max(axis=-1, keepdims=True)) / want_s[..., None] - onehot) * dloss.double().numpy()[..., None]
    assert m2(dz.float().cpu().numpy(), want_dz) <= TOL_BF16
    dz_ref = torch.from_numpy(want_dz).to(torch.bfloat16)                # the oracle's stored dz on both sides
    dzn = to_nt(dz_ref, (B, L, VOCAB))
    dw = mtf.einsum_local(_dev(cfg["x"]), (B, L, D), _dev(dz_ref), (B, L, VOCAB), (D, VOCAB), out_dtype=torch.float32)
    dx = mtf.einsum_local(_dev(dz_ref), (B, L, VOCAB), _dev(cfg["w_vocab"]), (D, VOCAB), (B, L, D),
                          out_dtype=torch.float32)
    assert m2(dw.cpu().numpy(), np.einsum("bld,blv->dv", x.data, dzn.data)) <= TOL_BF16
    assert m2(dx.cpu().numpy(), np.einsum("blv,dv->bld", dzn.data, w.data)) <= TOL_BF16


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
