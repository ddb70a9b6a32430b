"""The attention core behind mtf_attention_fwd / mtf_attention_bwd against the oracle: the fused
kernels at head widths 128 and 256 (the paper's translation and language models), and at any other
width two einsums on the GEMM kernel with a row softmax between them."""
import math

import numpy as np
import pytest
import torch

import mtf_inputs
from helpers import named as to_nt
from oracle import layer as OL
from oracle.layer import B, L, M, H, K, V
from oracle.metrics import m2

pytestmark = pytest.mark.gpu

TOL = 2e-2      # bf16 storage, fp32 accumulation


@pytest.fixture(scope="module")
def mtf():
    import paper_1811_02084_amd as m
    return m


CASES = [  # batch, length, heads, d_k, causal
    (2, 136, 3, 256, True),
    (2, 136, 3, 256, False),
    (1, 64, 2, 64, True),
    (3, 200, 2, 32, False),
    (2, 72, 2, 128, True),       # the fused kernels behind the same entry points
    (4, 256, 8, 256, True),      # a shard of the LM variant: 8 heads of width 256
    (2, 520, 4, 256, True),      # width 256 past one pass of row blocks, ragged tail of 8 rows
    (1, 1, 1, 256, True),        # a single position
    (1, 33, 2, 256, False),      # one row into the second 32-row tile
    (4, 200, 32, 128, True),     # fused kernels with 4 waves per workgroup (128 (batch, head) pairs), ragged
    (4, 256, 32, 128, False),
    (4, 384, 32, 128, True),     # 8-wave workgroups with an odd number of 128-row blocks (middle block unpaired)
    (4, 328, 32, 128, False),    # the same, ragged and unmasked
]


@pytest.mark.parametrize("case", CASES, ids=[f"b{c[0]}-l{c[1]}-h{c[2]}-k{c[3]}-{'causal' if c[4] else 'full'}" for c in CASES])
def test_attention_core_any_width(mtf, case):
    b, l, h, dk, causal = case
    scale = 1.0 / math.sqrt(dk)
    q = mtf_inputs.normal(51, 0, (b, l, h, dk))
    k = mtf_inputs.normal(51, 1, (b, l, h, dk))
    v = mtf_inputs.normal(51, 2, (b, l, h, dk))
    dctx = mtf_inputs.normal(51, 3, (b, l, h, dk))
    qn, kn, vn = to_nt(q, (B, L, H, K)), to_nt(k, (B, M, H, K)), to_nt(v, (B, M, H, V))
    ctx_ref, lse_ref = OL.attention_core_fwd(qn, kn, vn, scale, causal)
    ctx, lse = mtf.attention_fwd(q.cuda(), k.cuda(), v.cuda(), scale, causal)
    assert m2(ctx.float().cpu().numpy(), ctx_ref.data) <= TOL
    assert np.max(np.abs(lse.cpu().numpy() - lse_ref.data)) <= 1e-3 * max(1.0, np.max(np.abs(lse_ref.data)))
    # backward on the oracle's saved ctx / lse
    ctx_s = torch.from_numpy(ctx_ref.data).to(torch.bfloat16)
    lse_s = torch.from_numpy(lse_ref.data).float()
    dq_ref, dk_ref, dv_ref = OL.attention_core_bwd(qn, kn, vn, to_nt(ctx_s, (B, L, H, V)), to_nt(lse_s, (B, H, L)),
                                                   to_nt(dctx, (B, L, H, V)), scale, causal)
    dq, dk_, dv = mtf.attention_bwd(q.cuda(), k.cuda(), v.cuda(), ctx_s.cuda(), lse_s.cuda(), dctx.cuda(), scale, causal)
    for name, got, ref in (("dq", dq, dq_ref), ("dk", dk_, dk_ref), ("dv", dv, dv_ref)):
        err = m2(got.float().cpu().numpy(), ref.data)
        assert err <= TOL, (name, err)


@pytest.mark.parametrize("dk", [128, 256])
@pytest.mark.parametrize("scale", [-0.05, 0.0])
def test_attention_core_negative_and_zero_scale(mtf, dk, scale):
    """The kernels keep their running maximum on scale * logit with the scale's sign moved into an
    operand; a zero scale makes every visible logit equal."""
    b, l, h = 2, 100, 2
    q, k, v, dctx = (mtf_inputs.normal(52, i, (b, l, h, dk)) for i in range(4))
    qn, kn, vn = to_nt(q, (B, L, H, K)), to_nt(k, (B, M, H, K)), to_nt(v, (B, M, H, V))
    ctx_ref, lse_ref = OL.attention_core_fwd(qn, kn, vn, scale, True)
    ctx, lse = mtf.attention_fwd(q.cuda(), k.cuda(), v.cuda(), scale, True)
    assert m2(ctx.float().cpu().numpy(), ctx_ref.data) <= TOL
    assert np.max(np.abs(lse.cpu().numpy() - lse_ref.data)) <= 1e-3 * max(1.0, np.max(np.abs(lse_ref.data)))
    ctx_s = torch.from_numpy(ctx_ref.data).to(torch.bfloat16)
    lse_s = torch.from_numpy(lse_ref.data).float()
    refs = OL.attention_core_bwd(qn, kn, vn, to_nt(ctx_s, (B, L, H, V)), to_nt(lse_s, (B, H, L)),
                                 to_nt(dctx, (B, L, H, V)), scale, True)
    gots = mtf.attention_bwd(q.cuda(), k.cuda(), v.cuda(), ctx_s.cuda(), lse_s.cuda(), dctx.cuda(), scale, True)
    for name, got, ref in zip(("dq", "dk", "dv"), gots, refs):
        if scale == 0.0 and name != "dv":       # dq = dk = 0 exactly: nothing to scale an error by
            assert float(got.float().abs().max()) == 0.0, name
        else:
            assert m2(got.float().cpu().numpy(), ref.data) <= TOL, name


def test_attention_core_errors(mtf):
    q = torch.zeros((1, 12, 2, 64), dtype=torch.bfloat16, device="cuda")     # length % 8 != 0, unfused path
    with pytest.raises(mtf.MtfError) as e:
        mtf.attention_fwd(q, q, q, 1.0, False)
    assert e.value.name == "MTF_ERR_UNSUPPORTED"
    q = torch.zeros((1, 16, 2, 60), dtype=torch.bfloat16, device="cuda")     # d_k % 8 != 0
    with pytest.raises(mtf.MtfError) as e:
        mtf.attention_fwd(q, q, q, 1.0, False)
    assert e.value.name == "MTF_ERR_UNSUPPORTED"
