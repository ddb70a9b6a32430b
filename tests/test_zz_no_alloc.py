"""The entry point that allocates nothing (mtf_reduce_local_static: scratch in a static device
array inside the library) against the entry point it is a variant of (mtf_reduce_local with a
caller workspace), through the C ABI.  Same kernels and the same fixed summation order, so the
results must be identical bit for bit - on two calls in a row, the second with a smaller input
(the static array keeps the first call's partials), and for a reduction that exceeds the stated
maximum the call must be refused with nothing launched."""
import ctypes as C

import pytest
import torch

import mtf_inputs
import paper_1811_02084_amd as mtf
from paper_1811_02084_amd import binding

pytestmark = pytest.mark.gpu

DIMS = ("batch", "length", "d_ff")


def _both(x, out_dims, op):
    want = mtf.reduce_local(x, DIMS, out_dims, op)
    got = torch.full_like(want, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    mtf.reduce_local_static(x, DIMS, out_dims, op, out=got)
    assert torch.cuda.memory_allocated() == before            # nothing taken from torch's allocator either
    torch.cuda.synchronize()
    return got, want


def test_static_scratch_reduce_matches_workspace_reduce_on_two_calls_in_a_row():
    # first call: dbias of config 2's shape (4096 tokens x 4096 columns, 64 chunks: 1 MiB of partials)
    big = mtf_inputs.normal(41, 0, (16, 256, 4096)).cuda()
    small = mtf_inputs.normal(41, 1, (3, 50, 264)).cuda()     # ragged: fewer chunks, fewer columns
    for op in (mtf.REDUCE_SUM, mtf.REDUCE_MAX):
        print(f"static-scratch reduce, op {op}: x{tuple(big.shape)} then x{tuple(small.shape)}", flush=True)
        got, want = _both(big, ("d_ff",), op)
        assert torch.equal(got, want)
        got, want = _both(small, ("d_ff",), op)               # smaller input right after the larger one
        assert torch.equal(got, want)
        got, want = _both(big, ("d_ff",), op)                 # and the larger one again
        assert torch.equal(got, want)
    # fp32 input, bf16 output, kept dims (length, d_ff): still the column pattern
    xf = mtf_inputs.normal(41, 2, (5, 24, 64), dtype=torch.float32).cuda()
    want = mtf.reduce_local(xf, DIMS, ("length", "d_ff"), mtf.REDUCE_SUM, out_dtype=torch.bfloat16)
    got = mtf.reduce_local_static(xf, DIMS, ("length", "d_ff"), mtf.REDUCE_SUM, out_dtype=torch.bfloat16)
    assert torch.equal(got, want)
    # patterns that need no scratch at all go through unchanged
    got, want = _both(small, ("batch", "length"), mtf.REDUCE_MAX)
    assert torch.equal(got, want)


def test_static_scratch_reduce_refuses_what_does_not_fit():
    # 2 Mi columns: one chunk of 2 Mi fp32 partials = 8 MiB > the 4 MiB static array
    n = 1 << 21
    x = torch.zeros((16, 1, n), dtype=torch.bfloat16, device="cuda")
    k = binding._Keep()
    sx = k.shape(list(zip(DIMS, x.shape)))
    so = k.shape([("d_ff", n)])
    need = binding.lib.mtf_reduce_local_workspace_bytes(C.byref(sx), C.byref(so))
    assert need > binding.REDUCE_STATIC_MAX_SCRATCH
    out = torch.full((n,), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(mtf.MtfError) as e:
        mtf.reduce_local_static(x, DIMS, ("d_ff",), mtf.REDUCE_SUM, out=out)
    assert e.value.name == "MTF_ERR_WORKSPACE"
    assert "static" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                            # nothing was launched
    # the workspace entry point still takes it
    assert torch.equal(mtf.reduce_local(x, DIMS, ("d_ff",), mtf.REDUCE_SUM), torch.zeros_like(out))
