"""GPU parity tests of mtf_einsum_local against the oracle's named einsum: the MFMA GEMM in
all operand layouts (with ragged edges, batches, epilogues) and the generic fp32 kernel."""
import numpy as np
import pytest
import torch

import paper_1811_02084_amd as mtf
from oracle.bf16 import round_to_bf16
from oracle.einsum import NT, einsum, einsum_abs
from oracle.metrics import m1, m2
from helpers import f64, named, BF16_TOL, F32_TOL

pytestmark = pytest.mark.gpu

SIZES = dict(m=304, n=264, k=200, b=3, h=2, p=5)      # several tiles and ragged tails (tile 256, k 64)


def _rand(dims, dtype, seed, sizes=SIZES, ints=False):
    rng = np.random.default_rng(seed)
    shape = [sizes[d] for d in dims]
    a = rng.integers(-2, 3, shape).astype(np.float32) if ints else rng.standard_normal(shape).astype(np.float32)
    return torch.from_numpy(a).to(dtype)


GEMM_CASES = [
    ("nn", "mk", "kn", "mn"), ("nt", "mk", "nk", "mn"), ("tn", "km", "kn", "mn"), ("tt", "km", "nk", "mn"),
    ("out transposed", "mk", "kn", "nm"), ("batched", "bmk", "bkn", "bmn"),
    ("two batch dims, strided rows", "bmhk", "bnhk", "bhmn"),
    ("k folded from two dims", "mhk", "hkn", "mn"), ("vector out", "k", "kn", "n"),
]


@pytest.mark.parametrize("name,da,db,do", GEMM_CASES)
def test_bf16_contractions(name, da, db, do):
    print(f"einsum_local bf16 {name}: {da},{db}->{do}", flush=True)
    a, b = _rand(da, torch.bfloat16, 1), _rand(db, torch.bfloat16, 2)
    got = mtf.einsum_local(a.cuda(), da, b.cuda(), db, do, out_dtype=torch.float32)
    ins = [named(a, da), named(b, db)]
    ref, ref_abs = einsum(ins, do), einsum_abs(ins, do)
    assert m1(f64(got), ref.data, ref_abs.data) <= 1e-5      # fp32 accumulation of exact products
    assert m2(f64(got), ref.data) <= BF16_TOL
    got16 = mtf.einsum_local(a.cuda(), da, b.cuda(), db, do, out_dtype=torch.bfloat16)
    assert m2(f64(got16), round_to_bf16(ref.data)) <= BF16_TOL


@pytest.mark.parametrize("name,da,db,do", GEMM_CASES[:4])
def test_bf16_integer_inputs_are_exact(name, da, db, do):
    """Small integers: every product and partial sum is exact in fp32, whatever the order."""
    print(f"einsum_local exact ints {name}", flush=True)
    a, b = _rand(da, torch.bfloat16, 3, ints=True), _rand(db, torch.bfloat16, 4, ints=True)
    got = mtf.einsum_local(a.cuda(), da, b.cuda(), db, do, out_dtype=torch.float32)
    ref = einsum([named(a, da), named(b, db)], do)
    assert np.array_equal(f64(got), ref.data)


def test_epilogues_alpha_accumulate():
    da, db, do = "mk", "kn", "mn"
    a, b = _rand(da, torch.bfloat16, 5), _rand(db, torch.bfloat16, 6)
    ref = einsum([named(a, da), named(b, db)], do).data
    print("relu", flush=True)
    got = mtf.einsum_local(a.cuda(), da, b.cuda(), db, do, out_dtype=torch.bfloat16, epi=mtf.EPI_RELU)
    assert m2(f64(got), round_to_bf16(np.maximum(ref, 0))) <= BF16_TOL
    assert float(got.float().min()) >= 0.0
    print("mask", flush=True)
    aux = _rand(do, torch.bfloat16, 7)
    aux[0, :8] = 0.0                                          # exactly zero: masked (gradient 0 at 0)
    got = mtf.einsum_local(a.cuda(), da, b.cuda(), db, do, out_dtype=torch.float32, epi=mtf.EPI_MASK_GT0,
                           aux=aux.cuda())
    assert m2(f64(got), np.where(f64(aux) > 0, ref, 0.0)) <= BF16_TOL
    assert np.all(f64(got)[f64(aux) <= 0] == 0.0)
    print("alpha + accumulate", flush=True)
    init = _rand(do, torch.float32, 8)
    out = init.clone().cuda()
    mtf.einsum_local(a.cuda(), da, b.cuda(), db, do, alpha=0.25, accumulate=True, out=out)
    assert m2(f64(out), 0.25 * ref + f64(init)) <= BF16_TOL


@pytest.mark.parametrize("sizes", [dict(m=8, n=8, k=8), dict(m=1, n=8, k=16), dict(m=257, n=8, k=8),
                                   dict(m=64, n=512, k=72), dict(m=512, n=256, k=1024)])
def test_edge_sizes(sizes):
    print(f"einsum_local sizes {sizes}", flush=True)
    for da, db in (("mk", "kn"), ("mk", "nk"), ("km", "kn")):
        if da == "km" and sizes["m"] % 8:
            continue                                         # goes to the generic kernel; covered below
        a, b = _rand(da, torch.bfloat16, 9, sizes), _rand(db, torch.bfloat16, 10, sizes)
        got = mtf.einsum_local(a.cuda(), da, b.cuda(), db, "mn", out_dtype=torch.float32)
        ins = [named(a, da), named(b, db)]
        assert m1(f64(got), einsum(ins, "mn").data, einsum_abs(ins, "mn").data) <= 1e-5


def test_largest_grids():
    """The limits of the launch shapes: many tiles along m (thousands of tile rows through the
    XCD remap), the largest batch count the grid takes, and one past it (generic kernel)."""
    print("einsum_local tall: m=262144", flush=True)
    sizes = dict(m=262144, n=136, k=72)
    a, b = _rand("mk", torch.bfloat16, 21, sizes, ints=True), _rand("kn", torch.bfloat16, 22, sizes, ints=True)
    got = mtf.einsum_local(a.cuda(), "mk", b.cuda(), "kn", "mn", out_dtype=torch.float32)
    ref = a.float() @ b.float()                              # small integers: exact in any order
    assert torch.equal(got.cpu(), ref)
    # spot-check rows against the oracle's own einsum
    rows = [0, 1, 255, 256, 131071, 131072, 262143]
    ref_rows = einsum([named(a[rows], "mk"), named(b, "kn")], "mn").data
    assert np.array_equal(f64(got[rows]), ref_rows)
    for nb in (65535, 65536):
        print(f"einsum_local batch {nb}", flush=True)
        sizes = dict(b=nb, m=8, n=8, k=8)
        a, b = _rand("bmk", torch.bfloat16, 23, sizes, ints=True), _rand("bkn", torch.bfloat16, 24, sizes, ints=True)
        got = mtf.einsum_local(a.cuda(), "bmk", b.cuda(), "bkn", "bmn", out_dtype=torch.float32)
        assert torch.equal(got.cpu(), torch.bmm(a.float(), b.float()))
        pick = [0, 1, nb // 2, nb - 1]
        ref = einsum([named(a[pick], "bmk"), named(b[pick], "bkn")], "bmn").data
        assert np.array_equal(f64(got[pick]), ref)


def test_seeded_sweep_of_shapes_layouts_and_epilogues():
    """40 seeded random problems: sizes that are and are not multiples of the tile sizes, every
    operand layout, batches, output dtype, ReLU / bias / alpha / accumulate, all against the
    oracle.  Whatever does not fit the MFMA kernel must run on the generic one with the same
    result."""
    rng = np.random.default_rng(18110208)
    layouts = [("mk", "kn"), ("mk", "nk"), ("km", "kn"), ("km", "nk"), ("bmk", "bkn"), ("bmk", "bnk")]
    for case in range(40):
        da, db = layouts[rng.integers(len(layouts))]
        do = ("b" if "b" in da else "") + ("mn" if rng.random() < 0.8 else "nm")
        mult = 8 if rng.random() < 0.8 else 1
        sizes = dict(m=int(rng.integers(1, 60)) * mult, n=int(rng.integers(1, 60)) * mult,
                     k=int(rng.integers(1, 50)) * mult, b=int(rng.integers(1, 4)))
        out_dtype = torch.float32 if rng.random() < 0.5 else torch.bfloat16
        alpha = float(rng.choice([1.0, 0.5, -2.0]))
        epi = [mtf.EPI_NONE, mtf.EPI_RELU, mtf.EPI_BIAS, mtf.EPI_BIAS_RELU][rng.integers(4)]
        accumulate = bool(rng.random() < 0.3)
        print(f"sweep {case}: {da},{db}->{do} {sizes} {out_dtype} alpha={alpha} epi={epi} acc={accumulate}", flush=True)
        a, b = _rand(da, torch.bfloat16, 100 + case, sizes), _rand(db, torch.bfloat16, 200 + case, sizes)
        ref = alpha * einsum([named(a, da), named(b, db)], do).data
        out = None
        if accumulate:
            old = _rand(do, out_dtype, 300 + case, sizes)
            ref = ref + f64(old)
            out = old.cuda().clone()
        aux = None
        if epi in (mtf.EPI_BIAS, mtf.EPI_BIAS_RELU):
            aux = _rand(do[-1], torch.bfloat16, 400 + case, sizes)
            ref = ref + f64(aux)                                  # broadcast over the leading dims
        if epi in (mtf.EPI_RELU, mtf.EPI_BIAS_RELU):
            ref = np.maximum(ref, 0.0)
        got = mtf.einsum_local(a.cuda(), da, b.cuda(), db, do, out_dtype=out_dtype, epi=epi,
                               aux=aux.cuda() if aux is not None else None, alpha=alpha, accumulate=accumulate, out=out)
        want = round_to_bf16(ref) if out_dtype == torch.bfloat16 else ref
        assert m2(f64(got), want) <= BF16_TOL, case


GENERIC_CASES = [
    ("fp32 matmul", "bld", "df", "blf", torch.float32),
    ("fp32 outer + reduce", "bm", "pn", "mn", torch.float32),
    ("bf16 odd sizes", "mp", "pn", "mn", torch.bfloat16),
    ("bf16 batch innermost", "bmk", "bkn", "mnb", torch.bfloat16),
    ("scalar out", "mk", "mk", "", torch.float32),
]


@pytest.mark.parametrize("name,da,db,do,dtype", GENERIC_CASES)
def test_generic_kernel(name, da, db, do, dtype):
    print(f"einsum_local generic {name}", flush=True)
    sizes = dict(b=2, l=8, d=16, f=64, m=33, n=18, k=70, p=5)
    a, b = _rand(da, dtype, 11, sizes), _rand(db, dtype, 12, sizes)
    got = mtf.einsum_local(a.cuda(), da, b.cuda(), db, do, out_dtype=torch.float32)
    ins = [named(a, da), named(b, db)]
    ref, ref_abs = einsum(ins, do), einsum_abs(ins, do)
    assert tuple(got.shape) == ref.data.shape
    assert m1(f64(got), ref.data, ref_abs.data) <= F32_TOL


def test_one_operand_einsum_and_errors():
    a = _rand("bmk", torch.float32, 13, dict(b=3, m=4, k=5))
    got = mtf.einsum_local(a.cuda(), "bmk", None, None, "kb")           # reduce + transpose
    assert m2(f64(got), f64(a).sum(axis=1).T) <= F32_TOL
    with pytest.raises(mtf.MtfError) as e:
        mtf.einsum_local(a.cuda(), "bmk", None, None, "bq")
    assert e.value.name == "MTF_ERR_OUT_NOT_SUBSET"
    with pytest.raises(mtf.MtfError) as e:
        mtf.einsum_local(a.cuda(), "bmk", a.cuda()[:, :, :4].contiguous(), "bmk", "bm")
    assert e.value.name == "MTF_ERR_SIZE_MISMATCH"
    with pytest.raises(mtf.MtfError) as e:
        mtf.einsum_local(a.cuda(), "bmm", None, None, "b")
    assert e.value.name == "MTF_ERR_DUP_DIM"


def test_run_to_run_bitwise_determinism():
    a, b = _rand("mk", torch.bfloat16, 14), _rand("kn", torch.bfloat16, 15)
    outs = [mtf.einsum_local(a.cuda(), "mk", b.cuda(), "kn", "mn", out_dtype=torch.float32).cpu() for _ in range(3)]
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("n", [1, 2, 4])
@pytest.mark.parametrize("name,da,db,do", GEMM_CASES[:5] + [GEMM_CASES[7]])
def test_contracted_dim_cut_into_ranges(name, da, db, do, n):
    """mtf_einsum_local_kranges: range i of the contracted dim against the oracle's einsum of the
    operands sliced to that range, the ranges' sum against the whole einsum, and exactness on
    integers."""
    print(f"einsum_local_kranges {name} n={n}", flush=True)
    sizes = dict(SIZES, k=192, h=2)                    # contracted size 192 (384 when h folds in): divisible by 8 n
    a, b = _rand(da, torch.bfloat16, 21, sizes), _rand(db, torch.bfloat16, 22, sizes)
    parts = mtf.einsum_local_kranges(a.cuda(), da, b.cuda(), db, do, n)
    assert len(parts) == n and all(p.dtype == torch.float32 for p in parts)
    ins = [named(a, da), named(b, db)]
    ref, ref_abs = einsum(ins, do), einsum_abs(ins, do)
    total = sum(f64(p) for p in parts)
    assert m1(total, ref.data, ref_abs.data) <= 1e-5 and m2(total, ref.data) <= BF16_TOL
    if "h" not in da:                                  # one contracted dim: range i is a slice of k
        kr = sizes["k"] // n
        for i, p in enumerate(parts):
            cut = lambda t, dims: NT(np.take(t.data, range(i * kr, (i + 1) * kr), axis=dims.index("k")), t.dims)
            want = einsum([cut(ins[0], da), cut(ins[1], db)], do)
            assert m2(f64(p), want.data) <= BF16_TOL, i
    ai, bi = _rand(da, torch.bfloat16, 23, sizes, ints=True), _rand(db, torch.bfloat16, 24, sizes, ints=True)
    parts = mtf.einsum_local_kranges(ai.cuda(), da, bi.cuda(), db, do, n)
    assert np.array_equal(sum(f64(p) for p in parts), einsum([named(ai, da), named(bi, db)], do).data)


def test_ranges_refused():
    a, b = _rand("mk", torch.bfloat16, 25), _rand("kn", torch.bfloat16, 26)        # k = 200
    with pytest.raises(mtf.MtfError) as e:
        mtf.einsum_local_kranges(a.cuda(), "mk", b.cuda(), "kn", "mn", 4)          # 200 % 32 != 0
    assert e.value.name == "MTF_ERR_UNSUPPORTED"
    with pytest.raises(mtf.MtfError) as e:
        mtf.einsum_local_kranges(a.cuda(), "mk", b.cuda(), "kn", "mn", 5)
    assert e.value.name == "MTF_ERR_UNSUPPORTED"
    ab, bb = _rand("bmk", torch.bfloat16, 27, dict(SIZES, k=192)), _rand("bkn", torch.bfloat16, 28, dict(SIZES, k=192))
    with pytest.raises(mtf.MtfError) as e:
        mtf.einsum_local_kranges(ab.cuda(), "bmk", bb.cuda(), "bkn", "bmn", 2)     # batch dims: not this call
    assert e.value.name == "MTF_ERR_UNSUPPORTED"
