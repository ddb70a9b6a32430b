#!/usr/bin/env python3
"""Benchmark of the per-processor lowered-einsum path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input: forward and
backward of a full Transformer-layer shard (attention + feed-forward sublayers with their
residual adds), every contraction in the library's HIP kernels.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload layer|ffn|ffn_bias|mha|mesh|mesh3d|attention_lm|vocab|reshape|layer_norm]
  python bench.py --workload ceiling|copy      (measurement aids, see below)

`--workload copy` is not a benchmark of the path: it launches the library's plain copy kernel
(fp32 -> fp32 cast) on a buffer of known size, which is what the HBM counters of a profiler run
are scaled by (see roofline.traffic).
"""
import argparse
import gc
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
METRIC = "TFLOP/s per-shard Transformer einsum (bf16) + % of MFMA peak on 1 MI355X"


def flops_ffn(T, D, F):
    return 2 * 2.0 * T * D * F                       # two einsums


def flops_mha(B, L, D, H, K, causal):
    T = B * L
    pairs = L * (L + 1) / 2 if causal else L * L
    return 4 * 2.0 * T * D * H * K + 2 * 2.0 * B * H * pairs * K     # q,k,v,o projections + 2 attention einsums


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="layer", choices=["layer", "ffn", "ffn_bias", "mha", "mesh", "mesh3d", "attention_lm", "vocab", "reshape", "layer_norm", "copy", "ceiling"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of one captured HIP graph of the step instead of eager launches")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (one processor's share of the mesh); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch
    import mtf_inputs
    import paper_1811_02084_amd as mtf

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.workload == "copy":
        return copy_calibration(args, torch, mtf, dev)
    if args.workload == "reshape":
        return reshape_bench(args, torch, mtf, mtf_inputs, dev)
    if args.workload == "layer_norm":
        return layer_norm_bench(args, torch, mtf, mtf_inputs, dev)
    if args.workload == "ceiling":
        return ceiling_probe(args, torch, mtf, mtf_inputs, dev)

    # ---------------------------------------------------------------- workload
    if args.workload == "layer":
        cfg = mtf_inputs.config5()
        B, L, D = cfg["x"].shape
        H, K, F = cfg["w_q"].shape[1], cfg["w_q"].shape[2], cfg["w_in"].shape[1]
        causal = True
        fwd = flops_mha(B, L, D, H, K, causal) + flops_ffn(B * L, D, F)
        name = (f"config 5: full layer shard fwd+bwd, x[{B},{L},{D}] heads_local={H} d_k={K} "
                f"d_ff_local={F} causal")
        g = {k: (v.to(dev) if torch.is_tensor(v) else v) for k, v in cfg.items()}
        w = {k: g[k] for k in ("w_q", "w_k", "w_v", "w_o", "w_in", "w_out")}
        bufs = mtf.layer_alloc(g["x"], w)

        def step_fwd():
            mtf.layer_fwd(g["x"], w, cfg["scale"], causal, bufs)

        def step_bwd():
            mtf.layer_bwd(g["x"], w, bufs["saved"], g["dz"], cfg["scale"], causal, bufs)

        def step():
            step_fwd()
            step_bwd()
    elif args.workload in ("ffn", "ffn_bias"):
        cfg = mtf_inputs.config2()
        B, L, D = cfg["x"].shape
        F = cfg["w_in"].shape[1]
        fwd = flops_ffn(B * L, D, F)
        g = {k: v.to(dev) for k, v in cfg.items()}
        ws = torch.empty(B * L * F * 2 + (8 << 20), dtype=torch.uint8, device=dev)
        if args.workload == "ffn":
            name = f"config 2: FFN shard fwd+bwd, x[{B},{L},{D}] d_ff_local={F}"

            def step():
                a, _ = mtf.ffn_fwd(g["x"], g["w_in"], g["w_out"])
                mtf.ffn_bwd(g["x"], a, g["w_in"], g["w_out"], g["dy"], workspace=ws)
        else:       # the worked example as printed: y = Relu(x w + bias) v, and dbias in backward
            name = f"config 2 + bias: y = Relu(x w + bias) v fwd+bwd, x[{B},{L},{D}] d_ff_local={F}"
            bias = mtf_inputs.normal(2, 9, (F,), std=0.5).to(dev)
            cfg = dict(cfg, bias=bias.cpu())

            def step():
                a, _ = mtf.ffn_bias_fwd(g["x"], g["w_in"], bias, g["w_out"])
                mtf.ffn_bias_bwd(g["x"], a, g["w_in"], g["w_out"], g["dy"], workspace=ws)
    elif args.workload == "mesh":
        # config 4: the feed-forward sublayer on a VIRTUAL 4x4 mesh held on this one GPU (batch over
        # rows, d_ff over cols): 16 processors' local einsums, then the partial sums added up within
        # each mesh row (over the column index) - 4 groups of 4 - by the reduce kernel that stands
        # in for the Allreduce (section "Data-Parallel, Model-Parallel Layouts")
        cfg = mtf_inputs.config4()
        mesh, layout = cfg["mesh"], cfg["layout"]
        B, L, D = cfg["x"].shape
        F = cfg["w_in"].shape[1]
        fwd = flops_ffn(B * L, D, F) / 3.0                        # forward only: undo the x3 below
        name = f"config 4: FFN forward on a virtual 4x4 mesh, x[{B},{L},{D}] d_ff={F}, 16 slices + 4 group reduces"
        g = {k: v.to(dev) for k, v in cfg.items() if torch.is_tensor(v)}
        coords = [(r, c) for r in range(4) for c in range(4)]
        xs = {c: mtf.slice_copy(g["x"], ("batch", "length", "d_model"), mesh, layout, c) for c in coords}
        wi = {c: mtf.slice_copy(g["w_in"], ("d_model", "d_ff"), mesh, layout, c) for c in coords}
        wo = {c: mtf.slice_copy(g["w_out"], ("d_ff", "d_model"), mesh, layout, c) for c in coords}

        def step():
            parts = {c: mtf.ffn_fwd(xs[c], wi[c], wo[c])[1] for c in coords}
            return [mtf.reduce_partials([parts[(r, c)] for c in range(4)]) for r in range(4)]
    elif args.workload == "mesh3d":
        # config 7: the worked example's 3-D layout (batch -> rows, d_ff -> cols, d_model -> planes) on
        # a VIRTUAL 2x2x2 mesh held on this one GPU, forward and backward: on every processor each of
        # the six einsums leaves a partial sum (section "Data-Parallel, Model-Parallel Layouts",
        # last layout), which the reduce kernel sums over the mesh dim the einsum's plan names (once
        # per group of processors that differ only along that dim), applying the ReLU resp. its mask
        cfg = mtf_inputs.config7()
        mesh, layout = cfg["mesh"], cfg["layout"]
        B, L, D = cfg["x"].shape
        F = cfg["w_in"].shape[1]
        fwd = flops_ffn(B * L, D, F)
        name = (f"config 7: FFN fwd+bwd on a virtual 2x2x2 mesh (3-D layout), x[{B},{L},{D}] d_ff={F}: "
                "8 processors x 6 einsums, every one a partial sum + grouped reduce")
        g = {k: v.to(dev) for k, v in cfg.items() if torch.is_tensor(v)}
        coords = [(r, c, p) for r in range(2) for c in range(2) for p in range(2)]
        X, WI, WO, HID = ("batch", "length", "d_model"), ("d_model", "d_ff"), ("d_ff", "d_model"), ("batch", "length", "d_ff")
        sl = lambda n, dims: {c: mtf.slice_copy(g[n], dims, mesh, layout, c) for c in coords}
        xs, wi, wo, dys = sl("x", X), sl("w_in", WI), sl("w_out", WO), sl("dy", X)
        sizes = dict(zip(X, (B, L, D)))
        sizes["d_ff"] = F
        shp = lambda dims: [(d, sizes[d]) for d in dims]
        axes = lambda p, q, o: tuple(mtf.einsum_plan(shp(p), shp(q), shp(o), mesh, layout)["reduce_axes"])
        plan = {k: axes(*v) for k, v in dict(h=(X, WI, HID), y=(HID, WO, X), dwo=(HID, X, WO), da=(X, WO, HID),
                                             dwi=(X, HID, WI), dx=(HID, WI, X)).items()}
        group = lambda c, ax: [c2 for c2 in coords if all(c2[i] == c[i] for i in range(3) if i not in ax)]
        f32, bf16 = torch.float32, torch.bfloat16

        def reduced(parts, ax, dt, epi=mtf.EPI_NONE, aux=None):
            # every processor of a group ends with the same sum: taken once per group and shared
            done = {}
            for c in coords:
                members = tuple(group(c, ax))
                if members not in done:
                    bufs = [t for c2 in members for t in (parts[c2] if isinstance(parts[c2], list) else [parts[c2]])]
                    done[members] = mtf.reduce_partials(bufs, out_dtype=dt, epi=epi,
                                                        aux=None if aux is None else aux[c])
            return {c: done[tuple(group(c, ax))] for c in coords}

        def step():
            # the ReLU and the mask of its gradient ride on the reduce that completes their operand
            # the four einsums with a 512-wide output side run as 2 ranges of their contracted dim
            # (their partial sums go into the same reduce): 128 tiles for 256 CUs otherwise
            es = mtf.einsum_local
            kr = lambda p, pd, q, qd, od: mtf.einsum_local_kranges(p, pd, q, qd, od, 2)
            a = reduced({c: es(xs[c], X, wi[c], WI, HID, out_dtype=f32) for c in coords}, plan["h"], bf16,
                        mtf.EPI_RELU)
            y = reduced({c: kr(a[c], HID, wo[c], WO, X) for c in coords}, plan["y"], f32)
            dwo = reduced({c: kr(a[c], HID, dys[c], X, WO) for c in coords}, plan["dwo"], f32)
            dh = reduced({c: es(dys[c], X, wo[c], WO, HID, out_dtype=f32) for c in coords}, plan["da"], bf16,
                         mtf.EPI_MASK_GT0, a)
            dwi = reduced({c: kr(xs[c], X, dh[c], HID, WI) for c in coords}, plan["dwi"], f32)
            dx = reduced({c: kr(dh[c], HID, wi[c], WI, X) for c in coords}, plan["dx"], f32)
            return y, dwo, dwi, dx
    elif args.workload == "attention_lm":
        # the attention core at the head width of the paper's language models (d_k = d_v = 256):
        # 8 local heads of width 256 (the same 2048 columns as config 5), causal, 8 x 512 tokens
        B, L, H, K = 8, 512, 8, 256
        causal, scale = True, 1.0 / math.sqrt(K)
        pairs = L * (L + 1) / 2
        fwd = 2 * 2.0 * B * H * pairs * K
        name = f"attention core fwd+bwd, q/k/v[{B},{L},{H},{K}] causal (fused kernels at head width 256)"
        cfg = {n: mtf_inputs.normal(8, i, (B, L, H, K)) for i, n in enumerate(("q", "k", "v", "dctx"))}
        cfg.update(scale=scale, causal=causal)
        g = {n: (t.to(dev) if torch.is_tensor(t) else t) for n, t in cfg.items()}

        def step():
            ctx, lse = mtf.attention_fwd(g["q"], g["k"], g["v"], scale, causal)
            mtf.attention_bwd(g["q"], g["k"], g["v"], ctx, lse, g["dctx"], scale, causal)
    elif args.workload == "vocab":
        # one processor's share of the vocabulary-split operations (embedding; logits + softmax
        # cross-entropy with its three reductions; their gradients); the Allreduce group is this
        # one stripe, so the combining steps are identities and are left out
        cfg = mtf_inputs.config6()
        B, L, D = cfg["x"].shape
        VL, off = cfg["w_vocab"].shape[1], cfg["vocab_offset"]
        fwd = 2.0 * B * L * D * VL                                  # the logits einsum; the gathers count 0
        name = f"config 6: vocab-split ops fwd+bwd, x[{B},{L},{D}] vocab_local={VL} of {cfg['vocab_total']}"
        g = {k: (v.to(dev) if torch.is_tensor(v) else v) for k, v in cfg.items()}
        dims_x, dims_w, dims_z = ("batch", "length", "d_model"), ("d_model", "vocab"), ("batch", "length", "vocab")

        def step():
            mtf.embedding_local(g["ids"], g["table"], off)
            z = mtf.einsum_local(g["x"], dims_x, g["w_vocab"], dims_w, dims_z, out_dtype=torch.float32)
            m = mtf.reduce_local(z, dims_z, dims_z[:2], mtf.REDUCE_MAX)
            s, t = mtf.xent_stats_local(z, m, g["targets"], off)
            mtf.xent_loss(m, s, t)
            dz = mtf.xent_grad_local(z, m, s, g["targets"], off, g["dloss"])
            mtf.einsum_local(g["x"], dims_x, dz, dims_z, dims_w, out_dtype=torch.float32)
            mtf.einsum_local(dz, dims_z, g["w_vocab"], dims_w, dims_x, out_dtype=torch.float32)
            mtf.embedding_grad_local(g["ids"], g["de"], VL, off)
    else:
        cfg = mtf_inputs.config3()
        B, L, D = cfg["x"].shape
        H, K = cfg["w_q"].shape[1], cfg["w_q"].shape[2]
        causal = cfg["causal"]
        fwd = flops_mha(B, L, D, H, K, causal)
        name = f"config 3: attention shard fwd+bwd, x[{B},{L},{D}] heads_local={H} d_k={K}"
        g = {k: (v.to(dev) if torch.is_tensor(v) else v) for k, v in cfg.items()}

        def step():
            r = mtf.mha_fwd(g["x"], g["w_q"], g["w_k"], g["w_v"], g["w_o"], cfg["scale"], causal)
            mtf.mha_bwd(g["x"], g["w_q"], g["w_k"], g["w_v"], g["w_o"], r["q"], r["k"], r["v"], r["ctx"],
                        r["lse"], g["dy"], cfg["scale"], causal)
    step_flops = 3.0 * fwd          # every forward einsum has two gradient einsums of the same size

    # ---------------------------------------------------------------- timed region
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    run_step = step
    if args.graph:                   # the library allocates nothing and never synchronises: capturable
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run_step = graph.replay
        run_step()
        torch.cuda.synchronize()
    gc.collect()
    gc.disable()                     # as timeit does: no collector pause of the host inside the timed region
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    gc.enable()
    ms_per_step = elapsed * 1e3 / args.steps
    tflops = step_flops / (ms_per_step * 1e-3) / 1e12

    # ---------------------------------------------------------------- forward / backward split
    halves = None
    if args.workload == "layer":
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
        for e in ev:                     # the binding launches on torch's current stream
            e[0].record(); step_fwd(); e[1].record(); step_bwd(); e[2].record()
        torch.cuda.synchronize()
        f = sorted(e[0].elapsed_time(e[1]) for e in ev)
        b = sorted(e[1].elapsed_time(e[2]) for e in ev)
        halves = {"fwd_ms_median": round(f[len(f) // 2], 4), "fwd_ms_min": round(f[0], 4),
                  "bwd_ms_median": round(b[len(b) // 2], 4), "bwd_ms_min": round(b[0], 4)}

    # ---------------------------------------------------------------- dominant kernel, timed per launch
    # same steps again with every launch bracketed by HIP events on the launch stream
    mtf.timing_enable(True)
    for _ in range(args.steps):
        step()
    kinds = mtf.timing_collect()
    # what the matrix cores alone sustain here, operands distributed like the path's (N(0,1) bf16)
    ops = mtf_inputs.normal(0, 99, (4096,)).to(torch.bfloat16).to(dev)
    sink = torch.empty(66, dtype=torch.float32, device=dev)
    for _ in range(12):                  # ~0.6 ms each: long enough for the clock to settle
        mtf.mfma_ceiling(ops, 2000, sink)
    ceil = [r for r in mtf.timing_collect() if r["kernel"] == "mfma_ceiling_kernel"]
    mtf.timing_enable(False)
    mfma_only = round(ceil[0]["flops"] / (ceil[0]["total_ms"] * 1e-3) / 1e12, 1) if ceil else None
    kinds.sort(key=lambda r: -r["total_ms"])
    dom = kinds[0]
    avg_ms = dom["total_ms"] / dom["launches"]
    achieved = dom["flops"] / dom["launches"] / (avg_ms * 1e-3) / 1e12
    if dom["flops"] > 0:
        roofline = dict(bound="mfma", achieved=round(achieved, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                        frac=round(achieved / PEAK_BF16_TFLOPS, 4))
    else:                            # a step whose longest-running kernel moves bytes and multiplies nothing
        gbs = dom["bytes"] / dom["launches"] / (avg_ms * 1e-3) / 1e9
        roofline = dict(bound="hbm", achieved=round(gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(gbs / PEAK_HBM_GBS, 4))
    roofline.update(traffic=profile_field("dominant_kernel_hbm_traffic.txt", args.workload, dom["kernel"],
                                          "traffic_bytes_per_launch"),
                    mfma_busy=profile_field("layer_config5_counters.txt", args.workload, dom["kernel"], "mfma_busy"),
                    kernel=dom["kernel"], launches_per_step=dom["launches"] // args.steps,
                    avg_launch_us=round(avg_ms * 1e3, 2), mfma_only_measured_tflops=mfma_only)
    # the kernel above is the one with the most time per step (all its launches together); the
    # single longest launch of the step is reported beside it when it is another kernel
    longest = max(kinds, key=lambda r: r["total_ms"] / r["launches"])
    if longest is not dom and longest["flops"] > 0:
        l_ms = longest["total_ms"] / longest["launches"]
        l_tf = longest["flops"] / longest["launches"] / (l_ms * 1e-3) / 1e12
        roofline["longest_launch"] = dict(kernel=longest["kernel"], launches_per_step=longest["launches"] // args.steps,
                                          avg_launch_us=round(l_ms * 1e3, 2), achieved=round(l_tf, 1),
                                          frac=round(l_tf / PEAK_BF16_TFLOPS, 4))
    all_ms = sum(r["total_ms"] for r in kinds)
    gemm = [r for r in kinds if r["kernel"].startswith("gemm_bf16_kernel")]
    breakdown = {r["kernel"]: dict(us_per_step=round(r["total_ms"] * 1e3 / args.steps, 1),
                                   launches_per_step=r["launches"] // args.steps,
                                   tflops=round(r["flops"] / (r["total_ms"] * 1e-3) / 1e12, 1) if r["flops"] else None,
                                   gbs=round(r["bytes"] / (r["total_ms"] * 1e-3) / 1e9, 1) if r["bytes"] else None)
                 for r in kinds}
    gemm_tflops = sum(r["flops"] for r in gemm) / (sum(r["total_ms"] for r in gemm) * 1e-3) / 1e12 if gemm else None

    # ---------------------------------------------------------------- oracle on the host cores
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(args.workload, cfg)

    out = {
        "metric": METRIC, "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic", "launch": "hipGraph replay" if args.graph else "eager",
        "config": {"workload": name, "flop_per_step": step_flops,
                   "flop_counting": "2 x iteration-space size per einsum, causal pairs only"},
        "frac_of_bf16_mfma_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "fwd_bwd": halves,
        "kernels": breakdown,
        "all_gemm_launches_tflops": round(gemm_tflops, 1) if gemm_tflops else None,
        "kernel_time_ms_per_step": round(all_ms / args.steps, 4),
    }
    print(json.dumps(out))
    return 0


COPY_ELEMS = 1 << 28            # fp32 elements: 1 GiB read + 1 GiB written per launch


def copy_calibration(args, torch, mtf, dev):
    """Launches of the plain copy kernel on a buffer of known size (profiler calibration)."""
    x = torch.ones(COPY_ELEMS, dtype=torch.float32, device=dev)
    for _ in range(args.warmup):
        mtf.cast(x, torch.float32)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        y = mtf.cast(x, torch.float32)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    ok = bool((y[:: 1 << 16] == 1).all().item())
    print(json.dumps({"metric": "copy kernel (profiler calibration, not the hot path)", "kernel": "cast_kernel",
                      "bytes_read_per_launch": COPY_ELEMS * 4, "bytes_written_per_launch": COPY_ELEMS * 4,
                      "value": round(2 * COPY_ELEMS * 4 / dt / 1e9, 1), "unit": "GB/s", "steps": args.steps,
                      "warmup": args.warmup, "copied_correctly": ok}))
    return 0 if ok else 1


def reshape_bench(args, torch, mtf, mtf_inputs, dev):
    """Reshape on a virtual mesh of 8 processors: activations [16384 tokens, 4096 units] switch from
    data-parallel (tokens split) to model-parallel (units split): the alltoall case.  A step =
    the output slices of all 8 processors.  HBM-bound copy: GB/s against 8 TB/s."""
    mesh, layout = [("all", 8)], [("batch", "all"), ("hidden", "all")]
    in_shape, out_shape = [("batch", 16384), ("units", 4096)], [("examples", 16384), ("hidden", 4096)]
    full = mtf_inputs.normal(7, 0, (16384, 4096)).to(dev)
    slices = [mtf.slice_copy(full, ("batch", "units"), mesh, layout, (c,)) for c in range(8)]
    plan = mtf.reshape_plan(in_shape, out_shape, mesh, layout)

    outs = [torch.empty((16384, 512), dtype=full.dtype, device=dev) for _ in range(8)]

    def step():
        return [mtf.reshape_virtual(slices, in_shape, out_shape, mesh, layout, (c,), out=outs[c]) for c in range(8)]

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    gc.collect()
    gc.disable()                     # a full collection in this process pauses the host for ~40 ms
    t0 = time.perf_counter()
    for _ in range(args.steps):
        outs = step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    gc.enable()
    ok = all(torch.equal(outs[c], full[:, c * 512:(c + 1) * 512]) for c in range(8))
    nbytes = 2 * full.numel() * 2
    mtf.timing_enable(True)          # kernel time alone (the step above includes 8 host calls)
    for _ in range(args.steps):
        step()
    kern = [r for r in mtf.timing_collect() if r["kernel"] == "reshape_kernel"][0]
    mtf.timing_enable(False)
    kernel_gbs = kern["bytes"] / (kern["total_ms"] * 1e-3) / 1e9
    print(json.dumps({"metric": "reshape on a virtual mesh (alltoall case), HBM-bound copy", "plan": plan,
                      "value": round(nbytes / dt / 1e9, 1), "unit": "GB/s", "ms_per_step": round(dt * 1e3, 4),
                      "bytes_per_step": nbytes, "steps": args.steps, "warmup": args.warmup,
                      "roofline": {"bound": "hbm", "achieved": round(kernel_gbs, 1), "peak": 8000.0,
                                   "unit": "GB/s", "frac": round(kernel_gbs / 8000.0, 4), "kernel": "reshape_kernel",
                                   "avg_launch_us": round(kern["total_ms"] * 1e3 / kern["launches"], 2)},
                      "bit_exact": ok}))
    return 0 if ok else 1


def layer_norm_bench(args, torch, mtf, mtf_inputs, dev):
    """Layer normalisation at the layer shard's activation size (config 5: 8 x 512 tokens, d_model
    1024): a step = the pass that adds two fp32 partial sums to the residual and normalises the
    stored sum, and the backward pass.  HBM-bound: algorithmic bytes per step against 8 TB/s."""
    b, l, d = 8, 512, 1024
    x = mtf_inputs.normal(9, 0, (b, l, d)).to(dev)
    dy = mtf_inputs.normal(9, 1, (b, l, d)).to(dev)
    gain = (mtf_inputs.normal(9, 2, (d,), 0.25, torch.float32) + 1.0).to(torch.bfloat16).to(dev)
    bias = mtf_inputs.normal(9, 3, (d,), 0.5).to(dev)
    parts = [mtf_inputs.normal(9, 4 + i, (b, l, d), 0.7, torch.float32).to(dev) for i in range(2)]

    def step():
        u, y, mean, rstd = mtf.residual_layer_norm_fwd(parts, x, gain, bias, 1e-6)
        return mtf.layer_norm_bwd(u, gain, mean, rstd, dy)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    gc.collect()
    gc.disable()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    gc.enable()
    mtf.timing_enable(True)
    for _ in range(args.steps):
        step()
    kinds = {r["kernel"]: r for r in mtf.timing_collect()}
    mtf.timing_enable(False)
    nbytes = sum(r["bytes"] for r in kinds.values()) / args.steps
    dom = kinds["layer_norm_fwd_kernel"]
    gbs = dom["bytes"] / (dom["total_ms"] * 1e-3) / 1e9
    print(json.dumps({"metric": "layer normalisation after the residual sum, forward + backward, HBM-bound",
                      "value": round(nbytes / dt / 1e9, 1), "unit": "GB/s", "ms_per_step": round(dt * 1e3, 4),
                      "bytes_per_step": nbytes, "steps": args.steps, "warmup": args.warmup, "dtype": "bf16",
                      "config": {"workload": f"residual[{b},{l},{d}] + 2 fp32 partial sums -> layer norm; backward"},
                      "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                   "frac": round(gbs / PEAK_HBM_GBS, 4), "kernel": "layer_norm_fwd_kernel",
                                   "avg_launch_us": round(dom["total_ms"] * 1e3 / dom["launches"], 2)},
                      "kernels": {k: dict(us_per_step=round(r["total_ms"] * 1e3 / args.steps, 1),
                                          gbs=round(r["bytes"] / (r["total_ms"] * 1e-3) / 1e9, 1))
                                  for k, r in kinds.items()}}))
    return 0


def ceiling_probe(args, torch, mtf, mtf_inputs, dev):
    """What the matrix cores alone sustain (no memory traffic at all), by operand content: the
    power a matrix instruction draws, hence the clock the chip holds, depends on the operand bits.
    Not a benchmark of the path: the evidence behind roofline.mfma_only_measured_tflops."""
    sink = torch.empty(66, dtype=torch.float32, device=dev)
    out = {}
    for label, ops in (("normal", mtf_inputs.normal(0, 99, (4096,)).to(torch.bfloat16)),
                       ("ones", torch.ones(4096, dtype=torch.bfloat16)),
                       ("zeros", torch.zeros(4096, dtype=torch.bfloat16))):
        ops = ops.to(dev)
        for _ in range(max(args.warmup, 1)):
            mtf.mfma_ceiling(ops, 2000, sink)
        torch.cuda.synchronize()
        mtf.timing_enable(True)
        mhz = []
        for _ in range(args.steps):
            mtf.mfma_ceiling(ops, 2000, sink)
            cyc, ticks = sink[64:66].tolist()               # synchronises: one launch at a time
            mhz.append(100.0 * cyc / ticks)
        r = [k for k in mtf.timing_collect() if k["kernel"] == "mfma_ceiling_kernel"][0]
        mtf.timing_enable(False)
        out[label] = dict(tflops=round(r["flops"] / (r["total_ms"] * 1e-3) / 1e12, 1),
                          avg_launch_us=round(r["total_ms"] * 1e3 / r["launches"], 1),
                          shader_mhz_mean=round(sum(mhz) / len(mhz), 0), shader_mhz_min=round(min(mhz), 0))
    print(json.dumps({"workload": "MFMA-only kernel (v_mfma_f32_32x32x16_bf16, 8 waves per CU, no memory traffic)",
                      "peak_tflops_published": PEAK_BF16_TFLOPS, "operands": out}))
    return 0


def profile_field(filename, workload, kernel, key):
    """A figure of `kernel` from a committed rocprofv3 --pmc summary under profiles/ (HBM bytes per
    launch: FETCH_SIZE and WRITE_SIZE runs scaled by the same counters on the copy kernel; fraction
    of time the matrix pipe is busy: the profiler's MfmaUtil), or None if that summary is for
    another kernel or workload."""
    path = os.path.join(ROOT, "profiles", filename)
    try:
        fields = {}
        for line in open(path):
            if "=" in line and not line.lstrip().startswith("#"):
                k, v = line.split("=", 1)
                fields.setdefault(k.strip(), v.strip())
        if fields.get("workload") != workload or fields.get("kernel") != kernel:
            return None
        return float(fields[key])
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline_vocab(cfg, nb):
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import vocab as OV
    from oracle.einsum import NT
    f64 = lambda t: t.double().numpy()
    off, vl = cfg["vocab_offset"], cfg["w_vocab"].shape[1]
    x = NT(f64(cfg["x"][:nb]), (OV.B, OV.L, OV.D))
    w = NT(f64(cfg["w_vocab"]), (OV.D, OV.VOCAB))
    # the oracle works on a whole vocabulary: the stripe stands for it (ids folded into the stripe)
    tg = (cfg["targets"][:nb].numpy() - off) % vl
    ids = (cfg["ids"][:nb].numpy() - off) % vl
    t0 = time.perf_counter()
    OV.embedding_fwd(ids, NT(f64(cfg["table"]), (OV.VOCAB, OV.D)))
    f = OV.xent_fwd(x, w, tg)
    OV.xent_bwd(x, w, tg, f["logits"], f["m"], f["s"], NT(f64(cfg["dloss"][:nb]), (OV.B, OV.L)))
    OV.embedding_bwd(ids, NT(f64(cfg["de"][:nb]), (OV.B, OV.L, OV.D)), vl)
    dt = time.perf_counter() - t0
    flops = 3 * 2.0 * nb * cfg["x"].shape[1] * cfg["x"].shape[2] * vl
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": round(flops / dt / 1e12, 4), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"first {nb} of {cfg['x'].shape[0]} batch elements, forward + backward, fp64 "
                      f"(numpy; {dt:.1f} s)"}


def cpu_baseline(workload, cfg):
    """The oracle as it stands, timed on a bounded sample of the same workload."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_info
    from oracle import layer as OL
    from oracle.einsum import NT
    from oracle.layer import B, L, D, F, H, K, V

    f64 = lambda t: t.double().numpy()
    nb = {"layer": 4, "mesh": 64, "mesh3d": 16}.get(workload, 2)   # batch elements in the sample (~5-10 s of host work)
    if workload == "vocab":
        return cpu_baseline_vocab(cfg, nb)
    if workload == "mesh":                           # the unsplit forward on the first batch elements
        w_in, w_out = NT(f64(cfg["w_in"]), (D, F)), NT(f64(cfg["w_out"]), (F, D))
        xm = NT(f64(cfg["x"][:nb]), (B, L, D))
        t0 = time.perf_counter()
        OL.ffn_fwd(xm, w_in, w_out)
        dt = time.perf_counter() - t0
        flops = flops_ffn(nb * cfg["x"].shape[1], cfg["x"].shape[2], cfg["w_in"].shape[1])
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        return {"value": round(flops / dt / 1e12, 4), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
                "sample": f"first {nb} of {cfg['x'].shape[0]} batch elements, unsplit forward, fp64 (numpy; {dt:.1f} s)"}
    if workload == "attention_lm":
        from oracle import layer as OLA
        from oracle.einsum import NT as NTA
        qn, kn, vn, dn = (NTA(f64(cfg[n][:nb]), dims) for n, dims in
                          (("q", (OLA.B, OLA.L, OLA.H, OLA.K)), ("k", (OLA.B, OLA.M, OLA.H, OLA.K)),
                           ("v", (OLA.B, OLA.M, OLA.H, OLA.V)), ("dctx", (OLA.B, OLA.L, OLA.H, OLA.V))))
        t0 = time.perf_counter()
        ctx, lse = OLA.attention_core_fwd(qn, kn, vn, cfg["scale"], True)
        OLA.attention_core_bwd(qn, kn, vn, ctx, lse, dn, cfg["scale"], True)
        dt = time.perf_counter() - t0
        _, Lq, Hq, Kq = cfg["q"].shape
        flops = 3 * 2 * 2.0 * nb * Hq * (Lq * (Lq + 1) / 2) * Kq
        from threadpoolctl import threadpool_info as tpi
        threads = max([p.get("num_threads", 1) for p in tpi()] + [1])
        return {"value": round(flops / dt / 1e12, 4), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
                "sample": f"first {nb} of {cfg['q'].shape[0]} batch elements, forward + backward, fp64 "
                          f"(numpy; {dt:.1f} s)"}
    x = NT(f64(cfg["x"][:nb]), (B, L, D))
    t0 = time.perf_counter()
    if workload in ("ffn", "ffn_bias", "mesh3d"):      # mesh3d: the unsplit layer the mesh computes
        w_in, w_out = NT(f64(cfg["w_in"]), (D, F)), NT(f64(cfg["w_out"]), (F, D))
        dy = NT(f64(cfg["dy"][:nb]), (B, L, D))
        if workload != "ffn_bias":
            f = OL.ffn_fwd(x, w_in, w_out)
            OL.ffn_bwd(x, f["a"], w_in, w_out, dy)
        else:
            f = OL.ffn_bias_fwd(x, w_in, NT(f64(cfg["bias"]), (F,)), w_out)
            OL.ffn_bias_bwd(x, f["a"], w_in, w_out, dy)
        T = nb * cfg["x"].shape[1]
        flops = 3 * flops_ffn(T, cfg["x"].shape[2], cfg["w_in"].shape[1])
    else:
        names = dict(w_q=(D, H, K), w_k=(D, H, K), w_v=(D, H, V), w_o=(H, V, D), w_in=(D, F), w_out=(F, D))
        w = {k: NT(f64(cfg[k]), names[k]) for k in names if k in cfg}
        causal = bool(cfg.get("causal", False))
        Bq, Lq, Dq = nb, cfg["x"].shape[1], cfg["x"].shape[2]
        Hq, Kq = cfg["w_q"].shape[1], cfg["w_q"].shape[2]
        if workload == "layer":
            dz = NT(f64(cfg["dz"][:nb]), (B, L, D))
            f = OL.layer_fwd(x, w, cfg["scale"], causal)
            OL.layer_bwd(x, w, f["saved"], dz, cfg["scale"], causal)
            flops = 3 * (flops_mha(Bq, Lq, Dq, Hq, Kq, causal) + flops_ffn(Bq * Lq, Dq, cfg["w_in"].shape[1]))
        else:
            dy = NT(f64(cfg["dy"][:nb]), (B, L, D))
            f = OL.mha_fwd(x, w["w_q"], w["w_k"], w["w_v"], w["w_o"], cfg["scale"], causal)
            OL.mha_bwd(x, w["w_q"], w["w_k"], w["w_v"], w["w_o"], f["q"], f["k"], f["v"], f["ctx"], f["lse"],
                       dy, cfg["scale"], causal)
            flops = 3 * flops_mha(Bq, Lq, Dq, Hq, Kq, causal)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": round(flops / dt / 1e12, 4), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"first {nb} of {cfg['x'].shape[0]} batch elements, forward + backward, fp64 "
                      f"(numpy; {dt:.1f} s)"}


if __name__ == "__main__":
    sys.exit(main())
