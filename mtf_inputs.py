"""Seeded synthetic inputs shared by the CPU oracle's tests and the device path's tests and
benchmark.  This module holds no arithmetic of the method: it only draws random tensors
of the shapes of the paper's Transformer shards and fixes their storage dtype.

Shapes: d_model = 1024 and the (d_ff, heads) ladder with d_k = d_v = 128 come from the
machine-translation table of the experiments section; 16 x 256 tokens per processor row
from the language-model batch (256 sequences of 256 tokens split 16 ways); model dims
split 16- or 32-way as in the experiments.  Weights are N(0, 1/fan_in) with the GLOBAL
contracted size as fan_in (a processor holds a slice of a globally initialised weight).

Every tensor is drawn in fp32 from numpy's Philox keyed by (BASE_SEED, config, tensor
index), then converted once to its storage dtype by torch (bf16: round-to-nearest-even).
Both sides of every parity test receive these same bytes.
"""
import math
import numpy as np
import torch

BASE_SEED = 0x181102084

DIMS = dict(B="batch", L="length", M="memory_length", D="d_model", F="d_ff",
            H="heads", K="d_k", V="d_v")


def normal(cfg, index, shape, std=1.0, dtype=torch.bfloat16):
    """Tensor `index` of config `cfg`: N(0, std^2), fp32 draw, stored as `dtype`."""
    rng = np.random.Generator(np.random.Philox(key=[BASE_SEED, (cfg << 16) | index]))
    a = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return torch.from_numpy(a).to(dtype).contiguous()


def small_ints(cfg, index, shape, lo=-2, hi=2, dtype=torch.bfloat16):
    """Integers uniform in [lo, hi]: products and short sums are exact in every dtype."""
    rng = np.random.Generator(np.random.Philox(key=[BASE_SEED, (cfg << 16) | index]))
    a = rng.integers(lo, hi + 1, size=shape).astype(np.float32)
    return torch.from_numpy(a).to(dtype).contiguous()


def ffn_inputs(cfg, batch, length, d_model, d_ff_local, d_ff_total=None,
               dtype=torch.bfloat16):
    d_ff_total = d_ff_total or d_ff_local
    return dict(
        x=normal(cfg, 0, (batch, length, d_model), 1.0, dtype),
        w_in=normal(cfg, 1, (d_model, d_ff_local), 1.0 / math.sqrt(d_model), dtype),
        w_out=normal(cfg, 2, (d_ff_local, d_model), 1.0 / math.sqrt(d_ff_total), dtype),
        dy=normal(cfg, 3, (batch, length, d_model), 1.0, dtype),
    )


def mha_inputs(cfg, batch, length, d_model, heads_local, d_k, heads_total=None,
               dtype=torch.bfloat16):
    heads_total = heads_total or heads_local
    s_in = 1.0 / math.sqrt(d_model)
    return dict(
        x=normal(cfg, 0, (batch, length, d_model), 1.0, dtype),
        w_q=normal(cfg, 4, (d_model, heads_local, d_k), s_in, dtype),
        w_k=normal(cfg, 5, (d_model, heads_local, d_k), s_in, dtype),
        w_v=normal(cfg, 6, (d_model, heads_local, d_k), s_in, dtype),
        w_o=normal(cfg, 7, (heads_local, d_k, d_model), 1.0 / math.sqrt(heads_total * d_k), dtype),
        dy=normal(cfg, 3, (batch, length, d_model), 1.0, dtype),
        scale=1.0 / math.sqrt(d_k),
    )


def layer_inputs(cfg, batch, length, d_model, heads_local, d_k, d_ff_local,
                 heads_total=None, d_ff_total=None, dtype=torch.bfloat16):
    d = mha_inputs(cfg, batch, length, d_model, heads_local, d_k, heads_total, dtype)
    f = ffn_inputs(cfg, batch, length, d_model, d_ff_local, d_ff_total, dtype)
    d.update(w_in=f["w_in"], w_out=f["w_out"])
    d["dz"] = d.pop("dy")
    return d


# The five named workloads.
def config1():
    """Tiny fp32 FFN; mesh [("all",4)], layout [("d_ff","all")]."""
    d = ffn_inputs(1, 2, 8, 16, 64, dtype=torch.float32)
    d["w_in"] = normal(1, 1, (16, 64), 1.0, torch.float32)
    d["w_out"] = normal(1, 2, (64, 16), 1.0, torch.float32)
    d.update(mesh=[("all", 4)], layout=[("d_ff", "all")])
    return d


def config2():
    """One processor's FFN shard: d_ff = 65536 split 16 ways."""
    return ffn_inputs(2, 16, 256, 1024, 4096, 65536)


def config3():
    """One processor's attention shard: 8 of 128 heads, d_k = d_v = 128, no mask."""
    d = mha_inputs(3, 8, 256, 1024, 8, 128, 128)
    d["causal"] = False
    return d


def config4():
    """Unsplit FFN for the virtual 4x4 mesh (batch over rows, d_ff over cols)."""
    d = ffn_inputs(4, 64, 256, 1024, 16384, 16384)
    d.update(mesh=[("rows", 4), ("cols", 4)], layout=[("batch", "rows"), ("d_ff", "cols")])
    return d


def config5():
    """Full layer shard of the largest model: d_ff 262144 / 32, 512 heads-of-128 / 32."""
    d = layer_inputs(5, 8, 512, 1024, 16, 128, 8192, 512, 262144)
    d["causal"] = True
    return d


def token_ids(cfg, index, shape, vocab):
    """Integer token ids uniform in [0, vocab), int32."""
    rng = np.random.Generator(np.random.Philox(key=[BASE_SEED, (cfg << 16) | index]))
    return torch.from_numpy(rng.integers(0, vocab, size=shape).astype(np.int32)).contiguous()


def vocab_inputs(cfg, batch, length, d_model, vocab_local, vocab_total=None, dtype=torch.bfloat16):
    """Embedding table slice, output-layer weight slice, ids / targets (GLOBAL ids in
    [0, vocab_total)), activations and incoming gradients of the vocabulary-split operations."""
    vocab_total = vocab_total or vocab_local
    return dict(
        x=normal(cfg, 0, (batch, length, d_model), 1.0, dtype),
        table=normal(cfg, 10, (vocab_local, d_model), 1.0, dtype),
        w_vocab=normal(cfg, 11, (d_model, vocab_local), 1.0 / math.sqrt(d_model), dtype),
        ids=token_ids(cfg, 12, (batch, length), vocab_total),
        targets=token_ids(cfg, 13, (batch, length), vocab_total),
        de=normal(cfg, 14, (batch, length, d_model), 1.0, dtype),
        dloss=normal(cfg, 15, (batch, length), 1.0, torch.float32),
        vocab_total=vocab_total,
    )


def config6():
    """One processor's share of the vocabulary-split operations: 32768 tokens split 16 ways
    (this processor holds ids 2048 .. 4095), 16 x 256 tokens, d_model 1024."""
    d = vocab_inputs(6, 16, 256, 1024, 2048, 32768)
    d["vocab_offset"] = 2048
    return d


def config7():
    """The worked example's 3-D layout at shard size: batch -> rows, d_ff -> cols, d_model -> planes on
    a 2 x 2 x 2 mesh; every processor holds x[16, 256, 512], W_in[512, 4096], W_out[4096, 512] (the
    token and d_ff extents of config 2, d_model halved by the third mesh dim)."""
    d = ffn_inputs(7, 32, 256, 1024, 8192, 8192)
    d.update(mesh=[("rows", 2), ("cols", 2), ("planes", 2)],
             layout=[("batch", "rows"), ("d_ff", "cols"), ("d_model", "planes")])
    return d
