"""Shared helpers of the parity tests: conversions between torch tensors (device path) and
the oracle's named fp64 tensors.  No arithmetic of the method lives here."""
import numpy as np
import torch

from oracle.einsum import NT
from oracle.layer import B, L, M, D, F, H, K, V

BF16_TOL = 2e-2      # max relative error, bf16 in / fp32 accumulate
F32_TOL = 1e-5       # max relative error, fp32

WEIGHT_DIMS = dict(w_q=(D, H, K), w_k=(D, H, K), w_v=(D, H, V), w_o=(H, V, D), w_in=(D, F), w_out=(F, D))
SAVED_DIMS = dict(q=(B, L, H, K), k=(B, M, H, K), v=(B, M, H, V), ctx=(B, L, H, V), lse=(B, H, L),
                  u=(B, L, D), a=(B, L, F))


def f64(t):
    return t.detach().double().cpu().numpy()


def named(t, dims):
    return NT(f64(t), tuple(dims))


def to_dev(nt_or_array, dtype, dev="cuda"):
    arr = nt_or_array.data if isinstance(nt_or_array, NT) else nt_or_array
    return torch.from_numpy(np.ascontiguousarray(arr)).to(dtype).to(dev)


def on_device(cfg, dev="cuda"):
    return {k: (v.to(dev) if torch.is_tensor(v) else v) for k, v in cfg.items()}
