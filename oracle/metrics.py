"""Error measures used by the parity tests (test infrastructure only).

M1: forward-error measure of a contraction: |got - ref| relative to the same contraction
    of absolute values (the classical bound |fl(x.y) - x.y| <= gamma_K |x|.|y|).
M2: |got - ref| relative to max(|ref|, rms(ref)), element-wise maximum; this is the number
    compared with the stated tolerances (1e-5 fp32, 2e-2 bf16-in / fp32-accumulate).
"""
import numpy as np


def m1(got, ref, ref_abs):
    got, ref, ref_abs = (np.asarray(a, dtype=np.float64) for a in (got, ref, ref_abs))
    den = np.where(ref_abs > 0, ref_abs, 1.0)
    return float(np.max(np.abs(got - ref) / den)) if ref.size else 0.0


def m2(got, ref):
    got, ref = (np.asarray(a, dtype=np.float64) for a in (got, ref))
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), rms)
    den = np.where(den > 0, den, 1.0)
    return float(np.max(np.abs(got - ref) / den))
