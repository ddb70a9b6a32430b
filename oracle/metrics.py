"""Error measures used by the parity tests (test infrastructure only).

M1: forward-error measure of a contraction: |got - ref| relative to the same contraction
    of absolute values (the classical bound |fl(x.y) - x.y| <= gamma_K |x|.|y|).
M2: |got - ref| relative to max(|ref|, rms(ref)), element-wise maximum; this is the number
    compared with the stated tolerances (1e-5 fp32, 2e-2 bf16-in / fp32-accumulate).
L2: ||got - ref||_2 / ||ref||_2 over all elements; used where a result legitimately contains a
    few isolated large deviations (an integer decision taken from floating point differing at a
    handful of positions), which an element-wise maximum cannot grade.
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


def rel_l2(got, ref):
    got, ref = (np.asarray(a, dtype=np.float64) for a in (got, ref))
    if ref.size == 0:
        return 0.0
    den = float(np.sqrt(np.sum(ref * ref)))
    return float(np.sqrt(np.sum((got - ref) ** 2))) / (den if den > 0 else 1.0)
