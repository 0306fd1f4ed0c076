"""Shared helpers for the parity tests (error metrics, tensor conversion)."""
import numpy as np
import torch


def rel_l2(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((x - ref).ravel())
    return num / den if den > 0 else num


def max_abs(x, ref):
    return float(np.max(np.abs(np.asarray(x, dtype=np.float64) - np.asarray(ref, dtype=np.float64)))) if np.size(ref) else 0.0


def to_np64(t):
    """torch tensor (any float dtype, any device) -> float64 numpy, exactly."""
    return None if t is None else t.detach().to("cpu").to(torch.float64).numpy()


# parity bars: fp32 inputs rel-L2 <= 1e-4; bf16 inputs (fp32 accumulation) rel-L2 <= 5e-3, max-abs <= 2e-2.
# The max-abs bar is stated for tensors of order one (every benchmark workload); for a tensor whose
# largest reference entry exceeds 1 it is applied relative to that entry (bf16 carries 8 bits).
TOL = {"f32": dict(rel=1e-4, abs=None), "bf16": dict(rel=5e-3, abs=2e-2)}


def check(name, got, ref, dtype, report=None, abs_floor=None):
    """abs_floor: a tensor whose reference is a cancellation residue far below the magnitude of the
    intermediates it is computed from (e.g. dq when every slot holds the same row) cannot be judged
    by relative error; it passes if its max-abs error is below this floor."""
    r, a = rel_l2(got, ref), max_abs(got, ref)
    if report is not None:
        report.append((name, r, a))
    tol = TOL[dtype]
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), "%s has non-finite values" % name
    if abs_floor is not None and a <= abs_floor:
        return r, a
    assert r <= tol["rel"], "%s: rel-L2 %.3e > %.1e (max-abs %.3e)" % (name, r, tol["rel"], a)
    if tol["abs"] is not None:
        bar = tol["abs"] * max(1.0, float(np.max(np.abs(ref))) if np.size(ref) else 1.0)
        assert a <= bar, "%s: max-abs %.3e > %.1e (rel-L2 %.3e)" % (name, a, bar, r)
    return r, a
