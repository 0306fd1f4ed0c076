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


def rms(x):
    x = np.asarray(x, dtype=np.float64)
    return float(np.sqrt(np.mean(x * x))) if x.size else 0.0


def to_np64(t):
    """torch tensor (any float dtype, any device) -> float64 numpy, exactly."""
    return None if t is None else t.detach().to("cpu").to(torch.float64).numpy()


# parity bars: fp32 inputs rel-L2 <= 1e-4; bf16 inputs (fp32 accumulation) rel-L2 <= 5e-3, max-abs <= 2e-2.
# The max-abs bar is stated for tensors of order one (every benchmark workload); for a tensor whose
# largest reference entry exceeds 1 it is applied relative to that entry (bf16 carries 8 bits).
TOL = {"f32": dict(rel=1e-4, abs=None), "bf16": dict(rel=5e-3, abs=2e-2)}


def suffix_mass(terms, axis=1):
    """The gate gradient is a suffix sum over the later tokens of a sequence (Algorithm 1's reversed
    cumulative sum): dg_j = sum_{t >= j} (per-token terms of either sign).  Rounding errors of the terms add
    up like a random walk, so the error of the sum is relative to sqrt(sum_{t >= j} terms_t^2), which this
    returns for ORACLE terms [.., tokens of one sequence along `axis`, ..]."""
    x = np.moveaxis(np.asarray(terms, dtype=np.float64), axis, 0)
    mass = np.sqrt(np.cumsum((x * x)[::-1], axis=0)[::-1])
    return np.moveaxis(mass, 0, axis)


def check(name, got, ref, dtype, report=None, residue_of=None, widen=1.0):
    """Holds `got` to the parity bar against the oracle's `ref`.  Returns (rel-L2, max-abs, branch) and
    appends (name, rel-L2, max-abs, branch) to `report`; branch says which criterion passed:

      "relative"  rel-L2 and max-abs inside the bars above (the ordinary case);
      "residue"   only with residue_of: `ref` is a cancellation residue of larger ORACLE quantities (the
                  caller passes them: an array, or a list of arrays, computed from the oracle's outputs
                  and the inputs, never from the device result), so its error cannot be small next to
                  `ref` itself.  The bars are then applied against the magnitude of those quantities:
                  rms(got - ref) <= rel * rms(residue_of), and max|got - ref| <= 4 * rel *
                  max|residue_of| (the bf16 bars' own ratio of max-abs to rel-L2) and still inside the
                  max-abs bar.
    Anything else fails, whatever its absolute size.
    widen (>= 1, an oracle-side number) multiplies the bars: the bars are stated for scores of order one;
    the softmax turns an absolute error of a score into a relative error of its weight, and the error of a
    score is relative to the score, so a test that drives the scores far beyond order one (a large
    `scale`) passes widen = max(1, mean spread of the oracle's scores over the slots of a token)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert np.all(np.isfinite(got)), "%s has non-finite values" % name
    r, a = rel_l2(got, ref), max_abs(got, ref)
    assert widen >= 1.0
    tol = dict(rel=TOL[dtype]["rel"] * widen, abs=None if TOL[dtype]["abs"] is None else TOL[dtype]["abs"] * widen)
    bar = None if tol["abs"] is None else tol["abs"] * max(1.0, float(np.max(np.abs(ref))) if ref.size else 1.0)
    branch = None
    if r <= tol["rel"] and (bar is None or a <= bar):
        branch = "relative"
    elif residue_of is not None:
        parts = residue_of if isinstance(residue_of, (list, tuple)) else [residue_of]
        scale_rms = max(rms(p) for p in parts)
        scale_max = max(float(np.max(np.abs(p))) if np.size(p) else 0.0 for p in parts)
        if rms(got - ref) <= tol["rel"] * scale_rms and a <= 4.0 * tol["rel"] * scale_max and (bar is None or a <= bar):
            branch = "residue"
    if report is not None:
        report.append((name, r, a, branch))
    assert branch is not None, "%s: rel-L2 %.3e (bar %.1e), max-abs %.3e (bar %s)%s" % (
        name, r, tol["rel"], a, "none" if bar is None else "%.1e" % bar,
        "" if residue_of is None else "; not inside the residue bar either")
    if branch != "relative":
        print("  %s passed on the %s bar: rel-L2 %.3e, max-abs %.3e" % (name, branch, r, a))
    return r, a, branch
