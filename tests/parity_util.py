"""Error measures shared by the GPU parity tests.

A tensor passes when three bounds hold at once (tol = 1e-5 for the fp32
configuration, 1e-2 for bf16 operands with fp32 accumulation):

  * relative L2 error of the whole tensor <= tol (the stated bar);
  * relative L2 error of every row (last axis) <= ROW_FACTOR * tol, rows whose
    norm is below the typical row norm are measured against the typical one.
    A single wrong 128-element unit in a 5632-wide row is an error of about
    0.2 of the row, twenty times the bound, while it moves the whole-tensor
    figure of a 10^8-element gradient by 10^-4;
  * largest absolute error of every row <= MAX_FACTOR * tol * rms of that row
    of the reference (again with the typical row as the floor): one wrong
    element (error of the order of the rms) fails it.  Rounding a value of 5.5
    rms to bf16 is an error of 1.1e-2 rms and the observed accumulation errors
    are about 4e-3 rms, six sigma of which is 2.4e-2 rms; the bound of 0.1 rms
    leaves a factor of three.
"""
import numpy as np

ROW_FACTOR = 2.0
MAX_FACTOR = 10.0


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_l2(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / (den if den > 0 else 1.0))


def errors(got, ref):
    """(whole-tensor rel-L2, worst row rel-L2, worst |error| / row rms) of got against ref."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape)
    if ref.ndim == 0:
        ref, got = ref.reshape(1, 1), got.reshape(1, 1)
    r2 = ref.reshape(-1, ref.shape[-1])
    diff = got.reshape(r2.shape) - r2
    den = np.linalg.norm(r2)
    total = float(np.linalg.norm(diff) / (den if den > 0 else 1.0))
    row_norm = np.linalg.norm(r2, axis=1)
    typical = float(np.sqrt(np.mean(row_norm ** 2)))
    floor = typical if typical > 0 else 1.0
    row = float(np.max(np.linalg.norm(diff, axis=1) / np.maximum(row_norm, floor)))
    # largest absolute error of a row against that row's rms (rows below the typical size are
    # measured against the typical one)
    row_rms = np.maximum(row_norm, floor) / np.sqrt(r2.shape[1])
    worst = float(np.max(np.max(np.abs(diff), axis=1) / row_rms))
    return total, row, worst


def check(label, got, ref, tol):
    """Assert the three bounds; returns the whole-tensor rel-L2 error."""
    total, row, worst = errors(got, ref)
    print(f"[parity] {label}: rel-L2 {total:.2e}  worst row {row:.2e}  max|err|/rms {worst:.2e}", flush=True)
    assert np.isfinite(total) and total <= tol, (label, "rel-L2", total, tol)
    assert row <= ROW_FACTOR * tol, (label, "worst row rel-L2", row, ROW_FACTOR * tol)
    assert worst <= MAX_FACTOR * tol, (label, "max |error| / rms", worst, MAX_FACTOR * tol)
    return total
