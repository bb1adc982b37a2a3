"""Shared parity bars of the GPU tests (values against the fp64 oracle).

Two bars per tensor, both written here:
  * whole tensor: relative Frobenius error <= TOL = 1e-2 (the bar the benchmark definition states
    for bf16 inputs with fp32 accumulation);
  * per row: for every row r of the tensor viewed as [rows, last axis] -- a token of Y / dX, a
    (token, block) pair of Hsave, a hidden unit of dW1 / dW2, a query of an attention tensor --
    ||got_r - ref_r|| <= ROW_TOL * max(||ref_r||, ROW_FLOOR * rms_r ||ref_r||), ROW_TOL = 3e-2.
    The whole-tensor norm cannot see a localised fault: one token that misses one of its k block
    outputs moves its own row by about 1/sqrt(k) (18 % for k = 32) but the tensor's norm by far
    less than 1e-2; the row bar catches it.  bf16 rounding moves a row by 2e-3 ... 5e-3, so the
    bar leaves room for rounding only.  Rows whose reference norm is far below the typical row
    (a hidden unit that is almost never active, a gradient component in which large terms
    cancel) are measured against a floor of a quarter of the root-mean-square row norm, since
    their absolute error is set by the magnitudes that cancel in them.
The largest absolute error is printed with every check."""
import numpy as np

TOL = 1e-2
ROW_TOL = 3e-2
ROW_FLOOR = 0.25


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    n = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / n) if n > 0 else float(np.linalg.norm(got))


def row_errors(got, ref):
    """Per-row error relative to max(row norm, floor); rows = all axes but the last."""
    got = np.asarray(got, dtype=np.float64).reshape(-1, np.shape(ref)[-1])
    ref = np.asarray(ref, dtype=np.float64).reshape(got.shape)
    rn = np.linalg.norm(ref, axis=1)
    floor = ROW_FLOOR * float(np.sqrt(np.mean(rn * rn))) if rn.size else 0.0
    den = np.maximum(rn, floor)
    den[den == 0] = 1.0
    return np.linalg.norm(got - ref, axis=1) / den


def check(tag, name, got, ref, tol=TOL, row_tol=ROW_TOL):
    """Assert both bars; returns (relative Frobenius error, worst row error, max-abs error)."""
    got = np.asarray(got, dtype=np.float64).reshape(np.shape(ref))
    ref = np.asarray(ref, dtype=np.float64)
    fro = rel_err(got, ref)
    rows = row_errors(got, ref)
    worst = float(rows.max()) if rows.size else 0.0
    max_abs = float(np.max(np.abs(got - ref))) if ref.size else 0.0
    print(f"[parity] {tag}: {name}: rel Frobenius {fro:.3e}, worst row {worst:.3e} "
          f"(row {int(rows.argmax()) if rows.size else -1} of {rows.size}), max abs {max_abs:.3e}")
    assert fro <= tol, f"{tag}: {name}: relative Frobenius error {fro} > {tol}"
    assert worst <= row_tol, (f"{tag}: {name}: row {int(rows.argmax())} is off by {worst} of its norm "
                              f"(bar {row_tol}): a localised fault the tensor norm hides")
    return fro, worst, max_abs
