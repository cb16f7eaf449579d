"""Shared test helpers: the acceptance rule and small utilities (no GPU, no oracle arithmetic)."""
import numpy as np

ABS_TOL = 1e-2      # |Y - Yref| <= ABS_TOL + REL_TOL * |Yref| for every element ...
REL_TOL = 5e-3
FRO_TOL = 2e-3      # ... and ||Y - Yref||_F / ||Yref||_F <= FRO_TOL


def acceptance(Y, Yref):
    """Returns (ok, worst elementwise excess ratio, relative Frobenius error), all computed in fp64."""
    y = np.asarray(Y).astype(np.float64)
    r = np.asarray(Yref).astype(np.float64)
    if y.shape != r.shape:
        raise ValueError("shape mismatch")
    if y.size == 0:
        return True, 0.0, 0.0
    if not (np.isfinite(y).all() and np.isfinite(r).all()):
        same = np.array_equal(np.isnan(y), np.isnan(r)) and np.array_equal(y[~np.isfinite(y)], r[~np.isfinite(r)])
        if not same:
            return False, float("inf"), float("inf")
        fin = np.isfinite(r)
        y, r = y[fin], r[fin]
    err = np.abs(y - r)
    bound = ABS_TOL + REL_TOL * np.abs(r)
    worst = float((err / bound).max()) if err.size else 0.0
    den = float(np.linalg.norm(r))
    fro = float(np.linalg.norm(y - r)) / den if den > 0 else float(np.linalg.norm(y - r))
    return (worst <= 1.0 and fro <= FRO_TOL), worst, fro
