"""Index-time reduced-rank-regression fit in numpy float64.  TEST INFRASTRUCTURE ONLY.

A direct statement of the paper's estimators, used to pin the score model (full-rank identity, Theorem 1,
optimality of the reduced-rank solution) and to check the torch index builder on small clusters.
"""
from __future__ import annotations

import numpy as np


def projection_matrix(X_global: np.ndarray, s: int) -> np.ndarray:
    """Sec. 4.1: W_s [d x s] = the first s eigenvectors of X_global^T X_global (uncentered)."""
    X = np.asarray(X_global, np.float64)
    evals, evecs = np.linalg.eigh(X.T @ X)
    return evecs[:, np.argsort(evals)[::-1][:s]]


def rrr_fit(X: np.ndarray, C: np.ndarray, r: int, W: np.ndarray | None = None):
    """Sec. 3.2 / 4.1: reduced-rank regression of the true inner products Y = X C^T on the inputs.

    X [n_l x d] local training set, C [m_l x d] cluster points, W [d x s] projection or None.
    V_r = first r right singular vectors of Y; beta_OLS = (X W)^+ Y (= C^T when W is None and X has full
    column rank); A = beta_OLS V_r [s x r], B = V_r^T [r x m_l].
    """
    X, C = np.asarray(X, np.float64), np.asarray(C, np.float64)
    Y = X @ C.T
    _, _, Vt = np.linalg.svd(Y, full_matrices=False)
    Vr = Vt[:r].T
    Xin = X if W is None else X @ np.asarray(W, np.float64)
    beta_ols = np.linalg.pinv(Xin) @ Y
    return beta_ols @ Vr, Vr.T


def absmax_quantize(x: np.ndarray):
    """Sec. 3.3 absmax quantization with one multiplier for the whole array.

    Returns (codes int8, Delta) with codes = round(x * 127 / max|x|) and Delta = max|x| / 127, so that
    x ~= Delta * codes.
    """
    x = np.asarray(x, np.float64)
    a = np.abs(x).max() if x.size else 0.0
    if a == 0.0:
        return np.zeros(x.shape, np.int8), 0.0
    return np.clip(np.rint(x * (127.0 / a)), -127, 127).astype(np.int8), a / 127.0
