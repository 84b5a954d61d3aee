"""Oracle: one matrix's SOAP step in fp64.

Test infrastructure only (see the package docstring).

The paper runs SOAP through the same planner as Muon and Shampoo ("Generalization to
Other Optimizers (Shampoo & SOAP)", App. C) and describes it only as a matrix-based
optimizer whose cubic-cost operation is an eigendecomposition, under the generic update
W <- W - eta * MatrixOp(W, grad W) (App. B.3, Eq. 5).  The arithmetic is that of the
algorithm the paper cites for it (Vyas et al. 2024: Adam run in the eigenbasis of
Shampoo's statistics), for one matrix at step t = 1, 2, ...:

1. TP case: G = concatenation of its column fragments (as in the Muon step);
2. momentum in the original space:  M <- beta1 M + (1 - beta1) G;
3. rotation into the current eigenbasis:  G' = Q_L^T G Q_R,  M' = Q_L^T M Q_R;
4. second moment in the rotated space:  V <- beta2 V + (1 - beta2) G' * G'  (elementwise);
5. Adam's direction there:  N' = m / (sqrt(v) + eps)  with  m = M' / (1 - beta1^t),
   v = V / (1 - beta2^t)  when bias correction is on, else m = M', v = V;
6. rotation back and update:  N = Q_L N' Q_R^T;  P <- P (1 - lr wd) - lr N  or
   Delta W = - lr N  cut into column fragments;
7. statistics:  L <- beta2 L + (1 - beta2) G G^T,  R <- beta2 R + (1 - beta2) G^T G;
8. on a refresh step, one round of orthogonal (power) iteration per side from the new
   statistics:  Q_L <- Q factor of the QR decomposition of L Q_L, Q_R likewise from R Q_R.
   V is not rotated into the new basis.

A side whose extent exceeds max_precond_dim keeps no statistic and no basis (its Q is the
identity): the one-sided variant.  The columns of a basis are fixed only up to sign, and
nothing in steps 3-6 depends on those signs.

Inputs are the exact values the device sees, widened to fp64; numpy's matmul and
numpy.linalg.qr are the library steps.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class Hparams:
    beta1: float = float(np.float32(0.95))
    beta2: float = float(np.float32(0.95))
    lr: float = float(np.float32(3e-3))
    weight_decay: float = 0.0
    eps: float = float(np.float32(1e-8))
    bias_correction: bool = True
    max_precond_dim: int = 10000


def gather_columns(fragments) -> np.ndarray:
    """Whole matrix from its TP column fragments (step 1)."""
    return np.concatenate([np.asarray(f, dtype=np.float64) for f in fragments], axis=1)


def rotate_in(x: np.ndarray, q_left, q_right) -> np.ndarray:
    """Step 3: Q_L^T X Q_R; a side without a basis (None) is left alone."""
    y = np.asarray(x, dtype=np.float64)
    if q_left is not None:
        y = np.asarray(q_left, dtype=np.float64).T @ y
    if q_right is not None:
        y = y @ np.asarray(q_right, dtype=np.float64)
    return y


def rotate_out(x: np.ndarray, q_left, q_right) -> np.ndarray:
    """Step 6: Q_L X Q_R^T."""
    y = np.asarray(x, dtype=np.float64)
    if q_left is not None:
        y = np.asarray(q_left, dtype=np.float64) @ y
    if q_right is not None:
        y = y @ np.asarray(q_right, dtype=np.float64).T
    return y


def adam_direction(m_rot: np.ndarray, v_rot: np.ndarray, hp: Hparams, t: int) -> np.ndarray:
    """Step 5."""
    if hp.bias_correction:
        m_hat = m_rot / (1.0 - hp.beta1 ** t)
        v_hat = v_rot / (1.0 - hp.beta2 ** t)
    else:
        m_hat, v_hat = m_rot, v_rot
    return m_hat / (np.sqrt(v_hat) + hp.eps)


def refresh_basis(stat: np.ndarray, basis: np.ndarray) -> np.ndarray:
    """Step 8 for one side: the orthogonal factor of QR(S Q)."""
    s = np.asarray(stat, dtype=np.float64) @ np.asarray(basis, dtype=np.float64)
    q, _ = np.linalg.qr(s)
    return q


def soap_step(grad, state: dict, hp: Hparams, t: int, refresh: bool, param=None) -> dict:
    """One SOAP step for one matrix.

    grad    rows x cols array, or a list of tp column fragments
    state   dict with 'mom' (rows x cols), 'var' (rows x cols, rotated space), 'left'
            (rows x rows), 'right' (cols x cols), 'q_left', 'q_right' (orthogonal, columns are
            the basis vectors); the four entries of a side above max_precond_dim are ignored
    t       1-based step count (bias correction)
    refresh run step 8 at the end of this step

    Returns a dict with the new 'mom', 'var', 'left', 'right', 'q_left', 'q_right' (None for
    a side without a basis), 'grad_rot', 'mom_rot', 'direction' (N), 'delta' and, if param
    was given, 'param'.
    """
    g = gather_columns(grad) if isinstance(grad, (list, tuple)) else np.asarray(grad, dtype=np.float64)
    rows, cols = g.shape
    use_left, use_right = rows <= hp.max_precond_dim, cols <= hp.max_precond_dim
    q_left = np.asarray(state["q_left"], dtype=np.float64) if use_left else None
    q_right = np.asarray(state["q_right"], dtype=np.float64) if use_right else None

    mom = hp.beta1 * np.asarray(state["mom"], dtype=np.float64) + (1.0 - hp.beta1) * g
    grad_rot = rotate_in(g, q_left, q_right)
    mom_rot = rotate_in(mom, q_left, q_right)
    var = hp.beta2 * np.asarray(state["var"], dtype=np.float64) + (1.0 - hp.beta2) * grad_rot * grad_rot
    direction = rotate_out(adam_direction(mom_rot, var, hp, t), q_left, q_right)
    delta = -hp.lr * direction

    left = right = None
    if use_left:
        left = hp.beta2 * np.asarray(state["left"], dtype=np.float64) + (1.0 - hp.beta2) * (g @ g.T)
        if refresh:
            q_left = refresh_basis(left, q_left)
    if use_right:
        right = hp.beta2 * np.asarray(state["right"], dtype=np.float64) + (1.0 - hp.beta2) * (g.T @ g)
        if refresh:
            q_right = refresh_basis(right, q_right)

    out = {"mom": mom, "var": var, "left": left, "right": right, "q_left": q_left, "q_right": q_right,
           "grad_rot": grad_rot, "mom_rot": mom_rot, "direction": direction, "delta": delta}
    if param is not None:
        out["param"] = np.asarray(param, dtype=np.float64) * (1.0 - hp.lr * hp.weight_decay) + delta
    return out
