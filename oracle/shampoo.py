"""Oracle: one matrix's Shampoo step in fp64.

Test infrastructure only (see the package docstring).

The paper runs Shampoo through the same planner as Muon ("Generalization to Other
Optimizers (Shampoo & SOAP)", App. C) and describes it only as preconditioning
with matrices built from the gradients under the generic update
W <- W - eta * MatrixOp(W, grad W) (App. B.3, Eq. 5), with a cubic-cost
decomposition as the MatrixOp.  The arithmetic is that of the algorithm the
paper cites for it (Gupta, Koren and Singer 2018), for one matrix:

1. TP case: G = concatenation of its column fragments (as in the Muon step);
2. statistics:  L <- beta L + G G^T  (rows x rows),  R <- beta R + G^T G  (cols x cols);
   beta = 1 is the running sum of the original algorithm;
3. inverse fourth roots of the regularised statistics, by their definition through
   the symmetric eigendecomposition:  (S + eps I)^(-1/4) = V diag((lambda_i + eps)^(-1/4)) V^T;
4. preconditioned gradient  O = (L + eps I)^(-1/4) G (R + eps I)^(-1/4);
5. P <- P (1 - lr wd) - lr O   or   Delta W = - lr O  cut into column fragments.
Practical variants recompute the roots of step 3 only every n-th step and use the last ones in between
(the statistics of step 2 are still updated): shampoo_step takes such kept roots as an input.

Inputs are the exact values the device sees, widened to fp64; numpy's matmul and
numpy.linalg.eigh are the library steps.  The device reaches step 3 through a matmul-only
iteration that converges to the same matrix; the oracle is the definition itself.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class Hparams:
    beta: float = 1.0
    lr: float = float(np.float32(0.02))
    weight_decay: float = 0.0
    eps: float = float(np.float32(1e-6))


def gather_columns(fragments) -> np.ndarray:
    """Whole matrix from its TP column fragments (step 1)."""
    return np.concatenate([np.asarray(f, dtype=np.float64) for f in fragments], axis=1)


def inverse_fourth_root(stat: np.ndarray, eps: float) -> np.ndarray:
    """(S + eps I)^(-1/4) of a symmetric positive semi-definite S (step 3)."""
    s = np.asarray(stat, dtype=np.float64)
    s = 0.5 * (s + s.T)                      # the exactly symmetric part of the input
    lam, vec = np.linalg.eigh(s)
    lam = np.maximum(lam, 0.0) + eps         # S is PSD by construction; rounding may leave -1e-20
    return (vec * lam ** -0.25) @ vec.T


def statistics(grad: np.ndarray, left: np.ndarray, right: np.ndarray, beta: float):
    """Step 2: the two Kronecker-factor statistics after seeing `grad`."""
    g = np.asarray(grad, dtype=np.float64)
    new_left = beta * np.asarray(left, dtype=np.float64) + g @ g.T
    new_right = beta * np.asarray(right, dtype=np.float64) + g.T @ g
    return new_left, new_right


def shampoo_step(grad, left, right, hp: Hparams, param=None, kept_roots=None):
    """One Shampoo step for one matrix.

    grad   rows x cols array, or a list of tp column fragments
    left   rows x rows statistic before the step;  right  cols x cols likewise
    param  rows x cols parameter (optional)
    kept_roots  (left root, right root) from an earlier step: the amortised variant, in which the
           statistics are updated on every step and the roots only on some; None: the roots of the
           new statistics, as published

    Returns a dict with 'left', 'right' (statistics after the step), 'left_root',
    'right_root' (the inverse fourth roots), 'precond' (O), 'delta' (-lr O) and, if
    param was given, 'param'.
    """
    g = gather_columns(grad) if isinstance(grad, (list, tuple)) else np.asarray(grad, dtype=np.float64)
    new_left, new_right = statistics(g, left, right, hp.beta)
    if kept_roots is None:
        left_root = inverse_fourth_root(new_left, hp.eps)
        right_root = inverse_fourth_root(new_right, hp.eps)
    else:
        left_root = np.asarray(kept_roots[0], dtype=np.float64)
        right_root = np.asarray(kept_roots[1], dtype=np.float64)
    precond = left_root @ g @ right_root
    delta = -hp.lr * precond
    out = {"left": new_left, "right": new_right, "left_root": left_root, "right_root": right_root,
           "precond": precond, "delta": delta}
    if param is not None:
        out["param"] = np.asarray(param, dtype=np.float64) * (1.0 - hp.lr * hp.weight_decay) + delta
    return out
