"""Oracle: one matrix's Muon step in fp64.

Test infrastructure only (see the package docstring).

The paper treats the optimizer as a black box, Delta W = Muon_step(G, States)
(Sec. 4.1 stage (2)), naming only its ingredients: momentum and Newton-Schulz
orthogonalisation (App. B.3) under the generic update W <- W - eta * MatrixOp
(App. B.3, Eq. 5).  The arithmetic below is the benchmark's statement of that
operator, in this order, per matrix:

1. TP case: G = concatenation of its column fragments (column-parallel split,
   App. B.2; only gradients are gathered, Sec. 4.1 stage (1));
2. M <- beta * M + G;  U = M, or U = G + beta * M with Nesterov momentum;
3. X = U / (||U||_F + eps); when rows > cols the iteration runs on X^T;
4. ns_steps times:  A = X X^T;  B = b A + c A A;  X <- a X + B X;
5. O = X (transposed back), scale from scale_mode, and either
   P <- P (1 - lr wd) - lr scale O  (owner updates in place, Sec. 3.3 (2)) or
   Delta W = - lr scale O cut into column fragments (Sec. 4.1 stage (3); the
   receiver applies P_local += Delta W_local, stage (4)).

Inputs are the exact bf16 / fp32 values the device sees, widened to fp64; all
arithmetic is fp64; numpy's matmul is the only library step.  Scalars
(beta, lr, ...) must be passed as the fp32-representable values the C ABI
carries, widened to Python floats, so both sides use the same numbers.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

SCALE_NONE = 0          # scale = 1
SCALE_ASPECT = 1        # sqrt(max(1, rows / cols))
SCALE_RMS = 2           # 0.2 * sqrt(max(rows, cols))


@dataclass
class Hparams:
    beta: float = float(np.float32(0.95))
    lr: float = float(np.float32(0.02))
    weight_decay: float = 0.0
    eps: float = float(np.float32(1e-7))
    nesterov: bool = False
    ns_steps: int = 5
    a: float = float(np.float32(3.4445))
    b: float = float(np.float32(-4.7750))
    c: float = float(np.float32(2.0315))
    scale_mode: int = SCALE_RMS


def bf16_bits_to_f64(bits) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp64 exactly."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def gather_columns(fragments) -> np.ndarray:
    """Whole matrix from its TP column fragments (step 1)."""
    return np.concatenate([np.asarray(f, dtype=np.float64) for f in fragments], axis=1)


def scatter_columns(whole: np.ndarray, tp: int):
    """Column fragments of a whole matrix (the inverse of gather_columns)."""
    rows, cols = whole.shape
    if cols % tp:
        raise ValueError("cols must be divisible by tp")
    w = cols // tp
    return [whole[:, f * w:(f + 1) * w].copy() for f in range(tp)]


def newton_schulz(x0: np.ndarray, steps: int, a: float, b: float, c: float) -> np.ndarray:
    """ns_steps iterations of X <- a X + (b A + c A A) X with A = X X^T (step 4).

    x0 is used as given (the caller normalises).  For a tall matrix the
    iteration runs on the transpose and the result is transposed back.
    """
    tall = x0.shape[0] > x0.shape[1]
    x = np.array(x0.T if tall else x0, dtype=np.float64, copy=True)
    for _ in range(steps):
        gram = x @ x.T
        poly = b * gram + c * (gram @ gram)
        x = a * x + poly @ x
    return x.T.copy() if tall else x


def update_scale(rows: int, cols: int, scale_mode: int) -> float:
    if scale_mode == SCALE_NONE:
        return 1.0
    if scale_mode == SCALE_ASPECT:
        return math.sqrt(max(1.0, rows / cols))
    if scale_mode == SCALE_RMS:
        return 0.2 * math.sqrt(float(max(rows, cols)))
    raise ValueError("unknown scale_mode")


def muon_step(grad, mom, hp: Hparams, param=None):
    """One Muon step for one matrix.

    grad   rows x cols array, or a list of tp column fragments (TP case)
    mom    rows x cols momentum buffer before the step
    param  rows x cols parameter (optional)

    Returns a dict with
      'mom'    momentum after the step,
      'ortho'  O, the Newton-Schulz output in the rows x cols orientation,
      'delta'  -lr * scale * O,
      'param'  param * (1 - lr * wd) + delta (only if param was given).
    """
    g = gather_columns(grad) if isinstance(grad, (list, tuple)) else np.asarray(grad, dtype=np.float64)
    m_new = hp.beta * np.asarray(mom, dtype=np.float64) + g
    u = g + hp.beta * m_new if hp.nesterov else m_new
    norm = math.sqrt(float(np.sum(u * u)))
    x0 = u / (norm + hp.eps)
    ortho = newton_schulz(x0, hp.ns_steps, hp.a, hp.b, hp.c)
    rows, cols = g.shape
    delta = (-hp.lr * update_scale(rows, cols, hp.scale_mode)) * ortho
    out = {"mom": m_new, "ortho": ortho, "delta": delta}
    if param is not None:
        out["param"] = np.asarray(param, dtype=np.float64) * (1.0 - hp.lr * hp.weight_decay) + delta
    return out
