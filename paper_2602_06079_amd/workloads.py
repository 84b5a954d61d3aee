"""Seeded synthetic workloads: matrix sets and input values.

This module serves both the tests' CPU oracle and the device library with the
same bits.  It holds shapes, seeds and number-format conversion only - none of
the optimizer's or the planner's arithmetic - and depends on numpy alone.

The matrix sets stand in for the Qwen3 family the paper trains (Sec. 5,
App. C.1): per transformer layer the seven weight matrices q, k, v, o, gate,
up, down with the shapes the benchmark configurations list; one bucket per
layer, matrices in that order, layers in index order.  Gradient values are
i.i.d. normal with standard deviation 0.02 (1.0 for the tiny configuration),
rounded to bf16 with round-to-nearest-even where the configuration says bf16.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 20260206

DT_F32 = 0
DT_BF16 = 1

# per-layer matrices (name, rows, cols)
_LAYER_SHAPES = {
    "qwen3_0p6b": (28, [("q", 2048, 1024), ("k", 1024, 1024), ("v", 1024, 1024), ("o", 1024, 2048),
                        ("gate", 3072, 1024), ("up", 3072, 1024), ("down", 1024, 3072)]),
    "qwen3_8b": (36, [("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
                      ("gate", 12288, 4096), ("up", 12288, 4096), ("down", 4096, 12288)]),
    "qwen3_32b": (64, [("q", 8192, 5120), ("k", 1024, 5120), ("v", 1024, 5120), ("o", 5120, 8192),
                       ("gate", 25600, 5120), ("up", 25600, 5120), ("down", 5120, 25600)]),
}

# configuration number -> planner inputs.  "tp" is the number of column
# fragments each gradient arrives in (1 = whole).
CONFIGS = {
    1: dict(name="tiny", model=None, n_ranks=1, alpha=1.0, grad_dtype=DT_F32, grad_std=1.0, tp=1),
    2: dict(name="qwen3_0p6b_R8", model="qwen3_0p6b", n_ranks=8, alpha=1.0, grad_dtype=DT_BF16, grad_std=0.02, tp=1),
    3: dict(name="qwen3_8b_R32_a0p1", model="qwen3_8b", n_ranks=32, alpha=0.1, grad_dtype=DT_BF16, grad_std=0.02, tp=1),
    4: dict(name="qwen3_32b_R64", model="qwen3_32b", n_ranks=64, alpha=1.0, grad_dtype=DT_BF16, grad_std=0.02, tp=1),
    5: dict(name="qwen3_8b_tp4", model="qwen3_8b", n_ranks=1, alpha=1.0, grad_dtype=DT_BF16, grad_std=0.02, tp=4),
}


def matrix_set(cfg: int) -> dict:
    """Shapes, names and bucket layout of configuration ``cfg`` (1..5)."""
    c = CONFIGS[cfg]
    if c["model"] is None:
        names = ["w%d" % i for i in range(8)]
        rows = [256] * 8
        cols = [512] * 8
        bucket_off = [0, 8]
    else:
        layers, shapes = _LAYER_SHAPES[c["model"]]
        names, rows, cols, bucket_off = [], [], [], [0]
        for layer in range(layers):
            for nm, r, cc in shapes:
                names.append("layers.%d.%s" % (layer, nm))
                rows.append(r)
                cols.append(cc)
            bucket_off.append(len(rows))
    out = dict(c)
    out.update(cfg=cfg, names=names, rows=rows, cols=cols, bucket_off=bucket_off,
               dtype=[c["grad_dtype"]] * len(rows))
    return out


# ------------------------------------------------------------------ formats

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns uint16 bit patterns.
    Inputs are finite here, so NaN handling is not needed."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ------------------------------------------------------------------- values

def _rng(cfg: int, matrix_id: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([SEED_BASE, int(cfg), int(matrix_id), int(stream)])


def gen_normal_f32(cfg: int, matrix_id: int, stream: int, rows: int, cols: int, std: float) -> np.ndarray:
    x = _rng(cfg, matrix_id, stream).standard_normal((rows, cols), dtype=np.float32)
    x *= np.float32(std)
    return x


def gen_grad(cfg: int, matrix_id: int, rows: int, cols: int, step: int = 0, std=None, dtype=None):
    """Gradient of one matrix at optimizer step ``step``.

    Returns (values, dtype): a float32 array for DT_F32, a uint16 array of
    bf16 bit patterns for DT_BF16.  Stream numbers: 2*step for gradients,
    1 for parameters.
    """
    c = CONFIGS.get(cfg, {})
    std = c.get("grad_std", 0.02) if std is None else std
    dtype = c.get("grad_dtype", DT_BF16) if dtype is None else dtype
    x = gen_normal_f32(cfg, matrix_id, 2 * step, rows, cols, std)
    return (x if dtype == DT_F32 else f32_to_bf16_bits(x)), dtype


def gen_grad_decaying(cfg: int, matrix_id: int, rows: int, cols: int, rank: int = 8, std: float = 0.02,
                      dtype: int = DT_BF16):
    """A gradient with a decaying spectrum: a strong rank-``rank`` part plus
    i.i.d. noise, closer to real gradients than pure noise.  Used by parity
    tests to exercise small and large singular values together."""
    rng = _rng(cfg, matrix_id, 7)
    left = rng.standard_normal((rows, rank), dtype=np.float32)
    right = rng.standard_normal((rank, cols), dtype=np.float32)
    weights = (2.0 ** -np.arange(rank, dtype=np.float32))[:, None]
    x = (left @ (weights * right)) * np.float32(std) + \
        rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(std * 0.05)
    x = x.astype(np.float32)
    return (x if dtype == DT_F32 else f32_to_bf16_bits(x)), dtype


def gen_param(cfg: int, matrix_id: int, rows: int, cols: int, std: float = 0.02) -> np.ndarray:
    """fp32 master parameter values."""
    return gen_normal_f32(cfg, matrix_id, 1, rows, cols, std)


def gen_spd_f32(cfg: int, matrix_id: int, stream: int, d: int, level: float = 1.0, aspect: int = 2) -> np.ndarray:
    """A symmetric positive definite d x d matrix as an optimizer's accumulated statistic would be:
    level * H H^T / (aspect d) of a standard Gaussian d x (aspect d) factor (diagonal about `level`),
    exactly symmetric in fp32.  Its condition number is about ((1 + a) / (1 - a))^2 with
    a = aspect^-1/2 (34 at aspect 2)."""
    h = _rng(cfg, matrix_id, stream).standard_normal((d, aspect * d))
    s = (h @ h.T) * (level / (aspect * d))
    s = (0.5 * (s + s.T)).astype(np.float32)
    return np.ascontiguousarray(np.triu(s) + np.triu(s, 1).T)


def gen_orthogonal_f32(cfg: int, matrix_id: int, stream: int, d: int) -> np.ndarray:
    """A random orthogonal d x d matrix (orthonormal to fp32 rounding): the Q factor of a Gaussian matrix."""
    q, _ = np.linalg.qr(_rng(cfg, matrix_id, stream).standard_normal((d, d)))
    return np.ascontiguousarray(q.astype(np.float32))


def gen_soap_state(cfg: int, matrix_id: int, rows: int, cols: int, std: float = 0.02, identity_bases: bool = False) -> dict:
    """Seeded state of one matrix for a SOAP step that is under way: momentum and second moment of
    the size the gradients of gen_grad give, full-rank statistics, orthogonal bases (fp32 arrays)."""
    return {
        "mom": gen_normal_f32(cfg, matrix_id, 11, rows, cols, std),
        # an average of squared gradients over several steps: no mass near zero, unlike one squared sample
        "var": np.mean(np.square(gen_normal_f32(cfg, matrix_id, 12, 4 * rows, cols, std)).reshape(4, rows, cols), axis=0),
        "left": gen_spd_f32(cfg, matrix_id, 13, rows, std * std * cols),
        "right": gen_spd_f32(cfg, matrix_id, 14, cols, std * std * rows),
        "q_left": np.eye(rows, dtype=np.float32) if identity_bases else gen_orthogonal_f32(cfg, matrix_id, 15, rows),
        "q_right": np.eye(cols, dtype=np.float32) if identity_bases else gen_orthogonal_f32(cfg, matrix_id, 16, cols),
    }


def split_columns(x: np.ndarray, tp: int):
    """Column fragments (contiguous copies) of a rows x cols array."""
    rows, cols = x.shape
    if cols % tp:
        raise ValueError("cols not divisible by tp")
    w = cols // tp
    return [np.ascontiguousarray(x[:, f * w:(f + 1) * w]) for f in range(tp)]
