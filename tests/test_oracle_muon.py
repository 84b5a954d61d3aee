"""Pins for the Muon oracle: SVD closed forms, the polar factor, the scalar
quintic map, invariances and textbook reductions.  numpy.linalg.svd and
scipy.linalg.polar are the independent references."""
import math

import numpy as np
import pytest
import scipy.linalg

from oracle import muon as M
from paper_2602_06079_amd import workloads as W

QUINTIC = (3.4445, -4.7750, 2.0315)


def _rel(a, b):
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _scalar_map(sig, steps, a, b, c):
    sig = np.array(sig, dtype=np.float64)
    for _ in range(steps):
        sig = a * sig + b * sig ** 3 + c * sig ** 5
    return sig


# ------------------------------------------------------- Newton-Schulz core

@pytest.mark.parametrize("shape", [(16, 24), (24, 16), (32, 32), (64, 200), (256, 512), (300, 77)])
@pytest.mark.parametrize("coef", [QUINTIC, (1.5, -0.5, 0.0), (2.0, -1.5, 0.5)])
def test_iteration_acts_on_singular_values_only(shape, coef):
    """If X0 = U diag(s) V^T then X_k = U diag(p^k(s)) V^T with
    p(x) = a x + b x^3 + c x^5: pins every term, sign and operand order."""
    x0 = _rand(shape, 1)
    x0 /= np.linalg.norm(x0)
    u, s, vt = np.linalg.svd(x0, full_matrices=False)
    for steps in (1, 3, 5):
        want = (u * _scalar_map(s, steps, *coef)) @ vt
        got = M.newton_schulz(x0, steps, *coef)
        assert got.shape == x0.shape
        assert _rel(got, want) < 1e-10


def test_cubic_iteration_converges_to_polar_factor():
    """a, b, c = 1.5, -0.5, 0 is the classical Newton-Schulz iteration: for
    singular values in (0, sqrt(3)) it converges to the orthogonal polar factor U V^T."""
    for shape, seed in (((12, 20), 3), ((20, 12), 4), ((40, 40), 5)):
        x0 = _rand(shape, seed)
        x0 /= np.linalg.norm(x0, 2) * 1.01           # spectral norm < 1
        polar = scipy.linalg.polar(x0)[0] if shape[0] == shape[1] else None
        u, s, vt = np.linalg.svd(x0, full_matrices=False)
        steps = 80
        got = M.newton_schulz(x0, steps, 1.5, -0.5, 0.0)
        assert _rel(got, u @ vt) < 1e-9
        if polar is not None:
            assert _rel(got, polar) < 1e-9
        small = got @ got.T if shape[0] <= shape[1] else got.T @ got
        assert np.linalg.norm(small - np.eye(small.shape[0])) < 1e-8


def test_quintic_band():
    """Five quintic steps with (3.4445, -4.7750, 2.0315) send every singular value
    in [0.01, 1] into a band around 1 (it does not converge to 1).  The band is
    computed here from the scalar map on a fine grid, then checked on the singular
    values of the oracle's output for a matrix with a prescribed spectrum."""
    grid = np.linspace(0.01, 1.0, 200001)
    out = _scalar_map(grid, 5, *QUINTIC)
    lo, hi = out.min(), out.max()
    assert 0.68 < lo < 0.69 and 1.13 < hi < 1.14
    assert abs(_scalar_map(np.linspace(0, 1, 100001), 1, *QUINTIC).max() - 1.2024) < 1e-3
    rng = np.random.default_rng(8)
    q1, _ = np.linalg.qr(rng.standard_normal((48, 48)))
    q2, _ = np.linalg.qr(rng.standard_normal((80, 80)))
    s0 = np.sort(rng.uniform(0.01, 1.0, 48))[::-1]
    x0 = (q1 * s0) @ q2[:48, :]
    sv = np.linalg.svd(M.newton_schulz(x0, 5, *QUINTIC), compute_uv=False)
    assert sv.min() >= lo - 1e-9 and sv.max() <= hi + 1e-9
    assert np.allclose(np.sort(sv), np.sort(_scalar_map(s0, 5, *QUINTIC)), rtol=0, atol=1e-10)


def test_invariances():
    x0 = _rand((20, 36), 11)
    x0 /= np.linalg.norm(x0)
    base = M.newton_schulz(x0, 5, *QUINTIC)
    # transpose equivariance: NS(X^T) = NS(X)^T
    assert _rel(M.newton_schulz(x0.T.copy(), 5, *QUINTIC), base.T) < 1e-12
    # orthogonal equivariance: NS(Q1 X Q2) = Q1 NS(X) Q2
    q1, _ = np.linalg.qr(_rand((20, 20), 12))
    q2, _ = np.linalg.qr(_rand((36, 36), 13))
    assert _rel(M.newton_schulz(q1 @ x0 @ q2, 5, *QUINTIC), q1 @ base @ q2) < 1e-10
    # zero steps is the identity; zero input stays zero
    assert np.array_equal(M.newton_schulz(x0, 0, *QUINTIC), x0)
    assert not M.newton_schulz(np.zeros((4, 6)), 5, *QUINTIC).any()


# ---------------------------------------------------------------- full step

def test_step_reduces_to_normalised_gradient():
    """beta = 0 and zero Newton-Schulz steps: Delta W = -lr * scale * G / (||G||_F + eps)."""
    g = _rand((10, 30), 21)
    for mode, scale in ((M.SCALE_NONE, 1.0), (M.SCALE_ASPECT, 1.0), (M.SCALE_RMS, 0.2 * math.sqrt(30))):
        hp = M.Hparams(beta=0.0, ns_steps=0, lr=0.5, eps=1e-7, scale_mode=mode)
        out = M.muon_step(g, np.ones_like(g), hp)
        want = -0.5 * scale * g / (np.linalg.norm(g) + 1e-7)
        assert _rel(out["delta"], want) < 1e-14
        assert np.array_equal(out["mom"], g)
    # tall matrix: aspect scale sqrt(rows / cols)
    gt = g.T.copy()
    hp = M.Hparams(beta=0.0, ns_steps=0, lr=0.5, scale_mode=M.SCALE_ASPECT)
    want = -0.5 * math.sqrt(3.0) * gt / (np.linalg.norm(gt) + hp.eps)
    assert _rel(M.muon_step(gt, np.zeros_like(gt), hp)["delta"], want) < 1e-14


def test_momentum_recurrence_and_nesterov():
    """M_t = sum_i beta^(t-i) G_i after t steps from zero; Nesterov feeds G + beta M."""
    gs = [_rand((6, 9), 30 + i) for i in range(3)]
    beta = 0.9
    hp = M.Hparams(beta=beta, ns_steps=0, lr=1.0, scale_mode=M.SCALE_NONE)
    mom = np.zeros((6, 9))
    for g in gs:
        out = M.muon_step(g, mom, hp)
        mom = out["mom"]
    want = beta ** 2 * gs[0] + beta * gs[1] + gs[2]
    assert _rel(mom, want) < 1e-15
    assert _rel(out["delta"], -want / (np.linalg.norm(want) + hp.eps)) < 1e-14
    hpn = M.Hparams(beta=beta, ns_steps=0, lr=1.0, scale_mode=M.SCALE_NONE, nesterov=True)
    prev = beta * gs[0] + gs[1]
    outn = M.muon_step(gs[2], prev, hpn)
    u = gs[2] + beta * (beta * prev + gs[2])
    assert _rel(outn["delta"], -u / (np.linalg.norm(u) + hp.eps)) < 1e-14
    assert _rel(outn["mom"], beta * prev + gs[2]) < 1e-15


def test_step_output_is_scale_invariant_and_near_orthogonal():
    g = _rand((32, 96), 40)
    hp = M.Hparams(scale_mode=M.SCALE_NONE, lr=1.0)
    base = M.muon_step(g, np.zeros_like(g), hp)["ortho"]
    big = M.muon_step(1000.0 * g, np.zeros_like(g), hp)["ortho"]
    assert _rel(big, base) < 1e-6                      # only eps breaks exact invariance
    u, s, vt = np.linalg.svd(g, full_matrices=False)
    s0 = s / (np.linalg.norm(g) + hp.eps)
    want = (u * _scalar_map(s0, 5, hp.a, hp.b, hp.c)) @ vt
    assert _rel(base, want) < 1e-10
    sv = np.linalg.svd(base, compute_uv=False)
    assert sv.min() > 0.6 and sv.max() < 1.21


def test_param_update_and_weight_decay():
    g = _rand((8, 8), 50)
    p = _rand((8, 8), 51)
    hp = M.Hparams(lr=0.1, weight_decay=0.5, scale_mode=M.SCALE_NONE)
    out = M.muon_step(g, np.zeros_like(g), hp, param=p)
    assert _rel(out["param"], p * 0.95 - 0.1 * out["ortho"]) < 1e-15
    assert np.allclose(out["delta"], -0.1 * out["ortho"], rtol=1e-15, atol=0)


def test_zero_gradient_gives_zero_update():
    hp = M.Hparams()
    out = M.muon_step(np.zeros((5, 7)), np.zeros((5, 7)), hp, param=np.ones((5, 7)))
    assert not out["delta"].any() and np.isfinite(out["delta"]).all()
    assert np.array_equal(out["param"], np.ones((5, 7)))


def test_tp_fragments_round_trip_and_equal_whole():
    """Column fragments -> whole -> fragments is the identity, and the TP step on
    fragments equals the step on the concatenated matrix."""
    g = _rand((12, 32), 60)
    frags = M.scatter_columns(g, 4)
    assert [f.shape for f in frags] == [(12, 8)] * 4
    assert np.array_equal(M.gather_columns(frags), g)
    assert np.array_equal(frags[2], g[:, 16:24])
    hp = M.Hparams()
    a = M.muon_step(frags, np.zeros_like(g), hp)
    b = M.muon_step(g, np.zeros_like(g), hp)
    assert np.array_equal(a["delta"], b["delta"])
    with pytest.raises(ValueError):
        M.scatter_columns(g, 5)


def test_bf16_widening_is_exact():
    x = np.array([1.0, -2.5, 0.02, 3.0e-5, 65280.0], dtype=np.float32)
    bits = W.f32_to_bf16_bits(x)
    wide = M.bf16_bits_to_f64(bits)
    assert np.array_equal(wide, W.bf16_bits_to_f32(bits).astype(np.float64))
    assert wide[0] == 1.0 and wide[1] == -2.5 and wide[4] == 65280.0
    assert abs(wide[2] - 0.02) <= 0.02 * 2 ** -8
    # round-to-nearest-even at a halfway point: 1 + 2^-8 lies between 1 and 1 + 2^-7
    half = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], dtype=np.float32)
    assert list(M.bf16_bits_to_f64(W.f32_to_bf16_bits(half))) == [1.0, 1.0 + 2.0 ** -6]
