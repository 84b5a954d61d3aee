"""Pins of the Shampoo oracle (oracle/shampoo.py): what the mathematics fixes, checked
against something other than the oracle's own formula - defining identities of the
inverse fourth root, closed forms for diagonal, rank-one and 1 x 1 inputs, the SVD closed
form of a step from empty statistics (which is the polar factor as eps -> 0), covariance
under orthogonal similarity and scaling, and the state recurrence.  CPU only."""
import math

import numpy as np
import pytest

import oracle.partition as OP
import oracle.shampoo as SH


def _gauss(seed, rows, cols, std=0.02):
    return std * np.random.default_rng(seed).standard_normal((rows, cols))


def _orth(seed, n):
    q, r = np.linalg.qr(np.random.default_rng(seed).standard_normal((n, n)))
    return q * np.sign(np.diag(r))


@pytest.mark.parametrize("n,eps", [(5, 1e-3), (24, 1e-6), (40, 1e-9)])
def test_root_fourth_power_inverts_the_regularised_statistic(n, eps):
    """X = (S + eps I)^(-1/4)  <=>  X symmetric positive definite and X^4 (S + eps I) = I."""
    g = _gauss(n, n, n + 3, 1.0)
    s = g @ g.T
    x = SH.inverse_fourth_root(s, eps)
    a = s + eps * np.eye(n)
    assert np.allclose(x, x.T, atol=1e-12 * np.abs(x).max())
    assert np.linalg.eigvalsh(x).min() > 0
    x4 = x @ x @ x @ x
    assert np.linalg.norm(x4 @ a - np.eye(n)) <= 1e-8 * n * np.linalg.cond(a) ** 0.5
    assert np.linalg.norm(x @ s - s @ x) <= 1e-10 * np.linalg.norm(x) * np.linalg.norm(s)   # a function of S commutes with S


def test_root_of_a_diagonal_statistic():
    d = np.array([4.0, 1.0, 0.25, 0.0, 16.0])
    eps = 1e-4
    x = SH.inverse_fourth_root(np.diag(d), eps)
    assert np.allclose(x, np.diag((d + eps) ** -0.25), rtol=1e-13, atol=1e-13)
    # hand values: (16 + 0)^(-1/4) = 1/2, (1)^(-1/4) = 1, (0 + 1e-4)^(-1/4) = 10
    x0 = SH.inverse_fourth_root(np.diag([16.0, 1.0, 0.0]), 0.0 + 1e-4)
    assert abs(x0[2, 2] - 10.0) < 1e-9 and abs(x0[0, 0] - (16.0001) ** -0.25) < 1e-12 and abs(x0[1, 1] - 1.0001 ** -0.25) < 1e-12


def test_root_of_a_rank_one_statistic():
    """S = s^2 u u^T: the root acts as (s^2 + eps)^(-1/4) on u and as eps^(-1/4) on its complement."""
    n, eps, sig = 7, 1e-2, 3.0
    u = _gauss(1, n, 1, 1.0)[:, 0]
    u /= np.linalg.norm(u)
    x = SH.inverse_fourth_root(sig * sig * np.outer(u, u), eps)
    want = eps ** -0.25 * (np.eye(n) - np.outer(u, u)) + (sig * sig + eps) ** -0.25 * np.outer(u, u)
    assert np.allclose(x, want, rtol=1e-11, atol=1e-11)


def test_root_is_covariant_under_orthogonal_similarity():
    n, eps = 12, 1e-5
    g = _gauss(2, n, 20, 1.0)
    s = g @ g.T
    q = _orth(3, n)
    assert np.allclose(SH.inverse_fourth_root(q @ s @ q.T, eps), q @ SH.inverse_fourth_root(s, eps) @ q.T,
                       rtol=1e-9, atol=1e-10)


def test_statistics_recurrence_and_orientation():
    """L is rows x rows from G G^T, R is cols x cols from G^T G; two steps with decay beta."""
    rows, cols, beta = 3, 5, 0.9
    g1, g2 = _gauss(4, rows, cols, 1.0), _gauss(5, rows, cols, 1.0)
    l0, r0 = np.eye(rows) * 0.5, np.eye(cols) * 0.25
    l1, r1 = SH.statistics(g1, l0, r0, beta)
    l2, r2 = SH.statistics(g2, l1, r1, beta)
    assert l2.shape == (rows, rows) and r2.shape == (cols, cols)
    for i in range(rows):
        for j in range(rows):
            want = beta * beta * l0[i, j] + beta * sum(g1[i, k] * g1[j, k] for k in range(cols)) + \
                sum(g2[i, k] * g2[j, k] for k in range(cols))
            assert abs(l2[i, j] - want) < 1e-12
    for i in range(cols):
        for j in range(cols):
            want = beta * beta * r0[i, j] + beta * sum(g1[k, i] * g1[k, j] for k in range(rows)) + \
                sum(g2[k, i] * g2[k, j] for k in range(rows))
            assert abs(r2[i, j] - want) < 1e-12
    out = SH.shampoo_step(g1, l0, r0, SH.Hparams(beta=beta))
    assert np.array_equal(out["left"], l1) and np.array_equal(out["right"], r1)


def test_one_by_one_matrix_by_hand():
    """rows = cols = 1: L = R = g^2, Delta W = -lr g / sqrt(g^2 + eps); g = 3, eps = 7, lr = 0.5:
    -0.5 * 3 / sqrt(16) = -0.375.  With previous statistics l = 9 (beta 1): L = 18, R = 9 + r0."""
    out = SH.shampoo_step(np.array([[3.0]]), np.zeros((1, 1)), np.zeros((1, 1)), SH.Hparams(lr=0.5, eps=7.0))
    assert abs(out["delta"][0, 0] + 0.375) < 1e-15
    out = SH.shampoo_step(np.array([[3.0]]), np.array([[72.0]]), np.array([[0.0]]), SH.Hparams(lr=1.0, eps=0.0, beta=1.0))
    # L = 81 -> 81^(-1/4) = 1/3; R = 9 -> 9^(-1/4) = 1/sqrt(3)
    assert abs(out["delta"][0, 0] + 3.0 * (1.0 / 3.0) / math.sqrt(3.0)) < 1e-14


@pytest.mark.parametrize("shape", [(6, 6), (5, 9), (9, 5), (16, 40)])
def test_step_from_empty_statistics_is_the_svd_closed_form(shape):
    """With L0 = R0 = 0 and G = U diag(s) V^T:  L = U s^2 U^T, R = V s^2 V^T (plus null spaces
    that G annihilates), so  L^(-1/4) G R^(-1/4) = U diag(s / sqrt(s^2 + eps)) V^T."""
    rows, cols = shape
    g = _gauss(6, rows, cols, 1.0)
    u, s, vt = np.linalg.svd(g, full_matrices=False)
    for eps in (1e-2, 1e-8):
        out = SH.shampoo_step(g, np.zeros((rows, rows)), np.zeros((cols, cols)), SH.Hparams(lr=1.0, eps=eps))
        want = (u * (s / np.sqrt(s * s + eps))) @ vt
        assert np.linalg.norm(out["precond"] - want) <= 1e-9 * np.linalg.norm(want)
        assert np.array_equal(out["delta"], -out["precond"])
    # eps -> 0: the polar factor U V^T, the matrix Muon's iteration approximates
    out = SH.shampoo_step(g, np.zeros((rows, rows)), np.zeros((cols, cols)), SH.Hparams(lr=1.0, eps=1e-14))
    assert np.linalg.norm(out["precond"] - u @ vt) <= 1e-6 * math.sqrt(min(shape))


def test_step_scaling_and_rotation_covariance():
    """O(c G; c^2 L, c^2 R, c^2 eps) = O(G; L, R, eps) (degree 0), and
    O(Q1 G Q2; Q1 L Q1^T, Q2^T R Q2) = Q1 O Q2."""
    rows, cols, eps = 7, 10, 1e-3
    g = _gauss(7, rows, cols, 1.0)
    h = _gauss(8, rows, cols, 1.0)
    l0, r0 = h @ h.T, h.T @ h
    hp = SH.Hparams(lr=1.0, eps=eps, beta=0.7)
    base = SH.shampoo_step(g, l0, r0, hp)["precond"]
    c = 5.0
    scaled = SH.shampoo_step(c * g, c * c * l0, c * c * r0, SH.Hparams(lr=1.0, eps=c * c * eps, beta=0.7))["precond"]
    assert np.allclose(scaled, base, rtol=1e-10, atol=1e-12)
    q1, q2 = _orth(9, rows), _orth(10, cols)
    rot = SH.shampoo_step(q1 @ g @ q2, q1 @ l0 @ q1.T, q2.T @ r0 @ q2, hp)["precond"]
    assert np.allclose(rot, q1 @ base @ q2, rtol=1e-9, atol=1e-11)


def test_parameter_update_and_fragments():
    rows, cols, tp = 4, 8, 4
    g = _gauss(11, rows, cols, 1.0)
    p = _gauss(12, rows, cols, 1.0)
    hp = SH.Hparams(lr=0.1, weight_decay=0.5, eps=1e-3)
    whole = SH.shampoo_step(g, np.zeros((rows, rows)), np.zeros((cols, cols)), hp, param=p)
    frags = [g[:, f * 2:(f + 1) * 2].copy() for f in range(tp)]
    split = SH.shampoo_step(frags, np.zeros((rows, rows)), np.zeros((cols, cols)), hp, param=p)
    assert np.array_equal(whole["param"], split["param"])
    assert np.allclose(whole["param"], p * (1 - 0.1 * 0.5) - 0.1 * whole["precond"], rtol=1e-14, atol=1e-15)
    assert np.allclose(whole["precond"], whole["left_root"] @ g @ whole["right_root"], rtol=1e-13, atol=1e-14)


@pytest.mark.parametrize("shape", [(4, 6), (5, 5)])
def test_kept_roots_replace_the_roots_of_the_new_statistics(shape):
    """With kept roots the step is O = A G B for the matrices handed in (not their roots, not their transposes), while
    the statistics still move; identity roots give O = G; the roots a full step returns, kept, reproduce that step."""
    rows, cols = shape
    g = _gauss(21, rows, cols, 1.0)
    a, b = _gauss(22, rows, rows, 1.0), _gauss(23, cols, cols, 1.0)          # not symmetric on purpose
    hp = SH.Hparams(lr=1.0, eps=1e-3, beta=0.5)
    l0, r0 = np.eye(rows), np.eye(cols)
    out = SH.shampoo_step(g, l0, r0, hp, kept_roots=(a, b))
    want = np.array([[sum(a[i, k] * g[k, m] * b[m, j] for k in range(rows) for m in range(cols)) for j in range(cols)]
                     for i in range(rows)])
    assert np.allclose(out["precond"], want, rtol=1e-13, atol=1e-13)
    full = SH.shampoo_step(g, l0, r0, hp)
    assert np.array_equal(out["left"], full["left"]) and np.array_equal(out["right"], full["right"])
    assert np.array_equal(SH.shampoo_step(g, l0, r0, hp, kept_roots=(np.eye(rows), np.eye(cols)))["precond"], g)
    again = SH.shampoo_step(g, l0, r0, hp, kept_roots=(full["left_root"], full["right_root"]))
    assert np.array_equal(again["delta"], full["delta"])


def test_shampoo_cost_model_by_hand():
    """W(p) for the planner: r = 2, c = 3, 25 root rounds: 4*4*3 + 4*9*2 + 200*(8 + 27) = 7120 FLOPs;
    in the planner's units of 2^20 FLOPs a 4096 x 4096 matrix costs
    (8 * 4096^3 + 400 * 4096^3) / 2^20 = 408 * 65536."""
    assert OP.shampoo_flops(2, 3) == 7120
    assert OP.param_cost([4096], [4096], OP.COST_SHAMPOO_FLOPS) == [408 * 65536]
    assert OP.param_cost([2], [3], OP.COST_SHAMPOO_FLOPS) == [0]
    assert OP.shampoo_flops(3, 2) == OP.shampoo_flops(2, 3)
