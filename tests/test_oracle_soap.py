"""Pins of the SOAP oracle (oracle/soap.py), checked against something other than the oracle's
own formula: torch's Adam (the step is Adam when both bases are the identity, and Adam on the
rotated problem for any orthogonal bases), the polar factor (one step from empty state in the
singular bases of G), hand-worked 1 x 1 and 2 x 2 cases, the defining properties of the QR
refresh (orthonormal, triangular remainder, eigenvectors as fixed point and as limit), and the
state recurrences written out as loops.  CPU only."""
import math

import numpy as np
import pytest
import scipy.linalg
import torch

import oracle.partition as OP
import oracle.soap as SO


def _gauss(seed, rows, cols, std=1.0):
    return std * np.random.default_rng(seed).standard_normal((rows, cols))


def _orth(seed, n):
    q, r = np.linalg.qr(np.random.default_rng(seed).standard_normal((n, n)))
    return q * np.sign(np.diag(r))


def _state(rows, cols, q_left=None, q_right=None, mom=None, var=None, left=None, right=None):
    return {"mom": np.zeros((rows, cols)) if mom is None else mom,
            "var": np.zeros((rows, cols)) if var is None else var,
            "left": np.zeros((rows, rows)) if left is None else left,
            "right": np.zeros((cols, cols)) if right is None else right,
            "q_left": np.eye(rows) if q_left is None else q_left,
            "q_right": np.eye(cols) if q_right is None else q_right}


def _carry(state, out):
    new = dict(state)
    for k in ("mom", "var", "left", "right", "q_left", "q_right"):
        if out[k] is not None:
            new[k] = out[k]
    return new


def _torch_adam(grads, param, hp, mom=None, var=None, steps_before=0):
    """Parameter trajectory of torch.optim.Adam in fp64 (no weight decay) on the given gradients."""
    p = torch.nn.Parameter(torch.tensor(param, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=hp.lr, betas=(hp.beta1, hp.beta2), eps=hp.eps)
    if mom is not None:
        opt.state[p] = {"step": torch.tensor(float(steps_before)), "exp_avg": torch.tensor(mom, dtype=torch.float64),
                        "exp_avg_sq": torch.tensor(var, dtype=torch.float64)}
    traj = []
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        traj.append(p.detach().numpy().copy())
    return traj


def test_identity_bases_give_adam():
    rows, cols = 5, 7
    hp = SO.Hparams(beta1=0.9, beta2=0.99, lr=0.01, eps=1e-3)
    grads = [_gauss(10 + i, rows, cols) for i in range(4)]
    p0 = _gauss(3, rows, cols)
    want = _torch_adam(grads, p0, hp)
    st, p = _state(rows, cols), p0
    for i, g in enumerate(grads):
        out = SO.soap_step(g, st, hp, i + 1, False, param=p)
        st, p = _carry(st, out), out["param"]
        assert np.allclose(p, want[i], rtol=1e-12, atol=1e-14)


def test_one_by_one_by_hand():
    """g = 3 from empty state, beta1 = 0.9, beta2 = 0.99, eps = 1, lr = 0.5.
    With bias correction at t = 1: m = 0.3 / 0.1 = 3, v = 0.09 / 0.01 = 9, N = 3 / (3 + 1) = 0.75, delta = -0.375.
    Without: m = 0.3, v = 0.09, N = 0.3 / (0.3 + 1) = 3/13.
    Second step (g = 1, no correction): m = 0.27 + 0.1 = 0.37, v = 0.0891 + 0.01 = 0.0991."""
    hp = SO.Hparams(beta1=0.9, beta2=0.99, lr=0.5, eps=1.0)
    out = SO.soap_step(np.array([[3.0]]), _state(1, 1), hp, 1, False)
    assert abs(out["delta"][0, 0] + 0.375) < 1e-14
    assert abs(out["left"][0, 0] - 0.09) < 1e-15 and abs(out["right"][0, 0] - 0.09) < 1e-15
    hp.bias_correction = False
    out = SO.soap_step(np.array([[3.0]]), _state(1, 1), hp, 1, False)
    assert abs(out["direction"][0, 0] - 3.0 / 13.0) < 1e-14
    out2 = SO.soap_step(np.array([[1.0]]), _carry(_state(1, 1), out), hp, 2, False)
    assert abs(out2["mom"][0, 0] - 0.37) < 1e-15 and abs(out2["var"][0, 0] - 0.0991) < 1e-15
    assert abs(out2["direction"][0, 0] - 0.37 / (math.sqrt(0.0991) + 1.0)) < 1e-14
    assert abs(out2["left"][0, 0] - (0.99 * 0.09 + 0.01)) < 1e-15


@pytest.mark.parametrize("shape", [(4, 4), (5, 8), (9, 6)])
def test_any_orthogonal_bases_give_adam_on_the_rotated_problem(shape):
    """With Gt = Q_L^T G Q_R, Mt = Q_L^T M Q_R and the same V, the update is Q_L (Adam's update of
    the rotated problem) Q_R^T; torch's Adam takes the rotated step."""
    rows, cols = shape
    hp = SO.Hparams(beta1=0.8, beta2=0.9, lr=0.02, eps=1e-4)
    ql, qr = _orth(1, rows), _orth(2, cols)
    g, m0 = _gauss(3, rows, cols), _gauss(4, rows, cols)
    v0 = _gauss(5, rows, cols) ** 2
    p0 = _gauss(6, rows, cols)
    t = 3
    rotated = _torch_adam([ql.T @ g @ qr], ql.T @ p0 @ qr, hp, mom=ql.T @ m0 @ qr, var=v0, steps_before=t - 1)[0]
    out = SO.soap_step(g, _state(rows, cols, ql, qr, mom=m0, var=v0), hp, t, False, param=p0)
    assert np.allclose(out["param"], ql @ rotated @ qr.T, rtol=1e-11, atol=1e-13)
    assert np.allclose(out["mom"], 0.8 * m0 + 0.2 * g, rtol=1e-14, atol=1e-15)      # momentum stays in the original space
    assert np.allclose(out["var"], 0.9 * v0 + 0.1 * (ql.T @ g @ qr) ** 2, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("shape", [(6, 6), (5, 9), (9, 5)])
def test_first_step_in_the_singular_bases_is_the_polar_factor(shape):
    """G = U diag(s) W^T with Q_L = U, Q_R = W and empty state, no bias correction: the rotated gradient is
    diag(s), so N' = (1 - beta1) s / (sqrt(1 - beta2) s + eps) on the diagonal and 0 elsewhere, and
    N -> (1 - beta1) / sqrt(1 - beta2) times the polar factor U W^T as eps -> 0."""
    rows, cols = shape
    g = _gauss(7, rows, cols)
    u, s, wt = np.linalg.svd(g, full_matrices=True)
    hp = SO.Hparams(beta1=0.9, beta2=0.96, eps=1e-7, bias_correction=False)
    out = SO.soap_step(g, _state(rows, cols, u, wt.T), hp, 1, False)
    polar = scipy.linalg.polar(g)[0]
    assert np.allclose(out["direction"], 0.1 / 0.2 * polar, rtol=0, atol=1e-5)
    hp.bias_correction = True           # t = 1: m = G', v = G'^2: the polar factor itself
    out = SO.soap_step(g, _state(rows, cols, u, wt.T), hp, 1, False)
    assert np.allclose(out["direction"], polar, rtol=0, atol=1e-5)


def test_statistics_recurrence_and_orientation():
    rows, cols, b2 = 3, 5, 0.75
    hp = SO.Hparams(beta2=b2)
    g1, g2 = _gauss(8, rows, cols), _gauss(9, rows, cols)
    l0, r0 = 0.5 * np.eye(rows), 0.25 * np.eye(cols)
    st = _state(rows, cols, left=l0, right=r0)
    o1 = SO.soap_step(g1, st, hp, 1, False)
    o2 = SO.soap_step(g2, _carry(st, o1), hp, 2, False)
    assert o2["left"].shape == (rows, rows) and o2["right"].shape == (cols, cols)
    for i in range(rows):
        for j in range(rows):
            want = b2 * b2 * l0[i, j] + (1 - b2) * (b2 * sum(g1[i, k] * g1[j, k] for k in range(cols)) +
                                                    sum(g2[i, k] * g2[j, k] for k in range(cols)))
            assert abs(o2["left"][i, j] - want) < 1e-12
    for i in range(cols):
        for j in range(cols):
            want = b2 * b2 * r0[i, j] + (1 - b2) * (b2 * sum(g1[k, i] * g1[k, j] for k in range(rows)) +
                                                    sum(g2[k, i] * g2[k, j] for k in range(rows)))
            assert abs(o2["right"][i, j] - want) < 1e-12


def _same_up_to_sign(a, b, tol):
    signs = np.sign(np.sum(a * b, axis=0))
    return np.abs(a * signs - b).max() <= tol


def test_refresh_two_by_two_by_hand():
    """S = [[2, 1], [1, 2]], Q = I: the first column of S Q is (2, 1), so q1 = +-(2, 1) / sqrt 5 and
    q2 = +-(-1, 2) / sqrt 5."""
    q = SO.refresh_basis(np.array([[2.0, 1.0], [1.0, 2.0]]), np.eye(2))
    want = np.array([[2.0, -1.0], [1.0, 2.0]]) / math.sqrt(5.0)
    assert _same_up_to_sign(q, want, 1e-14)


def test_refresh_is_a_qr_factor_of_stat_times_basis():
    n = 9
    h = _gauss(11, n, 2 * n)
    stat, basis = h @ h.T, _orth(12, n)
    q = SO.refresh_basis(stat, basis)
    assert np.abs(q.T @ q - np.eye(n)).max() < 1e-13
    rem = q.T @ (stat @ basis)
    assert np.abs(np.tril(rem, -1)).max() < 1e-11 * np.abs(rem).max()      # upper triangular remainder
    assert np.abs(np.diag(rem)).min() > 1e-6                                  # which fixes q up to signs
    # multiplying the old basis from the wrong side breaks the property
    assert np.abs(np.tril(q.T @ (basis @ stat), -1)).max() > 1e-3 * np.abs(rem).max()


def test_refresh_keeps_eigenvectors_and_converges_to_them():
    n = 8
    lam = 2.0 ** -np.arange(n)
    vec = _orth(13, n)
    stat = (vec * lam) @ vec.T
    perm = np.array([3, 0, 7, 1, 2, 6, 4, 5])
    assert _same_up_to_sign(SO.refresh_basis(stat, vec[:, perm]), vec[:, perm], 1e-12)   # fixed point, any order
    q = np.eye(n)
    for _ in range(80):
        q = SO.refresh_basis(stat, q)
    assert _same_up_to_sign(q, vec, 1e-9)                       # orthogonal iteration: descending eigenvalues
    w, v = np.linalg.eigh(stat)
    assert _same_up_to_sign(q, v[:, ::-1], 1e-9)


@pytest.mark.parametrize("shape", [(6, 4), (5, 5)])
def test_refresh_runs_last_and_uses_the_new_statistics(shape):
    rows, cols = shape
    hp = SO.Hparams(beta2=0.5)
    g = _gauss(14, rows, cols)
    h = _gauss(15, rows, 3 * rows)
    k = _gauss(16, cols, 3 * cols)
    st = _state(rows, cols, _orth(17, rows), _orth(18, cols), mom=_gauss(19, rows, cols), var=_gauss(20, rows, cols) ** 2,
                left=h @ h.T, right=k @ k.T)
    plain = SO.soap_step(g, st, hp, 5, False)
    fresh = SO.soap_step(g, st, hp, 5, True)
    for key in ("direction", "var", "mom", "left", "right"):
        assert np.array_equal(plain[key], fresh[key])           # the step itself uses the old bases; V is not rotated
    assert np.array_equal(plain["q_left"], st["q_left"]) and np.array_equal(plain["q_right"], st["q_right"])
    new_left = 0.5 * st["left"] + 0.5 * np.array([[sum(g[i, c] * g[j, c] for c in range(cols)) for j in range(rows)]
                                                  for i in range(rows)])
    new_right = 0.5 * st["right"] + 0.5 * np.array([[sum(g[r, i] * g[r, j] for r in range(rows)) for j in range(cols)]
                                                    for i in range(cols)])
    for q_new, stat, q_old in ((fresh["q_left"], new_left, st["q_left"]), (fresh["q_right"], new_right, st["q_right"])):
        assert np.abs(q_new.T @ q_new - np.eye(len(stat))).max() < 1e-13
        rem = q_new.T @ (stat @ q_old)
        assert np.abs(np.tril(rem, -1)).max() < 1e-11 * np.abs(rem).max()
    # the old statistics would give another basis
    rem_old = fresh["q_left"].T @ (st["left"] @ st["q_left"])
    assert np.abs(np.tril(rem_old, -1)).max() > 1e-3 * np.abs(rem_old).max()


def test_column_signs_of_the_bases_do_not_matter():
    rows, cols = 5, 6
    hp = SO.Hparams()
    g = _gauss(21, rows, cols)
    ql, qr = _orth(22, rows), _orth(23, cols)
    st = _state(rows, cols, ql, qr, mom=_gauss(24, rows, cols), var=_gauss(25, rows, cols) ** 2)
    flip = dict(st)
    flip["q_left"] = ql * np.array([1, -1, 1, -1, -1.0])
    flip["q_right"] = qr * np.array([-1, -1, 1, 1, -1, 1.0])
    a, b = SO.soap_step(g, st, hp, 2, False), SO.soap_step(g, flip, hp, 2, False)
    assert np.allclose(a["direction"], b["direction"], rtol=1e-12, atol=1e-14)
    assert np.allclose(a["var"], b["var"], rtol=1e-12, atol=1e-16)


def test_side_above_the_limit_has_no_basis():
    rows, cols = 7, 4
    g = _gauss(26, rows, cols)
    qr = _orth(27, cols)
    base = _state(rows, cols, np.eye(rows), qr, mom=_gauss(28, rows, cols), var=_gauss(29, rows, cols) ** 2)
    poisoned = dict(base)
    poisoned["q_left"] = _orth(30, rows)                          # must be ignored: rows > max_precond_dim
    poisoned["left"] = np.full((rows, rows), np.nan)
    one = SO.soap_step(g, poisoned, SO.Hparams(max_precond_dim=5), 2, True)
    two = SO.soap_step(g, base, SO.Hparams(max_precond_dim=100), 2, False)
    assert one["left"] is None and one["q_left"] is None and one["right"] is not None
    assert np.allclose(one["direction"], two["direction"], rtol=1e-13, atol=1e-15)
    assert np.abs(one["q_right"].T @ one["q_right"] - np.eye(cols)).max() < 1e-13
    edge = SO.soap_step(g, base, SO.Hparams(max_precond_dim=7), 2, False)          # the limit itself is still allowed
    assert edge["left"] is not None and edge["q_left"] is not None
    wide = SO.soap_step(g.T, _state(cols, rows, qr, None, mom=base["mom"].T, var=base["var"].T),
                        SO.Hparams(max_precond_dim=5), 2, False)
    assert wide["right"] is None and np.allclose(wide["direction"], two["direction"].T, rtol=1e-13, atol=1e-15)


def test_parameter_update_and_fragments():
    rows, cols, tp = 4, 8, 4
    g, p = _gauss(31, rows, cols), _gauss(32, rows, cols)
    hp = SO.Hparams(lr=0.1, weight_decay=0.5)
    st = _state(rows, cols, _orth(33, rows), _orth(34, cols))
    whole = SO.soap_step(g, st, hp, 1, False, param=p)
    split = SO.soap_step([g[:, f * 2:(f + 1) * 2].copy() for f in range(tp)], st, hp, 1, False, param=p)
    assert np.array_equal(whole["param"], split["param"])
    assert np.allclose(whole["param"], p * (1 - 0.1 * 0.5) - 0.1 * whole["direction"], rtol=1e-14, atol=1e-15)
    assert np.array_equal(whole["delta"], -0.1 * whole["direction"])


def test_soap_cost_model_by_hand():
    """W(p) for the planner, r = 2, c = 3, refresh every 10th step: per step 4 * (2*4*3 + 2*2*9) = 240 FLOPs,
    per refresh 14/3 * (8 + 27) = 163.33, a tenth of it per step: floor(256.33) = 256.  In the planner's units of
    2^20 FLOPs a 4096 x 4096 matrix costs floor((16 + 14/15) * 65536) = 1109742."""
    assert OP.soap_flops(2, 3) == 256
    assert OP.soap_flops(3, 2) == 256
    assert OP.soap_flops(2, 3, refresh_every=1) == 240 + 163
    assert OP.param_cost([4096], [4096], OP.COST_SOAP_FLOPS) == [1109742]
    assert OP.param_cost([2], [3], OP.COST_SOAP_FLOPS) == [0]
    # A side above the limit keeps no basis and costs nothing: limit 2 leaves the side of extent 2 of a 2 x 3 matrix,
    # 4 * 2 * 2 * 3 * 2 = 96 per step and 14/3 * 8 = 37.33 per refresh, floor(96 + 3.73) = 99; the limit itself is
    # within; nothing is left of a matrix with both sides above it.
    assert OP.soap_flops(2, 3, max_precond_dim=2) == 99 and OP.soap_flops(3, 2, max_precond_dim=2) == 99
    assert OP.soap_flops(2, 3, max_precond_dim=3) == 256 and OP.soap_flops(2, 3, max_precond_dim=1) == 0
    # the model's own limit is 10000: a 25600 x 5120 matrix counts its 5120-long side only,
    # floor((8 * 25600 * 5120 * 5120 + 14/30 * 5120^3) / 2^20) = floor(5120000 + 59733.33) = 5179733
    assert OP.param_cost([25600, 5120], [5120, 25600], OP.COST_SOAP_FLOPS) == [5179733, 5179733]
    assert OP.param_cost([10000], [10001], OP.COST_SOAP_FLOPS) == [(8 * 10000 * 10001 * 10000 + 14 * 10000 ** 3 // 30) >> 20]
