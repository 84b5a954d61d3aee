"""GPU parity of canz_soap_step against the fp64 oracle (oracle/soap.py), through the C ABI.

What is compared, per matrix, on the same seeded inputs (the oracle gets the fp32 state and the
bf16 / fp32 gradients widened exactly):
  momentum M, second moment V, statistics L and R   relative Frobenius error;
  the update (parameters in place, or Delta W)        relative Frobenius error of the step taken;
  a refreshed basis Q                                 what is unique and what must hold: Q^T Q = I,
      Q^T (S Q_old) upper triangular, and column by column equality with the oracle's Q up to the
      column's sign where the QR factor is well conditioned (the columns of a QR factor are fixed
      up to sign only for a full-rank matrix, and their sensitivity grows with its condition).

Tolerances.  M: 1e-6 (one fused multiply-add per element).  L, R: 1e-5, V: 5e-6 (fp32 products of
up to 4096 terms, squared for V; measured 1e-7).  Update: 2e-5 (measured 1e-7 to 1.4e-6 with a second
moment that has history, 8e-6 on a first step).  A first step from V = 0 is N' = m / (|g'| sqrt(c) + eps),
i.e. the sign of g' for eps -> 0, so an element whose rotated gradient is below the fp32 rounding of the
rotation (about 1e-6 of the typical size) could flip: the first-step test uses eps = 1e-3 of the gradient
scale, which bounds the slope of N' in g'.  For the same reason the seeded second moment is an average of
several squared samples, as a real one is, not one squared sample (whose density piles up at zero).
Refreshed basis against the oracle's: 1e-4 max-abs per column at condition number 30 to 100 of the
statistic (measured 3e-7 to 5e-7; 2e-5 on the rank-deficient case, tolerance 1e-3 there);
orthonormality 5e-6 max-abs (measured 6e-7); triangular remainder below 5e-6 of the largest entry
(measured 2.5e-7)."""
import numpy as np
import pytest

from oracle import soap as SO
from paper_2602_06079_amd import workloads as W
from tests.gpu_harness import log, rel_fro, to_device, to_host64, widen

pytestmark = pytest.mark.gpu

TOL_MOM, TOL_STAT, TOL_VAR, TOL_UPDATE = 1e-6, 1e-5, 5e-6, 2e-5
TOL_ORTH, TOL_TRI, TOL_Q = 5e-6, 5e-6, 1e-4
TOL_MOM_ROT = 5e-6
STATE_KEYS = ("mom", "var", "left", "right", "q_left", "q_right")


def oracle_hparams(hp) -> SO.Hparams:
    f = lambda v: float(np.float32(v))
    return SO.Hparams(beta1=f(hp.beta1), beta2=f(hp.beta2), lr=f(hp.lr), weight_decay=f(hp.weight_decay), eps=f(hp.eps),
                      bias_correction=bool(hp.bias_correction), max_precond_dim=int(hp.max_precond_dim))


class SoapDevice:
    """One micro-group on the device.  grads: per matrix a host array or a list of tp fragments;
    states: per matrix a dict of fp32 host arrays (STATE_KEYS); outs: parameter arrays, or None
    for Delta W fragments."""

    def __init__(self, canz, rows, cols, grads, states, outs=None, tp=1, out_np_dtype=np.float32, max_precond_dim=10000,
                 mom_rot=None):
        import torch
        self.canz, self.rows, self.cols, self.tp, self.n = canz, rows, cols, tp, len(states)
        self.mom_rot_t = [] if mom_rot is None else [to_device(m) for m in mom_rot]     # the caller-held rotated momentum
        self.use_left, self.use_right = rows <= max_precond_dim, cols <= max_precond_dim
        self.t = {k: [to_device(st[k]) for st in states] for k in STATE_KEYS}
        if not self.use_left:
            self.t["left"], self.t["q_left"] = [], []
        if not self.use_right:
            self.t["right"], self.t["q_right"] = [], []
        self.set_grads(grads)
        self.delta = outs is None
        if self.delta:
            proto = np.zeros((rows, cols // tp), dtype=out_np_dtype)
            self.out_dtype = W.DT_BF16 if proto.dtype == np.uint16 else W.DT_F32
            self.out_t = [to_device(proto) for _ in range(self.n * tp)]
        else:
            self.out_dtype = W.DT_BF16 if outs[0].dtype == np.uint16 else W.DT_F32
            self.out_t = [to_device(p) for p in outs]
        torch.cuda.synchronize()

    def set_grads(self, grads):
        first = grads[0][0] if isinstance(grads[0], (list, tuple)) else grads[0]
        self.grad_dtype = W.DT_BF16 if first.dtype == np.uint16 else W.DT_F32
        self.grad_t = []
        for g in grads:
            frags = g if isinstance(g, (list, tuple)) else [g]
            assert len(frags) == self.tp
            self.grad_t += [to_device(f) for f in frags]

    def group(self):
        return self.canz.SoapGroup(rows=self.rows, cols=self.cols, grad=self.grad_t, mom=self.t["mom"], var=self.t["var"],
                                   left=self.t["left"], right=self.t["right"], qleft=self.t["q_left"],
                                   qright=self.t["q_right"], out=self.out_t, mom_rot=self.mom_rot_t, tp=self.tp,
                                   grad_dtype=self.grad_dtype, out_dtype=self.out_dtype)

    def out_host(self, i):
        if not self.delta:
            return to_host64(self.out_t[i])
        return np.concatenate([to_host64(self.out_t[i * self.tp + f]) for f in range(self.tp)], axis=1)

    def state_host(self, key, i):
        return to_host64(self.t[key][i])


def run(canz, devs, hp):
    import torch
    groups = [d.group() for d in devs]
    nbytes = canz.canz_soap_workspace_bytes(groups, hp)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)                                   # the workspace is scratch: NaN patterns must not leak
    canz.canz_soap_step(groups, hp, ws, nbytes, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()


def widen_state(st):
    return {k: widen(v) for k, v in st.items()}


def widen_grad(g):
    return [widen(f) for f in g] if isinstance(g, (list, tuple)) else widen(g)


def check_basis(got, ref, stat_new, q_old, label, unique_cols=None, tol_q=TOL_Q):
    """got: the device's refreshed basis; ref: the oracle's; stat_new, q_old: the oracle's new statistic and
    the basis before the step.  unique_cols: how many leading columns the QR factor fixes (all by default)."""
    d = got.shape[0]
    assert np.isfinite(got).all(), label
    orth = np.abs(got.T @ got - np.eye(d)).max()
    assert orth <= TOL_ORTH, "%s: Q^T Q - I = %.3g" % (label, orth)
    s = stat_new @ q_old
    rem = got.T @ s
    k = d if unique_cols is None else unique_cols
    tri = np.abs(np.tril(rem, -1)[:, :k]).max() / np.abs(rem).max()
    assert tri <= TOL_TRI, "%s: lower part of Q^T (S Q_old) = %.3g of the largest entry" % (label, tri)
    signs = np.sign(np.sum(got[:, :k] * ref[:, :k], axis=0))
    diff = np.abs(got[:, :k] * signs - ref[:, :k]).max() if k else 0.0
    assert diff <= tol_q, "%s: basis differs from the oracle's by %.3g" % (label, diff)
    return orth, tri, diff


def check(dev, grads, states, params, hp, label, tol_update=TOL_UPDATE, basis_kw=None, tol_var=TOL_VAR, tol_mom_rot=TOL_MOM_ROT):
    """Compares the device's state and output after one step with the oracle's step from `states`.
    Returns the oracle's results (for trajectories)."""
    ohp = oracle_hparams(hp)
    worst = {"update": 0.0, "var": 0.0, "orth": 0.0, "tri": 0.0, "q": 0.0}
    refs = []
    for i in range(dev.n):
        ref = SO.soap_step(widen_grad(grads[i]), widen_state(states[i]), ohp, int(hp.step), bool(hp.refresh),
                           param=None if params is None else widen(params[i]))
        refs.append(ref)
        assert rel_fro(dev.state_host("mom", i), ref["mom"]) <= TOL_MOM, "%s: M of matrix %d" % (label, i)
        ev = rel_fro(dev.state_host("var", i), ref["var"])
        worst["var"] = max(worst["var"], ev)
        assert ev <= tol_var, "%s: V of matrix %d: %.3g" % (label, i, ev)
        for side, stat_key, q_key in ((dev.use_left, "left", "q_left"), (dev.use_right, "right", "q_right")):
            if not side:
                continue
            got_s = dev.state_host(stat_key, i)
            assert rel_fro(got_s, ref[stat_key]) <= TOL_STAT, "%s: %s of matrix %d" % (label, stat_key, i)
            assert np.array_equal(got_s, got_s.T), "%s: statistic not symmetric" % label
            got_q = dev.state_host(q_key, i)
            if hp.refresh:
                orth, tri, diff = check_basis(got_q, ref[q_key], ref[stat_key], widen(states[i][q_key]),
                                              "%s: %s of matrix %d" % (label, q_key, i), **(basis_kw or {}).get(q_key, {}))
                worst["orth"], worst["tri"], worst["q"] = max(worst["orth"], orth), max(worst["tri"], tri), max(worst["q"], diff)
            else:
                assert np.array_equal(got_q, widen(states[i][q_key])), "%s: basis changed without a refresh" % label
        if dev.mom_rot_t:
            # the rotated momentum the device leaves: M of this step in the bases it returns (its own, whose columns
            # may differ in sign from the oracle's)
            ql = dev.state_host("q_left", i) if dev.use_left else None
            qr = dev.state_host("q_right", i) if dev.use_right else None
            er = rel_fro(to_host64(dev.mom_rot_t[i]), SO.rotate_in(ref["mom"], ql, qr))
            worst["mom_rot"] = max(worst.get("mom_rot", 0.0), er)
            assert er <= tol_mom_rot, "%s: rotated momentum of matrix %d: %.3g" % (label, i, er)
        got = dev.out_host(i)
        assert np.isfinite(got).all()
        want = ref["delta"] if params is None else ref["param"]
        den = np.linalg.norm(ref["delta"])
        err = np.linalg.norm(got - want) / den if den > 0 else np.linalg.norm(got - want)
        worst["update"] = max(worst["update"], err)
        assert err <= tol_update, "%s: matrix %d update error %.3g" % (label, i, err)
    log("%s: worst update %.3g (tol %.2g), V %.3g%s%s" % (
        label, worst["update"], tol_update, worst["var"], ", M' %.3g" % worst["mom_rot"] if "mom_rot" in worst else "",
        ", basis: orth %.3g tri %.3g vs oracle %.3g" % (worst["orth"], worst["tri"], worst["q"]) if hp.refresh else ""))
    return refs


RAGGED = [(300, 77), (77, 300), (200, 333), (256, 256), (130, 1), (1, 9), (520, 1032)]


@pytest.mark.parametrize("shape", RAGGED, ids=lambda s: "%dx%d" % s)
def test_ragged_shapes_one_step(canz, shape):
    """Shapes that do not fill the 128-wide tiles, tall and wide; bf16 gradients, fp32 parameters in place
    with weight decay, random orthogonal bases, a state with history."""
    rows, cols = shape
    n = 3
    grads = [W.gen_grad(60, i, rows, cols)[0] for i in range(n)]
    states = [W.gen_soap_state(60, i, rows, cols) for i in range(n)]
    params = [W.gen_param(60, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, weight_decay=0.1, eps=1e-8, step=7)
    dev = SoapDevice(canz, rows, cols, grads, states, outs=params)
    run(canz, [dev], hp)
    check(dev, grads, states, params, hp, "soap ragged %dx%d" % shape)


@pytest.mark.parametrize("shape", [(300, 77), (77, 300), (256, 256), (520, 1032), (33, 160), (1, 9), (129, 127), (255, 257), (384, 385)],
                         ids=lambda s: "%dx%d" % s)
def test_refresh_on_ragged_shapes(canz, shape):
    """A refresh step: extents that are no multiple of the 32-wide panels or the 128-wide tiles, and extents just below,
    at and just above the boundaries of the blocks of four panels (128 columns) that the factorisation applies at once."""
    rows, cols = shape
    n = 2
    grads = [W.gen_grad(61, i, rows, cols)[0] for i in range(n)]
    states = [W.gen_soap_state(61, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=10, refresh=True, out_mode=canz.OUT_DELTA)
    dev = SoapDevice(canz, rows, cols, grads, states)
    run(canz, [dev], hp)
    check(dev, grads, states, None, hp, "soap refresh %dx%d" % shape)


def test_first_step_from_empty_state_is_adam_in_the_given_bases(canz):
    """t = 1, M = V = 0, identity bases and random bases; eps at 1e-3 of the gradient scale (see the module text)."""
    rows, cols, n = 200, 136, 2
    for identity in (True, False):
        grads = [W.gen_grad(62, i, rows, cols)[0] for i in range(n)]
        states = [W.gen_soap_state(62, i, rows, cols, identity_bases=identity) for i in range(n)]
        for st in states:
            st["mom"][:] = 0
            st["var"][:] = 0
            st["left"][:] = 0
            st["right"][:] = 0
        hp = canz.SoapHparams(lr=0.01, eps=2e-5, step=1, out_mode=canz.OUT_DELTA)
        dev = SoapDevice(canz, rows, cols, grads, states)
        run(canz, [dev], hp)
        check(dev, grads, states, None, hp, "soap first step, %s bases" % ("identity" if identity else "random"))


@pytest.mark.parametrize("bf16_rot", [False, True], ids=["fp32", "bf16-rotations"])
@pytest.mark.parametrize("keep_rot", [False, True], ids=["rotate-every-step", "rotated-momentum-kept"])
def test_trajectory_with_refreshes(canz, keep_rot, bf16_rot):
    """Six steps, refresh on every second one; the oracle carries its own state and, after a refresh, takes the
    device's bases (they agree to TOL_Q up to column signs; the comparison of the following steps is then on the
    same bases instead of on two bases that differ by rounding).  With the rotated momentum kept by the caller the
    first step rotates M and every later one lets M' follow its own recurrence, across the refreshes; the oracle
    rotates M on every step.  With the rotations on bf16 operands every step is held to that mode's tolerances (the
    oracle restarts from the device's state, so the comparison is per step; the kept M' carries its rounding from
    step to step, decaying with beta1)."""
    rows, cols, n = 160, 288, 2
    states = [W.gen_soap_state(63, i, rows, cols) for i in range(n)]
    params = [W.gen_param(63, i, rows, cols) for i in range(n)]
    grads = [W.gen_grad(63, i, rows, cols, step=0)[0] for i in range(n)]
    dev = SoapDevice(canz, rows, cols, grads, states, outs=params,
                     mom_rot=[np.full((rows, cols), np.nan, np.float32) for _ in range(n)] if keep_rot else None)
    for step in range(1, 7):
        if step > 1:
            grads = [W.gen_grad(63, i, rows, cols, step=step - 1)[0] for i in range(n)]
            dev.set_grads(grads)
        hp = canz.SoapHparams(lr=0.02, weight_decay=0.01, eps=1e-8, beta1=0.9, beta2=0.95, step=step + 4, refresh=step % 2 == 0,
                              mom_rot_valid=keep_rot and step > 1, bf16_rotations=bf16_rot)
        run(canz, [dev], hp)
        tols = dict(tol_update=TOL16_UPDATE, tol_var=TOL16_VAR, tol_mom_rot=TOL16_MOM_ROT_WHOLE) if bf16_rot else {}
        check(dev, grads, states, params, hp, "soap trajectory step %d%s" % (step, ", bf16 rotations" if bf16_rot else ""), **tols)
        # next step starts from what the device holds (fp32), on both sides
        states = [{k: dev.t[k][i].cpu().numpy() for k in STATE_KEYS} for i in range(n)]
        params = [dev.out_t[i].cpu().numpy() for i in range(n)]


def test_tp_fragments_fp32_gradients_bf16_delta(canz):
    rows, cols, tp, n = 136, 256, 4, 3
    grads = [W.split_columns(W.gen_grad(64, i, rows, cols, dtype=W.DT_F32)[0], tp) for i in range(n)]
    states = [W.gen_soap_state(64, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=3, refresh=True, out_mode=canz.OUT_DELTA)
    dev = SoapDevice(canz, rows, cols, grads, states, tp=tp, out_np_dtype=np.uint16)
    run(canz, [dev], hp)
    check(dev, grads, states, None, hp, "soap tp=4 bf16 delta", tol_update=2 ** -8)     # bf16 storage of Delta W


@pytest.mark.parametrize("keep_rot", [False, True], ids=["rotate", "kept"])
@pytest.mark.parametrize("shape,limit", [((300, 100), 128), ((100, 300), 128), ((300, 100), 100), ((100, 300), 100)],
                         ids=lambda v: str(v).replace(" ", ""))
def test_one_sided_above_the_limit(canz, shape, limit, keep_rot):
    """The side longer than max_precond_dim has no statistic and no basis: its tables are not passed at all.  With the
    rotated momentum kept, the caller hands in a valid M' (the rotation of its M, computed here in fp64)."""
    rows, cols = shape
    n = 2
    grads = [W.gen_grad(65, i, rows, cols)[0] for i in range(n)]
    states = [W.gen_soap_state(65, i, rows, cols) for i in range(n)]
    params = [W.gen_param(65, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=5, refresh=True, max_precond_dim=limit, mom_rot_valid=keep_rot)
    rot = None
    if keep_rot:
        rot = [SO.rotate_in(widen(st["mom"]), widen(st["q_left"]) if rows <= limit else None,
                            widen(st["q_right"]) if cols <= limit else None).astype(np.float32) for st in states]
    dev = SoapDevice(canz, rows, cols, grads, states, outs=params, max_precond_dim=limit, mom_rot=rot)
    assert dev.use_left != dev.use_right
    run(canz, [dev], hp)
    check(dev, grads, states, params, hp, "soap one-sided %dx%d limit %d" % (rows, cols, limit))


def test_rank_deficient_refresh(canz):
    """From empty statistics a 96 x 40 gradient gives L = c G G^T of rank 40: the first 40 columns of the QR factor
    of L Q are fixed, the other 56 are some orthonormal completion (checked as such, not against the oracle)."""
    rows, cols, n = 96, 40, 2
    grads = [W.gen_grad(66, i, rows, cols)[0] for i in range(n)]
    states = [W.gen_soap_state(66, i, rows, cols) for i in range(n)]
    for st in states:
        st["left"][:] = 0
        st["right"][:] = 0
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=2, refresh=True, out_mode=canz.OUT_DELTA)
    dev = SoapDevice(canz, rows, cols, grads, states)
    run(canz, [dev], hp)
    # G G^T of a Gaussian 96 x 40 matrix: condition number of the rank-40 part about 20; its QR columns 30 .. 39
    # are the sensitive ones
    check(dev, grads, states, None, hp, "soap rank-deficient", basis_kw={"q_left": {"unique_cols": cols, "tol_q": 1e-3}})


def test_zero_gradient_and_empty_state(canz):
    """G = 0 from an empty state with a refresh: no update, every moment and statistic stays zero, and the QR of the
    zero matrix leaves every reflector switched off (tau = 0), so the refreshed bases are the identity."""
    rows, cols, n = 136, 72, 2
    grads = [np.zeros((rows, cols), np.uint16) for _ in range(n)]
    states = [W.gen_soap_state(70, i, rows, cols, identity_bases=False) for i in range(n)]
    for st in states:
        for k in ("mom", "var", "left", "right"):
            st[k][:] = 0
    params = [W.gen_param(70, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=1, refresh=True)
    dev = SoapDevice(canz, rows, cols, grads, states, outs=params)
    run(canz, [dev], hp)
    for i in range(n):
        assert np.array_equal(dev.out_host(i), widen(params[i]))
        for k in ("mom", "var", "left", "right"):
            assert not dev.state_host(k, i).any(), k
        assert np.array_equal(dev.state_host("q_left", i), np.eye(rows)) and np.array_equal(dev.state_host("q_right", i), np.eye(cols))


def test_first_refresh_from_identity_bases(canz):
    """The usual start: identity bases, a few steps of statistics, then the first refresh (the QR of S itself)."""
    rows, cols, n = 264, 200, 2
    states = [W.gen_soap_state(71, i, rows, cols, identity_bases=True) for i in range(n)]
    grads = [W.gen_grad(71, i, rows, cols)[0] for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=10, refresh=True, out_mode=canz.OUT_DELTA)
    dev = SoapDevice(canz, rows, cols, grads, states)
    run(canz, [dev], hp)
    check(dev, grads, states, None, hp, "soap first refresh from identity")


def test_two_groups_in_one_call_and_batches_are_independent(canz):
    """Two shape classes in one call; each matrix's results are bit-identical to a call with that matrix alone."""
    import torch
    shapes = [(200, 136), (72, 264)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=4, refresh=True, out_mode=canz.OUT_DELTA)
    devs, alone = [], []
    for gi, (rows, cols) in enumerate(shapes):
        grads = [W.gen_grad(67, 10 * gi + i, rows, cols)[0] for i in range(3)]
        states = [W.gen_soap_state(67, 10 * gi + i, rows, cols) for i in range(3)]
        devs.append((SoapDevice(canz, rows, cols, grads, states), grads, states))
        alone.append(SoapDevice(canz, rows, cols, grads[1:2], states[1:2]))
    run(canz, [d for d, _, _ in devs], hp)
    for d, grads, states in devs:
        check(d, grads, states, None, hp, "soap two groups %dx%d" % (d.rows, d.cols))
    for (d, _, _), a in zip(devs, alone):
        run(canz, [a], hp)
        for key in STATE_KEYS:
            assert torch.equal(d.t[key][1], a.t[key][0]), "%s differs between the batch and the matrix alone" % key
        assert torch.equal(d.out_t[1], a.out_t[0])


@pytest.mark.parametrize("bf16_rot", [False, True], ids=["fp32", "bf16-rotations"])
def test_like_shaped_groups_of_a_call_are_merged_and_unchanged(canz, bf16_rot):
    """Three groups in one call, the first two of one shape (the library runs them as one launch batch), the third of
    another; every matrix's state, output and kept rotated momentum are bit-identical to a call with its own group alone."""
    import torch
    shapes = [(264, 136), (264, 136), (136, 264)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=4, refresh=True, bf16_rotations=bf16_rot)

    def build():
        out = []
        for gi, (rows, cols) in enumerate(shapes):
            n = 2 + gi
            grads = [W.gen_grad(84, 10 * gi + i, rows, cols)[0] for i in range(n)]
            states = [W.gen_soap_state(84, 10 * gi + i, rows, cols) for i in range(n)]
            params = [W.gen_param(84, 10 * gi + i, rows, cols) for i in range(n)]
            rot = [np.full((rows, cols), np.nan, np.float32) for _ in range(n)]
            out.append((SoapDevice(canz, rows, cols, grads, states, outs=params, mom_rot=rot), grads, states, params))
        return out

    together, apart = build(), build()
    run(canz, [d for d, _, _, _ in together], hp)
    for d, _, _, _ in apart:
        run(canz, [d], hp)
    for (d, grads, states, params), (a, _, _, _) in zip(together, apart):
        for key in STATE_KEYS:
            for i in range(d.n):
                assert torch.equal(d.t[key][i], a.t[key][i]), "%s of matrix %d differs between one call and three" % (key, i)
        for i in range(d.n):
            assert torch.equal(d.out_t[i], a.out_t[i]) and torch.equal(d.mom_rot_t[i], a.mom_rot_t[i])
        if not bf16_rot:
            check(d, grads, states, params, hp, "soap merged groups %dx%d" % (d.rows, d.cols))


def test_more_matrices_than_one_launch_batch_holds(canz):
    """140 small matrices in two like-shaped groups of 70: the library merges them and cuts the 140 into launch batches
    of 128 and 12 (a pointer table holds 128 buffers).  A refresh step; every matrix against the oracle."""
    rows, cols, n = 40, 24, 70
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=10, refresh=True, out_mode=canz.OUT_DELTA)
    devs, ins = [], []
    for k in range(2):
        grads = [W.gen_grad(87, 100 * k + i, rows, cols)[0] for i in range(n)]
        states = [W.gen_soap_state(87, 100 * k + i, rows, cols) for i in range(n)]
        devs.append(SoapDevice(canz, rows, cols, grads, states))
        ins.append((grads, states))
    run(canz, devs, hp)
    for k, d in enumerate(devs):
        check(d, ins[k][0], ins[k][1], None, hp, "soap 2 x 70 matrices of 40x24, group %d" % k)


def test_config2_shape_with_refresh(canz):
    """Four 2048 x 1024 matrices (the 0.6B-shaped share's shape): state and update of every matrix against the oracle,
    refreshed bases of the first one against the oracle's QR, properties on all."""
    rows, cols, n = 2048, 1024, 4
    grads = [W.gen_grad(2, i, rows, cols)[0] for i in range(n)]
    states = [W.gen_soap_state(2, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.003, eps=1e-8, step=10, refresh=True, out_mode=canz.OUT_DELTA)
    dev = SoapDevice(canz, rows, cols, grads, states)
    run(canz, [dev], hp)
    check(dev, grads, states, None, hp, "soap 2048x1024")


def test_refresh_of_a_long_side(canz):
    """3200 rows: the first panels of the left side are longer than the 3072 rows the panel kernel can hold in
    registers (they stream the rows beyond the first 2048 from memory), the next ones use the 12-slot variant, the last ones the
    8-slot one; all three against the oracle's QR."""
    rows, cols, n = 3200, 384, 2
    grads = [W.gen_grad(69, i, rows, cols)[0] for i in range(n)]
    states = [W.gen_soap_state(69, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.003, eps=1e-8, step=20, refresh=True, out_mode=canz.OUT_DELTA)
    dev = SoapDevice(canz, rows, cols, grads, states)
    run(canz, [dev], hp)
    check(dev, grads, states, None, hp, "soap 3200x384")


def test_long_sums_take_the_symmetric_statistic_path(canz):
    """2000 x 8200 with a basis on the short side only, four matrices: the sums of G G^T are long enough for the
    library to compute the tiles on and above the diagonal only and mirror them (neither extent a multiple of the
    256-wide tiles, so diagonal and edge tiles are ragged).  Matrix 0 against the oracle in full - the statistic
    to 1e-5 and exactly symmetric - the others' statistics exactly symmetric and distinct."""
    import torch
    rows, cols, n, limit = 2000, 8200, 4, 4096
    grads = [W.gen_grad(85, i, rows, cols)[0] for i in range(n)]
    states = [{"mom": W.gen_normal_f32(85, i, 11, rows, cols, 0.02),
               "var": np.mean(np.square(W.gen_normal_f32(85, i, 12, 4 * rows, cols, 0.02)).reshape(4, rows, cols), axis=0),
               "left": W.gen_spd_f32(85, i, 13, rows, 0.02 * 0.02 * cols), "q_left": W.gen_orthogonal_f32(85, i, 15, rows),
               "right": np.zeros((1, 1), np.float32), "q_right": np.zeros((1, 1), np.float32)}      # not passed: no basis
              for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=6, out_mode=canz.OUT_DELTA, max_precond_dim=limit)
    dev = SoapDevice(canz, rows, cols, grads, states, max_precond_dim=limit)
    assert dev.use_left and not dev.use_right
    run(canz, [dev], hp)
    for i in range(1, n):
        assert torch.equal(dev.t["left"][i], dev.t["left"][i].T) and not torch.equal(dev.t["left"][i], dev.t["left"][0])
        assert bool(torch.isfinite(dev.out_t[i]).all())
    one = SoapDevice.__new__(SoapDevice)
    one.__dict__.update(dev.__dict__)
    one.n = 1
    check(one, grads[:1], states[:1], None, hp, "soap 2000x8200, left side only, symmetric statistic")


def test_config2_share_in_one_call(canz):
    """The share bench.py --optimizer soap runs by default, in its launch configuration: Algorithm 1 with W = SOAP
    FLOPs on the 0.6B-shaped set, the most loaded rank's 15 matrices of 3072 x 1024 as two micro-groups (8 + 7) in one
    call, a refresh step.  One matrix of each group is compared with the oracle in full; the others' bases are checked
    to be orthonormal and their outputs to be finite and different from one another."""
    import torch
    s = W.matrix_set(2)
    _, owner, load = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], s["n_ranks"], 1.0,
                                               cost_kind=canz.COST_SOAP_FLOPS)
    rank = int(np.argmax(load))
    groups = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, rank, max_mats=8)
    assert [len(g) for g in groups] == [8, 7] and {(s["rows"][p], s["cols"][p]) for g in groups for p in g} == {(3072, 1024)}
    rows, cols = 3072, 1024
    hp = canz.SoapHparams(lr=0.003, eps=1e-8, step=10, refresh=True, out_mode=canz.OUT_DELTA, mom_rot_valid=True)
    devs, inputs = [], []
    for g in groups:
        log("soap config 2: inputs of a group of %d" % len(g))
        grads = [W.gen_grad(2, p, rows, cols)[0] for p in g]
        states = [W.gen_soap_state(2, p, rows, cols, identity_bases=(k > 0)) for k, p in enumerate(g)]
        # the caller keeps the rotated momentum, as the benchmark does: a valid M' for every matrix
        rot = [SO.rotate_in(widen(st["mom"]), widen(st["q_left"]), widen(st["q_right"])).astype(np.float32) for st in states]
        devs.append(SoapDevice(canz, rows, cols, grads, states, mom_rot=rot))
        inputs.append((grads, states))
    run(canz, devs, hp)
    for dev, (grads, states) in zip(devs, inputs):
        for i in range(1, dev.n):
            for key, d in (("q_left", rows), ("q_right", cols)):
                q = dev.t[key][i]
                orth = float((q.T @ q - torch.eye(d, device="cuda")).abs().max())
                assert orth <= TOL_ORTH, "%s of matrix %d: Q^T Q - I = %.3g" % (key, i, orth)
            assert bool(torch.isfinite(dev.out_t[i]).all()) and not torch.equal(dev.out_t[i], dev.out_t[i - 1])
        one = SoapDevice.__new__(SoapDevice)
        one.__dict__.update(dev.__dict__)
        one.n = 1
        check(one, grads[:1], states[:1], None, hp, "soap config 2 share, group of %d, matrix 0" % dev.n)


def test_config4_share_in_one_call(canz):
    """The one-sided share bench.py --optimizer soap --config 4 --share 25600x5120x4 runs, in its launch configuration: four
    25600 x 5120 matrices in one call, one launch batch, max_precond_dim 10000 (the long side keeps no basis), a refresh step.  The first 64
    panels of the 5120-sided QR are longer than the panel kernel can hold in registers.  Matrix 0 is compared with the
    oracle in full (state, update, refreshed basis, re-rotated momentum); the bases of the others are checked to be
    orthonormal, and every output to be finite and distinct from matrix 0's.  The caller keeps the rotated momentum."""
    import torch
    rows, cols, n = 25600, 5120, 4
    log("soap config 4: inputs")
    grads = [W.gen_grad(4, i, rows, cols)[0] for i in range(n)]
    states = []
    for i in range(n):
        st = {"mom": W.gen_normal_f32(4, i, 11, rows, cols, 0.02),
              "var": np.mean(np.square(W.gen_normal_f32(4, i, 12, 2 * rows, cols, 0.02)).reshape(2, rows, cols), axis=0),
              "left": np.zeros((1, 1), np.float32), "q_left": np.zeros((1, 1), np.float32),      # not passed: no basis
              "right": W.gen_spd_f32(4, i, 14, cols, 0.02 * 0.02 * rows), "q_right": W.gen_orthogonal_f32(4, i, 16, cols)}
        states.append(st)
    hp = canz.SoapHparams(lr=0.003, eps=1e-8, step=10, refresh=True, out_mode=canz.OUT_DELTA, max_precond_dim=10000,
                          mom_rot_valid=True)
    rot = [SO.rotate_in(widen(st["mom"]), None, widen(st["q_right"])).astype(np.float32) for st in states]
    dev = SoapDevice(canz, rows, cols, grads, states, max_precond_dim=10000, mom_rot=rot)
    assert not dev.use_left and dev.use_right
    log("soap config 4: device step")
    run(canz, [dev], hp)
    for i in range(1, n):
        q = dev.t["q_right"][i]
        orth = float((q.T @ q - torch.eye(cols, device="cuda")).abs().max())
        assert orth <= TOL_ORTH, "basis of matrix %d: Q^T Q - I = %.3g" % (i, orth)
        assert bool(torch.isfinite(dev.out_t[i]).all()) and not torch.equal(dev.out_t[i], dev.out_t[0])
    log("soap config 4: oracle on matrix 0 (fp64)")
    one = SoapDevice.__new__(SoapDevice)
    one.__dict__.update(dev.__dict__)
    one.n = 1
    check(one, grads[:1], states[:1], None, hp, "soap 25600x5120, right side only")


# ---- rotations on bf16 operands (hparams.bf16_rotations) -------------------------------------------------------
# Each operand of the rotation products is rounded to bf16 once (relative error up to 2^-9 per element, 2.3e-3 rms):
# the bases, G (exact if it arrives as bf16), M, N' and the intermediate of a two-sided rotation.  So G' and M' carry
# a few 1e-3 of relative error (an orthogonal map carries the rounding error of its operand over at full size:
# about 1.7e-3 rms per rounded operand), V twice G's times 1 - beta2, and the update the sum of what M', V and the back
# rotation add.  A kept M' that follows its own recurrence takes 1 - beta1 of G's error per step (measured 1.3e-4
# to 1.8e-4); one that is rotated as a whole - on a step that does not take it from the caller, and after a
# refresh - carries the roundings of M, the bases and the intermediate (measured 3.3e-3).  The tolerances are three
# times what the cases below measure; momentum, statistics and a refreshed basis do not pass through bf16 and
# keep their fp32 tolerances.
TOL16_UPDATE, TOL16_VAR, TOL16_MOM_ROT, TOL16_MOM_ROT_WHOLE = 1.5e-2, 1.5e-3, 6e-4, 1e-2


@pytest.mark.parametrize("keep_rot", [False, True], ids=["rotate", "kept"])
@pytest.mark.parametrize("shape,limit", [((300, 77), 10000), ((77, 300), 10000), ((520, 1032), 10000), ((256, 256), 10000),
                                         ((130, 1), 10000), ((300, 100), 128), ((100, 300), 128)],
                         ids=lambda v: str(v).replace(" ", ""))
def test_bf16_rotations_one_step(canz, shape, limit, keep_rot):
    """Two-sided and one-sided (either side), ragged against the 256-wide padding of the bf16 operands; with the rotated
    momentum kept the caller hands in a valid M' and the step updates it by its own recurrence from the bf16 G'."""
    rows, cols = shape
    n = 3
    grads = [W.gen_grad(80, i, rows, cols)[0] for i in range(n)]
    states = [W.gen_soap_state(80, i, rows, cols) for i in range(n)]
    params = [W.gen_param(80, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, weight_decay=0.1, eps=1e-8, step=7, max_precond_dim=limit, mom_rot_valid=keep_rot,
                          bf16_rotations=True)
    rot = None
    if keep_rot:
        rot = [SO.rotate_in(widen(st["mom"]), widen(st["q_left"]) if rows <= limit else None,
                            widen(st["q_right"]) if cols <= limit else None).astype(np.float32) for st in states]
    dev = SoapDevice(canz, rows, cols, grads, states, outs=params, max_precond_dim=limit, mom_rot=rot)
    run(canz, [dev], hp)
    check(dev, grads, states, params, hp, "soap bf16 rotations %dx%d limit %d" % (rows, cols, limit), tol_update=TOL16_UPDATE,
          tol_var=TOL16_VAR, tol_mom_rot=TOL16_MOM_ROT)


def test_bf16_rotations_refresh_tp_fragments(canz):
    """A refresh step with fp32 gradient fragments and Delta W fragments out: statistics and the new bases come from the
    fp32 path and keep its tolerances; the rotated momentum is left in the new bases by bf16 products as well."""
    rows, cols, tp, n = 136, 256, 4, 3
    grads = [W.split_columns(W.gen_grad(81, i, rows, cols, dtype=W.DT_F32)[0], tp) for i in range(n)]
    states = [W.gen_soap_state(81, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=3, refresh=True, out_mode=canz.OUT_DELTA, bf16_rotations=True)
    dev = SoapDevice(canz, rows, cols, grads, states, tp=tp, mom_rot=[np.full((rows, cols), np.nan, np.float32) for _ in range(n)])
    run(canz, [dev], hp)
    check(dev, grads, states, None, hp, "soap bf16 rotations, refresh, tp=4", tol_update=TOL16_UPDATE, tol_var=TOL16_VAR,
          tol_mom_rot=TOL16_MOM_ROT_WHOLE)


def test_bf16_rotations_first_step_and_zero_gradient(canz):
    """The two degenerate inputs in the bf16 mode.  A first step from M = V = 0 is N' = g' / (|g'| sqrt(c) + eps): where
    |g'| is below the rounding the rotation adds (some 3e-3 of the typical size) the value is wrong by up to its own
    size, however the rotation is rounded, so the error of the update is that share of the elements (measured 0.074
    at eps = 1e-3 of the gradient scale, tolerance 0.15; V, which is (1 - beta2) g'^2 with no history to dilute
    the rounding, 4.7e-3) - a property of the step, stated in the header.  A zero
    gradient from an empty state leaves everything zero."""
    rows, cols, n = 200, 136, 2
    grads = [W.gen_grad(86, i, rows, cols)[0] for i in range(n)]
    states = [W.gen_soap_state(86, i, rows, cols) for i in range(n)]
    for st in states:
        for k in ("mom", "var", "left", "right"):
            st[k][:] = 0
    hp = canz.SoapHparams(lr=0.01, eps=2e-5, step=1, out_mode=canz.OUT_DELTA, bf16_rotations=True)
    dev = SoapDevice(canz, rows, cols, grads, states)
    run(canz, [dev], hp)
    check(dev, grads, states, None, hp, "soap bf16 rotations, first step", tol_update=0.15, tol_var=TOL16_VAR * 20)
    zero = [np.zeros((rows, cols), np.uint16) for _ in range(n)]
    params = [W.gen_param(86, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=1, refresh=True, bf16_rotations=True)
    dev = SoapDevice(canz, rows, cols, zero, states, outs=params, mom_rot=[np.full((rows, cols), np.nan, np.float32) for _ in range(n)])
    run(canz, [dev], hp)
    for i in range(n):
        assert np.array_equal(dev.out_host(i), widen(params[i]))
        for k in ("mom", "var", "left", "right"):
            assert not dev.state_host(k, i).any(), k
        assert not to_host64(dev.mom_rot_t[i]).any()
        assert np.array_equal(dev.state_host("q_left", i), np.eye(rows)) and np.array_equal(dev.state_host("q_right", i), np.eye(cols))


@pytest.mark.parametrize("shape,limit", [((264, 200), 10000), ((300, 100), 128), ((100, 300), 128)], ids=lambda v: str(v).replace(" ", ""))
def test_bf16_rotations_refresh_with_kept_rotated_momentum(canz, shape, limit):
    """A refresh step of the steady state (the caller's M' is valid on entry), two-sided and one-sided: bf16 gradients, so
    the statistics come from the bf16 matrix cores; after the refresh M' is rotated into the new bases."""
    rows, cols = shape
    n = 2
    grads = [W.gen_grad(83, i, rows, cols)[0] for i in range(n)]
    states = [W.gen_soap_state(83, i, rows, cols) for i in range(n)]
    params = [W.gen_param(83, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=10, refresh=True, max_precond_dim=limit, mom_rot_valid=True, bf16_rotations=True)
    rot = [SO.rotate_in(widen(st["mom"]), widen(st["q_left"]) if rows <= limit else None,
                        widen(st["q_right"]) if cols <= limit else None).astype(np.float32) for st in states]
    dev = SoapDevice(canz, rows, cols, grads, states, outs=params, max_precond_dim=limit, mom_rot=rot)
    run(canz, [dev], hp)
    check(dev, grads, states, params, hp, "soap bf16 rotations, refresh, kept M', %dx%d limit %d" % (rows, cols, limit),
          tol_update=TOL16_UPDATE, tol_var=TOL16_VAR, tol_mom_rot=TOL16_MOM_ROT_WHOLE)


def test_bf16_rotations_config2_shape(canz):
    """Eight matrices of 3072 x 1024 (one micro-group of the default benchmark share) with the rotated momentum kept;
    matrix 0 against the oracle, the others finite and distinct."""
    import torch
    rows, cols, n = 3072, 1024, 8
    grads = [W.gen_grad(82, i, rows, cols)[0] for i in range(n)]
    states = [W.gen_soap_state(82, i, rows, cols) for i in range(n)]
    rot = [SO.rotate_in(widen(st["mom"]), widen(st["q_left"]), widen(st["q_right"])).astype(np.float32) for st in states]
    hp = canz.SoapHparams(lr=0.003, eps=1e-8, step=10, out_mode=canz.OUT_DELTA, mom_rot_valid=True, bf16_rotations=True)
    dev = SoapDevice(canz, rows, cols, grads, states, mom_rot=rot)
    run(canz, [dev], hp)
    for i in range(1, n):
        assert bool(torch.isfinite(dev.out_t[i]).all()) and not torch.equal(dev.out_t[i], dev.out_t[i - 1])
    one = SoapDevice.__new__(SoapDevice)
    one.__dict__.update(dev.__dict__)
    one.n = 1
    check(one, grads[:1], states[:1], None, hp, "soap bf16 rotations 3072x1024", tol_update=TOL16_UPDATE, tol_var=TOL16_VAR,
          tol_mom_rot=TOL16_MOM_ROT)


def test_config4_planner_share_in_one_call(canz):
    """The share bench.py --optimizer soap --config 4 runs, in its launch configuration: Algorithm 1 with W = SOAP FLOPs
    on the 32B-shaped set gives the most loaded rank six matrices of 8192 x 5120, both sides with a basis; one call, one
    launch batch, a refresh step with the caller's rotated momentum valid.  The 8192-sided QR has 64 blocks of four
    panels, the first 160 panels longer than the panel kernel holds in registers.  Identity bases on entry (random ones
    of this size take the host a long time to draw; the 0.6B-shaped share's test has them): matrix 0 against the oracle in
    full, the others orthonormal, finite and distinct."""
    import torch
    s = W.matrix_set(4)
    _, owner, load = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], s["n_ranks"], 1.0,
                                               cost_kind=canz.COST_SOAP_FLOPS)
    rank = int(np.argmax(load))
    groups = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, rank, max_mats=8)
    assert [len(g) for g in groups] == [6] and {(s["rows"][p], s["cols"][p]) for p in groups[0]} == {(8192, 5120)}
    rows, cols, n = 8192, 5120, 6
    log("soap config 4 (planner share): inputs")
    grads = [W.gen_grad(4, p, rows, cols)[0] for p in groups[0]]
    # matrices 2 .. 5 start from the same state as matrix 1 (their gradients differ): the seeded 8192-sided statistics
    # take seconds each to draw on the host
    states = [W.gen_soap_state(4, groups[0][k], rows, cols, identity_bases=True) if k < 2 else None for k in range(n)]
    states = [st if st is not None else states[1] for st in states]
    rot = [st["mom"].copy() for st in states]                      # identity bases: M' = M
    hp = canz.SoapHparams(lr=0.003, eps=1e-8, step=10, refresh=True, out_mode=canz.OUT_DELTA, mom_rot_valid=True)
    dev = SoapDevice(canz, rows, cols, grads, states, mom_rot=rot)
    log("soap config 4 (planner share): device step")
    run(canz, [dev], hp)
    for i in range(1, n):
        for key, d in (("q_left", rows), ("q_right", cols)):
            q = dev.t[key][i].double()      # measured in fp64: an fp32 product of 8192 terms rounds at the tolerance itself
            orth = float((q.T @ q - torch.eye(d, device="cuda", dtype=torch.float64)).abs().max())
            assert orth <= TOL_ORTH, "%s of matrix %d: Q^T Q - I = %.3g" % (key, i, orth)
        assert bool(torch.isfinite(dev.out_t[i]).all()) and not torch.equal(dev.out_t[i], dev.out_t[i - 1])
    log("soap config 4 (planner share): oracle on matrix 0 (fp64)")
    one = SoapDevice.__new__(SoapDevice)
    one.__dict__.update(dev.__dict__)
    one.n = 1
    check(one, grads[:1], states[:1], None, hp, "soap 6 x 8192x5120, matrix 0")


@pytest.mark.parametrize("bf16_rot", [False, True], ids=["fp32", "bf16-rotations"])
@pytest.mark.parametrize("refresh", [False, True], ids=["plain", "refresh"])
def test_step_under_graph_capture_replays(canz, refresh, bf16_rot):
    """A step (plain, and with the basis refresh: a few hundred more kernels, one of them the fill of Q^T, no memset)
    captured in a HIP graph: three replays with eager work in between, each compared bit for bit with the eager
    result of the same step from the same state."""
    import torch
    rows, cols, n = 200, 136, 2
    grads = [W.gen_grad(68, i, rows, cols)[0] for i in range(n)]
    states = [W.gen_soap_state(68, i, rows, cols) for i in range(n)]
    hp = canz.SoapHparams(lr=0.01, eps=1e-8, step=3, out_mode=canz.OUT_DELTA, refresh=refresh, bf16_rotations=bf16_rot)
    eager = SoapDevice(canz, rows, cols, grads, states)
    run(canz, [eager], hp)
    dev = SoapDevice(canz, rows, cols, grads, states)
    groups = [dev.group()]
    nbytes = canz.canz_soap_workspace_bytes(groups, hp)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    saved = {k: [t.clone() for t in dev.t[k]] for k in STATE_KEYS}
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            canz.canz_soap_step(groups, hp, ws, nbytes, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for replay in range(3):
        for k, ts in saved.items():
            for dst, src in zip(dev.t[k], ts):
                dst.copy_(src)
        for o in dev.out_t:
            o.zero_()
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i in range(n):
            assert torch.equal(dev.out_t[i], eager.out_t[i]), "replay %d: Delta W differs from the eager step" % replay
            for k in saved:
                assert torch.equal(dev.t[k][i], eager.t[k][i]), "replay %d: %s differs" % (replay, k)
