"""GPU parity: canz_muon_step through the C ABI against the fp64 oracle, element by
element, on seeded inputs small enough for the oracle yet spanning several tiles and
ragged tails, plus the degenerate cases.  Tolerances (per matrix, relative Frobenius
error on Delta W): 3e-2 in bf16 mode, 1e-4 in fp32 verification mode; momentum 1e-6."""
import numpy as np
import pytest

from oracle import muon as OM
from paper_2602_06079_amd import workloads as W
from tests.gpu_harness import DeviceGroup, log, oracle_hparams, rel_fro, run_step, widen

pytestmark = pytest.mark.gpu

TOL = {0: 3e-2, 1: 1e-4}      # by precision code
TOL_MOM = 1e-6


def _check_group(canz, dg, grads, moms, params, hp, label):
    """Oracle on the same inputs; returns the worst errors."""
    ohp = oracle_hparams(hp)
    worst = 0.0
    for i in range(dg.n):
        g = grads[i]
        g64 = [widen(f) for f in g] if isinstance(g, (list, tuple)) else widen(g)
        ref = OM.muon_step(g64, widen(moms[i]), ohp, param=None if params is None else widen(params[i]))
        e_mom = rel_fro(dg.mom_host(i), ref["mom"])
        assert e_mom <= TOL_MOM, "%s: momentum of matrix %d off by %.3g" % (label, i, e_mom)
        got = dg.out_host(i)
        if params is None:
            err = rel_fro(got, ref["delta"])
        else:
            den = np.linalg.norm(ref["delta"])
            err = np.linalg.norm(got - ref["param"]) / den if den > 0 else np.linalg.norm(got - ref["param"])
        assert np.isfinite(got).all()
        assert err <= TOL[hp.precision], "%s: matrix %d error %.3g" % (label, i, err)
        worst = max(worst, err)
    log("%s: worst error %.3g (tol %.1g)" % (label, worst, TOL[hp.precision]))
    return worst


@pytest.mark.parametrize("precision", [0, 1])
def test_config1_tiny_two_steps(canz, precision):
    """Config 1: 8 fp32 matrices of 256 x 512, beta 0.95, 5 quintic steps; a second step
    with fresh gradients exercises the momentum recurrence."""
    s = W.matrix_set(1)
    n = len(s["rows"])
    grads = [W.gen_grad(1, i, 256, 512)[0] for i in range(n)]
    moms = [np.zeros((256, 512), np.float32) for _ in range(n)]
    hp = canz.Hparams(precision=precision, out_mode=canz.OUT_DELTA)
    dg = DeviceGroup(canz, 256, 512, grads, moms, outs=None)
    ws = run_step(canz, [dg], hp)
    _check_group(canz, dg, grads, moms, None, hp, "cfg1 step1 prec%d" % precision)
    moms2 = [dg.mom_host(i).astype(np.float32) for i in range(n)]
    grads2 = [W.gen_grad(1, i, 256, 512, step=1)[0] for i in range(n)]
    dg.set_grads(grads2)
    run_step(canz, [dg], hp, ws)
    _check_group(canz, dg, grads2, moms2, None, hp, "cfg1 step2 prec%d" % precision)


RAGGED = [(300, 77), (77, 300), (200, 333), (513, 257), (64, 1000), (256, 256), (1, 9), (520, 1032)]


@pytest.mark.parametrize("precision", [0, 1])
@pytest.mark.parametrize("shape", RAGGED, ids=lambda s: "%dx%d" % s)
def test_ragged_shapes_in_place_params(canz, shape, precision):
    """Shapes that do not fill the 256-wide tiles, tall and wide, unaligned columns;
    parameters updated in place with weight decay."""
    rows, cols = shape
    n = 3
    grads = [W.gen_grad(90, i, rows, cols)[0] for i in range(n)]
    moms = [W.gen_normal_f32(90, i, 3, rows, cols, 0.01) for i in range(n)]
    params = [W.gen_param(90, i, rows, cols) for i in range(n)]
    hp = canz.Hparams(precision=precision, out_mode=canz.OUT_PARAM, weight_decay=0.1, lr=0.05)
    dg = DeviceGroup(canz, rows, cols, grads, moms, outs=params)
    run_step(canz, [dg], hp)
    _check_group(canz, dg, grads, moms, params, hp, "ragged %dx%d prec%d" % (rows, cols, precision))


@pytest.mark.parametrize("precision", [0, 1])
def test_fp32_gradients_and_bf16_params(canz, precision):
    rows, cols = 384, 640
    grads = [W.gen_grad(91, i, rows, cols, dtype=W.DT_F32)[0] for i in range(2)]
    moms = [np.zeros((rows, cols), np.float32) for _ in range(2)]
    params = [W.f32_to_bf16_bits(W.gen_param(91, i, rows, cols, std=0.5)) for i in range(2)]
    hp = canz.Hparams(precision=precision, out_mode=canz.OUT_PARAM, lr=0.5)
    dg = DeviceGroup(canz, rows, cols, grads, moms, outs=params)
    run_step(canz, [dg], hp)
    # the bf16 store of the parameter adds up to 2^-9 relative rounding of |P| ~ 0.5
    ohp = oracle_hparams(hp)
    for i in range(2):
        ref = OM.muon_step(widen(grads[i]), widen(moms[i]), ohp, param=widen(params[i]))
        got = dg.out_host(i)
        assert np.max(np.abs(got - ref["param"])) <= 2.0 ** -8 * np.max(np.abs(ref["param"])) + \
            TOL[precision] * np.max(np.abs(ref["delta"])) * 4


@pytest.mark.parametrize("precision", [0, 1])
def test_decaying_spectrum(canz, precision):
    """A strong low-rank part plus weak noise: small and large singular values together."""
    rows, cols = 512, 1024
    grads = [W.gen_grad_decaying(92, i, rows, cols)[0] for i in range(2)]
    moms = [np.zeros((rows, cols), np.float32) for _ in range(2)]
    hp = canz.Hparams(precision=precision, out_mode=canz.OUT_DELTA)
    dg = DeviceGroup(canz, rows, cols, grads, moms)
    run_step(canz, [dg], hp)
    _check_group(canz, dg, grads, moms, None, hp, "decaying prec%d" % precision)


@pytest.mark.parametrize("precision", [0, 1])
def test_tp_fragments_gather_scatter(canz, precision):
    """Config 5 in miniature: gradients as 4 column fragments, Delta W scattered back to
    bf16 fragments.  Must equal the whole-matrix run bit for bit and match the oracle."""
    rows, cols, tp, n = 320, 768, 4, 3
    whole = [W.gen_grad(93, i, rows, cols)[0] for i in range(n)]
    frags = [W.split_columns(w, tp) for w in whole]
    moms = [W.gen_normal_f32(93, i, 3, rows, cols, 0.01) for i in range(n)]
    hp = canz.Hparams(precision=precision, out_mode=canz.OUT_DELTA)
    a = DeviceGroup(canz, rows, cols, frags, moms, tp=tp, out_np_dtype=np.uint16)
    b = DeviceGroup(canz, rows, cols, whole, moms, tp=1, out_np_dtype=np.uint16)
    run_step(canz, [a], hp)
    run_step(canz, [b], hp)
    for i in range(n):
        assert np.array_equal(a.out_host(i), b.out_host(i))
        assert np.array_equal(a.mom_host(i), b.mom_host(i))
    ohp = oracle_hparams(hp)
    for i in range(n):
        ref = OM.muon_step([widen(f) for f in frags[i]], widen(moms[i]), ohp)
        assert rel_fro(a.mom_host(i), ref["mom"]) <= TOL_MOM
        # bf16 output rounding (2^-9 per element) on top of the computation's tolerance
        assert rel_fro(a.out_host(i), ref["delta"]) <= TOL[precision] + 2.0 ** -8


def test_batch_independence_and_determinism(canz):
    """A matrix alone and inside a batch of 8 gives bit-identical output (the result does
    not depend on partition, grouping or batch order), and repeated runs agree bit for bit."""
    rows, cols, n = 512, 768, 8
    grads = [W.gen_grad(94, i, rows, cols)[0] for i in range(n)]
    zeros = [np.zeros((rows, cols), np.float32) for _ in range(n)]
    hp = canz.Hparams(out_mode=canz.OUT_DELTA)
    outs = []
    for _ in range(3):
        dg = DeviceGroup(canz, rows, cols, grads, zeros)
        run_step(canz, [dg], hp)
        outs.append([dg.out_host(i) for i in range(n)])
    for k in (1, 2):
        for i in range(n):
            assert np.array_equal(outs[0][i], outs[k][i])
    for i in (0, 5):
        solo = DeviceGroup(canz, rows, cols, [grads[i]], [zeros[i]])
        run_step(canz, [solo], hp)
        assert np.array_equal(solo.out_host(0), outs[0][i])
    # reversed batch order, and split across two groups in one call
    rev = DeviceGroup(canz, rows, cols, grads[::-1], zeros)
    run_step(canz, [rev], hp)
    for i in range(n):
        assert np.array_equal(rev.out_host(n - 1 - i), outs[0][i])
    g1 = DeviceGroup(canz, rows, cols, grads[:3], zeros[:3])
    g2 = DeviceGroup(canz, rows, cols, grads[3:], zeros[3:])
    run_step(canz, [g1, g2], hp)
    for i in range(n):
        got = g1.out_host(i) if i < 3 else g2.out_host(i - 3)
        assert np.array_equal(got, outs[0][i])


@pytest.mark.parametrize("precision", [0, 1])
def test_group_larger_than_launch_batch(canz, precision):
    """150 matrices in one group: split internally into launches of at most 128 (in bf16 mode
    the two launch batches, 128 + 22, then share their Gram, polynomial and update launches).
    Matrices on both sides of the cut also give the same bits as when run alone."""
    rows, cols, n = 256, 256, 150
    grads = [W.gen_grad(95, i, rows, cols)[0] for i in range(n)]
    zeros = [np.zeros((rows, cols), np.float32) for _ in range(n)]
    hp = canz.Hparams(out_mode=canz.OUT_DELTA, precision=precision)
    dg = DeviceGroup(canz, rows, cols, grads, zeros)
    run_step(canz, [dg], hp)
    _check_group(canz, dg, grads, zeros, None, hp, "150-matrix group prec%d" % precision)
    for i in (0, 127, 128, 149):
        solo = DeviceGroup(canz, rows, cols, [grads[i]], [zeros[i]])
        run_step(canz, [solo], hp)
        assert np.array_equal(solo.out_host(0), dg.out_host(i))


@pytest.mark.parametrize("precision", [0, 1])
def test_zero_steps_reduces_to_normalised_gradient(canz, precision):
    """beta = 0 and no Newton-Schulz step: Delta W = -lr * scale * G / (||G|| + eps)."""
    for rows, cols in ((130, 300), (300, 130)):
        grads = [W.gen_grad(96, 0, rows, cols, dtype=W.DT_F32)[0]]
        moms = [W.gen_normal_f32(96, 0, 3, rows, cols, 1.0)]
        hp = canz.Hparams(precision=precision, out_mode=canz.OUT_DELTA, beta=0.0, ns_steps=0, lr=0.5,
                          scale_mode=canz.SCALE_ASPECT)
        dg = DeviceGroup(canz, rows, cols, grads, moms)
        run_step(canz, [dg], hp)
        g = grads[0].astype(np.float64)
        want = -0.5 * np.sqrt(max(1.0, rows / cols)) * g / (np.linalg.norm(g) + float(np.float32(1e-7)))
        tol = 1e-6 if precision == 1 else 2.0 ** -8
        assert rel_fro(dg.out_host(0), want) <= tol
        assert rel_fro(dg.mom_host(0), g) <= 1e-7


@pytest.mark.parametrize("variant", ["cubic", "nesterov", "one_step", "three_steps", "scale_none"])
def test_hyper_parameter_variants(canz, variant):
    kw = dict(cubic=dict(a=1.5, b=-0.5, c=0.0, ns_steps=8), nesterov=dict(nesterov=True),
              one_step=dict(ns_steps=1), three_steps=dict(ns_steps=3), scale_none=dict(scale_mode=0))[variant]
    for rows, cols in ((256, 640), (640, 256)):        # wide, and tall (runs transposed)
        grads = [W.gen_grad(97, i, rows, cols)[0] for i in range(2)]
        moms = [W.gen_normal_f32(97, i, 3, rows, cols, 0.02) for i in range(2)]
        for precision in (0, 1):
            hp = canz.Hparams(precision=precision, out_mode=canz.OUT_DELTA, **kw)
            dg = DeviceGroup(canz, rows, cols, grads, moms)
            run_step(canz, [dg], hp)
            _check_group(canz, dg, grads, moms, None, hp, "%s %dx%d prec%d" % (variant, rows, cols, precision))


@pytest.mark.parametrize("precision", [0, 1])
def test_zero_gradient_gives_zero_update(canz, precision):
    rows, cols = 256, 300
    grads = [np.zeros((rows, cols), np.uint16)]
    moms = [np.zeros((rows, cols), np.float32)]
    params = [W.gen_param(98, 0, rows, cols)]
    hp = canz.Hparams(precision=precision)
    dg = DeviceGroup(canz, rows, cols, grads, moms, outs=params)
    run_step(canz, [dg], hp)
    assert np.array_equal(dg.out_host(0), params[0].astype(np.float64))
    assert not dg.mom_host(0).any()


def test_workspace_is_scratch(canz):
    """Garbage in the workspace (including NaN patterns) must not leak into results."""
    import torch
    rows, cols = 300, 500
    grads = [W.gen_grad(99, 0, rows, cols)[0]]
    zeros = [np.zeros((rows, cols), np.float32)]
    hp = canz.Hparams(out_mode=canz.OUT_DELTA)
    a = DeviceGroup(canz, rows, cols, grads, zeros)
    ws = run_step(canz, [a], hp)
    ws.fill_(0xFF)
    b = DeviceGroup(canz, rows, cols, grads, zeros)
    run_step(canz, [b], hp, ws)
    assert np.array_equal(a.out_host(0), b.out_host(0))


@pytest.mark.parametrize("shape", [(8, 300000), (70000, 16), (3, 4194240 // 16)], ids=lambda s: "%dx%d" % s)
def test_extreme_aspect_ratios(canz, shape):
    """Very wide and very tall matrices: one tile row, a k range of thousands of steps (the
    Gram product of a single tile is cut along k over the whole chip) and, the other way
    round, a k range of one panel."""
    rows, cols = shape
    grads = [W.gen_grad(96, i, rows, cols)[0] for i in range(2)]
    zeros = [np.zeros((rows, cols), np.float32) for _ in range(2)]
    for precision in (0, 1):
        hp = canz.Hparams(out_mode=canz.OUT_DELTA, precision=precision)
        dg = DeviceGroup(canz, rows, cols, grads, zeros)
        run_step(canz, [dg], hp)
        _check_group(canz, dg, grads, zeros, None, hp, "%dx%d prec%d" % (rows, cols, precision))


@pytest.mark.parametrize("precision", [0, 1])
@pytest.mark.parametrize("tp", [1, 2])
def test_transposed_shapes_share_a_launch(canz, precision, tp):
    """rows x cols and cols x rows matrices are batched into the same launches (both run in
    the wide orientation): parity for each, and the same bits as when run on their own."""
    shapes = [(320, 208, 3), (208, 320, 2), (320, 208, 1)]
    hp = canz.Hparams(out_mode=canz.OUT_DELTA if tp > 1 else canz.OUT_PARAM, precision=precision)

    def make(k):
        rows, cols, n = shapes[k]
        whole = [W.gen_grad(97 + k, i, rows, cols)[0] for i in range(n)]
        grads = [W.split_columns(g, tp) for g in whole] if tp > 1 else whole
        moms = [W.gen_normal_f32(97 + k, i, 5, rows, cols, 0.01) for i in range(n)]
        params = None if tp > 1 else [W.gen_param(97 + k, i, rows, cols) for i in range(n)]
        dg = DeviceGroup(canz, rows, cols, grads, moms, outs=params, tp=tp)
        return dg, grads, moms, params

    together = [make(k) for k in range(3)]
    run_step(canz, [t[0] for t in together], hp)
    for k, (dg, grads, moms, params) in enumerate(together):
        _check_group(canz, dg, grads, moms, params, hp, "merged batch, group %d, tp %d, prec %d" % (k, tp, precision))
    for k in range(3):
        alone = make(k)[0]
        run_step(canz, [alone], hp)
        for i in range(alone.n):
            assert np.array_equal(alone.out_host(i), together[k][0].out_host(i))
            assert np.array_equal(alone.mom_host(i), together[k][0].mom_host(i))


@pytest.mark.parametrize("precision", [0, 1])
def test_groups_of_different_shapes_share_launches(canz, precision):
    """Six small shape classes in one call: in bf16 mode their Gram, polynomial and update
    products run four classes to a launch.  Parity for each, and the same bits as alone."""
    shapes = [(300, 200, 3), (520, 1032, 2), (64, 1000, 2), (1000, 64, 1), (256, 256, 2), (130, 770, 1)]
    hp = canz.Hparams(out_mode=canz.OUT_PARAM, precision=precision, weight_decay=0.1)

    def make(k):
        rows, cols, n = shapes[k]
        grads = [W.gen_grad(60 + k, i, rows, cols)[0] for i in range(n)]
        moms = [W.gen_normal_f32(60 + k, i, 5, rows, cols, 0.01) for i in range(n)]
        params = [W.gen_param(60 + k, i, rows, cols) for i in range(n)]
        return DeviceGroup(canz, rows, cols, grads, moms, outs=params), grads, moms, params

    together = [make(k) for k in range(len(shapes))]
    run_step(canz, [t[0] for t in together], hp)
    for k, (dg, grads, moms, params) in enumerate(together):
        _check_group(canz, dg, grads, moms, params, hp, "mixed shapes, group %d, prec %d" % (k, precision))
    for k in range(len(shapes)):
        alone = make(k)[0]
        run_step(canz, [alone], hp)
        for i in range(alone.n):
            assert np.array_equal(alone.out_host(i), together[k][0].out_host(i))
            assert np.array_equal(alone.mom_host(i), together[k][0].mom_host(i))


@pytest.mark.parametrize("precision", [0, 1])
@pytest.mark.parametrize("log2_scale", [-40, 40])
def test_gradient_magnitudes_far_from_one(canz, precision, log2_scale):
    """Gradients scaled by 2^-40 and 2^+40 (exact in bf16): inside the documented magnitude range
    the step still matches the oracle, which carries the same eps in the normalisation (at
    2^-40 the norm is below eps and the update shrinks accordingly on both sides)."""
    rows, cols, n = 300, 520, 2
    scale = np.float32(2.0 ** log2_scale)
    grads = [W.f32_to_bf16_bits(W.bf16_bits_to_f32(W.gen_grad(89, i, rows, cols)[0]) * scale) for i in range(n)]
    zeros = [np.zeros((rows, cols), np.float32) for _ in range(n)]
    hp = canz.Hparams(out_mode=canz.OUT_DELTA, precision=precision)
    dg = DeviceGroup(canz, rows, cols, grads, zeros)
    run_step(canz, [dg], hp)
    _check_group(canz, dg, grads, zeros, None, hp, "scale 2^%d prec%d" % (log2_scale, precision))


def test_shared_launches_split_between_large_and_small_tiles(canz):
    """Two shape classes whose launch batches share launches, sized so that every shared launch
    has full rounds for the persistent 256 x 256 kernel AND left-over tiles for the 128 x 128 one
    (Gram: 120 + 180 = 300 tiles on 256 CUs, update: 240 + 360 = 600): the tile numbering runs across
    both products in both kernels.  Oracle parity on matrices of both classes, and the same bits as
    each matrix run alone (where every product runs on the small kernel only)."""
    classes = [(512, 768, 40), (768, 1024, 30)]
    hp = canz.Hparams(out_mode=canz.OUT_DELTA)
    devs, ins = [], []
    for k, (rows, cols, n) in enumerate(classes):
        grads = [W.gen_grad(70 + k, i, rows, cols)[0] for i in range(n)]
        zeros = [np.zeros((rows, cols), np.float32) for _ in range(n)]
        devs.append(DeviceGroup(canz, rows, cols, grads, zeros))
        ins.append((grads, zeros))
    run_step(canz, devs, hp)
    ohp = oracle_hparams(hp)
    for k, (rows, cols, n) in enumerate(classes):
        for i in (0, n // 2, n - 1):
            ref = OM.muon_step(widen(ins[k][0][i]), widen(ins[k][1][i]), ohp)
            err = rel_fro(devs[k].out_host(i), ref["delta"])
            assert err <= TOL[0], "class %d matrix %d: error %.3g" % (k, i, err)
            solo = DeviceGroup(canz, rows, cols, [ins[k][0][i]], [ins[k][1][i]])
            run_step(canz, [solo], hp)
            assert np.array_equal(solo.out_host(0), devs[k].out_host(i)), "class %d matrix %d differs from the run alone" % (k, i)
        for i in range(n):
            assert np.isfinite(devs[k].out_host(i)).all()
