"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times:
the planner picks the share, the micro-groups are run through canz_muon_step as
bench.py runs them, and the fp64 oracle is computed for sampled matrices of each group
(a full Newton-Schulz chain per sampled matrix; the oracle cannot sample single
elements of an orthogonalisation).  The remaining matrices are checked through
properties that hold at any size: exact momentum (element-wise, every matrix), finite
output, and the Frobenius norm implied by the quintic band.  Tolerances as in
test_gpu_muon.py."""
import numpy as np
import pytest

from oracle import muon as OM
from paper_2602_06079_amd import workloads as W
from tests.gpu_harness import DeviceGroup, log, oracle_hparams, rel_fro, run_step, widen

pytestmark = pytest.mark.gpu

TOL = {0: 3e-2, 1: 1e-4}
LR_SCALE_BAND = (0.68, 1.14)      # singular values after 5 quintic steps, inputs in [0.01, 1]


def _share(canz, cfg):
    s = W.matrix_set(cfg)
    cuts, owner, load = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], s["n_ranks"], s["alpha"])
    rank = 0 if cfg in (1, 2, 5) else int(np.argmax(load))
    groups = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, rank, max_mats=8)
    return s, groups


def _run_group(canz, cfg, s, ids, precision, sample, label, square_ok=False):
    """One micro-group as bench.py launches it; oracle on ids[k] for k in sample."""
    rows, cols, tp = s["rows"][ids[0]], s["cols"][ids[0]], s["tp"]
    log("%s: generating %d matrices of %dx%d" % (label, len(ids), rows, cols))
    grads = [W.gen_grad(cfg, p, rows, cols)[0] for p in ids]
    moms = [np.zeros((rows, cols), np.float32) for _ in ids]
    if tp > 1:
        hp = canz.Hparams(precision=precision, out_mode=canz.OUT_DELTA)
        dg = DeviceGroup(canz, rows, cols, [W.split_columns(g, tp) for g in grads], moms, tp=tp,
                         out_np_dtype=np.uint16)
        params = None
    else:
        hp = canz.Hparams(precision=precision, out_mode=canz.OUT_PARAM)
        params = [W.gen_param(cfg, p, rows, cols) for p in ids]
        dg = DeviceGroup(canz, rows, cols, grads, moms, outs=params)
    log("%s: device step" % label)
    run_step(canz, [dg], hp)
    ohp = oracle_hparams(hp)
    m = min(rows, cols)
    scale = abs(ohp.lr) * OM.update_scale(rows, cols, ohp.scale_mode)
    for k in range(len(ids)):
        g64 = widen(grads[k])
        # momentum: element-wise exact definition, every matrix (beta * 0 + G)
        assert rel_fro(dg.mom_host(k), g64) <= 1e-6
        out = dg.out_host(k)
        assert np.isfinite(out).all()
        delta = out if params is None else out - params[k].astype(np.float64)
        # all singular values of O in the band  =>  m lo^2 <= ||O||_F^2 <= m hi^2.  Square
        # Gaussian matrices have singular values near zero that are still climbing after
        # five steps, so only the upper bound applies to them.
        fro2 = float(np.sum(delta * delta)) / (scale * scale)
        assert fro2 <= m * LR_SCALE_BAND[1] ** 2 * 1.02, "%s: matrix %d norm too large" % (label, k)
        if not square_ok:
            assert fro2 >= m * LR_SCALE_BAND[0] ** 2 * 0.9, "%s: matrix %d norm too small" % (label, k)
    for k in sample:
        log("%s: oracle on matrix %d (fp64, %.1f TFLOP)" % (label, ids[k], 5 * (4 * m * m * max(rows, cols) + 2 * m ** 3) / 1e12))
        ref = OM.muon_step(widen(grads[k]), widen(moms[k]), ohp,
                           param=None if params is None else widen(params[k]))
        got = dg.out_host(k)
        if params is None:
            err = rel_fro(got, ref["delta"])
            tol = TOL[precision] + 2.0 ** -8       # bf16 rounding of the stored Delta W
        else:
            err = float(np.linalg.norm(got - ref["param"]) / np.linalg.norm(ref["delta"]))
            # fp32 parameters: |P| ~ 0.02 stored with 2^-24 relative rounding, against |Delta W| ~ lr * scale
            tol = TOL[precision] + 1e-5
        log("%s: matrix %d error %.3g (tol %.2g)" % (label, ids[k], err, tol))
        assert err <= tol, "%s: matrix %d error %.3g" % (label, ids[k], err)


@pytest.mark.parametrize("precision", [0, 1])
def test_config2_rank0_share(canz, precision):
    """Qwen3-0.6B-shaped set, R = 8, alpha = 1: rank 0 owns 26 matrices of 2048 x 1024 in
    groups of 8, 8, 8, 2; every group runs, three matrices per group are checked."""
    s, groups = _share(canz, 2)
    assert [len(g) for g in groups] == [8, 8, 8, 2]
    for gi, ids in enumerate(groups):
        _run_group(canz, 2, s, ids, precision, sample=sorted({0, len(ids) // 2, len(ids) - 1}),
                   label="cfg2 group %d prec%d" % (gi, precision))


def test_config3_heaviest_rank_first_group(canz):
    """Qwen3-8B-shaped set, R = 32, alpha = 0.1: the heaviest rank owns every layer's
    12288 x 4096 gate matrix; its first micro-group (8 matrices) runs as bench.py launches it."""
    s, groups = _share(canz, 3)
    assert [len(g) for g in groups] == [8, 8, 8, 8, 4]
    assert all((s["rows"][p], s["cols"][p]) == (12288, 4096) for g in groups for p in g)
    _run_group(canz, 3, s, groups[0], 0, sample=[3], label="cfg3 group 0")


@pytest.mark.parametrize("precision", [0, 1])
def test_config4_heaviest_rank_share(canz, precision):
    """Qwen3-32B-shaped set, R = 64: the heaviest rank's share is one micro-group of four
    25600 x 5120 matrices - exactly what bench.py times by default."""
    s, groups = _share(canz, 4)
    assert len(groups) == 1 and len(groups[0]) == 4
    _run_group(canz, 4, s, groups[0], precision, sample=[1], label="cfg4 prec%d" % precision)


def test_config5_tp_fragments_one_group_per_shape(canz):
    """The 8B set as TP = 4 column fragments: the first micro-group of each shape class
    (gather fused into the momentum pass, bf16 Delta W scattered back to fragments)."""
    s, groups = _share(canz, 5)
    assert len(groups) == 32 and sum(len(g) for g in groups) == 252
    seen = set()
    for ids in groups:
        shape = (s["rows"][ids[0]], s["cols"][ids[0]])
        if shape in seen:
            continue
        seen.add(shape)
        _run_group(canz, 5, s, ids, 0, sample=[len(ids) - 1], label="cfg5 %dx%d" % shape,
                   square_ok=shape[0] == shape[1])
    assert seen == {(4096, 4096), (1024, 4096), (12288, 4096), (4096, 12288)}
