"""GPU parity of canz_shampoo_step against the fp64 oracle (oracle/shampoo.py), through the C ABI.

Tolerances, per matrix.  Statistics L, R: 1e-5 relative Frobenius error (fp32 accumulation
of products that are exact in fp32 for bf16 gradients).  Delta W: 5e-3 relative Frobenius
error for eps >= 1e-5 lambda_max(S).  Where that figure comes from: the statistics are held in
fp32, so the eigenvalues of S + eps I near eps carry a relative perturbation of about
2^-24 lambda_max / eps, which the inverse fourth root passes on at a quarter of its size and the
multiplication by G damps again; measured on the device: 4.9e-3 at eps = 2.7e-6 lambda_max
(1024 x 4096, rank-deficient R), falling in proportion to lambda_max / eps - 2e-3 and below from
1e-5 lambda_max on, 1e-4 to 5e-4 on small Gaussian matrices.  The iteration itself converges to
2.4e-7 (residual of M - I) within 18-23 of the 25 default rounds for cond <= 1e6 and stays finite
down to eps = 1e-6 lambda_max (an fp32 emulation on the CPU shows the same figures)."""
import numpy as np
import pytest

from oracle import shampoo as SH
from paper_2602_06079_amd import workloads as W
from tests.gpu_harness import log, rel_fro, to_device, to_host64, widen

pytestmark = pytest.mark.gpu

TOL_DELTA = 5e-3
TOL_STAT = 1e-5


def oracle_hparams(hp) -> SH.Hparams:
    f = lambda v: float(np.float32(v))
    return SH.Hparams(beta=f(hp.beta), lr=f(hp.lr), weight_decay=f(hp.weight_decay), eps=f(hp.eps))


class ShampooDevice:
    """One micro-group on the device.  grads: per matrix a host array or a list of tp fragments;
    lefts / rights: fp32 host arrays; outs: parameter arrays, or None for Delta W fragments."""

    def __init__(self, canz, rows, cols, grads, lefts, rights, outs=None, tp=1, out_np_dtype=np.float32, keep_roots=False):
        import torch
        self.canz, self.rows, self.cols, self.tp, self.n = canz, rows, cols, tp, len(lefts)
        # caller-held inverse roots (NaN until a full step writes them)
        self.lroot_t = [to_device(np.full((rows, rows), np.nan, np.float32)) for _ in lefts] if keep_roots else []
        self.rroot_t = [to_device(np.full((cols, cols), np.nan, np.float32)) for _ in lefts] if keep_roots else []
        first = grads[0][0] if isinstance(grads[0], (list, tuple)) else grads[0]
        self.grad_dtype = W.DT_BF16 if first.dtype == np.uint16 else W.DT_F32
        self.grad_t = []
        for g in grads:
            frags = g if isinstance(g, (list, tuple)) else [g]
            assert len(frags) == tp
            self.grad_t += [to_device(f) for f in frags]
        self.left_t = [to_device(x) for x in lefts]
        self.right_t = [to_device(x) for x in rights]
        self.delta = outs is None
        if self.delta:
            proto = np.zeros((rows, cols // tp), dtype=out_np_dtype)
            self.out_dtype = W.DT_BF16 if proto.dtype == np.uint16 else W.DT_F32
            self.out_t = [to_device(proto) for _ in range(self.n * tp)]
        else:
            self.out_dtype = W.DT_BF16 if outs[0].dtype == np.uint16 else W.DT_F32
            self.out_t = [to_device(p) for p in outs]
        torch.cuda.synchronize()

    def group(self):
        return self.canz.ShampooGroup(rows=self.rows, cols=self.cols, grad=self.grad_t, left=self.left_t,
                                      right=self.right_t, out=self.out_t, lroot=self.lroot_t, rroot=self.rroot_t, tp=self.tp,
                                      grad_dtype=self.grad_dtype, out_dtype=self.out_dtype)

    def out_host(self, i):
        if not self.delta:
            return to_host64(self.out_t[i])
        return np.concatenate([to_host64(self.out_t[i * self.tp + f]) for f in range(self.tp)], axis=1)


def run(canz, devs, hp):
    import torch
    groups = [d.group() for d in devs]
    nbytes = canz.canz_shampoo_workspace_bytes(groups, hp)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)                                   # the workspace is scratch: NaN patterns must not leak
    canz.canz_shampoo_step(groups, hp, ws, nbytes, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()


def check(dev, grads, lefts, rights, params, hp, label, tol=TOL_DELTA):
    ohp = oracle_hparams(hp)
    worst = 0.0
    for i in range(dev.n):
        g = grads[i]
        g64 = [widen(f) for f in g] if isinstance(g, (list, tuple)) else widen(g)
        ref = SH.shampoo_step(g64, widen(lefts[i]), widen(rights[i]), ohp, param=None if params is None else widen(params[i]))
        got_l, got_r = to_host64(dev.left_t[i]), to_host64(dev.right_t[i])
        assert rel_fro(got_l, ref["left"]) <= TOL_STAT, "%s: L of matrix %d" % (label, i)
        assert rel_fro(got_r, ref["right"]) <= TOL_STAT, "%s: R of matrix %d" % (label, i)
        assert np.array_equal(got_l, got_l.T) and np.array_equal(got_r, got_r.T), "%s: statistics not symmetric" % label
        got = dev.out_host(i)
        assert np.isfinite(got).all()
        if params is None:
            err = rel_fro(got, ref["delta"])
        else:
            den = np.linalg.norm(ref["delta"])
            err = np.linalg.norm(got - ref["param"]) / den if den > 0 else np.linalg.norm(got - ref["param"])
        worst = max(worst, err)
        assert err <= tol, "%s: matrix %d error %.3g" % (label, i, err)
    log("%s: worst Delta W error %.3g (tol %.2g)" % (label, worst, tol))


RAGGED = [(300, 77), (77, 300), (200, 333), (256, 256), (130, 1), (1, 9), (520, 1032)]


@pytest.mark.parametrize("shape", RAGGED, ids=lambda s: "%dx%d" % s)
def test_ragged_shapes_from_empty_statistics(canz, shape):
    """Shapes that do not fill the 128-wide tiles, tall and wide; bf16 gradients, fp32 parameters in
    place with weight decay.  From empty statistics the update is U diag(s / sqrt(s^2 + eps)) V^T."""
    rows, cols = shape
    n = 3
    grads = [W.gen_grad(40, i, rows, cols)[0] for i in range(n)]
    lefts = [np.zeros((rows, rows), np.float32) for _ in range(n)]
    rights = [np.zeros((cols, cols), np.float32) for _ in range(n)]
    params = [W.gen_param(40, i, rows, cols) for i in range(n)]
    hp = canz.ShampooHparams(lr=0.05, weight_decay=0.1, eps=1e-5)
    dev = ShampooDevice(canz, rows, cols, grads, lefts, rights, outs=params)
    run(canz, [dev], hp)
    check(dev, grads, lefts, rights, params, hp, "shampoo ragged %dx%d" % shape)


def test_two_steps_with_decay_and_fp32_gradients(canz):
    """The state recurrence: a second step with fresh gradients on the statistics the first left."""
    rows, cols, n = 192, 320, 2
    hp = canz.ShampooHparams(beta=0.9, lr=0.1, eps=1e-4, out_mode=canz.OUT_DELTA)
    g1 = [W.gen_grad(41, i, rows, cols, dtype=W.DT_F32)[0] for i in range(n)]
    l0 = [np.eye(rows, dtype=np.float32) * np.float32(0.01) for _ in range(n)]
    r0 = [np.eye(cols, dtype=np.float32) * np.float32(0.02) for _ in range(n)]
    dev = ShampooDevice(canz, rows, cols, g1, l0, r0)
    run(canz, [dev], hp)
    check(dev, g1, l0, r0, None, hp, "shampoo step 1")
    l1 = [dev.left_t[i].cpu().numpy() for i in range(n)]
    r1 = [dev.right_t[i].cpu().numpy() for i in range(n)]
    g2 = [W.gen_grad(41, i, rows, cols, step=1, dtype=W.DT_F32)[0] for i in range(n)]
    for i in range(n):
        dev.grad_t[i].copy_(to_device(g2[i]))
    run(canz, [dev], hp)
    check(dev, g2, l1, r1, None, hp, "shampoo step 2")


def test_kept_roots_between_steps(canz):
    """The amortised variant: a full step leaves its roots with the caller (compared with the oracle's roots), the next
    step takes them from there while its statistics move on; the oracle gets the device's kept roots as they are."""
    rows, cols, n = 200, 328, 2
    g1 = [W.gen_grad(47, i, rows, cols)[0] for i in range(n)]
    l0 = [np.eye(rows, dtype=np.float32) * np.float32(0.02) for _ in range(n)]
    r0 = [np.eye(cols, dtype=np.float32) * np.float32(0.01) for _ in range(n)]
    hp = canz.ShampooHparams(beta=0.9, lr=0.1, eps=1e-3, out_mode=canz.OUT_DELTA)
    dev = ShampooDevice(canz, rows, cols, g1, l0, r0, keep_roots=True)
    run(canz, [dev], hp)
    check(dev, g1, l0, r0, None, hp, "shampoo full step with roots kept")
    ohp = oracle_hparams(hp)
    for i in range(n):
        ref = SH.shampoo_step(widen(g1[i]), widen(l0[i]), widen(r0[i]), ohp)
        for got, want in ((dev.lroot_t[i], ref["left_root"]), (dev.rroot_t[i], ref["right_root"])):
            got = to_host64(got)
            assert rel_fro(got, want) <= 1e-4 and np.abs(got - got.T).max() <= 1e-5 * np.abs(got).max()
    l1 = [dev.left_t[i].cpu().numpy() for i in range(n)]
    r1 = [dev.right_t[i].cpu().numpy() for i in range(n)]
    kept = [(to_host64(dev.lroot_t[i]), to_host64(dev.rroot_t[i])) for i in range(n)]
    g2 = [W.gen_grad(47, i, rows, cols, step=1)[0] for i in range(n)]
    for i in range(n):
        dev.grad_t[i].copy_(to_device(g2[i]))
    hp2 = canz.ShampooHparams(beta=0.9, lr=0.1, eps=1e-3, out_mode=canz.OUT_DELTA, keep_roots=True)
    run(canz, [dev], hp2)
    worst = 0.0
    for i in range(n):
        ref = SH.shampoo_step(widen(g2[i]), widen(l1[i]), widen(r1[i]), ohp, kept_roots=kept[i])
        assert rel_fro(to_host64(dev.left_t[i]), ref["left"]) <= TOL_STAT and rel_fro(to_host64(dev.right_t[i]), ref["right"]) <= TOL_STAT
        assert np.array_equal(to_host64(dev.lroot_t[i]), kept[i][0]), "a step with keep_roots must not touch the roots"
        worst = max(worst, rel_fro(dev.out_host(i), ref["delta"]))
    log("shampoo step on kept roots: worst Delta W error %.3g (tol 1e-5: two fp32 products)" % worst)
    assert worst <= 1e-5


def test_tp_fragments_equal_the_whole_matrix(canz):
    """Gradients as 4 column fragments, bf16 Delta W scattered back: same bits as the whole-matrix run."""
    rows, cols, tp, n = 160, 384, 4, 2
    whole = [W.gen_grad(42, i, rows, cols)[0] for i in range(n)]
    frags = [W.split_columns(w, tp) for w in whole]
    lefts = [np.zeros((rows, rows), np.float32) for _ in range(n)]
    rights = [np.zeros((cols, cols), np.float32) for _ in range(n)]
    hp = canz.ShampooHparams(eps=1e-5, out_mode=canz.OUT_DELTA)
    a = ShampooDevice(canz, rows, cols, frags, lefts, rights, tp=tp, out_np_dtype=np.uint16)
    b = ShampooDevice(canz, rows, cols, whole, lefts, rights, tp=1, out_np_dtype=np.uint16)
    run(canz, [a], hp)
    run(canz, [b], hp)
    for i in range(n):
        assert np.array_equal(a.out_host(i), b.out_host(i))
        assert np.array_equal(to_host64(a.left_t[i]), to_host64(b.left_t[i]))
    check(a, frags, lefts, rights, None, hp, "shampoo tp fragments", tol=TOL_DELTA + 2.0 ** -8)


def test_decaying_spectrum_and_batch_independence(canz):
    """A strong low-rank part over weak noise, several groups in one call; a matrix alone gives the
    same bits as inside its group.  lambda_max(G G^T) is about 0.02^2 * 256 * 384 = 39 here, so
    eps = 1e-3 sits at 2.5e-5 lambda_max (condition number 4e4)."""
    shapes = [(256, 384, 3), (384, 256, 2)]
    hp = canz.ShampooHparams(eps=1e-3, out_mode=canz.OUT_DELTA)
    devs, ins = [], []
    for k, (rows, cols, n) in enumerate(shapes):
        grads = [W.gen_grad_decaying(43 + k, i, rows, cols)[0] for i in range(n)]
        lefts = [np.zeros((rows, rows), np.float32) for _ in range(n)]
        rights = [np.zeros((cols, cols), np.float32) for _ in range(n)]
        devs.append(ShampooDevice(canz, rows, cols, grads, lefts, rights))
        ins.append((grads, lefts, rights))
    run(canz, devs, hp)
    for k, d in enumerate(devs):
        check(d, ins[k][0], ins[k][1], ins[k][2], None, hp, "shampoo decaying spectrum, group %d" % k)
    rows, cols, _ = shapes[0]
    solo = ShampooDevice(canz, rows, cols, [ins[0][0][1]], [ins[0][1][1]], [ins[0][2][1]])
    run(canz, [solo], hp)
    assert np.array_equal(solo.out_host(0), devs[0].out_host(1))


def test_like_shaped_groups_of_a_call_are_merged_and_unchanged(canz):
    """Three groups in one call, the first two of one shape (the library runs them as one launch batch), the third of
    another, with caller-held roots: statistics, roots and parameters are bit-identical to one call per group."""
    import torch
    shapes = [(264, 136, 2), (264, 136, 3), (136, 264, 2)]
    hp = canz.ShampooHparams(eps=1e-3)

    def build():
        out = []
        for k, (rows, cols, n) in enumerate(shapes):
            grads = [W.gen_grad(47, 10 * k + i, rows, cols)[0] for i in range(n)]
            lefts = [np.zeros((rows, rows), np.float32) for _ in range(n)]
            rights = [np.zeros((cols, cols), np.float32) for _ in range(n)]
            params = [W.gen_param(47, 10 * k + i, rows, cols) for i in range(n)]
            out.append((ShampooDevice(canz, rows, cols, grads, lefts, rights, outs=params, keep_roots=True), grads, lefts, rights, params))
        return out

    together, apart = build(), build()
    run(canz, [d for d, *_ in together], hp)
    for d, *_ in apart:
        run(canz, [d], hp)
    for (d, grads, lefts, rights, params), (a, *_) in zip(together, apart):
        for i in range(d.n):
            for got, want in ((d.left_t, a.left_t), (d.right_t, a.right_t), (d.lroot_t, a.lroot_t), (d.rroot_t, a.rroot_t), (d.out_t, a.out_t)):
                assert torch.equal(got[i], want[i]), "matrix %d differs between one call and three" % i
        check(d, grads, lefts, rights, params, hp, "shampoo merged groups %dx%d" % (d.rows, d.cols))


def test_zero_gradient_and_empty_group(canz):
    """A zero gradient on empty statistics gives a zero update (A = eps I, no NaN); empty groups are skipped."""
    import torch
    rows, cols = 130, 70
    hp = canz.ShampooHparams(eps=1e-6)
    params = [W.gen_param(44, 0, rows, cols)]
    dev = ShampooDevice(canz, rows, cols, [np.zeros((rows, cols), np.uint16)], [np.zeros((rows, rows), np.float32)],
                        [np.zeros((cols, cols), np.float32)], outs=params)
    run(canz, [dev], hp)
    assert np.array_equal(dev.out_host(0), params[0].astype(np.float64))
    assert not to_host64(dev.left_t[0]).any()
    empty = canz.ShampooGroup(rows=64, cols=64, n_mats=0)
    assert canz.canz_shampoo_workspace_bytes([empty], hp) <= 256
    canz.canz_shampoo_step([empty], hp, None, 0, torch.cuda.current_stream().cuda_stream)


def test_round_count_for_condition_1e6(canz):
    """22 rounds are what the header promises for cond(S + eps I) = 1e6: at that condition number the update after 22
    rounds must agree with the update after 40 (both at the fp32 floor of the iteration), and 12 rounds must not (so
    the case does need its rounds).  L starts with eigenvalues from 1 down to 1e-6 in a random basis; the gradient is
    small against them and has components along all of them, the smallest amplified 31-fold by the root."""
    rows, cols = 256, 320
    q = W.gen_orthogonal_f32(46, 0, 3, rows).astype(np.float64)
    left = ((q * np.logspace(0, -6, rows)) @ q.T).astype(np.float32)
    left = np.triu(left) + np.triu(left, 1).T
    right = np.eye(cols, dtype=np.float32)
    g = W.gen_grad(46, 0, rows, cols, std=1e-5, dtype=W.DT_F32)[0]
    outs = {}
    for rounds in (12, 22, 40):
        hp = canz.ShampooHparams(lr=1.0, eps=1e-7, root_iters=rounds, out_mode=canz.OUT_DELTA)
        dev = ShampooDevice(canz, rows, cols, [g], [left.copy()], [right.copy()])
        run(canz, [dev], hp)
        outs[rounds] = dev.out_host(0)
        assert np.isfinite(outs[rounds]).all()
    late = rel_fro(outs[22], outs[40])
    early = rel_fro(outs[12], outs[40])
    log("shampoo cond 1e6: 22 vs 40 rounds %.3g, 12 vs 40 rounds %.3g" % (late, early))
    assert late <= 5e-3 and early >= 0.05


def test_8b_shaped_class_1024x4096(canz):
    """The k / v projection shape of the Qwen3-8B-shaped set: a 1024 x 1024 and a 4096 x 4096 root per matrix."""
    rows, cols, n = 1024, 4096, 2
    grads = [W.gen_grad(3, 1 + 7 * i, rows, cols)[0] for i in range(n)]
    lefts = [np.zeros((rows, rows), np.float32) for _ in range(n)]
    rights = [np.zeros((cols, cols), np.float32) for _ in range(n)]
    params = [W.gen_param(3, 1 + 7 * i, rows, cols) for i in range(n)]
    # lambda_max(G G^T) ~ 0.02^2 (sqrt(4096) + sqrt(1024))^2 = 3.7; eps = 1e-4 is 2.7e-5 of that
    hp = canz.ShampooHparams(eps=1e-4)
    dev = ShampooDevice(canz, rows, cols, grads, lefts, rights, outs=params)
    log("shampoo 1024x4096: device step")
    run(canz, [dev], hp)
    log("shampoo 1024x4096: oracle (two eigendecompositions per matrix)")
    check(dev, grads, lefts, rights, params, hp, "shampoo 1024x4096")


def test_hip_graph_replay_matches_eager(canz):
    """canz_shampoo_step issues kernels only, so it can be captured; replays with eager work in
    between reproduce the eager result bit for bit (statistics and parameters)."""
    import torch
    rows, cols, n = 200, 333, 2
    hp = canz.ShampooHparams(beta=0.9, eps=1e-5)
    grads = [W.gen_grad(45, i, rows, cols)[0] for i in range(n)]
    lefts = [np.eye(rows, dtype=np.float32) * np.float32(1e-3) for _ in range(n)]
    rights = [np.eye(cols, dtype=np.float32) * np.float32(1e-3) for _ in range(n)]
    params = [W.gen_param(45, i, rows, cols) for i in range(n)]
    dev = ShampooDevice(canz, rows, cols, grads, lefts, rights, outs=params)
    groups = [dev.group()]
    state = dev.left_t + dev.right_t + dev.out_t
    saved = [t.clone() for t in state]
    nbytes = canz.canz_shampoo_workspace_bytes(groups, hp)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    canz.canz_shampoo_step(groups, hp, ws, nbytes, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = [t.clone() for t in state]
    assert any(not torch.equal(a, b) for a, b in zip(want, saved))

    def restore():
        for t, s0 in zip(state, saved):
            t.copy_(s0)

    restore()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        canz.canz_shampoo_step(groups, hp, ws, nbytes, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(state, saved))     # capture runs nothing
    for rep in range(3):
        restore()
        ws.fill_(0x5A if rep % 2 else 0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(state, want)):
            assert torch.equal(a, b), "replay %d: state tensor %d differs from the eager result" % (rep, i)
