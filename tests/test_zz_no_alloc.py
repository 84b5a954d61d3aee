"""GPU: canz_muon_step_static, the entry point that allocates nothing (its scratch is an
array inside the library), against canz_muon_step with a caller-owned workspace: same bits
for momentum and output, on two calls in a row, the second with a smaller input (the
array keeps the first call's contents and nothing may depend on them); a share above the
array's size is refused before anything is enqueued."""
import numpy as np
import pytest

from paper_2602_06079_amd import workloads as W
from tests.gpu_harness import DeviceGroup, log, run_step

pytestmark = pytest.mark.gpu


def _make(canz, seed, rows, cols, n, in_place):
    grads = [W.gen_grad(seed, i, rows, cols)[0] for i in range(n)]
    moms = [W.gen_normal_f32(seed, i, 5, rows, cols, 0.01) for i in range(n)]
    params = [W.gen_param(seed, i, rows, cols) for i in range(n)] if in_place else None
    return DeviceGroup(canz, rows, cols, grads, moms, outs=params)


@pytest.mark.parametrize("precision", [0, 1])
def test_static_workspace_matches_caller_workspace(canz, precision):
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    hp = canz.Hparams(precision=precision, out_mode=canz.OUT_PARAM, weight_decay=0.1)
    # first call: two shape classes, several tiles and ragged edges; second call: smaller
    calls = [[(70, 520, 1032, 3), (71, 300, 77, 2)], [(72, 200, 333, 2)]]
    for k, spec in enumerate(calls):
        want = [_make(canz, *sp, in_place=True) for sp in spec]
        got = [_make(canz, *sp, in_place=True) for sp in spec]
        need = canz.canz_muon_workspace_bytes([d.group() for d in want], hp)
        assert need <= canz.STATIC_WORKSPACE_BYTES
        run_step(canz, want, hp)
        log("static workspace call %d (precision %d): %d bytes of scratch" % (k, precision, need))
        canz.canz_muon_step_static([d.group() for d in got], hp, stream)
        torch.cuda.synchronize()
        for a, b in zip(want, got):
            for i in range(a.n):
                assert np.array_equal(a.mom_host(i), b.mom_host(i)), "call %d: momentum differs" % k
                assert np.array_equal(a.out_host(i), b.out_host(i)), "call %d: parameters differ" % k
        # and the step did something
        assert not np.array_equal(got[0].out_host(0), W.gen_param(spec[0][0], 0, spec[0][1], spec[0][2]).astype(np.float64))


def test_static_workspace_refuses_larger_steps(canz):
    """Above the array's size the call fails with CANZ_EWORKSPACE and enqueues nothing
    (no device buffer is touched: the tables hold small valid buffers for one matrix only,
    the size check comes before the pointer checks)."""
    hp = canz.Hparams()
    big = canz.Group(rows=4096, cols=4096, n_mats=8, grad_dtype=W.DT_BF16, out_dtype=W.DT_F32)
    assert canz.canz_muon_workspace_bytes([big], hp) > canz.STATIC_WORKSPACE_BYTES
    with pytest.raises(canz.CanzError) as e:
        canz.canz_muon_step_static([big], hp, 0)
    assert e.value.code == canz.EWORKSPACE
    # an empty call needs nothing
    canz.canz_muon_step_static([], hp, 0)
