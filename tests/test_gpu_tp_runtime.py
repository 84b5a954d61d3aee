"""GPU: the TP-scheduled execution (Sec. 4.1 stages (1)-(4); Sec. 4.2, "Integration with
Runtime Workflow"): canz_tp_schedule fixes the micro-group sequence and the host rank of
every tensor; each host rank then walks the sequence with one canz_muon_step per micro-group
(paper_2602_06079_amd.tp_runtime).  On a scaled-down 8B-shaped set held as TP = 4 column
fragments, the Delta W fragments of every tensor - computed by whichever rank hosts it, in
whichever micro-group - must match the fp64 oracle and be bit-identical to the plain run
that takes all tensors in same-shape chunks of 8 in one call."""
import numpy as np
import pytest

from oracle import muon as OM
from oracle import tp_schedule as OT
from paper_2602_06079_amd import workloads as W
from tests.gpu_harness import DeviceGroup, log, oracle_hparams, rel_fro, run_step, widen

pytestmark = pytest.mark.gpu

TP = 4
LAYERS = 6
# the 8B layer with every extent divided by 8
LAYER = [(512, 512), (128, 512), (128, 512), (512, 512), (1536, 512), (1536, 512), (512, 1536)]
CMAX = 1_600_000          # elements per host rank and micro-group
SEED = 55


def _set():
    rows = [r for _ in range(LAYERS) for r, _c in LAYER]
    cols = [c for _ in range(LAYERS) for _r, c in LAYER]
    return rows, cols


def _device(canz, rows, cols, ids):
    grads = [W.gen_grad(SEED, p, rows[ids[0]], cols[ids[0]])[0] for p in ids]
    moms = [W.gen_normal_f32(SEED, p, 5, rows[ids[0]], cols[ids[0]], 0.01) for p in ids]
    dg = DeviceGroup(canz, rows[ids[0]], cols[ids[0]], [W.split_columns(g, TP) for g in grads], moms, tp=TP,
                     out_np_dtype=np.uint16)
    return dg, grads, moms


def test_tp_schedule_walked_per_host_rank(canz):
    import torch
    from paper_2602_06079_amd import tp_runtime as T
    rows, cols = _set()
    n = len(rows)
    cost = [r * c for r, c in zip(rows, cols)]
    dtype = [W.DT_BF16] * n
    schedule, loads = canz.canz_tp_schedule(cost, TP, CMAX)
    assert (schedule, loads) == OT.tp_schedule(cost, TP, CMAX)
    assert len(schedule) >= 3 and max(loads) <= CMAX
    hp = canz.Hparams(out_mode=canz.OUT_DELTA)
    stream = torch.cuda.current_stream().cuda_stream

    # plain run: every tensor, same-shape chunks of 8, one call
    plain_groups = canz.canz_microgroup_plan(rows, cols, dtype, [0] * n, 0, max_mats=8)
    plain = {}
    dgs = []
    for ids in plain_groups:
        dg, _, _ = _device(canz, rows, cols, ids)
        dgs.append(dg)
        for k, p in enumerate(ids):
            plain[p] = (dg, k)
    run_step(canz, dgs, hp)

    seen = set()
    shapes_per_call = []
    for rank in range(TP):
        calls = T.host_rank_calls(schedule, rank, rows, cols, dtype)
        assert len(calls) == len(schedule)
        hosted = {}
        inputs = {}

        def make_group(ids):
            dg, grads, moms = _device(canz, rows, cols, ids)
            for k, p in enumerate(ids):
                hosted[p] = (dg, k)
                inputs[p] = (grads[k], moms[k])
            return dg.group()

        # the walk itself: one library call per micro-group on this rank's tensors
        nbytes = T.workspace_bytes(calls, lambda ids: canz.Group(rows=rows[ids[0]], cols=cols[ids[0]], n_mats=len(ids), tp=TP,
                                                                  grad_dtype=W.DT_BF16, out_dtype=W.DT_BF16), hp)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        issued = T.run_host_rank(calls, make_group, hp, ws, nbytes, stream)
        torch.cuda.synchronize()
        assert issued == sum(1 for c in calls if c)
        for mg, batches in zip(schedule, calls):
            mine = sorted(t for t, h in mg if h == rank)
            assert sorted(p for ids in batches for p in ids) == mine
            shapes_per_call.append(len(batches))
        ohp = oracle_hparams(hp)
        worst = 0.0
        for p, (dg, k) in hosted.items():
            assert p not in seen
            seen.add(p)
            ref = OM.muon_step([widen(f) for f in W.split_columns(inputs[p][0], TP)], widen(inputs[p][1]), ohp)
            assert rel_fro(dg.mom_host(k), ref["mom"]) <= 1e-6
            err = rel_fro(dg.out_host(k), ref["delta"])
            worst = max(worst, err)
            assert err <= 3e-2 + 2.0 ** -8, "rank %d tensor %d: error %.3g" % (rank, p, err)
            pdg, pk = plain[p]
            assert np.array_equal(dg.out_host(k), pdg.out_host(pk)), "rank %d tensor %d differs from the plain run" % (rank, p)
            assert np.array_equal(dg.mom_host(k), pdg.mom_host(pk))
        log("host rank %d: %d tensors in %d calls, worst error %.3g" % (rank, len(hosted), issued, worst))
    assert seen == set(range(n))
    # the shared-launch path ran: some call held several shape classes
    assert max(shapes_per_call) >= 2
