"""Measured optimizer-step latency of every rank's share on one MI355X (needs a GPU).

The planner balances a proxy (elements, or Newton-Schulz FLOPs); what a job waits for is
the slowest rank's step (the straggler effect of Sec. 3.1 and the per-rank latency plot
of the load-balance study in Sec. 5).  This tool partitions a synthetic Qwen3-shaped set
with the static rule (Eq. 1) and with Algorithm 1 (both cost metrics), runs
canz_muon_step on each distinct share (ranks that own the same multiset of shapes take
the same time and are measured once) and prints the largest, mean and smallest latency
and the ratio max / mean (Eq. 6 applied to time).

With --optimizer shampoo or soap the same is done for the other two matrix optimizers the
paper runs through the planner ("Generalization to Other Optimizers (Shampoo & SOAP)",
App. C): the step is canz_shampoo_step (inverse roots on every step) or canz_soap_step
(averaged over a refresh period of ten steps, the rotated momentum kept), and Algorithm 1
is also run with that operator's FLOPs as W(p) (App. D.5).  Shampoo is measured on the
0.6B-shaped set only (its root iteration is cubic in the long side too).  Their state is
several times the parameters, so a share is timed one shape class at a time, a class of
more than 16 matrices on 16 of them and scaled by the count.

Usage: python -m paper_2602_06079_amd.rank_latency [--optimizer muon] [--configs 2 3 4] [--steps 3]
Gradient and parameter values are drawn on the device (seeded torch.randn): the timing
does not depend on the values.
"""
from __future__ import annotations

import argparse
import collections
import sys

import numpy as np

from . import binding as canz
from . import workloads as W


def _log(msg):
    sys.stderr.write("[rank-latency] %s\n" % msg)
    sys.stderr.flush()


CLASS_CAP = 16   # matrices of one shape class held on the device at a time by the Shampoo / SOAP measurement


def measure_share_other(torch, s, ids, optimizer, steps):
    """Latency in ms of canz_shampoo_step (median of `steps` steps) or canz_soap_step (mean over a refresh period of
    ten steps, repeated `steps` times) over the matrices ``ids`` of set ``s``."""
    if not ids:
        return 0.0
    owner = np.zeros(len(s["rows"]), dtype=np.int32)
    owner[list(ids)] = 1
    plan = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, 1, max_mats=8)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(W.SEED_BASE)
    limit = 10000
    groups, keep = [], []
    for g in plan:
        rows, cols = s["rows"][g[0]], s["cols"][g[0]]
        new = lambda r, c: [torch.zeros(r, c, device="cuda") for _ in g]
        grads = [(torch.randn(rows, cols, device="cuda", generator=gen) * s["grad_std"]).to(torch.bfloat16) for _ in g]
        outs = [torch.randn(rows, cols, device="cuda", generator=gen) * 0.02 for _ in g]
        if optimizer == "shampoo":
            st = (new(rows, rows), new(cols, cols))
            groups.append(canz.ShampooGroup(rows=rows, cols=cols, grad=grads, left=st[0], right=st[1], out=outs,
                                            grad_dtype=canz.DT_BF16, out_dtype=canz.DT_F32))
        else:
            use_l, use_r = rows <= limit, cols <= limit
            st = (new(rows, cols), new(rows, cols), new(rows, rows) if use_l else [], new(cols, cols) if use_r else [],
                  [torch.eye(rows, device="cuda") for _ in g] if use_l else [], [torch.eye(cols, device="cuda") for _ in g] if use_r else [],
                  new(rows, cols))
            groups.append(canz.SoapGroup(rows=rows, cols=cols, grad=grads, mom=st[0], var=st[1], left=st[2], right=st[3], qleft=st[4],
                                         qright=st[5], out=outs, mom_rot=st[6], grad_dtype=canz.DT_BF16, out_dtype=canz.DT_F32))
        keep.append((grads, outs, st))
    stream = torch.cuda.current_stream().cuda_stream
    if optimizer == "shampoo":
        hp = canz.ShampooHparams(beta=0.9, eps=1e-2, lr=0.02, root_iters=22)
        nbytes = canz.canz_shampoo_workspace_bytes(groups, hp)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        one = lambda t: canz.canz_shampoo_step(groups, hp, ws, nbytes, stream)
        per_sample = 1
    else:
        hps = lambda t: canz.SoapHparams(beta1=0.95, beta2=0.95, lr=3e-3, eps=1e-8, step=t, refresh=(t % 10 == 0), max_precond_dim=limit,
                                         mom_rot_valid=t > 1)
        nbytes = max(canz.canz_soap_workspace_bytes(groups, hps(1)), canz.canz_soap_workspace_bytes(groups, hps(10)))
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        one = lambda t: canz.canz_soap_step(groups, hps(t), ws, nbytes, stream)
        per_sample = 10
    one(1)                                             # warm-up (and the step that leaves a valid rotated momentum)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    t = 1
    for i in range(steps):
        for _ in range(per_sample):
            t += 1
            one(t)
        ev[i + 1].record()
    torch.cuda.synchronize()
    ms = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)])) / per_sample
    del keep, groups, ws
    torch.cuda.empty_cache()
    return ms


def measure_share(torch, s, ids, hp, steps, warmup=1):
    """Median latency in ms of canz_muon_step over the matrices ``ids`` of set ``s``."""
    if not ids:
        return 0.0
    owner = np.zeros(len(s["rows"]), dtype=np.int32)
    owner[list(ids)] = 1
    plan = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, 1, max_mats=8)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(W.SEED_BASE)
    gdt = torch.bfloat16 if s["grad_dtype"] == W.DT_BF16 else torch.float32
    groups, keep = [], []
    for g in plan:
        rows, cols = s["rows"][g[0]], s["cols"][g[0]]
        grads = [(torch.randn(rows, cols, device="cuda", generator=gen) * s["grad_std"]).to(gdt) for _ in g]
        moms = [torch.zeros(rows, cols, device="cuda") for _ in g]
        outs = [torch.randn(rows, cols, device="cuda", generator=gen) * 0.02 for _ in g]
        keep.append((grads, moms, outs))
        groups.append(canz.Group(rows=rows, cols=cols, grad=grads, mom=moms, out=outs, tp=1,
                                 grad_dtype=s["grad_dtype"], out_dtype=canz.DT_F32))
    nbytes = canz.canz_muon_workspace_bytes(groups, hp)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(warmup):
        canz.canz_muon_step(groups, hp, ws, nbytes, stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for i in range(steps):
        canz.canz_muon_step(groups, hp, ws, nbytes, stream)
        ev[i + 1].record()
    torch.cuda.synchronize()
    ms = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]))
    del keep, groups, ws
    torch.cuda.empty_cache()
    return ms


def layouts(s, optimizer="muon"):
    """name -> owner array for the partitions compared."""
    R = s["n_ranks"]
    numel = [r * c for r, c in zip(s["rows"], s["cols"])]
    kind, label = {"muon": (canz.COST_NS_FLOPS, "FLOPs"), "shampoo": (canz.COST_SHAMPOO_FLOPS, "Shampoo FLOPs"),
                   "soap": (canz.COST_SOAP_FLOPS, "SOAP FLOPs")}[optimizer]
    out = collections.OrderedDict()
    out["static, Eq. 1 per bucket"] = canz.canz_partition_naive(numel, R, s["bucket_off"])[0]
    out["Alg. 1, alpha = 1, W = numel"] = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], R, 1.0)[1]
    out["Alg. 1, alpha = 1, W = %s" % label] = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], R, 1.0, cost_kind=kind)[1]
    return out


def report(cfgs=(2, 3, 4), steps=3, max_share_elems=12_000_000_000, optimizer="muon"):
    import torch
    assert torch.cuda.is_available(), "rank_latency needs a GPU"
    if optimizer == "shampoo" and any(c != 2 for c in cfgs):
        raise ValueError("shampoo is measured on config 2 only")
    hp = canz.Hparams()
    lines = ["| set | partition | distinct shares | max ms | mean ms | min ms | max / mean | slowest rank's share |",
             "|---|---|---|---|---|---|---|---|"]
    for cfg in cfgs:
        s = W.matrix_set(cfg)
        R = s["n_ranks"]
        memo, class_memo = {}, {}
        for name, owner in layouts(s, optimizer).items():
            per_rank, sig_of = [], []
            for r in range(R):
                ids = [p for p in range(len(owner)) if owner[p] == r]
                sig = tuple(sorted(collections.Counter((s["rows"][p], s["cols"][p]) for p in ids).items()))
                elems = sum(s["rows"][p] * s["cols"][p] for p in ids)
                if sig not in memo:
                    if elems > max_share_elems:
                        raise RuntimeError("share of %d elements exceeds the memory bound of this tool" % elems)
                    if optimizer == "muon":
                        memo[sig] = measure_share(torch, s, ids, hp, steps)
                    else:
                        # one shape class at a time (their launches do not overlap anyway), at most CLASS_CAP matrices
                        # of a class on the device: a larger class is timed on CLASS_CAP of them and scaled by count
                        total = 0.0
                        for shape, n in sig:
                            some = [p for p in ids if (s["rows"][p], s["cols"][p]) == shape][:CLASS_CAP]
                            key = (shape, len(some))
                            if key not in class_memo:
                                class_memo[key] = measure_share_other(torch, s, some, optimizer, steps)
                            total += class_memo[key] * n / len(some)
                        memo[sig] = total
                    _log("config %d, %s: %s -> %.3f ms" % (cfg, name, sig, memo[sig]))
                per_rank.append(memo[sig])
                sig_of.append(sig)
            t = np.array(per_rank)
            worst = int(np.argmax(t))
            share = ", ".join("%d x %dx%d" % (n, a, b) for (a, b), n in sig_of[worst]) or "nothing"
            lines.append("| %d %s R=%d | %s | %d | %.2f | %.2f | %.2f | %.2f | rank %d: %s |" %
                         (cfg, s["name"], R, name, len(set(sig_of)), t.max(), t.mean(), t.min(),
                          t.max() / t.mean() if t.mean() > 0 else 1.0, worst, share))
    return "\n".join(lines)


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", type=int, nargs="+", default=[2, 3, 4])
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--optimizer", choices=["muon", "shampoo", "soap"], default="muon")
    a = ap.parse_args()
    cfgs = tuple(a.configs) if a.optimizer != "shampoo" or "--configs" in sys.argv else (2,)
    print(report(cfgs, a.steps, optimizer=a.optimizer))
