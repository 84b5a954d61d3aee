"""Measured optimizer-step latency of every rank's share on one MI355X (needs a GPU).

The planner balances a proxy (elements, or Newton-Schulz FLOPs); what a job waits for is
the slowest rank's step (the straggler effect of Sec. 3.1 and the per-rank latency plot
of the load-balance study in Sec. 5).  This tool partitions a synthetic Qwen3-shaped set
with the static rule (Eq. 1) and with Algorithm 1 (both cost metrics), runs
canz_muon_step on each distinct share (ranks that own the same multiset of shapes take
the same time and are measured once) and prints the largest, mean and smallest latency
and the ratio max / mean (Eq. 6 applied to time).

Usage: python -m paper_2602_06079_amd.rank_latency [--configs 2 3 4] [--steps 3]
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


def layouts(s):
    """name -> owner array for the partitions compared."""
    R = s["n_ranks"]
    numel = [r * c for r, c in zip(s["rows"], s["cols"])]
    out = collections.OrderedDict()
    out["static, Eq. 1 per bucket"] = canz.canz_partition_naive(numel, R, s["bucket_off"])[0]
    out["Alg. 1, alpha = 1, W = numel"] = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], R, 1.0)[1]
    out["Alg. 1, alpha = 1, W = FLOPs"] = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], R, 1.0,
                                                                  cost_kind=canz.COST_NS_FLOPS)[1]
    return out


def report(cfgs=(2, 3, 4), steps=3, max_share_elems=12_000_000_000):
    import torch
    assert torch.cuda.is_available(), "rank_latency needs a GPU"
    hp = canz.Hparams()
    lines = ["| set | partition | distinct shares | max ms | mean ms | min ms | max / mean | slowest rank's share |",
             "|---|---|---|---|---|---|---|---|"]
    for cfg in cfgs:
        s = W.matrix_set(cfg)
        R = s["n_ranks"]
        memo = {}
        for name, owner in layouts(s).items():
            per_rank, sig_of = [], []
            for r in range(R):
                ids = [p for p in range(len(owner)) if owner[p] == r]
                sig = tuple(sorted(collections.Counter((s["rows"][p], s["cols"][p]) for p in ids).items()))
                elems = sum(s["rows"][p] * s["cols"][p] for p in ids)
                if sig not in memo:
                    if elems > max_share_elems:
                        raise RuntimeError("share of %d elements exceeds the memory bound of this tool" % elems)
                    memo[sig] = measure_share(torch, s, ids, hp, steps)
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
    a = ap.parse_args()
    print(report(tuple(a.configs), a.steps))
