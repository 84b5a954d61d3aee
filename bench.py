#!/usr/bin/env python3
"""Benchmark of one rank's Muon optimizer step (canz_muon_step) on one MI355X.

A "step" is one pass of the whole hot path - momentum, normalisation, ns_steps
Newton-Schulz iterations and the fused update - over the share of the matrix set that
the alpha-balanced partitioner assigns to the chosen rank.  Inputs are seeded synthetic
Qwen3-shaped gradients already resident in HBM when timing starts.  One JSON line is
printed on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6     # 256 CUs x 4096 FLOP/clk/CU x 2.4 GHz, dense
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch (read + written) of the GEMM kernels on the default workload, from the
# two rocprofv3 --pmc runs summarised in profiles/hbm_traffic_config4.md (FETCH_SIZE scaled by
# 2.000, WRITE_SIZE by 1.000, the factors a plain 1 GiB copy gives).  Counters cannot be read
# from inside this process, so the figures are carried here, keyed by the library version they
# were measured on (a library whose kernels changed since reports null until the profile is
# taken again); other workloads report null.
MEASURED_TRAFFIC_BYTES = {("0.4.0", 4, "bf16", 1): {"gram": 3.94e9 + 0.21e9, "poly": 0.97e9 + 0.21e9,
                                           "update": 10.03e9 + 2.24e9, "final": 10.78e9 + 2.37e9}}


def log(msg):
    sys.stderr.write("[bench] %s\n" % msg)
    sys.stderr.flush()


class ClockSampler:
    """Best-effort sampler of the current shader clock from the amdgpu sysfs file
    pp_dpm_sclk (the line marked with '*'), read every few milliseconds on a host thread
    while the timed steps run.  Reports None where the file is absent or unreadable."""

    def __init__(self):
        import glob
        import threading
        self.paths = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.samples, self.stop = [], threading.Event()
        self.thread = threading.Thread(target=self._run, daemon=True)

    def _read(self):
        best = None
        for p in self.paths:
            try:
                for line in open(p).read().splitlines():
                    if line.rstrip().endswith("*"):
                        mhz = float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
                        best = mhz if best is None else max(best, mhz)
            except (OSError, ValueError, IndexError):
                pass
        return best

    def max_level_mhz(self):
        """Highest level the file lists (the nominal peak clock)."""
        best = None
        for p in self.paths:
            try:
                for line in open(p).read().splitlines():
                    mhz = float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
                    best = mhz if best is None else max(best, mhz)
            except (OSError, ValueError, IndexError):
                pass
        return best

    def _run(self):
        while not self.stop.is_set():
            v = self._read()
            if v is not None:
                self.samples.append(v)
            self.stop.wait(0.005)

    def __enter__(self):
        if self.paths:
            self.thread.start()
        return self

    def __exit__(self, *exc):
        self.stop.set()
        if self.paths:
            self.thread.join(timeout=1.0)

    def mean_mhz(self):
        return sum(self.samples) / len(self.samples) if self.samples else None


def pick_tp_share(canz, W, cfg, cmax_bytes):
    """TP planner (Algorithms 2-4): micro-groups with a host rank per tensor; the share is what
    the most loaded host rank computes, one library call per micro-group of the sequence
    (paper_2602_06079_amd.tp_runtime holds the walk; here only the share is chosen)."""
    from paper_2602_06079_amd import tp_runtime as T
    s = W.matrix_set(cfg)
    cost = [r * c for r, c in zip(s["rows"], s["cols"])]
    t0 = time.perf_counter()
    mgroups, loads = canz.canz_tp_schedule(cost, s["tp"], cmax_bytes // 2)      # capacity in bf16 elements
    per_rank = T.host_rank_loads(mgroups, cost, s["tp"])
    rank = max(range(s["tp"]), key=lambda r: (per_rank[r], -r))
    per_call = T.host_rank_calls(mgroups, rank, s["rows"], s["cols"], s["dtype"])
    plan_ms = (time.perf_counter() - t0) * 1e3
    groups, calls = [], []
    for batches in per_call:
        if batches:
            calls.append((len(groups), len(groups) + len(batches)))
            groups += batches
    mean = sum(per_rank) / len(per_rank)
    diag = dict(rank=rank, n_ranks=s["tp"], alpha=None, r_lb_numel=max(per_rank) / mean if mean else 1.0,
                planner_ms=plan_ms, tp_micro_groups=len(mgroups), cmax_bytes=cmax_bytes, calls=calls,
                largest_group_load_elems=max(loads) if loads else 0)
    return s, rank, groups, diag


def pick_share(canz, W, cfg):
    """Planner calls (timed) -> (set, rank, groups of matrix ids, diagnostics)."""
    import numpy as np
    s = W.matrix_set(cfg)
    t0 = time.perf_counter()
    cuts, owner, load = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], s["n_ranks"], s["alpha"])
    rank = 0 if cfg in (1, 2, 5) else int(np.argmax(load))   # argmax: lowest rank among equals
    groups = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, rank, max_mats=8)
    plan_ms = (time.perf_counter() - t0) * 1e3
    mean = float(load.sum()) / len(load)
    diag = dict(rank=rank, n_ranks=s["n_ranks"], alpha=s["alpha"], r_lb_numel=float(load.max()) / mean if mean else 1.0,
                planner_ms=plan_ms)
    return s, rank, groups, diag


def ns_flops(rows, cols, steps):
    m, n = min(rows, cols), max(rows, cols)
    return steps * (4 * m * m * n + 2 * m ** 3)


def main_shampoo(args, canz, W, np, torch):
    """One rank's Shampoo step (canz_shampoo_step): Algorithm 1 with W(p) = Shampoo FLOPs
    (App. D.5) on the set of --config, alpha = 1, the most loaded rank's share."""
    cfg = 2 if args.config is None else args.config
    s = W.matrix_set(cfg)
    R = s["n_ranks"]
    t0 = time.perf_counter()
    cuts, owner, load = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], R, 1.0,
                                                  cost_kind=canz.COST_SHAMPOO_FLOPS)
    rank = int(np.argmax(load))
    groups = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, rank, max_mats=8)
    plan_ms = (time.perf_counter() - t0) * 1e3
    mean = float(load.sum()) / len(load)
    n_share = sum(len(g) for g in groups)
    log("shampoo on config %d (%s): rank %d owns %d matrices in %d groups; planner %.2f ms, R_LB(FLOPs) %.3f" %
        (cfg, s["name"], rank, n_share, len(groups), plan_ms, float(load.max()) / mean))
    # 22 rounds: what covers a condition number of 1e6 at these extents (25, the library default, covers 1e7)
    hp = canz.ShampooHparams(beta=0.9, eps=1e-2, lr=0.02, root_iters=22)
    every = max(1, args.roots_every)       # 1: the roots on every step, as published
    gen = torch.Generator(device="cuda")
    gen.manual_seed(W.SEED_BASE + cfg)
    dgroups, keep = [], []
    for g in groups:
        rows, cols = s["rows"][g[0]], s["cols"][g[0]]
        grads = [(torch.randn(rows, cols, device="cuda", generator=gen) * s["grad_std"]).to(torch.bfloat16) for _ in g]
        lefts = [torch.zeros(rows, rows, device="cuda") for _ in g]
        rights = [torch.zeros(cols, cols, device="cuda") for _ in g]
        outs = [torch.randn(rows, cols, device="cuda", generator=gen) * 0.02 for _ in g]
        lroots = [torch.zeros(rows, rows, device="cuda") for _ in g] if every > 1 else []
        rroots = [torch.zeros(cols, cols, device="cuda") for _ in g] if every > 1 else []
        keep.append((grads, lefts, rights, outs, lroots, rroots))
        dgroups.append(canz.ShampooGroup(rows=rows, cols=cols, grad=grads, left=lefts, right=rights, out=outs, lroot=lroots,
                                         rroot=rroots, grad_dtype=canz.DT_BF16, out_dtype=canz.DT_F32))
    ws_bytes = canz.canz_shampoo_workspace_bytes(dgroups, hp)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    hp_keep = canz.ShampooHparams(beta=0.9, eps=1e-2, lr=0.02, root_iters=22, keep_roots=True)
    t_now = [0]

    def step():   # step t computes the roots if t = 1 (mod every), else it keeps the last ones
        t_now[0] += 1
        canz.canz_shampoo_step(dgroups, hp if (t_now[0] - 1) % every == 0 else hp_keep, ws, ws_bytes, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    canz.canz_profile_enable(n_share * (12 + 8 * hp.root_iters) + 8)
    t_now[0] = 0                           # a step with the roots: the longest there is
    step()
    torch.cuda.synchronize()
    launches_per_step = sum(n for _ms, n in canz.canz_profile_collect().values())
    t_now[0] = args.warmup
    canz.canz_profile_enable(launches_per_step * args.steps + 8)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t_start) * 1e3 / args.steps
    prof = canz.canz_profile_collect()
    canz.canz_profile_disable()
    log("timed %d steps: %.3f ms/step" % (args.steps, ms_per_step))

    # FLOPs.  A product of two commuting symmetric d x d matrices has d (d + 1) / 2 distinct entries of
    # 2 d FLOPs each: that is the algorithmic count of the statistics and of the four products of a
    # root round; the kernels compute whole 128 x 128 tiles on or above the diagonal ("issued").
    def pad(x):
        return (x + 127) // 128 * 128

    def sym(d, k):
        return d * (d + 1) * k, (pad(d) // 128) * (pad(d) // 128 + 1) // 2 * 128 * 128 * 2 * pad(k)

    alg = dict(sh_stat=0.0, sh_root=0.0, sh_apply=0.0)
    iss = dict(sh_stat=0.0, sh_root=0.0, sh_apply=0.0)
    # share of the timed steps that computed the roots
    root_share = sum(1 for t in range(args.warmup + 1, args.warmup + args.steps + 1) if (t - 1) % every == 0) / args.steps
    for g in groups:
        r, c = s["rows"][g[0]], s["cols"][g[0]]
        n = len(g)
        for d, k in ((r, c), (c, r)):
            a, i = sym(d, k)
            alg["sh_stat"] += n * a
            iss["sh_stat"] += n * i
            a, i = sym(d, d)
            alg["sh_root"] += n * a * (4 * hp.root_iters - 3 + 2) * root_share      # + A'A' and A'^2 A'^2 for the starting bound
            iss["sh_root"] += n * i * (4 * hp.root_iters - 3 + 2) * root_share
        alg["sh_apply"] += n * (2.0 * r * r * c + 2.0 * r * c * c)
        iss["sh_apply"] += n * (2.0 * pad(r) * pad(r) * pad(c) + 2.0 * pad(r) * pad(c) * pad(c))
    kernels = {}
    for k, (ms, n) in prof.items():
        if n:
            kernels[k] = dict(ms_per_step=ms / args.steps, launches_per_step=n / args.steps, avg_ms=ms / n)
            if k in alg:
                kernels[k]["tflops_algorithmic"] = alg[k] * args.steps / (ms * 1e-3) / 1e12
                kernels[k]["tflops_issued"] = iss[k] * args.steps / (ms * 1e-3) / 1e12
    dom = max((k for k in kernels if k in alg), key=lambda k: kernels[k]["ms_per_step"])
    peak = 157.3
    per_launch = alg[dom] / kernels[dom]["launches_per_step"]
    achieved = per_launch / (kernels[dom]["avg_ms"] * 1e-3) / 1e12
    issued = iss[dom] / kernels[dom]["launches_per_step"] / (kernels[dom]["avg_ms"] * 1e-3) / 1e12
    roofline = dict(bound="mfma", kernel="k_sh_gemm (%s)" % dom, achieved=achieved, peak=peak, unit="TFLOP/s",
                    frac=achieved / peak, traffic=None, achieved_issued=issued, frac_issued=issued / peak,
                    flops_per_launch=per_launch, avg_launch_ms=kernels[dom]["avg_ms"])
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import shampoo as OS
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [os.cpu_count()])
        except Exception:
            cores = os.cpu_count()
        g0 = groups[0]
        rows, cols = s["rows"][g0[0]], s["cols"][g0[0]]
        g64 = keep[0][0][0].float().cpu().numpy().astype(np.float64)
        t0 = time.perf_counter()
        OS.shampoo_step(g64, np.zeros((rows, rows)), np.zeros((cols, cols)), OS.Hparams(eps=1e-2), param=np.zeros((rows, cols)))
        t_one = time.perf_counter() - t0
        cost = lambda r, c: r ** 3 + c ** 3
        est_s = sum(len(g) * t_one * cost(s["rows"][g[0]], s["cols"][g[0]]) / cost(rows, cols) for g in groups)
        cpu = dict(value=est_s * 1e3, unit="ms", cores=int(cores), kind="oracle",
                   sample="fp64 oracle (two symmetric eigendecompositions and the products), one whole step of matrix "
                          "%d (%dx%d): %.2f s, scaled by rows^3 + cols^3 to the %d-matrix share" % (g0[0], rows, cols, t_one, n_share))
    total_alg, total_iss = sum(alg.values()), sum(iss.values())
    out = {
        "metric": "optimizer_step_latency_ms", "value": ms_per_step, "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic", "launch": "eager",
        "config": {"workload": "shampoo step, config %d %s partitioned by Shampoo FLOPs: rank %d of %d (alpha=1), %d matrices %s "
                               "in %d micro-groups, %d root rounds, roots %s" %
                               (cfg, s["name"], rank, R, n_share, sorted({(s["rows"][p], s["cols"][p]) for g in groups for p in g}),
                                len(groups), hp.root_iters, "on every step" if every == 1 else "on every %d-th step" % every),
                   "elements": sum(s["rows"][p] * s["cols"][p] for g in groups for p in g)},
        "tflops_algorithmic": total_alg / (ms_per_step * 1e-3) / 1e12, "tflops_issued": total_iss / (ms_per_step * 1e-3) / 1e12,
        "frac_mfma_peak_issued": total_iss / (ms_per_step * 1e-3) / 1e12 / peak,
        "planner": dict(rank=rank, n_ranks=R, alpha=1.0, cost="shampoo_flops", r_lb_flops=float(load.max()) / mean, planner_ms=plan_ms),
        "kernels": kernels, "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def main_soap(args, canz, W, np, torch):
    """One rank's SOAP step (canz_soap_step): Algorithm 1 with W(p) = SOAP FLOPs (App. D.5) on the set of
    --config, alpha = 1, the most loaded rank's share.  Steps t = 1, 2, ... with a basis refresh on every
    --refresh-every-th one; with the defaults (3 warm-up + 10 timed steps, refresh every 10th) the timed
    region holds nine plain steps and one refresh step, one whole refresh period."""
    cfg = 2 if args.config is None else args.config
    s = W.matrix_set(cfg)
    R = s["n_ranks"]
    t0 = time.perf_counter()
    cuts, owner, load = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], R, 1.0,
                                                  cost_kind=canz.COST_SOAP_FLOPS)
    rank = int(np.argmax(load))
    groups = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, rank, max_mats=8)
    plan_ms = (time.perf_counter() - t0) * 1e3
    if args.share:
        # a share given by hand instead of the planner's: N matrices of one shape (e.g. a one-sided case)
        r_, c_, n_ = (int(v) for v in args.share.lower().split("x"))
        s = dict(s, rows=list(s["rows"]) + [r_] * n_, cols=list(s["cols"]) + [c_] * n_)
        first = len(s["rows"]) - n_
        groups = [list(range(first + i, min(first + i + 8, first + n_))) for i in range(0, n_, 8)]
    mean = float(load.sum()) / len(load)
    n_share = sum(len(g) for g in groups)
    log("soap on config %d (%s): rank %d owns %d matrices in %d groups; planner %.2f ms, R_LB(FLOPs) %.3f" %
        (cfg, s["name"], rank, n_share, len(groups), plan_ms, float(load.max()) / mean))
    f = args.refresh_every
    limit = args.max_precond_dim

    keep_rot = not args.rotate_momentum_every_step

    def hparams(t):
        # the rotated momentum is valid from the second step on (the first one rotates M and leaves M' behind)
        return canz.SoapHparams(beta1=0.95, beta2=0.95, lr=3e-3, eps=1e-8, step=t, refresh=(t % f == 0), max_precond_dim=limit,
                                mom_rot_valid=keep_rot and t > 1, bf16_rotations=args.bf16_rotations)

    gen = torch.Generator(device="cuda")
    gen.manual_seed(W.SEED_BASE + cfg)
    dgroups, keep = [], []
    for g in groups:
        rows, cols = s["rows"][g[0]], s["cols"][g[0]]
        use_l, use_r = rows <= limit, cols <= limit
        grads = [(torch.randn(rows, cols, device="cuda", generator=gen) * s["grad_std"]).to(torch.bfloat16) for _ in g]
        moms = [torch.zeros(rows, cols, device="cuda") for _ in g]
        vars_ = [torch.zeros(rows, cols, device="cuda") for _ in g]
        lefts = [torch.zeros(rows, rows, device="cuda") for _ in g] if use_l else []
        rights = [torch.zeros(cols, cols, device="cuda") for _ in g] if use_r else []
        qls = [torch.eye(rows, device="cuda") for _ in g] if use_l else []
        qrs = [torch.eye(cols, device="cuda") for _ in g] if use_r else []
        outs = [torch.randn(rows, cols, device="cuda", generator=gen) * 0.02 for _ in g]
        rots = [torch.zeros(rows, cols, device="cuda") for _ in g] if keep_rot else []
        keep.append((grads, moms, vars_, lefts, rights, qls, qrs, outs, rots))
        dgroups.append(canz.SoapGroup(rows=rows, cols=cols, grad=grads, mom=moms, var=vars_, left=lefts, right=rights,
                                      qleft=qls, qright=qrs, out=outs, mom_rot=rots, grad_dtype=canz.DT_BF16,
                                      out_dtype=canz.DT_F32))
    ws_bytes = max(canz.canz_soap_workspace_bytes(dgroups, hparams(1)), canz.canz_soap_workspace_bytes(dgroups, hparams(f)))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    t_now = [0]

    def step():
        t_now[0] += 1
        canz.canz_soap_step(dgroups, hparams(t_now[0]), ws, ws_bytes, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # launches of a refresh step: per side and panel of 32 columns 4 + 3, plus a few dozen per batch
    max_d = max(max(s["rows"][g[0]], s["cols"][g[0]]) for g in groups)
    per_refresh = len(groups) * 8 * (2 * (7 * (max_d // 32 + 1) + 8) + 16)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t_start) * 1e3 / args.steps
    n_refresh_timed = sum(1 for t in range(args.warmup + 1, args.warmup + args.steps + 1) if t % f == 0)
    log("timed %d steps (%d with a refresh): %.3f ms/step" % (args.steps, n_refresh_timed, ms_per_step))
    # the per-kernel breakdown comes from a second pass of the same length outside the timed region: a refresh
    # issues thousands of short launches, and a pair of events around each would weigh on the timed figure
    canz.canz_profile_enable(per_refresh * (args.steps // f + 2) + 64 * args.steps * len(groups))
    first_profiled = t_now[0] + 1
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = canz.canz_profile_collect()
    canz.canz_profile_disable()
    n_refresh = sum(1 for t in range(first_profiled, first_profiled + args.steps) if t % f == 0)

    def pad(x, to=128):
        return (x + to - 1) // to * to

    def sym(d, k, n):
        # the statistic is symmetric (d (d + 1) k FLOPs); from bf16 gradients, as here, the bf16 kernels compute its
        # 256 x 256 tiles on operands padded to 256: those on and above the diagonal where the sums are long (the
        # library's rule, restated here for the count), else the whole square
        t = pad(d, 256) // 256
        saved_us = t * (t - 1) // 2 * n / 256.0 * (pad(k, 256) // 32) * 0.65
        tiles = t * (t + 1) // 2 if saved_us > 1.5 * (15.0 + d * d * n * 4.0 / 4.0e6) else t * t
        return d * (d + 1) * k, tiles * 256 * 256 * 2 * pad(k, 256)

    alg = dict(soap_rotate=0.0, soap_stat=0.0, soap_qr=0.0)
    iss = dict(soap_rotate=0.0, soap_stat=0.0)
    for g in groups:
        r, c = s["rows"][g[0]], s["cols"][g[0]]
        n = len(g)
        use_l, use_r = r <= limit, c <= limit
        per_rot = (2.0 * r * r * c if use_l else 0.0) + (2.0 * r * c * c if use_r else 0.0)
        pr, pc = (pad(r, 256), pad(c, 256)) if args.bf16_rotations else (pad(r), pad(c))   # the bf16 kernels' tiles are 256 wide
        per_rot_iss = (2.0 * pr * pr * pc if use_l else 0.0) + (2.0 * pr * pc * pc if use_r else 0.0)
        # G (and M, unless its rotated image is kept) in, the direction back; M again after a refresh if it is kept
        n_rot = (2 * args.steps + n_refresh) if keep_rot else 3 * args.steps
        alg["soap_rotate"] += n_rot * n * per_rot
        iss["soap_rotate"] += n_rot * n * per_rot_iss
        for d, k, used in ((r, c, use_l), (c, r, use_r)):
            if used:
                # like-shaped consecutive groups run as one launch batch
                a, i = sym(d, k, sum(len(h) for h in groups if (s["rows"][h[0]], s["cols"][h[0]]) == (r, c)))
                alg["soap_stat"] += n * a * args.steps
                iss["soap_stat"] += n * i * args.steps
                alg["soap_qr"] += n * (2.0 + 4.0 / 3.0 + 4.0 / 3.0) * d ** 3 * n_refresh
    kernels = {}
    for k, (ms, n) in prof.items():
        if n:
            kernels[k] = dict(ms_per_step=ms / args.steps, launches_per_step=n / args.steps, avg_ms=ms / n)
            if k in alg and alg[k] > 0:
                kernels[k]["tflops_algorithmic"] = alg[k] / (ms * 1e-3) / 1e12
            if k in iss and iss[k] > 0:
                kernels[k]["tflops_issued"] = iss[k] / (ms * 1e-3) / 1e12
    refresh_ms = sum(kernels[k]["ms_per_step"] * args.steps for k in ("soap_qr", "soap_panel") if k in kernels) / max(n_refresh, 1)
    plain_ms = sum(v["ms_per_step"] for k, v in kernels.items() if k not in ("soap_qr", "soap_panel"))
    # the dominant kernel: the rotations, unless they run on the bf16 matrix cores and the fp32 statistics take longer
    dom = max(("soap_rotate", "soap_stat"), key=lambda k: kernels[k]["ms_per_step"])
    peak = 2500.0 if (dom == "soap_stat" or args.bf16_rotations) else 157.3
    launches = kernels[dom]["launches_per_step"] * args.steps
    per_launch = alg[dom] / launches
    achieved = per_launch / (kernels[dom]["avg_ms"] * 1e-3) / 1e12
    issued = iss[dom] / launches / (kernels[dom]["avg_ms"] * 1e-3) / 1e12
    roofline = dict(bound="mfma", kernel="%s (%s)" % ("k_gemm_nt_bf16" if peak > 1000 else "k_sh_gemm", dom), achieved=achieved, peak=peak, unit="TFLOP/s",
                    frac=achieved / peak, traffic=None, achieved_issued=issued, frac_issued=issued / peak,
                    flops_per_launch=per_launch, avg_launch_ms=kernels[dom]["avg_ms"])
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import soap as OS
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [os.cpu_count()])
        except Exception:
            cores = os.cpu_count()
        g0 = groups[0]
        rows, cols = s["rows"][g0[0]], s["cols"][g0[0]]
        # seeded state; a side above the limit keeps no statistic and no basis (the oracle ignores its entries)
        side = lambda d, stream, level: (W.gen_spd_f32(cfg, g0[0], stream, d, level).astype(np.float64) if d <= limit else np.zeros((1, 1)))
        st = {"mom": W.gen_normal_f32(cfg, g0[0], 11, rows, cols, 0.02).astype(np.float64),
              "var": np.square(W.gen_normal_f32(cfg, g0[0], 12, rows, cols, 0.02)).astype(np.float64),
              "left": side(rows, 13, 0.02 * 0.02 * cols), "right": side(cols, 14, 0.02 * 0.02 * rows),
              "q_left": np.eye(rows) if rows <= limit else np.zeros((1, 1)), "q_right": np.eye(cols) if cols <= limit else np.zeros((1, 1))}
        g64 = keep[0][0][0].float().cpu().numpy().astype(np.float64)
        ohp = OS.Hparams(max_precond_dim=limit)
        t0 = time.perf_counter()
        OS.soap_step(g64, st, ohp, 5, False, param=np.zeros((rows, cols)))
        t_plain = time.perf_counter() - t0
        t0 = time.perf_counter()
        OS.soap_step(g64, st, ohp, 10, True, param=np.zeros((rows, cols)))
        t_fresh = time.perf_counter() - t0
        per_step = (t_plain * (args.steps - n_refresh_timed) + t_fresh * n_refresh_timed) / args.steps
        cost = lambda r, c: r * c * ((r if r <= limit else 0) + (c if c <= limit else 0))
        est_s = sum(len(g) * per_step * cost(s["rows"][g[0]], s["cols"][g[0]]) / cost(rows, cols) for g in groups)
        cpu = dict(value=est_s * 1e3, unit="ms", cores=int(cores), kind="oracle",
                   sample="fp64 oracle, matrix %d (%dx%d): one plain step %.2f s and one refresh step %.2f s, weighted as in "
                          "the timed region and scaled by rows cols (sum of the sides with a basis) to the %d-matrix share" %
                          (g0[0], rows, cols, t_plain, t_fresh, n_share))
    total_alg = sum(alg.values())
    out = {
        "metric": "optimizer_step_latency_ms", "value": ms_per_step, "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (rotations on bf16 operands)" if args.bf16_rotations else "f32", "data": "synthetic", "launch": "eager",
        "config": {"workload": ("soap step, share given by hand (--share %s; the planner figures below are of config %d %s, rank %d of %d): " % (args.share, cfg, s["name"], rank, R) if args.share else "soap step, config %d %s partitioned by SOAP FLOPs: rank %d of %d (alpha=1), " % (cfg, s["name"], rank, R)) + "%d matrices %s in %d "
                               "micro-groups, basis refresh every %d steps (%d of the %d timed steps), max_precond_dim %d, %s" %
                               (n_share, sorted({(s["rows"][p], s["cols"][p]) for g in groups for p in g}),
                                len(groups), f, n_refresh_timed, args.steps, limit,
                                "rotated momentum kept between steps" if keep_rot else "momentum rotated on every step"),
                   "elements": sum(s["rows"][p] * s["cols"][p] for g in groups for p in g)},
        "plain_step_ms": plain_ms, "refresh_ms": refresh_ms,
        "tflops_algorithmic": total_alg / (ms_per_step * args.steps * 1e-3) / 1e12,
        "planner": dict(rank=rank, n_ranks=R, alpha=1.0, cost="soap_flops", r_lb_flops=float(load.max()) / mean, planner_ms=plan_ms),
        "kernels": kernels, "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=None, help="benchmark configuration 1..5 (default 4: Qwen3-32B share; "
                                                             "2 with --optimizer shampoo or soap)")
    ap.add_argument("--optimizer", choices=["muon", "shampoo", "soap"], default="muon",
                    help="muon (default): canz_muon_step on the share of --config; shampoo / soap: canz_shampoo_step / "
                         "canz_soap_step on the share Algorithm 1 assigns under that operator's FLOPs cost (default set: "
                         "config 2, the 0.6B shapes)")
    ap.add_argument("--refresh-every", type=int, default=10, help="soap: basis refresh on every n-th step")
    ap.add_argument("--roots-every", type=int, default=1,
                    help="shampoo: inverse roots on every n-th step, kept in between (default 1: on every step, as published)")
    ap.add_argument("--max-precond-dim", type=int, default=10000, help="soap: a longer side keeps no basis")
    ap.add_argument("--rotate-momentum-every-step", action="store_true",
                    help="soap: do not keep the rotated momentum between steps (three rotations per step instead of two)")
    ap.add_argument("--share", default="", metavar="RxCxN",
                    help="soap: run N matrices of R x C instead of the share the planner assigns (e.g. 25600x5120x4)")
    ap.add_argument("--bf16-rotations", action="store_true",
                    help="soap: the rotation products on bf16 operands with fp32 accumulation (state, statistics, refresh stay fp32)")
    ap.add_argument("--precision", choices=["bf16", "f32"], default="bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tp-schedule", type=int, default=0, metavar="MB",
                    help="config 5 only: plan with canz_tp_schedule at this micro-group capacity (MB of bf16 per host "
                         "rank) and run the share of the most loaded host rank instead of all matrices")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time replays of it (the per-kernel breakdown then "
                         "comes from one extra eager pass outside the timed region)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy before the warm-up: under `rocprofv3 --pmc FETCH_SIZE` / "
                         "`WRITE_SIZE` its known traffic gives the scale of the counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py measures one rank's share on ONE GPU; this build has no multi-GPU path "
                         "(--gpus %d refused).\n" % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_06079_amd import build as _build
    if not os.path.exists(_build.OUT):
        _build.build()
    from paper_2602_06079_amd import binding as canz
    from paper_2602_06079_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.optimizer == "shampoo":
        return main_shampoo(args, canz, W, np, torch)
    if args.optimizer == "soap":
        return main_soap(args, canz, W, np, torch)
    cfg = 4 if args.config is None else args.config
    if args.tp_schedule:
        assert cfg == 5, "--tp-schedule applies to the TP configuration (5)"
        s, rank, groups, diag = pick_tp_share(canz, W, cfg, args.tp_schedule << 20)
    else:
        s, rank, groups, diag = pick_share(canz, W, cfg)
    tp = s["tp"]
    n_share = sum(len(g) for g in groups)
    log("config %d (%s): rank %d owns %d matrices in %d groups; planner %.2f ms" %
        (cfg, s["name"], rank, n_share, len(groups), diag["planner_ms"]))

    # ---- inputs, resident in HBM before timing
    hp = canz.Hparams(precision=canz.PREC_BF16 if args.precision == "bf16" else canz.PREC_F32,
                      out_mode=canz.OUT_DELTA if tp > 1 else canz.OUT_PARAM)
    total_elems = sum(s["rows"][p] * s["cols"][p] for g in groups for p in g)
    host_gen = total_elems <= 700_000_000
    dgroups, keep, first_host = [], [], None
    t0 = time.perf_counter()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(W.SEED_BASE + cfg)
    for g in groups:
        rows, cols = s["rows"][g[0]], s["cols"][g[0]]
        grads, moms, outs = [], [], []
        for p in g:
            if host_gen:
                bits, dt = W.gen_grad(cfg, p, rows, cols)
                if first_host is None:
                    first_host = (p, bits)
                frags = W.split_columns(bits, tp) if tp > 1 else [bits]
                for f in frags:
                    t = torch.from_numpy(f)
                    grads.append((t.view(torch.bfloat16) if f.dtype == np.uint16 else t).cuda())
            else:
                for _ in range(tp):
                    grads.append((torch.randn(rows, cols // tp, device="cuda", generator=gen) * s["grad_std"])
                                 .to(torch.bfloat16 if s["grad_dtype"] == W.DT_BF16 else torch.float32))
            moms.append(torch.zeros(rows, cols, device="cuda"))
            if tp > 1:
                outs += [torch.zeros(rows, cols // tp, device="cuda", dtype=torch.bfloat16) for _ in range(tp)]
            else:
                outs.append(torch.randn(rows, cols, device="cuda", generator=gen) * 0.02)
        keep.append((grads, moms, outs))
        dgroups.append(canz.Group(rows=rows, cols=cols, grad=grads, mom=moms, out=outs, tp=tp,
                                  grad_dtype=s["grad_dtype"],
                                  out_dtype=canz.DT_BF16 if tp > 1 else canz.DT_F32))
    ws_bytes = canz.canz_muon_workspace_bytes(dgroups, hp)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    log("inputs ready in %.1f s (%s); %.2f G elements; workspace %.2f GB" %
        (time.perf_counter() - t0, "host numpy" if host_gen else "device torch.randn", total_elems / 1e9,
         ws_bytes / 1e9))

    stream = torch.cuda.current_stream().cuda_stream

    calls = diag.pop("calls", [(0, len(dgroups))])

    def step():
        for lo, hi in calls:
            canz.canz_muon_step(dgroups[lo:hi], hp, ws, ws_bytes, stream)

    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                                                    # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for i in range(args.warmup):
        step()
    torch.cuda.synchronize()
    log("warm-up done")

    # launch records of one step, counted by the library itself in one profiled step (so the
    # event pool of the timed run holds every launch whatever batches the library forms)
    canz.canz_profile_enable(n_share * (6 + 3 * hp.ns_steps) + 8)
    step()
    torch.cuda.synchronize()
    launches_per_step = sum(n for _ms, n in canz.canz_profile_collect().values())
    canz.canz_profile_disable()
    graph = None
    if args.graph:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for lo, hi in calls:
                canz.canz_muon_step(dgroups[lo:hi], hp, ws, ws_bytes, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        canz.canz_profile_enable(launches_per_step * args.steps + 8)
        for i in range(args.steps):                 # eager pass for the per-kernel breakdown, not timed
            step()
        torch.cuda.synchronize()
        prof_eager = canz.canz_profile_collect()
        canz.canz_profile_disable()
        step = graph.replay
        step()
        torch.cuda.synchronize()
        log("graph captured; timing replays")
    else:
        canz.canz_profile_enable(launches_per_step * args.steps + 8)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    clock = ClockSampler()
    with clock:
        t_start = time.perf_counter()
        ev[0].record()
        for i in range(args.steps):
            step()
            ev[i + 1].record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t_start) * 1e3
    if graph is None:
        prof = canz.canz_profile_collect()
        canz.canz_profile_disable()
    else:
        prof = prof_eager
    per_step = [ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)]
    ms_per_step = wall_ms / args.steps
    log("timed %d steps: %.3f ms/step (events: median %.3f, min %.3f)" %
        (args.steps, ms_per_step, float(np.median(per_step)), min(per_step)))

    # ---- work accounting
    flops_step = float(sum(ns_flops(s["rows"][p], s["cols"][p], hp.ns_steps) for g in groups for p in g))
    tflops = flops_step / (ms_per_step * 1e-3) / 1e12
    # FLOPs per launch kind and step: "algorithmic" as the method writes them (2 m^2 n for the
    # Gram and update products, 2 m^3 for the square); "issued" = what the MFMA units execute:
    # padded extents, and only the tiles on or above the diagonal for the symmetric products.
    def pad(x):
        return (x + 255) // 256 * 256

    kind_flops = dict(gram=0.0, poly=0.0, update=0.0, final=0.0)
    kind_issued = dict(gram=0.0, poly=0.0, update=0.0, final=0.0)
    bf16 = args.precision == "bf16"
    for g in groups:
        rows, cols = s["rows"][g[0]], s["cols"][g[0]]
        m, n = min(rows, cols), max(rows, cols)
        mp, np_ = pad(m), pad(n)
        tri = (mp // 256) * (mp // 256 + 1) // 2 * 65536 if bf16 else mp * mp
        kind_flops["gram"] += 2.0 * m * m * n * len(g) * hp.ns_steps
        kind_flops["poly"] += 2.0 * m ** 3 * len(g) * hp.ns_steps
        kind_flops["update"] += 2.0 * m * m * n * len(g) * (hp.ns_steps - 1)
        kind_flops["final"] += 2.0 * m * m * n * len(g)
        kind_issued["gram"] += 2.0 * tri * np_ * len(g) * hp.ns_steps
        kind_issued["poly"] += 2.0 * tri * mp * len(g) * hp.ns_steps
        kind_issued["update"] += 2.0 * mp * mp * np_ * len(g) * (hp.ns_steps - 1)
        kind_issued["final"] += 2.0 * mp * mp * np_ * len(g)
    issued_step = sum(kind_issued.values())
    kernels = {}
    for k, (ms, n) in prof.items():
        if n:
            kernels[k] = dict(ms_per_step=ms / args.steps, launches_per_step=n / args.steps, avg_ms=ms / n)
            if k in kind_flops:
                # "issued" is what the MFMA units execute and what belongs next to a peak;
                # "effective" counts the method's nominal FLOPs (the symmetric products compute
                # only the tiles on or above the diagonal, so it can exceed the peak)
                kernels[k]["tflops_issued"] = kind_issued[k] * args.steps / (ms * 1e-3) / 1e12
                kernels[k]["tflops_effective"] = kind_flops[k] * args.steps / (ms * 1e-3) / 1e12
    dom = max((k for k in kernels if k in kind_flops), key=lambda k: kernels[k]["ms_per_step"])
    dom_flops_per_launch = kind_flops[dom] / kernels[dom]["launches_per_step"]
    dom_issued_per_launch = kind_issued[dom] / kernels[dom]["launches_per_step"]
    achieved = dom_flops_per_launch / (kernels[dom]["avg_ms"] * 1e-3) / 1e12
    achieved_issued = dom_issued_per_launch / (kernels[dom]["avg_ms"] * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if bf16 else 157.3
    # the same peak from what the device reports, and at the shader clock sampled during the run
    props = torch.cuda.get_device_properties(0)
    cus = int(props.multi_processor_count)
    nominal_mhz = float(getattr(props, "clock_rate", 0)) / 1e3 or clock.max_level_mhz() or 2400.0
    flop_per_clk_cu = 4096.0 if bf16 else 256.0
    seen_mhz = clock.mean_mhz()
    device = dict(name=props.name, compute_units=cus, nominal_clock_mhz=nominal_mhz,
                  peak_tflops_at_nominal_clock=cus * flop_per_clk_cu * nominal_mhz * 1e6 / 1e12,
                  sampled_clock_mhz=seen_mhz, clock_samples=len(clock.samples),
                  peak_tflops_at_sampled_clock=(cus * flop_per_clk_cu * seen_mhz * 1e6 / 1e12) if seen_mhz else None)
    roofline = dict(bound="mfma", kernel="k_gemm_nt_%s<%s>" % (args.precision, dom), achieved=achieved, peak=peak,
                    unit="TFLOP/s", frac=achieved / peak,
                    traffic=MEASURED_TRAFFIC_BYTES.get((canz.canz_version(), cfg, args.precision, tp), {}).get(dom), traffic_unit="B",
                    achieved_issued=achieved_issued, frac_issued=achieved_issued / peak,
                    flops_per_launch=dom_flops_per_launch, issued_flops_per_launch=dom_issued_per_launch,
                    avg_launch_ms=kernels[dom]["avg_ms"])
    if "momentum" in kernels:
        grad_b = 2 if s["grad_dtype"] == W.DT_BF16 else 4
        esz = 2 if args.precision == "bf16" else 4
        bytes_step = total_elems * (grad_b + 8 + 2 * esz)
        kernels["momentum"]["gbs"] = bytes_step / (kernels["momentum"]["ms_per_step"] * 1e-3) / 1e9
        kernels["momentum"]["frac_hbm_peak"] = kernels["momentum"]["gbs"] / PEAK_HBM_GBS

    # ---- the oracle on the host cores, bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import muon as OM
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [os.cpu_count()])
        except Exception:
            cores = os.cpu_count()
        f = lambda v: float(np.float32(v))
        g0 = groups[0]
        rows, cols = s["rows"][g0[0]], s["cols"][g0[0]]
        if first_host is not None and first_host[0] == g0[0]:
            bits = first_host[1]
        else:
            bits = W.gen_grad(cfg, g0[0], rows, cols)[0]
        g64 = OM.bf16_bits_to_f64(bits) if bits.dtype == np.uint16 else bits.astype(np.float64)
        mom0 = np.zeros((rows, cols))
        base = dict(beta=f(hp.beta), lr=f(hp.lr), eps=f(hp.eps), a=f(hp.a), b=f(hp.b), c=f(hp.c),
                    scale_mode=hp.scale_mode)
        t0 = time.perf_counter()
        OM.muon_step(g64, mom0, OM.Hparams(ns_steps=hp.ns_steps, **base), param=mom0)
        t_one = time.perf_counter() - t0
        f0 = ns_flops(rows, cols, hp.ns_steps)
        est_s = sum(len(g) * t_one * ns_flops(s["rows"][g[0]], s["cols"][g[0]], hp.ns_steps) / f0 for g in groups)
        cpu = dict(value=est_s * 1e3, unit="ms", cores=int(cores), kind="oracle",
                   sample="fp64 oracle, one whole step (momentum, normalisation, %d Newton-Schulz iterations, update) "
                          "of matrix %d (%dx%d): %.2f s (%.0f GFLOP/s), scaled by FLOPs to the %d-matrix share"
                          % (hp.ns_steps, g0[0], rows, cols, t_one, f0 / max(t_one, 1e-9) / 1e9, n_share))
        log("oracle sample: %.2f s measured, share estimated at %.1f s on %d threads" % (t_one, est_s, cores))

    out = {
        "metric": "optimizer_step_latency_ms", "value": ms_per_step, "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": args.precision, "data": "synthetic", "launch": "hip graph replay" if graph is not None else "eager",
        "config": {"workload": "config %d %s: %s, %d matrices %s in %d micro-groups, "
                               "%d Newton-Schulz steps" %
                               (cfg, s["name"],
                                ("host rank %d of %d under the TP schedule (capacity %d MB)" % (rank, tp, args.tp_schedule))
                                if args.tp_schedule else
                                "rank %d of %d (alpha=%.2g)" % (rank, s["n_ranks"], s["alpha"]), n_share,
                                sorted({(s["rows"][p], s["cols"][p]) for g in groups for p in g}), len(groups),
                                hp.ns_steps),
                   "tp": tp, "elements": total_elems},
        "tflops_algorithmic": tflops, "ns_flops_per_step": flops_step,
        "tflops_issued": issued_step / (ms_per_step * 1e-3) / 1e12, "issued_flops_per_step": issued_step,
        "frac_mfma_peak_issued": issued_step / (ms_per_step * 1e-3) / 1e12 / peak,
        "frac_mfma_peak_algorithmic": tflops / peak,
        "step_ms_events": {"median": float(np.median(per_step)), "min": float(min(per_step))},
        "device": device, "planner": diag, "kernels": kernels, "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
