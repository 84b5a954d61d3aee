"""Load-balance study of the planner on the synthetic Qwen3-shaped sets (CPU only).

Prints, for each set, the load-balance ratio R_LB = max_r / avg_r (Eq. 6) of the element
count ("memory"), of the Newton-Schulz FLOPs and of the Shampoo- and SOAP-step FLOPs per rank (the
load-balance analysis for Shampoo / SOAP of App. C), for the naive atomic ownership
rule (Eq. 1) and for Algorithm 1 at several alpha, with numel and with exact FLOPs as the
cost W(p) (the ablation of App. D.5), plus J_DP (Eq. 2) in elements.

Usage: python -m paper_2602_06079_amd.balance_report
"""
from __future__ import annotations

import numpy as np

from . import binding as canz
from . import workloads as W


def _ns_flops(rows, cols, steps=5):
    m, n = min(rows, cols), max(rows, cols)
    return steps * (4 * m * m * n + 2 * m ** 3)


def _shampoo_flops(rows, cols, root_iters=25):
    return 4 * rows * cols * (rows + cols) + 8 * root_iters * (rows ** 3 + cols ** 3)


def _soap_flops(rows, cols, refresh_every=10, max_precond_dim=10000):
    sides = [d for d in (rows, cols) if d <= max_precond_dim]      # a longer side keeps no basis and costs nothing
    return 8 * rows * cols * sum(sides) + 14 * sum(d ** 3 for d in sides) / (3 * refresh_every)


def _ratio(v):
    v = np.asarray(v, dtype=np.float64)
    return float(v.max() / v.mean()) if v.mean() > 0 else 1.0


def report(cfgs=(2, 3, 4)):
    lines = []
    for cfg in cfgs:
        s = W.matrix_set(cfg)
        R = s["n_ranks"]
        numel = np.array([r * c for r, c in zip(s["rows"], s["cols"])], dtype=np.int64)
        flops = np.array([_ns_flops(r, c) for r, c in zip(s["rows"], s["cols"])], dtype=np.float64)
        sh_flops = np.array([_shampoo_flops(r, c) for r, c in zip(s["rows"], s["cols"])], dtype=np.float64)
        so_flops = np.array([_soap_flops(r, c) for r, c in zip(s["rows"], s["cols"])], dtype=np.float64)

        def row(name, owner):
            per_n = np.bincount(owner, weights=numel.astype(np.float64), minlength=R)
            per_f = np.bincount(owner, weights=flops, minlength=R)
            per_s = np.bincount(owner, weights=sh_flops, minlength=R)
            per_o = np.bincount(owner, weights=so_flops, minlength=R)
            lines.append("| %d %s R=%d | %s | %.3f | %.3f | %.3f | %.3f | %.3g |" %
                         (cfg, s["name"], R, name, _ratio(per_n), _ratio(per_f), _ratio(per_s), _ratio(per_o),
                          np.abs(per_n - per_n.mean()).max()))

        owner, _ = canz.canz_partition_naive(numel, R, s["bucket_off"])
        row("naive (Eq. 1 per bucket)", owner)
        owner, _ = canz.canz_partition_naive(numel, R)
        row("naive (Eq. 1, whole buffer)", owner)
        for alpha in (0.0, 0.1, 0.5, 1.0):
            _, owner, _ = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], R, alpha)
            row("Alg. 1, W = numel, alpha = %.1f" % alpha, owner)
        _, owner, _ = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], R, 1.0,
                                                cost_kind=canz.COST_NS_FLOPS)
        row("Alg. 1, W = FLOPs, alpha = 1.0", owner)
        _, owner, _ = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], R, 1.0,
                                                cost_kind=canz.COST_SHAMPOO_FLOPS)
        row("Alg. 1, W = Shampoo FLOPs, alpha = 1.0", owner)
        _, owner, _ = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], R, 1.0,
                                                cost_kind=canz.COST_SOAP_FLOPS)
        row("Alg. 1, W = SOAP FLOPs, alpha = 1.0", owner)
    head = ["| set | partition | R_LB elements | R_LB Muon FLOPs | R_LB Shampoo FLOPs | R_LB SOAP FLOPs | J_DP (elements) |",
            "|---|---|---|---|---|---|---|"]
    return "\n".join(head + lines)


if __name__ == "__main__":
    print(report())
