"""Oracle: alpha-balanced greedy LPT partitioning (Algorithm 1, Sec. 3.2).

Test infrastructure only (see the package docstring).  Plain Python: integer
loads are Python ints, every real quantity is a Python float (IEEE fp64) and
the operations are taken in the order the algorithm lists them, so that an
independent implementation using the same order reproduces every decision
bit for bit.  ``partition_alpha_exact`` replays the same algorithm in exact
rationals and reports how close any decision came to a tie.

Readings of points the paper leaves open (the design notes of the repository list them too):

* cuts are parameter indices inside the bucket (the domain of Phi_i in the
  "Define" lines of Algorithm 1), not element offsets;
* ranks are numbered 0..R-1 here (the paper counts from 1);
* buckets of equal total load are visited in ascending original index
  (a stable sort for the "Sort" line);
* when two feasible cuts are equally close to the running target C the
  smaller index wins ("arg min" line of Step (4));
* a rank may receive an empty slice of a bucket (0 is a feasible cut).
"""
from __future__ import annotations

from fractions import Fraction

COST_NUMEL = 0      # W(p) = numel(p), the paper's default (Sec. 3.2)
COST_NS_FLOPS = 1   # W(p) = FLOPs of the Newton-Schulz chain (App. D.5 ablation)
COST_SHAMPOO_FLOPS = 2  # W(p) = FLOPs of a Shampoo step in units of 2^20 (App. D.5: cost follows the operator)
COST_SOAP_FLOPS = 3     # W(p) = FLOPs of a SOAP step, refresh every 10th step, in units of 2^20


def ns_flops(rows: int, cols: int, ns_steps: int = 5) -> int:
    """FLOPs of ns_steps quintic Newton-Schulz steps on a rows x cols matrix.

    With m = min(rows, cols) and n = max(rows, cols) one step is the Gram
    product X X^T (2 m^2 n), the square A A (2 m^3) and the product B X
    (2 m^2 n).  This is the "exact FLOPs" cost of App. D.5.
    """
    m, n = (rows, cols) if rows <= cols else (cols, rows)
    return ns_steps * (4 * m * m * n + 2 * m * m * m)


def shampoo_flops(rows: int, cols: int, root_iters: int = 25) -> int:
    """FLOPs of one Shampoo step on a rows x cols matrix (the non-linear cost of
    App. D.5 for this operator): the two statistics G G^T and G^T G
    (2 r^2 c + 2 c^2 r), the two preconditioning products L^(-1/4) G and (.) R^(-1/4)
    (the same again), and the two inverse fourth roots, each root_iters rounds of four
    d x d products of 2 d^3 (the matmul-only root finder): 8 root_iters (r^3 + c^3).
    """
    r, c = int(rows), int(cols)
    return 4 * r * r * c + 4 * c * c * r + 8 * root_iters * (r ** 3 + c ** 3)


SOAP_COST_MAX_PRECOND_DIM = 10000   # the limit the cost model assumes: the cited implementation's default


def soap_flops(rows: int, cols: int, refresh_every: int = 10, max_precond_dim: int = SOAP_COST_MAX_PRECOND_DIM) -> int:
    """FLOPs of one SOAP step on a rows x cols matrix, averaged over a refresh period.  The cost follows the
    operator (App. D.5), and the operator keeps no basis on a side longer than max_precond_dim: only a side of
    extent d within the limit costs, per step, its share of the rotation of G and of M into the bases, of the
    rotation of the direction back and its statistic, four times 2 r c d; and per refresh the product S Q
    (2 d^3), the Householder QR (4/3 d^3) and the accumulation of its orthogonal factor (4/3 d^3).
    Rounded down.  A matrix with both sides above the limit costs nothing here (the step does not take it).
    """
    r, c = int(rows), int(cols)
    sides = [d for d in (r, c) if d <= max_precond_dim]
    return (3 * refresh_every * 8 * r * c * sum(sides) + 14 * sum(d ** 3 for d in sides)) // (3 * refresh_every)


def param_cost(rows, cols, cost_kind: int = COST_NUMEL, ns_steps: int = 5):
    """W(p) for every parameter, as Python ints."""
    if cost_kind == COST_SOAP_FLOPS:
        return [soap_flops(int(r), int(c)) >> 20 for r, c in zip(rows, cols)]
    if cost_kind == COST_SHAMPOO_FLOPS:
        # in units of 2^20 FLOPs, rounded down, so that the loads of a large model stay exact in fp64
        return [shampoo_flops(int(r), int(c)) >> 20 for r, c in zip(rows, cols)]
    if cost_kind == COST_NUMEL:
        return [int(r) * int(c) for r, c in zip(rows, cols)]
    if cost_kind == COST_NS_FLOPS:
        return [ns_flops(int(r), int(c), ns_steps) for r, c in zip(rows, cols)]
    raise ValueError("unknown cost_kind %r" % (cost_kind,))


def _check_inputs(n_params, bucket_off, n_ranks, alpha):
    if n_ranks < 1:
        raise ValueError("n_ranks must be >= 1")
    if not (0.0 <= alpha <= 1.0):
        raise ValueError("alpha must lie in [0, 1]")
    if len(bucket_off) < 1 or bucket_off[0] != 0 or bucket_off[-1] != n_params:
        raise ValueError("bucket_off must start at 0 and end at n_params")
    for lo, hi in zip(bucket_off[:-1], bucket_off[1:]):
        if hi < lo:
            raise ValueError("bucket_off must be non-decreasing")


def _prefix_loads(cost, lo, hi):
    """Phi of one bucket: load of its first u parameters, u = 0 .. size (the boundaries a cut may use)."""
    acc = [0]
    for p in range(lo, hi):
        acc.append(acc[-1] + cost[p])
    return acc


def _rank_shares(load, mu, alpha, real):
    """The fraction of the next bucket each rank should take: alpha times its share of the total
    deficit below the mean load mu (an even share if nobody is below), plus 1 - alpha times an even share."""
    n_ranks = len(load)
    deficit = []
    for r in range(n_ranks):
        gap = mu - real(load[r])
        deficit.append(gap if gap > 0 else real(0))
    total_deficit = real(0)
    for r in range(n_ranks):
        total_deficit = total_deficit + deficit[r]
    even = real(1) / real(n_ranks)
    shares = []
    for r in range(n_ranks):
        fill = deficit[r] / total_deficit if total_deficit > 0 else even
        shares.append((real(1) - real(alpha)) * even + real(alpha) * fill)
    return shares


def _nearest_boundary(prefix, goal, real):
    """Index u whose prefix load is closest to goal (the smaller u on a tie), and by how much the
    runner-up is further away (None if there is no other boundary)."""
    dist = [abs(real(x) - goal) for x in prefix]
    best = 0
    for u in range(1, len(dist)):
        if dist[u] < dist[best]:
            best = u
    others = [g for u, g in enumerate(dist) if u != best]
    return best, (min(others) - dist[best] if others else None)


def _algorithm1(cost, bucket_off, n_ranks, alpha, real, margin_log=None):
    """Algorithm 1 (Sec. 3.2) with the real-number type given by ``real``.

    ``real`` converts an int (or the float alpha) into the number type used for the mean load,
    the deficits, the shares and the running goal: ``float`` for the fp64 oracle, ``Fraction``
    for the exact replay.  Buckets are taken heaviest first; each is cut at the parameter
    boundaries nearest to the running sums of (bucket load x rank share).
    """
    n_buckets = len(bucket_off) - 1
    prefix = [_prefix_loads(cost, bucket_off[i], bucket_off[i + 1]) for i in range(n_buckets)]
    bucket_load = [prefix[i][-1] for i in range(n_buckets)]
    load = [0] * n_ranks
    mu = real(sum(bucket_load)) / real(n_ranks)
    heaviest_first = sorted(range(n_buckets), key=lambda i: (-bucket_load[i], i))
    cuts = [[0] * (n_ranks + 1) for _ in range(n_buckets)]
    for k in heaviest_first:
        shares = _rank_shares(load, mu, alpha, real)
        goal = real(0)
        for r in range(n_ranks - 1):
            goal = goal + real(bucket_load[k]) * shares[r]
            cut, margin = _nearest_boundary(prefix[k], goal, real)
            if margin_log is not None and margin is not None:
                margin_log.append((margin, k, r + 1))
            cuts[k][r + 1] = cut
            load[r] += prefix[k][cut] - prefix[k][cuts[k][r]]
        cuts[k][n_ranks] = len(prefix[k]) - 1
        load[n_ranks - 1] += prefix[k][-1] - prefix[k][cuts[k][n_ranks - 1]]
    return cuts, load


def _owners(cuts, bucket_off, n_ranks, n_params):
    owner = [-1] * n_params
    for i in range(len(bucket_off) - 1):
        for r in range(n_ranks):
            for u in range(cuts[i][r], cuts[i][r + 1]):
                owner[bucket_off[i] + u] = r
    return owner


def partition_alpha(rows, cols, bucket_off, n_ranks, alpha,
                    cost=None, cost_kind=COST_NUMEL):
    """Algorithm 1 in fp64.  Returns (cuts, owner, load).

    cuts[i][r] .. cuts[i][r+1] is the half-open range of parameter indices
    (relative to bucket i) owned by rank r; owner[p] is the owning rank of
    parameter p; load[r] is the final accumulated load L_r in cost units.
    """
    n_params = len(rows)
    bucket_off = [int(x) for x in bucket_off]
    _check_inputs(n_params, bucket_off, n_ranks, alpha)
    if cost is None:
        cost = param_cost(rows, cols, cost_kind)
    cost = [int(c) for c in cost]
    if any(c < 0 for c in cost):
        raise ValueError("costs must be non-negative")
    cuts, load = _algorithm1(cost, bucket_off, n_ranks, float(alpha), float)
    owner = _owners(cuts, bucket_off, n_ranks, n_params)
    return cuts, owner, load


def partition_alpha_exact(rows, cols, bucket_off, n_ranks, alpha,
                          cost=None, cost_kind=COST_NUMEL):
    """The same algorithm in exact rationals.

    Returns (cuts, owner, load, min_margin, n_ties): min_margin is the
    smallest non-zero difference between the best and the second-best
    |Phi(u) - C| over all decisions (None if there was no decision with two
    candidates), n_ties the number of decisions with an exact tie.  alpha is
    taken as the exact value of the fp64 number passed in.
    """
    n_params = len(rows)
    bucket_off = [int(x) for x in bucket_off]
    _check_inputs(n_params, bucket_off, n_ranks, alpha)
    if cost is None:
        cost = param_cost(rows, cols, cost_kind)
    cost = [int(c) for c in cost]
    log = []
    cuts, load = _algorithm1(cost, bucket_off, n_ranks, float(alpha), Fraction, log)
    owner = _owners(cuts, bucket_off, n_ranks, n_params)
    nonzero = [m for m, _, _ in log if m != 0]
    n_ties = sum(1 for m, _, _ in log if m == 0)
    return cuts, owner, load, (min(nonzero) if nonzero else None), n_ties


# --------------------------------------------------------------------------
# Diagnostics: Eq. 2 (J_DP), Eq. 3 (J_Comm), Eq. 6 (R_LB), Eq. 1 (naive rule)
# --------------------------------------------------------------------------

def r_lb(values) -> float:
    """Load-balance ratio max_r v_r / avg_r v_r (Eq. 6)."""
    values = [float(v) for v in values]
    avg = sum(values) / len(values)
    return max(values) / avg if avg > 0 else 1.0


def j_dp(load) -> float:
    """Largest deviation of a rank's total load from the mean (Eq. 2)."""
    mu = float(sum(load)) / len(load)
    return max(abs(float(l) - mu) for l in load)


def j_comm(cuts, numel, bucket_off) -> float:
    """Sum over buckets and ranks of |S_{i,r} - |B_i|/R| in elements (Eq. 3)."""
    total = 0.0
    for i in range(len(bucket_off) - 1):
        sizes = [int(numel[p]) for p in range(bucket_off[i], bucket_off[i + 1])]
        pre = [0]
        for s in sizes:
            pre.append(pre[-1] + s)
        R = len(cuts[i]) - 1
        for r in range(R):
            s_ir = pre[cuts[i][r + 1]] - pre[cuts[i][r]]
            total += abs(s_ir - pre[-1] / R)
    return total


def rank_loads(owner, values, n_ranks):
    """Sum of values[p] over the parameters each rank owns."""
    out = [0] * n_ranks
    for p, r in enumerate(owner):
        out[r] += values[p]
    return out


def ownership_naive(numel, n_ranks, bucket_off=None):
    """Atomic Ownership Rule (Eq. 1), 0-based, applied to every bucket on its own (the
    uniform partition rule of App. B.1 cuts each bucket into R equal segments): with stride
    S = |B_i|/R, rank r owns p iff r*S <= Start_Index(p) < (r+1)*S, the start index taken
    inside the bucket.  Integer arithmetic: r = floor(start * R / |B_i|).  Without
    bucket_off the whole buffer is one bucket (the reading of Sec. 3.1's "total buffer")."""
    if bucket_off is None:
        bucket_off = [0, len(numel)]
    owner = []
    for lo, hi in zip(bucket_off[:-1], bucket_off[1:]):
        total = sum(int(x) for x in numel[lo:hi])
        start = 0
        for x in numel[lo:hi]:
            owner.append(min(n_ranks - 1, (start * n_ranks) // total) if total > 0 else 0)
            start += int(x)
    return owner
