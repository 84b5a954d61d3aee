"""Oracle: TP micro-group construction with greedy rollback (Algorithm 2 in Sec. 4.2;
detailed as Algorithms 3 and 4 in App. C "Detailed Walkthrough").

Test infrastructure only (see the package docstring).

Tensors are taken in LPT order (cost descending; equal costs in ascending id - the
deterministic (W(p), ID_p) key of Algorithm 2 read as a stable sort).  A candidate group
grows one tensor at a time; after each addition the group is scheduled onto the R host
ranks with the LPT rule on a min-heap of (load, rank) pairs, and if the largest rank load
L_max exceeds the capacity C_max the addition is rolled back: the group without that tensor
is final, and the tensor opens the next group.  A tensor that alone exceeds C_max is an
error.  Inside a group the solver assigns, in cost order, each tensor to the rank whose
(load, rank) pair is smallest.
"""
from __future__ import annotations

def min_heap_solver(costs, n_ranks):
    """The group solver (Algorithm 4): items in the given (descending) order, each to the rank
    whose (load, rank) pair is smallest - what popping a min-heap of such pairs yields, written
    here as a plain minimum over the ranks.  Returns (host rank per item, L_max)."""
    load = [0] * n_ranks
    host = []
    for c in costs:
        r = min(range(n_ranks), key=lambda q: (load[q], q))
        host.append(r)
        load[r] += c
    return host, max(load)


def tp_schedule(cost, n_ranks, cmax):
    """Returns a list of groups; each group is a list of (tensor id, host rank) in the order
    the solver assigned them, plus the list of L_max per group."""
    if n_ranks < 1:
        raise ValueError("n_ranks must be >= 1")
    if cmax < 0 or any(c < 0 for c in cost):
        raise ValueError("costs and capacity must be non-negative")
    order = sorted(range(len(cost)), key=lambda p: (-cost[p], p))
    groups, loads = [], []
    current = []
    for p in order:
        trial = current + [p]
        _, l_max = min_heap_solver([cost[q] for q in trial], n_ranks)
        if l_max <= cmax:
            current = trial
            continue
        if not current:
            raise ValueError("tensor %d alone exceeds the capacity" % p)
        host, l_fin = min_heap_solver([cost[q] for q in current], n_ranks)
        groups.append(list(zip(current, host)))
        loads.append(l_fin)
        # the tensor that did not fit opens the next group (it must fit alone)
        _, l_one = min_heap_solver([cost[p]], n_ranks)
        if l_one > cmax:
            raise ValueError("tensor %d alone exceeds the capacity" % p)
        current = [p]
    if current:
        host, l_fin = min_heap_solver([cost[q] for q in current], n_ranks)
        groups.append(list(zip(current, host)))
        loads.append(l_fin)
    return groups, loads
