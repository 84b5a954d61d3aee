"""Runtime side of the TP schedule: walk the pre-computed micro-group sequence on one host rank.

The offline planner (canz_tp_schedule: Algorithm 2, Sec. 4.2; Algorithms 3 and 4, App. C)
fixes, once, the sequence of micro-groups and the host rank of every tensor.  At run time a
rank simply iterates through that sequence (Sec. 4.2, "Integration with Runtime Workflow"):
for micro-group k it receives the fragments of the tensors it hosts (stage (1), the
All-to-All, outside this build), computes their updates (stage (2)) and returns the Delta W
fragments (stage (3)).  Stage (2) for one micro-group is one canz_muon_step call on the
tensors this rank hosts in it, batched by shape with canz_microgroup_plan (owner = host rank,
restricted to the members of the micro-group).

Everything here is call sequencing and argument marshalling; the planning runs in the
library's host code and the arithmetic in its kernels.
"""
from __future__ import annotations

from typing import Callable, List, Sequence

import numpy as np

from . import binding as canz


def host_rank_loads(schedule, cost, n_ranks) -> List[int]:
    """Total cost each host rank computes over the whole sequence."""
    load = [0] * n_ranks
    for mg in schedule:
        for t, h in mg:
            load[h] += int(cost[t])
    return load


def host_rank_calls(schedule, rank, rows, cols, dtype) -> List[List[List[int]]]:
    """For every micro-group of the sequence, in order: the same-shape batches (lists of
    tensor ids, largest shape first, ids ascending) of the tensors ``rank`` hosts in it.
    A micro-group in which the rank hosts nothing gives an empty list (the rank still takes
    part in that micro-group's exchanges)."""
    n = len(rows)
    calls = []
    for mg in schedule:
        owner = np.full(n, -1, dtype=np.int32)
        for t, h in mg:
            owner[t] = h
        calls.append(canz.canz_microgroup_plan(rows, cols, dtype, owner, rank, max_mats=0))
    return calls


def run_host_rank(calls: Sequence[Sequence[Sequence[int]]], make_group: Callable[[Sequence[int]], "canz.Group"],
                  hp: "canz.Hparams", workspace, workspace_bytes: int, stream=0) -> int:
    """One canz_muon_step per micro-group, in sequence order, on ``stream``.
    make_group(ids) returns the canz.Group (device buffers) of one same-shape batch.
    Returns the number of library calls issued."""
    issued = 0
    for batches in calls:
        if not batches:
            continue
        canz.canz_muon_step([make_group(ids) for ids in batches], hp, workspace, workspace_bytes, stream)
        issued += 1
    return issued


def workspace_bytes(calls, make_group, hp) -> int:
    """The largest workspace any call of the sequence needs."""
    need = 0
    for batches in calls:
        if batches:
            need = max(need, canz.canz_muon_workspace_bytes([make_group(ids) for ids in batches], hp))
    return need
