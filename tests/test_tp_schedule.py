"""TP micro-group scheduler (Algorithm 2 / 3 / 4): oracle pins and bit-exact parity of
canz_tp_schedule with the oracle."""
import itertools
import random

import pytest

from oracle import tp_schedule as TS
from paper_2602_06079_amd import workloads as W


def _check_valid(cost, R, cmax, groups, loads):
    flat = [p for g in groups for p, _ in g]
    assert sorted(flat) == list(range(len(cost)))                       # every tensor exactly once
    order = sorted(range(len(cost)), key=lambda p: (-cost[p], p))
    assert flat == order                                                # groups are consecutive runs of the LPT order
    for g, l in zip(groups, loads):
        per_rank = [0] * R
        for p, r in g:
            assert 0 <= r < R
            per_rank[r] += cost[p]
        assert max(per_rank) == l and l <= cmax                         # reported makespan, capacity respected


def test_hand_worked_rollback():
    # costs 5,4,3,3,2 on 2 ranks, capacity 7 (derivation in the comments)
    cost = [5, 4, 3, 3, 2]
    groups, loads = TS.tp_schedule(cost, 2, 7)
    # {5}->r0; {5,4}->r0,r1; third: 3 joins r1 (4 < 5): loads 5,7; fourth: 3 joins r0: 8 > 7 -> roll back
    assert groups[0] == [(0, 0), (1, 1), (2, 1)] and loads[0] == 7
    # next group: 3 -> r0, 2 -> r1
    assert groups[1] == [(3, 0), (4, 1)] and loads[1] == 3
    assert len(groups) == 2


def test_heap_order_is_load_then_rank():
    groups, loads = TS.tp_schedule([2, 2, 2, 2], 3, 100)
    assert groups == [[(0, 0), (1, 1), (2, 2), (3, 0)]] and loads == [4]
    assert TS.min_heap_solver([7, 5, 5, 3], 2) == ([0, 1, 1, 0], 10)


def test_single_tensor_above_capacity_is_an_error():
    with pytest.raises(ValueError):
        TS.tp_schedule([3, 9, 1], 4, 8)
    with pytest.raises(ValueError):
        TS.tp_schedule([1], 0, 8)


def test_groups_are_maximal_prefixes():
    """Greedy packing: a group is closed only because the next tensor would break the
    capacity (Priority 2 of Sec. 4.2: pack as much as fits)."""
    rng = random.Random(3)
    for _ in range(200):
        n, R = rng.randint(1, 14), rng.randint(1, 4)
        cost = [rng.randint(1, 20) for _ in range(n)]
        cmax = max(cost) + rng.randint(0, 25)
        groups, loads = TS.tp_schedule(cost, R, cmax)
        _check_valid(cost, R, cmax, groups, loads)
        order = sorted(range(n), key=lambda p: (-cost[p], p))
        pos = 0
        for g in groups[:-1]:
            pos += len(g)
            trial = [cost[p] for p, _ in g] + [cost[order[pos]]]
            assert TS.min_heap_solver(trial, R)[1] > cmax


def test_lpt_bound_against_brute_force():
    """Graham's bound for LPT: L_max <= (4/3 - 1/(3R)) * OPT, OPT by enumeration."""
    rng = random.Random(5)
    for _ in range(150):
        n, R = rng.randint(1, 8), rng.randint(1, 3)
        cost = sorted((rng.randint(1, 30) for _ in range(n)), reverse=True)
        host, l_max = TS.min_heap_solver(cost, R)
        opt = min(max(sum(c for c, r in zip(cost, assign) if r == k) for k in range(R))
                  for assign in itertools.product(range(R), repeat=n))
        assert opt <= l_max <= (4.0 / 3.0 - 1.0 / (3 * R)) * opt + 1e-9


def test_library_matches_oracle(canz):
    rng = random.Random(11)
    for _ in range(300):
        n, R = rng.randint(0, 40), rng.randint(1, 8)
        cost = [rng.choice([0, 1, 5, 64, 1000, 4096, 10 ** 6]) * rng.randint(1, 9) for _ in range(n)]
        cmax = (max(cost) if cost else 0) + rng.choice([0, 1, 10 ** 3, 10 ** 7])
        assert canz.canz_tp_schedule(cost, R, cmax) == TS.tp_schedule(cost, R, cmax)
    with pytest.raises(canz.CanzError) as e:
        canz.canz_tp_schedule([3, 9, 1], 4, 8)
    assert e.value.code == canz.ESHAPE
    with pytest.raises(canz.CanzError) as e:
        canz.canz_tp_schedule([3], 0, 8)
    assert e.value.code == canz.EINVAL


def test_config5_schedule(canz):
    """The 8B-shaped set under TP = 4 with numel costs and a 512 MB (bf16) group capacity."""
    s = W.matrix_set(5)
    cost = [r * c for r, c in zip(s["rows"], s["cols"])]
    cmax = 512 * 1024 * 1024 // 2
    groups, loads = canz.canz_tp_schedule(cost, 4, cmax)
    assert (groups, loads) == TS.tp_schedule(cost, 4, cmax)
    _check_valid(cost, 4, cmax, groups, loads)
    # the heaviest matrices (12288 x 4096 = 50 M elements) fill a rank alone 5 times over
    assert all(l <= cmax for l in loads) and len(groups) >= 252 * 33_554_432 // (4 * cmax)


def test_host_rank_walk_of_the_schedule(canz):
    """tp_runtime.host_rank_calls: per micro-group of the sequence, the tensors one host rank hosts,
    batched by shape - every tensor exactly once over all ranks, batches shape-homogeneous and equal
    to the oracle's micro-group plan restricted to that micro-group (CPU only)."""
    from oracle import microgroup as OMG
    from paper_2602_06079_amd import tp_runtime as T
    layer = [(512, 512), (128, 512), (128, 512), (512, 512), (1536, 512), (1536, 512), (512, 1536)]
    rows = [r for _ in range(5) for r, _c in layer]
    cols = [c for _ in range(5) for _r, c in layer]
    cost = [r * c for r, c in zip(rows, cols)]
    dtype = [1] * len(rows)
    schedule, loads = canz.canz_tp_schedule(cost, 4, 1_600_000)
    assert (schedule, loads) == TS.tp_schedule(cost, 4, 1_600_000)
    seen = []
    for rank in range(4):
        calls = T.host_rank_calls(schedule, rank, rows, cols, dtype)
        assert len(calls) == len(schedule)
        for mg, batches in zip(schedule, calls):
            owner = [-1] * len(rows)
            for t, h in mg:
                owner[t] = h
            assert batches == OMG.microgroup_plan(rows, cols, dtype, owner, rank, max_mats=0)
            for ids in batches:
                assert len({(rows[p], cols[p]) for p in ids}) == 1
                seen += ids
    assert sorted(seen) == list(range(len(rows)))
    assert T.host_rank_loads(schedule, cost, 4) == [sum(cost[t] for mg in schedule for t, h in mg if h == r) for r in range(4)]
