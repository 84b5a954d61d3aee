"""canz_partition_alpha and canz_microgroup_plan (host C++) against the oracle:
bit-exact on the five benchmark configurations and on randomised small cases."""
import random

import numpy as np
import pytest

from oracle import microgroup as OMG
from oracle import partition as OP
from paper_2602_06079_amd import workloads as W


def _same_partition(canz, rows, cols, off, R, alpha, cost=None, cost_kind=0):
    cuts, owner, load = canz.canz_partition_alpha(rows, cols, off, R, alpha, cost=cost, cost_kind=cost_kind)
    ocuts, oowner, oload = OP.partition_alpha(rows, cols, off, R, alpha, cost=cost, cost_kind=cost_kind)
    assert cuts.tolist() == ocuts
    assert owner.tolist() == oowner
    assert load.tolist() == oload
    return owner.tolist(), load.tolist()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_configs_bit_exact(canz, cfg):
    s = W.matrix_set(cfg)
    for alpha in sorted({s["alpha"], 0.0, 0.1, 0.5, 1.0}):
        for kind in (OP.COST_NUMEL, OP.COST_NS_FLOPS, OP.COST_SHAMPOO_FLOPS, OP.COST_SOAP_FLOPS):
            owner, load = _same_partition(canz, s["rows"], s["cols"], s["bucket_off"], s["n_ranks"], alpha,
                                          cost_kind=kind)
    owner, load = _same_partition(canz, s["rows"], s["cols"], s["bucket_off"], s["n_ranks"], s["alpha"])
    for rank in range(s["n_ranks"]):
        got = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, rank, max_mats=8)
        assert got == OMG.microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, rank, max_mats=8)


def test_config_shares(canz):
    """The shares the benchmark runs (rank 0 of config 2, heaviest rank of configs 3 and 4)."""
    s = W.matrix_set(2)
    _, owner, load = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], 8, 1.0)
    groups = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, 0)
    assert [len(g) for g in groups] == [8, 8, 8, 2]
    s = W.matrix_set(4)
    _, owner, load = canz.canz_partition_alpha(s["rows"], s["cols"], s["bucket_off"], 64, 1.0)
    heavy = int(np.argmax(load))
    groups = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], owner, heavy)
    assert len(groups) == 1 and [(s["rows"][p], s["cols"][p]) for p in groups[0]] == [(25600, 5120)] * 4
    s = W.matrix_set(5)
    groups = canz.canz_microgroup_plan(s["rows"], s["cols"], s["dtype"], [0] * len(s["rows"]), 0)
    assert len(groups) == 32 and sum(len(g) for g in groups) == 252


def test_random_cases_bit_exact(canz):
    rng = random.Random(77)
    for _ in range(400):
        nb = rng.randint(1, 6)
        off, rows, cols = [0], [], []
        for _ in range(nb):
            for _ in range(rng.randint(0, 9)):
                rows.append(rng.choice([1, 3, 64, 100, 1024, 4096]))
                cols.append(rng.choice([1, 7, 64, 300, 1024, 5120]))
            off.append(len(rows))
        R = rng.randint(1, 9)
        alpha = rng.choice([0.0, 0.1, 1 / 3, 0.5, 0.9, 1.0])
        kind = rng.randint(0, 2)
        if not rows:
            continue
        owner, _ = _same_partition(canz, rows, cols, off, R, alpha, cost_kind=kind)
        cost = [rng.randint(0, 10 ** 9) for _ in rows]
        _same_partition(canz, rows, cols, off, R, alpha, cost=cost)
        dtype = [rng.randint(0, 1) for _ in rows]
        for cap, cmax in ((0, 0), (3, 0), (8, 10 ** 7)):
            try:
                want = OMG.microgroup_plan(rows, cols, dtype, owner, 0, max_mats=cap, cmax_bytes=cmax)
            except ValueError:
                with pytest.raises(canz.CanzError) as e:
                    canz.canz_microgroup_plan(rows, cols, dtype, owner, 0, max_mats=cap, cmax_bytes=cmax)
                assert e.value.code == canz.ESHAPE
                continue
            assert canz.canz_microgroup_plan(rows, cols, dtype, owner, 0, max_mats=cap, cmax_bytes=cmax) == want


def test_tie_heavy_inputs_bit_exact(canz):
    """Equal costs put the running target exactly between boundaries again and again;
    the tie rule and the fp64 operation order must agree on both sides."""
    for R in (2, 3, 4, 6, 8):
        for per in (1, 2, 3, 5, 7):
            for nb in (1, 2, 5):
                rows = [16] * (per * nb)
                cols = [16] * (per * nb)
                off = [i * per for i in range(nb + 1)]
                for alpha in (0.0, 0.25, 0.5, 1.0):
                    _same_partition(canz, rows, cols, off, R, alpha)


def test_partition_errors(canz):
    def code(*a, **k):
        with pytest.raises(canz.CanzError) as e:
            canz.canz_partition_alpha(*a, **k)
        return e.value.code

    assert code([2, 2], [2, 2], [0, 2], 0, 0.5) == canz.EINVAL
    assert code([2, 2], [2, 2], [0, 2], 2, 1.5) == canz.EINVAL
    assert code([2, 2], [2, 2], [0, 2], 2, float("nan")) == canz.EINVAL
    assert code([2, 2], [2, 2], [0, 1], 2, 0.5) == canz.EINVAL
    assert code([2, 2], [2, 2], [0, 2, 1, 2], 2, 0.5) == canz.EINVAL
    assert code([2, 2], [2, 2], [0, 2], 2, 0.5, cost=[1, -1]) == canz.EINVAL
    assert code([2, 2], [2, 2], [0, 2], 2, 0.5, cost_kind=5) == canz.EUNSUPPORTED
    assert "cost_kind" in canz.canz_last_error()


def test_partition_naive_matches_oracle_and_eq1(canz):
    """Eq. 1 per bucket: rank r owns p iff r*S <= start(p) < (r+1)*S, S = |B_i|/R."""
    from fractions import Fraction
    rng = random.Random(5)
    for _ in range(200):
        nb, R = rng.randint(1, 4), rng.randint(1, 9)
        numel, off = [], [0]
        for _ in range(nb):
            numel += [rng.choice([0, 1, 7, 1024, 4096 * 4096, 25600 * 5120]) for _ in range(rng.randint(0, 9))]
            off.append(len(numel))
        owner, load = canz.canz_partition_naive(numel, R, off)
        assert owner.tolist() == OP.ownership_naive(numel, R, off)
        assert load.tolist() == OP.rank_loads(owner.tolist(), numel, R)
        for lo, hi in zip(off[:-1], off[1:]):
            total, start = sum(numel[lo:hi]), 0
            for p in range(lo, hi):
                if total > 0 and owner[p] < R - 1:
                    S = Fraction(total, R)
                    assert owner[p] * S <= start < (owner[p] + 1) * S
                start += numel[p]
    # one bucket = the whole buffer
    assert canz.canz_partition_naive([4, 2, 6], 3)[0].tolist() == [0, 1, 1]
    with pytest.raises(canz.CanzError):
        canz.canz_partition_naive([1, 2], 0)


def test_balance_report_runs_and_alpha1_beats_naive(canz):
    from paper_2602_06079_amd import balance_report
    text = balance_report.report((2,))
    rows = [l for l in text.splitlines() if l.startswith("| 2 ")]
    naive = float([l for l in rows if "per bucket" in l][0].split("|")[3])
    best = float([l for l in rows if "numel, alpha = 1.0" in l][0].split("|")[3])
    assert best < naive and best < 1.05


def test_overflowing_loads_are_errors_not_wraparound(canz):
    """Loads that do not stay exact (2^53 and above) and sums that would wrap int64 are refused."""
    big = 1 << 52
    with pytest.raises(canz.CanzError):
        canz.canz_partition_alpha([1, 1], [1, 1], [0, 2], 2, 1.0, cost=[big, big])
    with pytest.raises(canz.CanzError):
        canz.canz_partition_alpha([1], [1], [0, 1], 2, 1.0, cost=[1 << 62])
    with pytest.raises(canz.CanzError):        # 5 * (4 m^2 n + 2 m^3) far above 2^53
        canz.canz_partition_alpha([1 << 20], [1 << 20], [0, 1], 2, 1.0, cost_kind=canz.COST_NS_FLOPS)
    with pytest.raises(canz.CanzError):        # rows * cols would wrap int64
        canz.canz_partition_alpha([1 << 40], [1 << 40], [0, 1], 2, 1.0)
    with pytest.raises(canz.CanzError):
        canz.canz_tp_schedule([1 << 61, 1 << 61, 1 << 61], 2, (1 << 63) - 1)
    with pytest.raises(canz.CanzError):
        canz.canz_microgroup_plan([1 << 40], [8], [1], [0], 0)
    # just below the limits still works, bit-exact against the oracle
    ok = (1 << 51) - 3
    got = canz.canz_partition_alpha([1, 1], [1, 1], [0, 2], 2, 1.0, cost=[ok, ok])
    assert got[1].tolist() == OP.partition_alpha([1, 1], [1, 1], [0, 2], 2, 1.0, cost=[ok, ok])[1]
