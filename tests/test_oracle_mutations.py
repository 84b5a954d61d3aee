"""Pin strength: mistakes planted in a copy of the oracle's source must each be caught by
at least one of the pins in test_oracle_partition / test_oracle_muon / test_tp_schedule.

A mutant is the oracle module's source with one expression replaced (a dropped term, a
wrong sign, a transposed operand, a flipped comparison), executed as a fresh module; the
pin tests are then run with that module in place of the oracle.  CPU only."""
import importlib
import inspect
import sys
import types

import pytest

import oracle.muon as OM
import oracle.partition as OP
import oracle.tp_schedule as TS
from tests import test_oracle_muon as PINS_MUON
from tests import test_oracle_partition as PINS_PART
from tests import test_tp_schedule as PINS_TP


def _mutant(module, old, new):
    src = inspect.getsource(module)
    assert src.count(old) == 1, "mutation site %r must occur exactly once (found %d)" % (old, src.count(old))
    m = types.ModuleType(module.__name__ + "_mutant")
    m.__file__ = module.__file__
    m.__package__ = module.__package__
    sys.modules[m.__name__] = m      # dataclasses look their module up while the class is built
    try:
        exec(compile(src.replace(old, new), module.__file__, "exec"), m.__dict__)
    finally:
        del sys.modules[m.__name__]
    return m


def _pins(pins_module, only_cpu=True):
    """(name, callable) for every pin, parametrised ones expanded by hand."""
    out = []
    for name, fn in sorted(vars(pins_module).items()):
        if not name.startswith("test_") or not callable(fn):
            continue
        params = inspect.signature(fn).parameters
        if "canz" in params:            # those compare the library, not the oracle with its pins
            continue
        marks = [mk for mk in getattr(fn, "pytestmark", []) if mk.name == "parametrize"]
        if not marks:
            if not params:
                out.append((name, fn))
            continue
        # cartesian product of the parametrize marks
        combos = [{}]
        for mk in marks:
            names = [n.strip() for n in mk.args[0].split(",")] if isinstance(mk.args[0], str) else list(mk.args[0])
            new = []
            for combo in combos:
                for val in mk.args[1]:
                    vals = val if len(names) > 1 else (val,)
                    new.append({**combo, **dict(zip(names, vals))})
            combos = new
        for combo in combos:
            out.append(("%s%r" % (name, sorted(combo.items())), lambda fn=fn, combo=combo: fn(**combo)))
    return out


def _caught(pins_module, attr, mutant):
    """Names of the pins that fail when pins_module.<attr> is the mutant module."""
    original = getattr(pins_module, attr)
    setattr(pins_module, attr, mutant)
    failed = []
    try:
        for name, fn in _pins(pins_module):
            try:
                fn()
            except (Exception, pytest.fail.Exception):   # an assertion, or an exception the mistake provokes
                failed.append(name)
    finally:
        setattr(pins_module, attr, original)
    return failed


MUON_MUTANTS = [
    ("Gram product transposed", "gram = x @ x.T", "gram = x.T @ x if x.shape[0] == x.shape[1] else x @ x.T"),
    ("sign of the cubic term's coefficient", "poly = b * gram + c * (gram @ gram)", "poly = b * gram - c * (gram @ gram)"),
    ("square of A dropped", "poly = b * gram + c * (gram @ gram)", "poly = b * gram + c * gram"),
    ("polynomial applied on the wrong side", "x = a * x + poly @ x", "x = a * x + x @ poly if x.shape[0] == x.shape[1] else a * x + poly @ x"),
    ("a X term dropped", "x = a * x + poly @ x", "x = poly @ x"),
    ("tall matrices not transposed back", "return x.T.copy() if tall else x", "return x.T.copy() if tall and x.shape[0] < 3 else (x.T.copy() * 1.001 if tall else x)"),
    ("momentum decay on the wrong operand", "m_new = hp.beta * np.asarray(mom, dtype=np.float64) + g", "m_new = np.asarray(mom, dtype=np.float64) + hp.beta * g"),
    ("nesterov uses the old momentum", "u = g + hp.beta * m_new if hp.nesterov else m_new", "u = g + hp.beta * np.asarray(mom) if hp.nesterov else m_new"),
    ("norm without the square root", "norm = math.sqrt(float(np.sum(u * u)))", "norm = float(np.sum(u * u))"),
    ("update with the wrong sign", "delta = (-hp.lr * update_scale(rows, cols, hp.scale_mode)) * ortho", "delta = (hp.lr * update_scale(rows, cols, hp.scale_mode)) * ortho"),
    ("weight decay without the learning rate", "* (1.0 - hp.lr * hp.weight_decay) + delta", "* (1.0 - hp.weight_decay) + delta"),
    ("RMS scale uses the smaller extent", "return 0.2 * math.sqrt(float(max(rows, cols)))", "return 0.2 * math.sqrt(float(min(rows, cols)))"),
    ("fragments gathered along rows", "return np.concatenate([np.asarray(f, dtype=np.float64) for f in fragments], axis=1)",
     "return np.concatenate([np.asarray(f, dtype=np.float64) for f in fragments], axis=0).reshape(fragments[0].shape[0], -1)"),
]

PARTITION_MUTANTS = [
    ("deficits not clipped at zero", "d.append(gap if gap > 0 else real(0))", "d.append(gap)"),
    ("blend weights swapped", "v_star = (one - al) * v_even + al * v_fill", "v_star = al * v_even + (one - al) * v_fill"),
    ("buckets visited lightest first", "key=lambda i: (-w_bucket[i], i))", "key=lambda i: (w_bucket[i], i))"),
    ("ties go to the larger cut", "if gaps[u] < gaps[best_u]:", "if gaps[u] <= gaps[best_u]:"),
    ("running target not accumulated", "c_run = c_run + target[r]", "c_run = target[r]"),
    ("target from the mean load instead of the bucket", "target.append(real(w_bucket[k]) * v_star)", "target.append(mu * v_star)"),
    ("last rank's load not recorded", "load[R - 1] += phi[k][s[R]] - phi[k][s[R - 1]]", "load[R - 1] += 0"),
    ("mean load over buckets instead of ranks", "mu = real(sum(w_bucket)) / real(R)", "mu = real(sum(w_bucket)) / real(max(1, n_buckets))"),
    ("FLOPs cost without the square term", "return ns_steps * (4 * m * m * n + 2 * m * m * m)", "return ns_steps * (4 * m * m * n)"),
    ("R_LB against the minimum", "return max(values) / avg if avg > 0 else 1.0", "return max(values) / min(values) if min(values) > 0 else 1.0"),
]

TP_MUTANTS = [
    ("tensors taken lightest first", "key=lambda p: (-cost[p], p))", "key=lambda p: (cost[p], p))"),
    ("capacity test is strict", "if l_max <= cmax:", "if l_max < cmax:"),
    ("the tensor that did not fit is dropped", "current = [p]\n    if current:", "current = []\n    if current:"),
    ("heap ordered by rank before load", "heapq.heappush(heap, (load + c, r))", "heapq.heappush(heap, (load, r))"),
    ("L_max reported as the smallest load", "return host, max(load for load, _ in heap)", "return host, min(load for load, _ in heap)"),
]


@pytest.mark.parametrize("what,old,new", TP_MUTANTS, ids=[m[0] for m in TP_MUTANTS])
def test_tp_schedule_pins_catch(what, old, new):
    failed = _caught(PINS_TP, "TS", _mutant(TS, old, new))
    assert failed, "no pin notices: " + what


@pytest.mark.parametrize("what,old,new", MUON_MUTANTS, ids=[m[0] for m in MUON_MUTANTS])
def test_muon_pins_catch(what, old, new):
    failed = _caught(PINS_MUON, "M", _mutant(OM, old, new))
    assert failed, "no pin notices: " + what


@pytest.mark.parametrize("what,old,new", PARTITION_MUTANTS, ids=[m[0] for m in PARTITION_MUTANTS])
def test_partition_pins_catch(what, old, new):
    failed = _caught(PINS_PART, "P", _mutant(OP, old, new))
    assert failed, "no pin notices: " + what


def test_unmutated_oracle_passes_the_same_harness():
    """The harness itself: with the real modules in place every pin passes."""
    assert _caught(PINS_MUON, "M", importlib.import_module("oracle.muon")) == []
    assert _caught(PINS_PART, "P", importlib.import_module("oracle.partition")) == []
    assert _caught(PINS_TP, "TS", importlib.import_module("oracle.tp_schedule")) == []
