"""Pin strength: mistakes planted in a copy of the oracle's source must each be caught by
at least one of the pins in test_oracle_partition / test_oracle_muon / test_oracle_shampoo /
test_oracle_soap / test_tp_schedule.

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
import oracle.shampoo as SHO
import oracle.soap as SOO
import oracle.tp_schedule as TS
from tests import test_oracle_muon as PINS_MUON
from tests import test_oracle_partition as PINS_PART
from tests import test_oracle_shampoo as PINS_SHAMPOO
from tests import test_oracle_soap as PINS_SOAP
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
    ("deficits not clipped at zero", "deficit.append(gap if gap > 0 else real(0))", "deficit.append(gap)"),
    ("blend weights swapped", "shares.append((real(1) - real(alpha)) * even + real(alpha) * fill)", "shares.append(real(alpha) * even + (real(1) - real(alpha)) * fill)"),
    ("buckets visited lightest first", "key=lambda i: (-bucket_load[i], i))", "key=lambda i: (bucket_load[i], i))"),
    ("ties go to the larger cut", "if dist[u] < dist[best]:", "if dist[u] <= dist[best]:"),
    ("running target not accumulated", "goal = goal + real(bucket_load[k]) * shares[r]", "goal = real(bucket_load[k]) * shares[r]"),
    ("target from the mean load instead of the bucket", "goal = goal + real(bucket_load[k]) * shares[r]", "goal = goal + mu * shares[r]"),
    ("last rank's load not recorded", "load[n_ranks - 1] += prefix[k][-1] - prefix[k][cuts[k][n_ranks - 1]]", "load[n_ranks - 1] += 0"),
    ("mean load over buckets instead of ranks", "mu = real(sum(bucket_load)) / real(n_ranks)", "mu = real(sum(bucket_load)) / real(max(1, n_buckets))"),
    ("FLOPs cost without the square term", "return ns_steps * (4 * m * m * n + 2 * m * m * m)", "return ns_steps * (4 * m * m * n)"),
    ("R_LB against the minimum", "return max(values) / avg if avg > 0 else 1.0", "return max(values) / min(values) if min(values) > 0 else 1.0"),
]

TP_MUTANTS = [
    ("tensors taken lightest first", "key=lambda p: (-cost[p], p))", "key=lambda p: (cost[p], p))"),
    ("capacity test is strict", "if l_max <= cmax:", "if l_max < cmax:"),
    ("the tensor that did not fit is dropped", "current = [p]\n    if current:", "current = []\n    if current:"),
    ("ranks ordered by rank before load", "key=lambda q: (load[q], q))", "key=lambda q: (q, load[q]))"),
    ("L_max reported as the smallest load", "return host, max(load)", "return host, min(load)"),
]


SHAMPOO_MUTANTS = [
    ("left statistic from G^T G", "+ g @ g.T", "+ (g.T @ g if g.shape[0] == g.shape[1] else g @ g.T)"),
    ("right statistic from G G^T", "+ g.T @ g", "+ (g @ g.T if g.shape[0] == g.shape[1] else g.T @ g)"),
    ("decay on the new term", "new_left = beta * np.asarray(left, dtype=np.float64) + g @ g.T",
     "new_left = np.asarray(left, dtype=np.float64) + beta * (g @ g.T)"),
    ("inverse square root instead of fourth root", "return (vec * lam ** -0.25) @ vec.T", "return (vec * lam ** -0.5) @ vec.T"),
    ("ridge not added", "lam = np.maximum(lam, 0.0) + eps", "lam = np.maximum(lam, 0.0) + 0.0 * eps + 1e-300"),
    ("eigenvectors transposed", "return (vec * lam ** -0.25) @ vec.T", "return (vec.T * lam ** -0.25) @ vec"),
    ("preconditioned on the left only", "precond = left_root @ g @ right_root", "precond = left_root @ g"),
    ("roots on the wrong sides", "precond = left_root @ g @ right_root",
     "precond = right_root @ g @ left_root if g.shape[0] == g.shape[1] else left_root @ g @ right_root"),
    ("update with the wrong sign", "delta = -hp.lr * precond", "delta = hp.lr * precond"),
    ("weight decay without the learning rate", "* (1.0 - hp.lr * hp.weight_decay) + delta", "* (1.0 - hp.weight_decay) + delta"),
    ("right root taken of the left statistic", "right_root = inverse_fourth_root(new_right, hp.eps)",
     "right_root = inverse_fourth_root(new_left if new_left.shape == new_right.shape else new_right, hp.eps)"),
    ("roots of the statistics before the update", "left_root = inverse_fourth_root(new_left, hp.eps)",
     "left_root = inverse_fourth_root(np.asarray(left, dtype=np.float64), hp.eps)"),
    ("fragments gathered along rows", "return np.concatenate([np.asarray(f, dtype=np.float64) for f in fragments], axis=1)",
     "return np.concatenate([np.asarray(f, dtype=np.float64) for f in fragments], axis=0).reshape(fragments[0].shape[0], -1)"),
    ("kept roots ignored", "if kept_roots is None:", "if True:"),
    ("kept roots swapped", "left_root = np.asarray(kept_roots[0], dtype=np.float64)",
     "left_root = np.asarray(kept_roots[0] if np.shape(kept_roots[0]) != np.shape(kept_roots[1]) else kept_roots[1], dtype=np.float64)"),
    ("kept right root transposed", "right_root = np.asarray(kept_roots[1], dtype=np.float64)",
     "right_root = np.asarray(kept_roots[1], dtype=np.float64).T"),
]

SHAMPOO_COST_MUTANTS = [
    ("cubic cost of the roots dropped", "+ 8 * root_iters * (r ** 3 + c ** 3)", ""),
    ("cost of the statistics counted for one side", "return 4 * r * r * c + 4 * c * c * r", "return 4 * r * r * c"),
    ("cost units not scaled", "return [shampoo_flops(int(r), int(c)) >> 20", "return [shampoo_flops(int(r), int(c))"),
]


@pytest.mark.parametrize("what,old,new", SHAMPOO_MUTANTS, ids=[m[0] for m in SHAMPOO_MUTANTS])
def test_shampoo_pins_catch(what, old, new):
    failed = _caught(PINS_SHAMPOO, "SH", _mutant(SHO, old, new))
    assert failed, "no pin notices: " + what


SOAP_MUTANTS = [
    ("momentum without the (1 - beta1) weight", "+ (1.0 - hp.beta1) * g", "+ g"),
    ("momentum decays with beta2", "mom = hp.beta1 *", "mom = hp.beta2 *"),
    ("left basis not transposed on the way in", "np.asarray(q_left, dtype=np.float64).T @ y", "np.asarray(q_left, dtype=np.float64) @ y"),
    ("right basis not transposed on the way out", "y @ np.asarray(q_right, dtype=np.float64).T", "y @ np.asarray(q_right, dtype=np.float64)"),
    ("second moment of the unrotated gradient", "* grad_rot * grad_rot", "* g * g"),
    ("second moment of the momentum", "* grad_rot * grad_rot", "* mom_rot * mom_rot"),
    ("second moment without the (1 - beta2) weight", "+ (1.0 - hp.beta2) * grad_rot * grad_rot", "+ grad_rot * grad_rot"),
    ("eps inside the square root", "np.sqrt(v_hat) + hp.eps", "np.sqrt(v_hat + hp.eps)"),
    ("second moment corrected with beta1", "v_hat = v_rot / (1.0 - hp.beta2 ** t)", "v_hat = v_rot / (1.0 - hp.beta1 ** t)"),
    ("bias correction one step late", "m_hat = m_rot / (1.0 - hp.beta1 ** t)", "m_hat = m_rot / (1.0 - hp.beta1 ** (t + 1))"),
    ("update with the wrong sign", "delta = -hp.lr * direction", "delta = hp.lr * direction"),
    ("weight decay without the learning rate", "* (1.0 - hp.lr * hp.weight_decay) + delta", "* (1.0 - hp.weight_decay) + delta"),
    ("left statistic from G^T G", "* (g @ g.T)", "* (g.T @ g if g.shape[0] == g.shape[1] else g @ g.T)"),
    ("statistics decay with beta1", "left = hp.beta2 *", "left = hp.beta1 *"),
    ("statistics without the (1 - beta2) weight", "+ (1.0 - hp.beta2) * (g.T @ g)", "+ (g.T @ g)"),
    ("basis multiplied from the wrong side", "s = np.asarray(stat, dtype=np.float64) @ np.asarray(basis, dtype=np.float64)",
     "s = np.asarray(basis, dtype=np.float64) @ np.asarray(stat, dtype=np.float64)"),
    ("triangular factor returned", "q, _ = np.linalg.qr(s)", "_, q = np.linalg.qr(s)"),
    ("refresh from the statistics before the step", "q_left = refresh_basis(left, q_left)",
     "q_left = refresh_basis(np.asarray(state['left'], dtype=np.float64), q_left)"),
    ("right basis refreshed from the left statistic", "q_right = refresh_basis(right, q_right)",
     "q_right = refresh_basis(left if left is not None and left.shape == right.shape else right, q_right)"),
    ("step uses the refreshed basis of an earlier call", "grad_rot = rotate_in(g, q_left, q_right)",
     "grad_rot = rotate_in(g, q_left, None if q_right is None else np.asarray(q_right)[:, ::-1])"),
    ("limit excludes the extent equal to it", "use_left, use_right = rows <= hp.max_precond_dim, cols <= hp.max_precond_dim",
     "use_left, use_right = rows < hp.max_precond_dim, cols <= hp.max_precond_dim"),
    ("side above the limit still rotated", "q_left = np.asarray(state[\"q_left\"], dtype=np.float64) if use_left else None",
     "q_left = np.asarray(state[\"q_left\"], dtype=np.float64)"),
    ("fragments gathered along rows", "return np.concatenate([np.asarray(f, dtype=np.float64) for f in fragments], axis=1)",
     "return np.concatenate([np.asarray(f, dtype=np.float64) for f in fragments], axis=0).reshape(fragments[0].shape[0], -1)"),
]


SOAP_COST_MUTANTS = [
    ("refresh not spread over the period", "+ 14 * sum(d ** 3 for d in sides)) // (3 * refresh_every)",
     "+ 14 * sum(d ** 3 for d in sides) * refresh_every) // (3 * refresh_every)"),
    ("three rotations instead of four products", "3 * refresh_every * 8 * r * c * sum(sides)", "3 * refresh_every * 6 * r * c * sum(sides)"),
    ("side above the limit still counted", "sides = [d for d in (r, c) if d <= max_precond_dim]", "sides = [r, c]"),
    ("limit itself excluded", "sides = [d for d in (r, c) if d <= max_precond_dim]", "sides = [d for d in (r, c) if d < max_precond_dim]"),
    ("model's limit off by a factor", "SOAP_COST_MAX_PRECOND_DIM = 10000", "SOAP_COST_MAX_PRECOND_DIM = 100000"),
    ("cost units not scaled", "return [soap_flops(int(r), int(c)) >> 20", "return [soap_flops(int(r), int(c))"),
]


@pytest.mark.parametrize("what,old,new", SOAP_COST_MUTANTS, ids=[m[0] for m in SOAP_COST_MUTANTS])
def test_soap_cost_pins_catch(what, old, new):
    failed = _caught(PINS_SOAP, "OP", _mutant(OP, old, new))
    assert failed, "no pin notices: " + what


@pytest.mark.parametrize("what,old,new", SOAP_MUTANTS, ids=[m[0] for m in SOAP_MUTANTS])
def test_soap_pins_catch(what, old, new):
    failed = _caught(PINS_SOAP, "SO", _mutant(SOO, old, new))
    assert failed, "no pin notices: " + what


@pytest.mark.parametrize("what,old,new", SHAMPOO_COST_MUTANTS, ids=[m[0] for m in SHAMPOO_COST_MUTANTS])
def test_shampoo_cost_pins_catch(what, old, new):
    failed = _caught(PINS_SHAMPOO, "OP", _mutant(OP, old, new))
    assert failed, "no pin notices: " + what


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
    assert _caught(PINS_SHAMPOO, "SH", importlib.import_module("oracle.shampoo")) == []
    assert _caught(PINS_SOAP, "SO", importlib.import_module("oracle.soap")) == []
