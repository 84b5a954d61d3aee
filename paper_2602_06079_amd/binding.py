"""ctypes binding of libcanz.so: argument marshalling only.

The functions carry the names of the C ABI (include/canz.h).  Device buffers are
passed as integer addresses (``tensor.data_ptr()``) or as objects that have a
``data_ptr()`` method; the stream as an integer (``torch.cuda.current_stream().cuda_stream``).
If the library has not been built the import of this module fails loudly - there is
no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcanz.so")

OK, EINVAL, ESHAPE, EWORKSPACE, EHIP, EUNSUPPORTED = 0, -1, -2, -3, -4, -5
COST_NUMEL, COST_NS_FLOPS, COST_SHAMPOO_FLOPS, COST_SOAP_FLOPS = 0, 1, 2, 3
DT_F32, DT_BF16 = 0, 1
SCALE_NONE, SCALE_ASPECT, SCALE_RMS = 0, 1, 2
PREC_BF16, PREC_F32 = 0, 1
OUT_PARAM, OUT_DELTA = 0, 1

EXPORTS = ("canz_last_error", "canz_version", "canz_partition_alpha", "canz_partition_naive", "canz_microgroup_plan", "canz_tp_schedule",
           "canz_muon_workspace_bytes", "canz_muon_step", "canz_muon_step_static",
           "canz_shampoo_workspace_bytes", "canz_shampoo_step", "canz_soap_workspace_bytes", "canz_soap_step",
           "canz_profile_enable", "canz_profile_collect", "canz_profile_disable")
KERNEL_KINDS = ("momentum", "norm", "gram", "poly", "update", "final", "apply",
                "sh_load", "sh_stat", "sh_init", "sh_root", "sh_apply",
                "soap_load", "soap_rotate", "soap_adam", "soap_stat", "soap_qr", "soap_panel")


class CanzError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("canz error %d: %s" % (code, message))
        self.code = code


class _Group(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("n_mats", C.c_int32), ("tp", C.c_int32),
                ("grad_dtype", C.c_int32), ("out_dtype", C.c_int32),
                ("grad", C.POINTER(C.c_void_p)), ("mom", C.POINTER(C.c_void_p)), ("out", C.POINTER(C.c_void_p))]


class _Hparams(C.Structure):
    _fields_ = [("beta", C.c_float), ("lr", C.c_float), ("weight_decay", C.c_float), ("eps", C.c_float),
                ("nesterov", C.c_int32), ("ns_steps", C.c_int32),
                ("a", C.c_float), ("b", C.c_float), ("c", C.c_float),
                ("scale_mode", C.c_int32), ("precision", C.c_int32), ("out_mode", C.c_int32)]


class _ShGroup(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("n_mats", C.c_int32), ("tp", C.c_int32),
                ("grad_dtype", C.c_int32), ("out_dtype", C.c_int32),
                ("grad", C.POINTER(C.c_void_p)), ("left", C.POINTER(C.c_void_p)), ("right", C.POINTER(C.c_void_p)),
                ("out", C.POINTER(C.c_void_p)), ("lroot", C.POINTER(C.c_void_p)), ("rroot", C.POINTER(C.c_void_p))]


class _ShHparams(C.Structure):
    _fields_ = [("beta", C.c_float), ("lr", C.c_float), ("weight_decay", C.c_float), ("eps", C.c_float),
                ("root_iters", C.c_int32), ("out_mode", C.c_int32), ("keep_roots", C.c_int32)]


class _SoapGroup(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("n_mats", C.c_int32), ("tp", C.c_int32),
                ("grad_dtype", C.c_int32), ("out_dtype", C.c_int32),
                ("grad", C.POINTER(C.c_void_p)), ("mom", C.POINTER(C.c_void_p)), ("var", C.POINTER(C.c_void_p)),
                ("left", C.POINTER(C.c_void_p)), ("right", C.POINTER(C.c_void_p)),
                ("qleft", C.POINTER(C.c_void_p)), ("qright", C.POINTER(C.c_void_p)), ("out", C.POINTER(C.c_void_p)),
                ("mom_rot", C.POINTER(C.c_void_p))]


class _SoapHparams(C.Structure):
    _fields_ = [("beta1", C.c_float), ("beta2", C.c_float), ("lr", C.c_float), ("weight_decay", C.c_float),
                ("eps", C.c_float), ("step", C.c_int32), ("bias_correction", C.c_int32), ("refresh", C.c_int32),
                ("max_precond_dim", C.c_int32), ("out_mode", C.c_int32), ("mom_rot_valid", C.c_int32),
                ("bf16_rotations", C.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libcanz.so is missing at %s - build it with "
                           "`python -m paper_2602_06079_amd.build` (there is no fallback)" % LIB_PATH)
    # One process must use one HIP runtime.  PyTorch ships its own copy and supplies the
    # device memory and streams here, so it is loaded first; libcanz.so then binds to the
    # runtime that is already in the process (same soname) instead of a second one.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    lib.canz_last_error.restype = C.c_char_p
    lib.canz_version.restype = C.c_char_p
    i64p, i32p = C.POINTER(C.c_int64), C.POINTER(C.c_int32)
    lib.canz_partition_alpha.argtypes = [C.c_int64, i64p, i64p, i64p, C.c_int32, C.c_int64, i64p, C.c_int32,
                                         C.c_double, i64p, i32p, i64p]
    lib.canz_partition_alpha.restype = C.c_int
    lib.canz_microgroup_plan.argtypes = [C.c_int64, i64p, i64p, i32p, i32p, C.c_int32, C.c_int32, C.c_int64,
                                         i64p, i64p, i64p]
    lib.canz_microgroup_plan.restype = C.c_int
    lib.canz_partition_naive.argtypes = [C.c_int64, i64p, C.c_int64, i64p, C.c_int32, i32p, i64p]
    lib.canz_partition_naive.restype = C.c_int
    lib.canz_tp_schedule.argtypes = [C.c_int64, i64p, C.c_int32, C.c_int64, i64p, i64p, i64p, i32p, i64p]
    lib.canz_tp_schedule.restype = C.c_int
    lib.canz_muon_workspace_bytes.argtypes = [C.POINTER(_Group), C.c_int32, C.POINTER(_Hparams),
                                              C.POINTER(C.c_size_t)]
    lib.canz_muon_workspace_bytes.restype = C.c_int
    lib.canz_muon_step.argtypes = [C.POINTER(_Group), C.c_int32, C.POINTER(_Hparams), C.c_void_p, C.c_size_t,
                                   C.c_void_p]
    lib.canz_muon_step.restype = C.c_int
    lib.canz_muon_step_static.argtypes = [C.POINTER(_Group), C.c_int32, C.POINTER(_Hparams), C.c_void_p]
    lib.canz_muon_step_static.restype = C.c_int
    lib.canz_shampoo_workspace_bytes.argtypes = [C.POINTER(_ShGroup), C.c_int32, C.POINTER(_ShHparams),
                                                 C.POINTER(C.c_size_t)]
    lib.canz_shampoo_workspace_bytes.restype = C.c_int
    lib.canz_shampoo_step.argtypes = [C.POINTER(_ShGroup), C.c_int32, C.POINTER(_ShHparams), C.c_void_p, C.c_size_t,
                                      C.c_void_p]
    lib.canz_shampoo_step.restype = C.c_int
    lib.canz_soap_workspace_bytes.argtypes = [C.POINTER(_SoapGroup), C.c_int32, C.POINTER(_SoapHparams),
                                              C.POINTER(C.c_size_t)]
    lib.canz_soap_workspace_bytes.restype = C.c_int
    lib.canz_soap_step.argtypes = [C.POINTER(_SoapGroup), C.c_int32, C.POINTER(_SoapHparams), C.c_void_p, C.c_size_t,
                                   C.c_void_p]
    lib.canz_soap_step.restype = C.c_int
    lib.canz_profile_enable.argtypes = [C.c_int32]
    lib.canz_profile_enable.restype = C.c_int
    lib.canz_profile_collect.argtypes = [C.POINTER(C.c_double), i64p]
    lib.canz_profile_collect.restype = C.c_int
    lib.canz_profile_disable.argtypes = []
    lib.canz_profile_disable.restype = C.c_int
    return lib


_lib = _load()


def _check(rc: int):
    if rc != OK:
        raise CanzError(rc, _lib.canz_last_error().decode())


def canz_version() -> str:
    return _lib.canz_version().decode()


def canz_last_error() -> str:
    return _lib.canz_last_error().decode()


def _i64(x):
    return np.ascontiguousarray(x, dtype=np.int64)


def _i32(x):
    return np.ascontiguousarray(x, dtype=np.int32)


def _p64(a):
    return a.ctypes.data_as(C.POINTER(C.c_int64))


def _p32(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def canz_partition_alpha(rows, cols, bucket_off, n_ranks, alpha, cost=None, cost_kind=COST_NUMEL):
    """Algorithm 1.  Returns (cuts [n_buckets][n_ranks+1], owner [n_mats], load [n_ranks]) as numpy arrays."""
    rows, cols, bucket_off = _i64(rows), _i64(cols), _i64(bucket_off)
    n_mats, n_buckets = rows.shape[0], bucket_off.shape[0] - 1
    cost_a = None if cost is None else _i64(cost)
    cuts = np.zeros((max(n_buckets, 0), max(int(n_ranks), 0) + 1), dtype=np.int64)
    owner = np.full(n_mats, -1, dtype=np.int32)
    load = np.zeros(max(int(n_ranks), 0), dtype=np.int64)
    _check(_lib.canz_partition_alpha(n_mats, _p64(rows), _p64(cols), None if cost_a is None else _p64(cost_a),
                                     int(cost_kind), n_buckets, _p64(bucket_off), int(n_ranks), float(alpha),
                                     _p64(cuts), _p32(owner), _p64(load)))
    return cuts, owner, load


def canz_partition_naive(numel, n_ranks, bucket_off=None):
    """Eq. 1 per bucket (atomic ownership without balancing).  Returns (owner, load)."""
    numel = _i64(numel)
    bucket_off = _i64([0, numel.shape[0]] if bucket_off is None else bucket_off)
    owner = np.full(numel.shape[0], -1, dtype=np.int32)
    load = np.zeros(max(int(n_ranks), 0), dtype=np.int64)
    _check(_lib.canz_partition_naive(numel.shape[0], _p64(numel), bucket_off.shape[0] - 1, _p64(bucket_off),
                                     int(n_ranks), _p32(owner), _p64(load)))
    return owner, load


def canz_microgroup_plan(rows, cols, dtype, owner, rank, max_mats=8, cmax_bytes=0) -> List[List[int]]:
    """Same-shape batches of the matrices ``rank`` owns; a list of id lists."""
    rows, cols, dtype, owner = _i64(rows), _i64(cols), _i32(dtype), _i32(owner)
    n = rows.shape[0]
    n_groups = C.c_int64(0)
    off = np.zeros(n + 1, dtype=np.int64)
    member = np.zeros(max(n, 1), dtype=np.int64)
    _check(_lib.canz_microgroup_plan(n, _p64(rows), _p64(cols), _p32(dtype), _p32(owner), int(rank), int(max_mats),
                                     int(cmax_bytes), C.byref(n_groups), _p64(off), _p64(member)))
    return [[int(x) for x in member[off[i]:off[i + 1]]] for i in range(n_groups.value)]


def canz_tp_schedule(cost, n_ranks, cmax):
    """Algorithm 2/3/4.  Returns (groups, loads): groups is a list of lists of
    (tensor id, host rank) in assignment order, loads the largest rank load of each group."""
    cost = _i64(cost)
    n = cost.shape[0]
    n_groups = C.c_int64(0)
    off = np.zeros(n + 1, dtype=np.int64)
    member = np.zeros(max(n, 1), dtype=np.int64)
    host = np.zeros(max(n, 1), dtype=np.int32)
    load = np.zeros(max(n, 1), dtype=np.int64)
    _check(_lib.canz_tp_schedule(n, _p64(cost), int(n_ranks), int(cmax), C.byref(n_groups), _p64(off), _p64(member),
                                 _p32(host), _p64(load)))
    groups = [[(int(member[i]), int(host[i])) for i in range(off[k], off[k + 1])] for k in range(n_groups.value)]
    return groups, [int(x) for x in load[:n_groups.value]]


@dataclass
class Hparams:
    beta: float = 0.95
    lr: float = 0.02
    weight_decay: float = 0.0
    eps: float = 1e-7
    nesterov: bool = False
    ns_steps: int = 5
    a: float = 3.4445
    b: float = -4.7750
    c: float = 2.0315
    scale_mode: int = SCALE_RMS
    precision: int = PREC_BF16
    out_mode: int = OUT_PARAM

    def _c(self) -> _Hparams:
        return _Hparams(self.beta, self.lr, self.weight_decay, self.eps, int(bool(self.nesterov)), int(self.ns_steps),
                        self.a, self.b, self.c, int(self.scale_mode), int(self.precision), int(self.out_mode))


@dataclass
class Group:
    """One micro-group: device buffers given as addresses or objects with data_ptr()."""
    rows: int
    cols: int
    grad: Sequence = field(default_factory=list)   # n_mats * tp
    mom: Sequence = field(default_factory=list)    # n_mats
    out: Sequence = field(default_factory=list)    # n_mats (params) or n_mats * tp (delta fragments)
    tp: int = 1
    grad_dtype: int = DT_BF16
    out_dtype: int = DT_F32
    n_mats: int = -1                               # -1: len(mom)


def _addr(x) -> int:
    if x is None:
        return 0
    return int(x.data_ptr()) if hasattr(x, "data_ptr") else int(x)


def _marshal(groups: Sequence[Group]):
    arr = (_Group * max(len(groups), 1))()
    keep = []
    for i, g in enumerate(groups):
        n_mats = len(g.mom) if g.n_mats < 0 else g.n_mats
        tabs = []
        for seq in (g.grad, g.mom, g.out):
            t = (C.c_void_p * max(len(seq), 1))(*[_addr(x) for x in seq])
            keep.append(t)
            tabs.append(C.cast(t, C.POINTER(C.c_void_p)) if len(seq) else None)
        arr[i] = _Group(int(g.rows), int(g.cols), int(n_mats), int(g.tp), int(g.grad_dtype), int(g.out_dtype),
                        tabs[0], tabs[1], tabs[2])
    return arr, keep


def canz_muon_workspace_bytes(groups: Sequence[Group], hp: Hparams) -> int:
    arr, _keep = _marshal(groups)
    out = C.c_size_t(0)
    h = hp._c()
    _check(_lib.canz_muon_workspace_bytes(arr, len(groups), C.byref(h), C.byref(out)))
    return int(out.value)


def canz_muon_step(groups: Sequence[Group], hp: Hparams, workspace, workspace_bytes: int, stream=0) -> None:
    """Enqueue one optimizer step on ``stream`` (an integer hipStream_t)."""
    arr, _keep = _marshal(groups)
    h = hp._c()
    _check(_lib.canz_muon_step(arr, len(groups), C.byref(h), C.c_void_p(_addr(workspace)), int(workspace_bytes),
                               C.c_void_p(int(stream))))


@dataclass
class ShampooHparams:
    beta: float = 1.0
    lr: float = 0.02
    weight_decay: float = 0.0
    eps: float = 1e-6
    root_iters: int = 25
    out_mode: int = OUT_PARAM
    keep_roots: bool = False

    def _c(self) -> _ShHparams:
        return _ShHparams(self.beta, self.lr, self.weight_decay, self.eps, int(self.root_iters), int(self.out_mode),
                          int(bool(self.keep_roots)))


@dataclass
class ShampooGroup:
    """One micro-group of canz_shampoo_step: device buffers given as addresses or objects with data_ptr()."""
    rows: int
    cols: int
    grad: Sequence = field(default_factory=list)    # n_mats * tp
    left: Sequence = field(default_factory=list)    # n_mats, fp32 rows x rows
    right: Sequence = field(default_factory=list)   # n_mats, fp32 cols x cols
    out: Sequence = field(default_factory=list)     # n_mats (params) or n_mats * tp (delta fragments)
    lroot: Sequence = field(default_factory=list)   # n_mats, fp32 rows x rows: the kept inverse fourth roots, or empty
    rroot: Sequence = field(default_factory=list)   # n_mats, fp32 cols x cols
    tp: int = 1
    grad_dtype: int = DT_BF16
    out_dtype: int = DT_F32
    n_mats: int = -1                                # -1: len(left)


def _marshal_shampoo(groups: Sequence[ShampooGroup]):
    arr = (_ShGroup * max(len(groups), 1))()
    keep = []
    for i, g in enumerate(groups):
        n_mats = len(g.left) if g.n_mats < 0 else g.n_mats
        tabs = []
        for seq in (g.grad, g.left, g.right, g.out, g.lroot, g.rroot):
            t = (C.c_void_p * max(len(seq), 1))(*[_addr(x) for x in seq])
            keep.append(t)
            tabs.append(C.cast(t, C.POINTER(C.c_void_p)) if len(seq) else None)
        arr[i] = _ShGroup(int(g.rows), int(g.cols), int(n_mats), int(g.tp), int(g.grad_dtype), int(g.out_dtype), *tabs)
    return arr, keep


def canz_shampoo_workspace_bytes(groups: Sequence[ShampooGroup], hp: ShampooHparams) -> int:
    arr, _keep = _marshal_shampoo(groups)
    out = C.c_size_t(0)
    h = hp._c()
    _check(_lib.canz_shampoo_workspace_bytes(arr, len(groups), C.byref(h), C.byref(out)))
    return int(out.value)


def canz_shampoo_step(groups: Sequence[ShampooGroup], hp: ShampooHparams, workspace, workspace_bytes: int, stream=0) -> None:
    """Enqueue one Shampoo step on ``stream`` (an integer hipStream_t)."""
    arr, _keep = _marshal_shampoo(groups)
    h = hp._c()
    _check(_lib.canz_shampoo_step(arr, len(groups), C.byref(h), C.c_void_p(_addr(workspace)), int(workspace_bytes),
                                  C.c_void_p(int(stream))))


@dataclass
class SoapHparams:
    beta1: float = 0.95
    beta2: float = 0.95
    lr: float = 3e-3
    weight_decay: float = 0.0
    eps: float = 1e-8
    step: int = 1
    bias_correction: bool = True
    refresh: bool = False
    max_precond_dim: int = 10000
    out_mode: int = OUT_PARAM
    mom_rot_valid: bool = False
    bf16_rotations: bool = False

    def _c(self) -> _SoapHparams:
        return _SoapHparams(self.beta1, self.beta2, self.lr, self.weight_decay, self.eps, int(self.step),
                            int(bool(self.bias_correction)), int(bool(self.refresh)), int(self.max_precond_dim),
                            int(self.out_mode), int(bool(self.mom_rot_valid)), int(bool(self.bf16_rotations)))


@dataclass
class SoapGroup:
    """One micro-group of canz_soap_step: device buffers given as addresses or objects with data_ptr()."""
    rows: int
    cols: int
    grad: Sequence = field(default_factory=list)    # n_mats * tp
    mom: Sequence = field(default_factory=list)     # n_mats, fp32 rows x cols
    var: Sequence = field(default_factory=list)     # n_mats, fp32 rows x cols (rotated space)
    left: Sequence = field(default_factory=list)    # n_mats, fp32 rows x rows (empty if rows > max_precond_dim)
    right: Sequence = field(default_factory=list)   # n_mats, fp32 cols x cols
    qleft: Sequence = field(default_factory=list)   # n_mats, fp32 rows x rows, columns are the basis vectors
    qright: Sequence = field(default_factory=list)  # n_mats, fp32 cols x cols
    out: Sequence = field(default_factory=list)     # n_mats (params) or n_mats * tp (delta fragments)
    mom_rot: Sequence = field(default_factory=list) # n_mats, fp32 rows x cols: the rotated momentum, or empty
    tp: int = 1
    grad_dtype: int = DT_BF16
    out_dtype: int = DT_F32
    n_mats: int = -1                                # -1: len(mom)


def _marshal_soap(groups: Sequence[SoapGroup]):
    arr = (_SoapGroup * max(len(groups), 1))()
    keep = []
    for i, g in enumerate(groups):
        n_mats = len(g.mom) if g.n_mats < 0 else g.n_mats
        tabs = []
        for seq in (g.grad, g.mom, g.var, g.left, g.right, g.qleft, g.qright, g.out, g.mom_rot):
            t = (C.c_void_p * max(len(seq), 1))(*[_addr(x) for x in seq])
            keep.append(t)
            tabs.append(C.cast(t, C.POINTER(C.c_void_p)) if len(seq) else None)
        arr[i] = _SoapGroup(int(g.rows), int(g.cols), int(n_mats), int(g.tp), int(g.grad_dtype), int(g.out_dtype), *tabs)
    return arr, keep


def canz_soap_workspace_bytes(groups: Sequence[SoapGroup], hp: SoapHparams) -> int:
    arr, _keep = _marshal_soap(groups)
    out = C.c_size_t(0)
    h = hp._c()
    _check(_lib.canz_soap_workspace_bytes(arr, len(groups), C.byref(h), C.byref(out)))
    return int(out.value)


def canz_soap_step(groups: Sequence[SoapGroup], hp: SoapHparams, workspace, workspace_bytes: int, stream=0) -> None:
    """Enqueue one SOAP step on ``stream`` (an integer hipStream_t)."""
    arr, _keep = _marshal_soap(groups)
    h = hp._c()
    _check(_lib.canz_soap_step(arr, len(groups), C.byref(h), C.c_void_p(_addr(workspace)), int(workspace_bytes),
                               C.c_void_p(int(stream))))


STATIC_WORKSPACE_BYTES = 128 << 20


def canz_muon_step_static(groups: Sequence[Group], hp: Hparams, stream=0) -> None:
    """canz_muon_step on the workspace built into the library (no device allocation)."""
    arr, _keep = _marshal(groups)
    h = hp._c()
    _check(_lib.canz_muon_step_static(arr, len(groups), C.byref(h), C.c_void_p(int(stream))))


def canz_profile_enable(max_launches: int) -> None:
    _check(_lib.canz_profile_enable(int(max_launches)))


def canz_profile_collect():
    """Returns {kind: (milliseconds, launches)} for the period since the last collection."""
    ms = (C.c_double * len(KERNEL_KINDS))()
    n = (C.c_int64 * len(KERNEL_KINDS))()
    _check(_lib.canz_profile_collect(ms, n))
    return {k: (float(ms[i]), int(n[i])) for i, k in enumerate(KERNEL_KINDS)}


def canz_profile_disable() -> None:
    _check(_lib.canz_profile_disable())
