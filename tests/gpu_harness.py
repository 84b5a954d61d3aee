"""Helpers for the GPU parity tests: move seeded host inputs to the device bit for bit,
call canz_muon_step through the binding, bring results back as fp64, and run the
oracle on the very same input values.  torch is used for device memory only."""
from __future__ import annotations

import sys

import numpy as np

from oracle import muon as OM
from paper_2602_06079_amd import workloads as W


def log(msg: str):
    sys.stderr.write("[gpu-test] %s\n" % msg)
    sys.stderr.flush()


def oracle_hparams(hp) -> OM.Hparams:
    """The oracle takes the fp32 values the ABI carries, widened to Python floats."""
    f = lambda v: float(np.float32(v))
    return OM.Hparams(beta=f(hp.beta), lr=f(hp.lr), weight_decay=f(hp.weight_decay), eps=f(hp.eps),
                      nesterov=bool(hp.nesterov), ns_steps=int(hp.ns_steps), a=f(hp.a), b=f(hp.b), c=f(hp.c),
                      scale_mode=int(hp.scale_mode))


def widen(x: np.ndarray) -> np.ndarray:
    """Host array (float32, or uint16 bf16 bits) -> fp64, exactly."""
    return OM.bf16_bits_to_f64(x) if x.dtype == np.uint16 else x.astype(np.float64)


def to_device(x: np.ndarray):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x))
    if x.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def to_host64(t) -> np.ndarray:
    import torch
    if t.dtype == torch.bfloat16:
        return OM.bf16_bits_to_f64(t.view(torch.uint16).cpu().numpy())
    return t.cpu().numpy().astype(np.float64)


def dtype_code(x: np.ndarray) -> int:
    return W.DT_BF16 if x.dtype == np.uint16 else W.DT_F32


class DeviceGroup:
    """One micro-group on the device.

    grads  per matrix: a host array, or a list of tp column fragments
    moms   per matrix: float32 host array (rows x cols)
    outs   per matrix: the parameter array (in-place mode), or None for delta mode, in
           which case zero-filled fragment buffers of out_np_dtype are created
    """

    def __init__(self, canz, rows, cols, grads, moms, outs=None, tp=1, out_np_dtype=np.float32):
        import torch
        self.canz, self.rows, self.cols, self.tp = canz, rows, cols, tp
        self.n = len(moms)
        self.grad_t, self.out_t = [], []
        first = grads[0][0] if isinstance(grads[0], (list, tuple)) else grads[0]
        self.grad_dtype = dtype_code(first)
        for g in grads:
            frags = g if isinstance(g, (list, tuple)) else [g]
            assert len(frags) == tp
            self.grad_t += [to_device(f) for f in frags]
        self.mom_t = [to_device(m) for m in moms]
        self.delta = outs is None
        if self.delta:
            w = cols // tp
            proto = np.zeros((rows, w), dtype=out_np_dtype)
            self.out_dtype = dtype_code(proto)
            self.out_t = [to_device(proto) for _ in range(self.n * tp)]
        else:
            self.out_dtype = dtype_code(outs[0])
            self.out_t = [to_device(p) for p in outs]
        torch.cuda.synchronize()

    def group(self):
        return self.canz.Group(rows=self.rows, cols=self.cols, grad=self.grad_t, mom=self.mom_t, out=self.out_t,
                               tp=self.tp, grad_dtype=self.grad_dtype, out_dtype=self.out_dtype)

    def set_grads(self, grads):
        for i, g in enumerate(grads):
            frags = g if isinstance(g, (list, tuple)) else [g]
            for f, frag in enumerate(frags):
                self.grad_t[i * self.tp + f].copy_(to_device(frag))

    def mom_host(self, i):
        return to_host64(self.mom_t[i])

    def out_host(self, i):
        """Parameter (in-place mode) or the whole Delta W reassembled from its fragments."""
        if not self.delta:
            return to_host64(self.out_t[i])
        return np.concatenate([to_host64(self.out_t[i * self.tp + f]) for f in range(self.tp)], axis=1)


def run_step(canz, dgroups, hp, workspace=None):
    """One canz_muon_step over the given DeviceGroups on torch's current stream."""
    import torch
    groups = [d.group() for d in dgroups]
    nbytes = canz.canz_muon_workspace_bytes(groups, hp)
    if workspace is None or workspace.numel() < nbytes:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    canz.canz_muon_step(groups, hp, workspace, workspace.numel(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return workspace


def rel_fro(got: np.ndarray, want: np.ndarray) -> float:
    den = float(np.linalg.norm(want))
    return float(np.linalg.norm(got - want)) / den if den > 0 else float(np.linalg.norm(got))


TILE = 256


def tile_errors(diff, ref):
    """(largest per-tile relative Frobenius error, largest |diff| / rms(ref)) over the grid of
    256 x 256 tiles; edge tiles are smaller.  A tile whose reference is all zero counts by its
    absolute error against the matrix rms."""
    rows, cols = ref.shape
    rms = float(np.sqrt(np.mean(ref * ref)))
    pr, pc = -rows % TILE, -cols % TILE
    d2 = np.pad(diff * diff, ((0, pr), (0, pc)))
    r2 = np.pad(ref * ref, ((0, pr), (0, pc)))
    shape = (d2.shape[0] // TILE, TILE, d2.shape[1] // TILE, TILE)
    dt = d2.reshape(shape).sum(axis=(1, 3))
    rt = r2.reshape(shape).sum(axis=(1, 3))
    floor = (rms * 1e-3) ** 2
    worst_tile = float(np.sqrt(np.max(dt / np.maximum(rt, floor))))
    return worst_tile, float(np.max(np.abs(diff))) / rms if rms > 0 else float(np.max(np.abs(diff)))
