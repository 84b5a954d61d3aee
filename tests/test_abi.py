"""The C-ABI library loads and exports every symbol include/canz.h declares; host-side
validation of canz_muon_step (everything that is rejected before any device work)."""
import ctypes
import os
import re

import pytest

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "canz.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(canz_[a-z_]+)\s*\(", text)))


def test_header_functions_are_exported(canz):
    names = _declared_functions()
    assert set(names) == set(canz.EXPORTS)
    lib = ctypes.CDLL(canz.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None
    assert canz.canz_version() == "0.4.0"


def test_struct_layouts_match_header(canz):
    # canz_group: 2 x int64, 4 x int32, 3 pointers; canz_muon_hparams: 12 four-byte fields
    assert ctypes.sizeof(canz._Group) == 16 + 16 + 24
    assert ctypes.sizeof(canz._Hparams) == 48


def test_workspace_bytes_formula(canz):
    hp = canz.Hparams()
    g = canz.Group(rows=256, cols=512, n_mats=8)
    # bf16: 3 X buffers of 8*256*512*2 B, A and B of 8*256*256*2 B, 8*(4*8) tile sums, two scale arrays
    # and 256 parked accumulator tiles of 256 KiB for the k-split of left-over tiles
    split = 256 * 256 * 256 * 4
    want = 3 * 8 * 256 * 512 * 2 + 2 * 8 * 256 * 256 * 2 + 8 * 32 * 4 + 256 + 256 + split
    assert canz.canz_muon_workspace_bytes([g], hp) == want
    # ragged shapes are padded to multiples of 256; fp32 mode doubles the element size
    g2 = canz.Group(rows=300, cols=77, n_mats=1)
    hp32 = canz.Hparams(precision=canz.PREC_F32)
    want2 = 3 * 256 * 512 * 4 + 2 * 256 * 256 * 4 + 256 + 256 + 256
    assert canz.canz_muon_workspace_bytes([g2], hp32) == want2
    # the maximum over runs.  A launch batch takes at most 128 matrices (the pointer-table size); batches
    # too small to fill the chip for long share a run (up to 4 of them), side by side in the workspace
    def batch_bytes(n):
        up = lambda x: (x + 255) // 256 * 256
        return 3 * n * 256 * 512 * 2 + 2 * n * 256 * 256 * 2 + up(n * 32 * 4) + 2 * up(n * 4)
    g3 = canz.Group(rows=256, cols=512, n_mats=150)
    assert canz.canz_muon_workspace_bytes([g, g3], hp) == batch_bytes(128) + batch_bytes(30) + split
    # ... at most 128 / tp with column fragments, and at most 2^30 padded elements
    g4 = canz.Group(rows=256, cols=512, n_mats=150, tp=4)
    assert canz.canz_muon_workspace_bytes([g4], hp) == 4 * batch_bytes(32) + split
    # the fp32 verification path keeps one batch per run
    assert canz.canz_muon_workspace_bytes([g4], hp32) == 2 * (batch_bytes(32) - 32 * 32 * 4 - 512) + 32 * 32 * 4 + 512
    g5 = canz.Group(rows=12288, cols=4096, n_mats=36)
    nb = (1 << 30) // (12288 * 4096)
    want5 = 3 * nb * 12288 * 4096 * 2 + 2 * nb * 4096 * 4096 * 2 + nb * (192 * 64) * 4 + 256 + 256 + split
    assert nb == 21 and canz.canz_muon_workspace_bytes([g5], hp) == want5
    assert canz.canz_muon_workspace_bytes([], hp) == 256


def test_step_argument_errors_without_device(canz):
    hp = canz.Hparams()
    ok = dict(rows=256, cols=512, grad=[4096], mom=[8192], out=[12288])

    def code(groups, hp_, ws=256 * 1024, ws_bytes=1 << 40):
        with pytest.raises(canz.CanzError) as e:
            canz.canz_muon_step(groups, hp_, ws, ws_bytes, 0)
        return e.value.code

    assert code([canz.Group(**{**ok, "grad": [4100]})], hp) == canz.EINVAL          # misaligned
    assert code([canz.Group(**{**ok, "mom": [0]})], hp) == canz.EINVAL              # null
    assert code([canz.Group(**{**ok, "tp": 9})], hp) == canz.EINVAL
    assert code([canz.Group(**{**ok, "tp": 3})], hp) == canz.ESHAPE                 # 512 % 3
    assert code([canz.Group(**{**ok, "cols": 36, "tp": 3, "grad": [4096] * 3})], hp) == canz.ESHAPE  # width 12
    assert code([canz.Group(**{**ok, "rows": 65535 * 64 + 1})], hp) == canz.ESHAPE  # above the documented limit
    assert code([canz.Group(**{**ok, "grad_dtype": 7})], hp) == canz.EUNSUPPORTED
    assert code([canz.Group(**ok)], canz.Hparams(ns_steps=-1)) == canz.EINVAL
    assert code([canz.Group(**ok)], canz.Hparams(scale_mode=9)) == canz.EUNSUPPORTED
    assert code([canz.Group(**ok)], canz.Hparams(precision=2)) == canz.EUNSUPPORTED
    assert code([canz.Group(**ok)], hp, ws=0) == canz.EWORKSPACE
    assert code([canz.Group(**ok)], hp, ws=4096 + 16) == canz.EWORKSPACE            # not 256-aligned
    assert code([canz.Group(**ok)], hp, ws_bytes=1024) == canz.EWORKSPACE
    assert "workspace too small" in canz.canz_last_error()
    # nothing to do: no device work, no workspace needed
    canz.canz_muon_step([], hp, 0, 0, 0)
    canz.canz_muon_step([canz.Group(rows=4, cols=4, n_mats=0)], hp, 0, 0, 0)


def test_shampoo_argument_errors_and_workspace_without_device(canz):
    hp = canz.ShampooHparams()
    ok = dict(rows=256, cols=512, grad=[4096], left=[8192], right=[12288], out=[16384])

    def code(groups, hp_, ws=256 * 1024, ws_bytes=1 << 40):
        with pytest.raises(canz.CanzError) as e:
            canz.canz_shampoo_step(groups, hp_, ws, ws_bytes, 0)
        return e.value.code

    G = canz.ShampooGroup
    assert code([G(**{**ok, "grad": [4100]})], hp) == canz.EINVAL
    assert code([G(**{**ok, "right": [0]})], hp) == canz.EINVAL
    assert code([G(**{**ok, "tp": 9})], hp) == canz.EINVAL
    assert code([G(**{**ok, "tp": 3})], hp) == canz.ESHAPE
    assert code([G(**{**ok, "rows": 32769})], hp) == canz.ESHAPE
    assert code([G(**{**ok, "out_dtype": 7})], hp) == canz.EUNSUPPORTED
    assert code([G(**ok)], canz.ShampooHparams(root_iters=0)) == canz.EINVAL
    assert code([G(**ok)], canz.ShampooHparams(eps=-1.0)) == canz.EINVAL
    assert code([G(**ok)], canz.ShampooHparams(out_mode=3)) == canz.EUNSUPPORTED
    assert code([G(**ok)], hp, ws=0) == canz.EWORKSPACE
    assert code([G(**ok)], hp, ws_bytes=1024) == canz.EWORKSPACE
    canz.canz_shampoo_step([], hp, 0, 0, 0)
    # workspace: fp32 working matrices padded to multiples of 128; rows 256, cols 512, one matrix:
    # G in two orientations and L^(-1/4) G (3 x 256 x 512), the two roots (256^2 + 512^2), eight
    # 512 x 512 matrices of the root iteration, twice 64 partial sums
    want = 4 * (3 * 256 * 512 + 256 * 256 + 512 * 512 + 8 * 512 * 512 + 128)
    assert canz.canz_shampoo_workspace_bytes([G(rows=256, cols=512, n_mats=1)], hp) == want
    assert canz.canz_shampoo_workspace_bytes([G(rows=200, cols=500, n_mats=1)], hp) == want
    assert ctypes.sizeof(canz._ShGroup) == 16 + 16 + 48 and ctypes.sizeof(canz._ShHparams) == 28
    assert code([G(**{**ok, "lroot": [20480]})], hp) == canz.EINVAL                              # one root table without the other
    assert code([G(**ok)], canz.ShampooHparams(keep_roots=True)) == canz.EINVAL                  # nothing to keep them in


def test_soap_argument_errors_and_workspace_without_device(canz):
    hp = canz.SoapHparams()
    ok = dict(rows=256, cols=512, grad=[4096], mom=[8192], var=[12288], left=[16384], right=[20480], qleft=[24576],
              qright=[28672], out=[32768])

    def code(groups, hp_, ws=256 * 1024, ws_bytes=1 << 40):
        with pytest.raises(canz.CanzError) as e:
            canz.canz_soap_step(groups, hp_, ws, ws_bytes, 0)
        return e.value.code

    G = canz.SoapGroup
    assert code([G(**{**ok, "grad": [4100]})], hp) == canz.EINVAL
    assert code([G(**{**ok, "var": [0]})], hp) == canz.EINVAL
    assert code([G(**{**ok, "qright": []})], hp) == canz.EINVAL                      # a side within the limit needs its tables
    assert code([G(**{**ok, "tp": 9})], hp) == canz.EINVAL
    assert code([G(**{**ok, "tp": 3})], hp) == canz.ESHAPE
    assert code([G(**{**ok, "rows": 32769})], hp) == canz.ESHAPE
    assert code([G(**{**ok, "out_dtype": 7})], hp) == canz.EUNSUPPORTED
    assert code([G(**ok)], canz.SoapHparams(beta1=1.0)) == canz.EINVAL
    assert code([G(**ok)], canz.SoapHparams(eps=-1.0)) == canz.EINVAL
    assert code([G(**ok)], canz.SoapHparams(step=0)) == canz.EINVAL
    assert code([G(**ok)], canz.SoapHparams(max_precond_dim=0)) == canz.EINVAL
    assert code([G(**ok)], canz.SoapHparams(out_mode=3)) == canz.EUNSUPPORTED
    assert code([G(**ok)], canz.SoapHparams(max_precond_dim=255)) == canz.EUNSUPPORTED     # neither side has a basis
    assert code([G(**{**ok, "rows": 12289})], canz.SoapHparams(max_precond_dim=20000)) == canz.ESHAPE   # too long for a basis
    assert canz.canz_soap_workspace_bytes([G(rows=12289, cols=512, n_mats=1)], hp) > 0                   # fine one-sided
    assert "max_precond_dim" in canz.canz_last_error()
    assert code([G(**ok)], hp, ws=0) == canz.EWORKSPACE
    assert code([G(**ok)], hp, ws_bytes=1024) == canz.EWORKSPACE
    canz.canz_soap_step([], hp, 0, 0, 0)
    # workspace in floats, rows 256, cols 512, one matrix, both sides: G and M in two orientations, the half-rotated
    # and the rotated pair (4 x 2 planes), N' and its half-rotated image (2 planes), the bases in two orientations,
    # one padded statistic of the larger side; a refresh step adds four square matrices of that side (working copy,
    # reflectors, the panels' Y2 = V T, Q^T), strips of 128 columns (one block's Y, W twice, U2^T of every block) and of 32
    # (T of every panel), 32 tau (one 256-byte unit) and three 128 x 128 matrices (C, C2, U^T of one block)
    plane, sq = 256 * 512, 512 * 512
    plain = 4 * (10 * plane + 2 * 256 * 256 + 2 * sq + sq)
    fresh = plain + 4 * (4 * sq + (128 + 2 * 128 + 32 + 128) * 512 + 64 + 3 * 128 * 128)
    one = [G(rows=256, cols=512, n_mats=1, grad_dtype=canz.DT_F32)]
    assert canz.canz_soap_workspace_bytes(one, hp) == plain
    assert canz.canz_soap_workspace_bytes([G(rows=200, cols=500, n_mats=1, grad_dtype=canz.DT_F32)], hp) == plain
    assert canz.canz_soap_workspace_bytes(one, canz.SoapHparams(refresh=True)) == fresh
    # one-sided: no half-rotated images, no basis of the long side, the statistic of the short side only
    one_sided = 4 * (7 * plane + 3 * 256 * 256)
    assert canz.canz_soap_workspace_bytes(one, canz.SoapHparams(max_precond_dim=256)) == one_sided
    # bf16 gradients: their bf16 image padded to 256, one orientation per side with a statistic
    one16 = [G(rows=256, cols=512, n_mats=1, grad_dtype=canz.DT_BF16)]
    assert canz.canz_soap_workspace_bytes(one16, hp) == plain + 2 * 2 * plane
    assert canz.canz_soap_workspace_bytes(one16, canz.SoapHparams(max_precond_dim=256)) == one_sided + 2 * plane
    # bf16 rotations add bf16 images padded to 256: sixteen planes (G, M, their half-rotated and rotated images, N', its
    # half-rotated image, each in two orientations) and the bases in two orientations
    want16 = plain + 2 * (16 * plane + 2 * 256 * 256 + 2 * sq)
    assert canz.canz_soap_workspace_bytes(one, canz.SoapHparams(bf16_rotations=True)) == want16
    assert canz.canz_soap_workspace_bytes(one16, canz.SoapHparams(bf16_rotations=True)) == want16
    assert ctypes.sizeof(canz._SoapGroup) == 16 + 16 + 72 and ctypes.sizeof(canz._SoapHparams) == 48
