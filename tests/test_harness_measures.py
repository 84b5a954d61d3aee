"""CPU checks of the measures the full-size GPU parity tests rely on."""
import numpy as np

from tests.gpu_harness import rel_fro, tile_errors

TILE_TOL_BF16, MAXABS_TOL_BF16 = 2e-2, 0.25     # the bounds tests/test_gpu_configs.py applies in bf16 mode


def test_tile_error_measure_sees_one_lost_tile():
    """The per-tile measure on a 25600 x 5120 sized problem in miniature: an error spread evenly
    at 1e-2 passes; the same with one 256 x 256 tile zeroed fails the tile bound while the
    matrix-level error stays under 3e-2 (which is why the tile bound exists)."""
    rng = np.random.default_rng(5)
    ref = rng.standard_normal((2560, 2560))
    got = ref + 1e-2 * rng.standard_normal(ref.shape)
    t, a = tile_errors(got - ref, ref)
    assert t <= TILE_TOL_BF16 and a <= MAXABS_TOL_BF16
    got[512:768, 1024:1280] = 0.0
    assert rel_fro(got, ref) <= 0.11          # sqrt(1/100): at full size 2.2e-2, under the matrix tolerance
    t, a = tile_errors(got - ref, ref)
    assert t > 0.9 and a > 1.0
