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


def test_products_of_bf16_values_are_exact_in_fp32():
    """What lets the SOAP statistics of bf16 gradients run on the bf16 matrix cores at no loss: a bf16 number has 8
    significant bits, so the product of two has at most 16 and is an fp32 number exactly (exponent range permitting);
    only the sums round, as in the fp32 kernel.  Checked on 2^20 random pairs over the gradient's range, and on the
    widening itself (bf16 -> fp32 -> bf16 is the identity)."""
    from paper_2602_06079_amd import workloads as W
    rng = np.random.default_rng(11)
    a = W.bf16_bits_to_f32(W.f32_to_bf16_bits((0.02 * rng.standard_normal(1 << 20)).astype(np.float32)))
    b = W.bf16_bits_to_f32(W.f32_to_bf16_bits((0.02 * rng.standard_normal(1 << 20) * 10.0 ** rng.integers(-3, 4, 1 << 20)).astype(np.float32)))
    assert np.array_equal(W.bf16_bits_to_f32(W.f32_to_bf16_bits(a)), a)
    exact = a.astype(np.float64) * b.astype(np.float64)
    assert np.array_equal((a * b).astype(np.float64), exact)                 # the fp32 product did not round
    assert np.array_equal(exact.astype(np.float32).astype(np.float64), exact)
