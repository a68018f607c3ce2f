"""Pins of the oracle's product with the stored (packed, mixed-precision) weights, paper Sec. 5.3."""
import numpy as np
import pytest

from test_oracle_pack import unpack_block


def _pack(orc, Wb, m, n, bits, level, base=0):
    off = orc.offsets(level, m, n, bits)
    codes = np.zeros(off[-1], np.uint8)
    scale = np.zeros(level.size * m, np.float32)
    zero = np.zeros(level.size * m, np.float32)
    orc.pack(Wb, m, n, bits, level, off, base, codes, scale, zero)
    return off, codes, scale, zero


def test_hand_example_on_the_grid(orc):
    """One 8 x 8 block whose rows are the ramp 0..7 at 3 bits (scale 1, zero 0: stored exactly);
    x = e_2 + 2 e_5 gives y_i = 2 + 2 * 5 = 12 for every row; a second batch row of ones gives 28."""
    W = orc.f32_to_bf16(np.tile(np.arange(8, dtype=np.float32), (8, 1)))
    level = np.array([0], np.uint8)
    off, codes, scale, zero = _pack(orc, W, 8, 8, [3], level)
    x = np.zeros((2, 8), np.float32); x[0, 2] = 1; x[0, 5] = 2; x[1] = 1
    y = orc.mp_gemm(codes, scale, zero, level, off, 0, 8, 8, 8, 8, [3], orc.f32_to_bf16(x))
    np.testing.assert_array_equal(y, np.array([[12.0] * 8, [28.0] * 8]))


@pytest.mark.parametrize("m,n,bits", [(8, 8, [1, 2, 3, 4, 8]), (16, 64, [2, 4, 8]), (64, 128, [1, 2, 3, 4, 5, 6, 7, 8])])
def test_dequant_against_numpy_unpacking_and_product_against_matmul(orc, m, n, bits):
    rng = np.random.default_rng(m + n)
    R, C, base = 2 * m, 3 * n, 4
    Wb = orc.f32_to_bf16(0.02 * rng.standard_t(4, size=(R, C)))
    N = base + 6 + 1
    level = rng.integers(0, len(bits), size=N).astype(np.uint8)
    off, codes, scale, zero = _pack(orc, Wb, m, n, bits, level, base)
    What = orc.dequant(codes, scale, zero, level, off, base, R, C, m, n, bits)
    for I in range(2):
        for J in range(3):
            b = base + I * 3 + J
            q = unpack_block(codes[off[b]:off[b + 1]], bits[level[b]], m, n)        # numpy's bit unpacking
            want = (q.astype(np.float64) * scale[b * m:(b + 1) * m, None] + zero[b * m:(b + 1) * m, None])
            got = What[I * m:(I + 1) * m, J * n:(J + 1) * n]
            assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -23 + 1e-45)  # one fp32 rounding of q*s+z
            W = orc.bf16_to_f32(Wb)[I * m:(I + 1) * m, J * n:(J + 1) * n]
            assert np.all(np.abs(got - W) <= 0.5 * scale[b * m:(b + 1) * m, None] * (1 + 1e-5) + np.abs(W) * 2.0 ** -22)
    xb = orc.f32_to_bf16(rng.standard_normal((5, C)))
    y = orc.mp_gemm(codes, scale, zero, level, off, base, R, C, m, n, bits, xb)
    ref = orc.bf16_to_f32(xb).astype(np.float64) @ What.astype(np.float64).T
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12 * np.abs(ref).max())
    assert y.shape == (5, R)


def test_integer_weights_at_eight_bits_give_the_exact_product(orc):
    """Integer weights 0..255 with both extremes in every row group are stored exactly at 8 bits
    (scale 1, zero 0): the product is the integer matrix product."""
    rng = np.random.default_rng(9)
    m, n, R, C = 8, 16, 16, 32
    Wi = rng.integers(0, 256, (R, C))
    Wi[:, 0::n] = 0; Wi[:, 1::n] = 255
    level = np.zeros(4, np.uint8)
    off, codes, scale, zero = _pack(orc, orc.f32_to_bf16(Wi.astype(np.float32)), m, n, [8], level)
    assert np.all(scale == 1) and np.all(zero == 0)
    xi = rng.integers(-8, 9, (3, C))
    y = orc.mp_gemm(codes, scale, zero, level, off, 0, R, C, m, n, [8], orc.f32_to_bf16(xi.astype(np.float32)))
    np.testing.assert_array_equal(y, (xi @ Wi.T).astype(np.float64))


def test_a_transposed_or_mislabelled_block_would_show(orc):
    """Blocks with distinct constant rows: y picks out row sums per output channel, per block column."""
    m = n = 8
    R, C = 16, 16
    W = np.zeros((R, C), np.float32)
    for i in range(R):
        W[i, :8] = i + 1                                   # block column 0: value = row + 1
        W[i, 8:] = 100 + i                                 # block column 1
    W[:, 0] = 0; W[:, 8] = 0                               # a second grid point per group (range > 0)
    level = np.array([4, 4, 4, 4], np.uint8)
    bits = [1, 2, 3, 4, 8]
    off, codes, scale, zero = _pack(orc, orc.f32_to_bf16(W), m, n, bits, level)
    What = orc.dequant(codes, scale, zero, level, off, 0, R, C, m, n, bits)
    np.testing.assert_allclose(What, W, rtol=2.0 ** -8)
    x = np.zeros((1, C), np.float32); x[0, 3] = 1          # picks column 3 (block column 0)
    y = orc.mp_gemm(codes, scale, zero, level, off, 0, R, C, m, n, bits, orc.f32_to_bf16(x))
    np.testing.assert_allclose(y[0], np.arange(1, 17), rtol=2.0 ** -8)
    x[:] = 0; x[0, 12] = 1                                 # block column 1
    y = orc.mp_gemm(codes, scale, zero, level, off, 0, R, C, m, n, bits, orc.f32_to_bf16(x))
    np.testing.assert_allclose(y[0], 100 + np.arange(16), rtol=2.0 ** -8)
