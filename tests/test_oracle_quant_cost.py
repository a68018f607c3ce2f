"""Pins for the oracle's round-to-nearest quantizer and the block x bitwidth cost table.

The expected values are closed forms and hand-worked cases of the definition
(paper Sec. 5 "Implementation": round-to-nearest uniform scalar quantizer, group
size = block width; cost = sensitivity-weighted squared error summed per block),
plus an independent float64 evaluation for the 1e-5 relative bound.
"""
import numpy as np
import pytest


# ------------------------------------------------------------------ quantizer

@pytest.mark.parametrize("bits", [1, 2, 3, 4, 8])
def test_group_on_the_grid_has_zero_error_and_recovers_indices(orc, bits):
    # values mn + q*step with step a power of two: every operation is exact
    qmax = 2 ** bits - 1
    rng = np.random.default_rng(bits)
    q_true = rng.integers(0, qmax + 1, size=128)
    q_true[0], q_true[1] = 0, qmax                  # both extremes present
    step, mn = 0.25, -3.0
    w = (mn + step * q_true).astype(np.float32)
    q, scale, zero = orc.quant_group(w, bits)
    np.testing.assert_array_equal(q, q_true)
    assert zero == np.float32(mn)
    what = q.astype(np.float32) * scale + zero
    if qmax & (qmax + 1) == 0 and bits in (1,):       # qmax = 1: scale exactly the range
        assert scale == np.float32(step * qmax)
    np.testing.assert_allclose(what, w, rtol=0, atol=float(scale) * 2.0 ** -22)


def test_constant_group(orc):
    w = np.full(64, 0.37, np.float32)
    for bits in (1, 2, 3, 4, 8):
        q, scale, zero = orc.quant_group(w, bits)
        assert not q.any() and scale == 0.0 and zero == np.float32(0.37)


def test_one_bit_is_a_midpoint_threshold(orc):
    rng = np.random.default_rng(7)
    w = rng.normal(size=128).astype(np.float32)
    q, scale, zero = orc.quant_group(w, 1)
    mn, mx = w.min(), w.max()
    assert zero == mn and scale == np.float32(mx - mn)
    mid = (np.float64(mn) + np.float64(mx)) / 2
    far = np.abs(w.astype(np.float64) - mid) > 1e-6   # away from the rounding boundary
    np.testing.assert_array_equal(q[far], (w[far] > mid).astype(np.int32))


def test_round_half_to_even(orc):
    # range 3 at 2 bits: inv = scale = 1 exactly, codes are rint(w)
    w = np.array([0.0, 0.5, 1.5, 2.5, 3.0, 1.0, 2.0, 0.25], np.float32)
    q, scale, zero = orc.quant_group(w, 2)
    assert scale == 1.0 and zero == 0.0
    np.testing.assert_array_equal(q, [0, 0, 2, 2, 3, 1, 2, 0])


def test_zero_is_the_group_minimum_not_an_integer_zero_point(orc):
    w = np.array([-1.0, 2.0, 0.5, 0.0, 1.0, -0.5, 1.5, 2.0], np.float32)
    q, scale, zero = orc.quant_group(w, 2)     # range 3, qmax 3
    assert zero == -1.0 and scale == 1.0
    np.testing.assert_array_equal(q, [0, 3, 2, 1, 2, 0, 2, 3])   # 1.5 -> rint(1.5) = 2, 0.5 -> rint(0.5) = 0


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 8])
def test_codes_in_range_and_error_at_most_half_a_step(orc, bits):
    rng = np.random.default_rng(100 + bits)
    w = orc.bf16_to_f32(orc.f32_to_bf16(0.02 * rng.standard_t(4, size=128)))
    q, scale, zero = orc.quant_group(w, bits)
    qmax = 2 ** bits - 1
    assert q.min() == 0 and q.max() == qmax       # min and max land on the grid ends
    what = q.astype(np.float64) * np.float64(scale) + np.float64(zero)
    assert np.max(np.abs(w - what)) <= 0.5 * float(scale) * (1 + 1e-5)
    # matches the textbook formulation in float64 away from rounding boundaries
    t = (w.astype(np.float64) - w.min()) / ((np.float64(w.max()) - w.min()) / qmax)
    safe = np.abs(t - np.floor(t) - 0.5) > 1e-4
    np.testing.assert_array_equal(q[safe], np.rint(t[safe]).astype(np.int32))


def test_tiny_range_overflowing_reciprocal_falls_back_to_constant_group(orc):
    # range = smallest bf16 subnormal: qmax / range overflows float -> scale = inv = 0
    tiny = np.array([0x0001], np.uint16)
    w = np.zeros(8, np.float32)
    w[3] = orc.bf16_to_f32(tiny)[0]
    q, scale, zero = orc.quant_group(w, 8)
    assert not q.any() and scale == 0.0 and zero == 0.0


# ----------------------------------------------------------------- cost table

def _bf16_mat(orc, x):
    return orc.f32_to_bf16(np.asarray(x, np.float32))


def test_hand_worked_block(orc):
    # 8x8 block, every row [0,1,2,3,0,0,0,3].
    # 1 bit: levels {0,3}; 1 -> 0 (error 1), 2 -> 3 (error -1); cost = sum S over columns 1, 2
    # 2 bits: levels {0,1,2,3}: exact, cost 0
    row = np.array([0, 1, 2, 3, 0, 0, 0, 3], np.float32)
    W = _bf16_mat(orc, np.tile(row, (8, 1)))
    S = np.arange(64, dtype=np.float32).reshape(8, 8)
    cost = orc.cost_table(W, S, 8, 8, [1, 2])
    assert cost.shape == (1, 2)
    assert cost[0, 0] == S[:, 1].sum() + S[:, 2].sum()
    assert cost[0, 1] == 0.0


def test_error_is_squared_and_weighted(orc):
    # row [0, 1, 0, 0, 0, 0, 0, 4] at 1 bit: only the "1" is off the grid, by 1 -> d^2 = 1
    # row [0, 3, 0, 0, 0, 0, 0, 8] at 1 bit: "3" is off by 3 -> d^2 = 9 (not |d| = 3)
    W = np.zeros((8, 8), np.float32)
    W[:, 7] = 4.0
    W[:, 1] = 1.0
    W[5, 7], W[5, 1] = 8.0, 3.0
    S = np.zeros((8, 8), np.float32)
    S[2, 1] = 5.0          # weight 5 on an error of 1  -> 5
    S[5, 1] = 2.0          # weight 2 on an error of 3  -> 18
    S[5, 7] = 100.0        # on-grid element: contributes nothing
    cost = orc.cost_table(_bf16_mat(orc, W), S, 8, 8, [1])
    assert cost[0, 0] == 23.0


def test_power_one_weighs_the_absolute_change(orc):
    # the same block as above under the first-order form (Eq. 3, element-wise): 5*1 + 2*3
    W = np.zeros((8, 8), np.float32)
    W[:, 7] = 4.0
    W[:, 1] = 1.0
    W[5, 7], W[5, 1] = 8.0, 3.0
    S = np.zeros((8, 8), np.float32)
    S[2, 1] = 5.0
    S[5, 1] = 2.0
    S[5, 7] = 100.0
    assert orc.cost_table(_bf16_mat(orc, W), S, 8, 8, [1], power=1)[0, 0] == 11.0
    # a change of 1/2: squared 1/4, absolute 1/2.  Row [0, 0.5, 0, 0, 0, 0, 0, 1] at 1 bit: 0.5 is a tie -> 0
    W = np.zeros((8, 8), np.float32)
    W[:, 7] = 1.0
    W[3, 1] = 0.5
    S = np.full((8, 8), 8.0, np.float32)
    assert orc.cost_table(_bf16_mat(orc, W), S, 8, 8, [1], power=2)[0, 0] == 2.0
    assert orc.cost_table(_bf16_mat(orc, W), S, 8, 8, [1], power=1)[0, 0] == 4.0


def test_block_order_and_group_is_one_block_row(orc):
    # 16 x 24 matrix, blocks 8 x 8 -> 2 x 3 blocks, index I*3 + J.
    # Only block (1, 2) holds off-grid data; the groups are block rows of 8 columns,
    # so the large values in the neighbouring block must not widen its grid.
    W = np.zeros((16, 24), np.float32)
    W[8:, 16:] = np.tile(np.array([0, 1, 2, 3, 0, 0, 0, 3], np.float32), (8, 1))
    W[8:, 8:16] = np.tile(np.array([0, 96, 0, 0, 0, 0, 0, 96], np.float32), (8, 1))   # on its own grids (96/3 exact)
    S = np.ones((16, 24), np.float32)
    cost = orc.cost_table(_bf16_mat(orc, W), S, 8, 8, [1, 2])
    expect = np.zeros((6, 2), np.float32)
    expect[5, 0] = 16.0
    np.testing.assert_array_equal(cost, expect)


def test_non_square_blocks(orc):
    # blocks of 8 rows x 16 columns: group = 16 columns
    row = np.array([0, 1, 2, 3] * 3 + [0, 0, 0, 3], np.float32)        # 1-bit: three 1s and three 2s are off by 1
    W = _bf16_mat(orc, np.tile(row, (16, 1)))
    S = np.ones((16, 16), np.float32)
    cost = orc.cost_table(W, S, 8, 16, [1, 2])
    np.testing.assert_array_equal(cost, [[48.0, 0.0], [48.0, 0.0]])
    cost = orc.cost_table(W, S, 16, 16, [1])
    np.testing.assert_array_equal(cost, [[96.0]])


def test_canonical_order_rows_inside_an_octet_before_columns(orc):
    # 8 x 16 block, 1 bit, rows [0,1,0,0,0,0,0,2 | 0,1,0,0,0,0,0,2]: the error is 1 at columns 1 and 9,
    # so chunk sums are E[r][0] = S[r][1], E[r][1] = S[r][9].
    # E[0][0] = 2^24, E[0][1] = 1, E[1][1] = 1, rest 0:
    #   rows first (canonical): column 0 -> 2^24, column 1 -> 1 + 1 = 2, total 2^24 + 2
    #   columns first would give (2^24 + 1 -> 2^24) + (0 + 1) -> 2^24
    row = np.array([0, 1, 0, 0, 0, 0, 0, 2] * 2, np.float32)
    W = _bf16_mat(orc, np.tile(row, (8, 1)))
    S = np.zeros((8, 16), np.float32)
    S[0, 1], S[0, 9], S[1, 9] = 2.0 ** 24, 1.0, 1.0
    cost = orc.cost_table(W, S, 8, 16, [1])
    assert cost[0, 0] == 2.0 ** 24 + 2.0


def test_canonical_order_chunk_is_sequential_and_octets_pair_up(orc):
    # 16 x 8 block (two octets), 1 bit, rows [0,1,1,1,1,1,1,2]: columns 1..6 are off by 1
    # row 0: S = [.,2^24,1,1,1,1,1,.] -> sequential chain keeps 2^24 (each +1 is a tie to even)
    #        a pairwise order inside the chunk would give 2^24 + 4
    # rows 8 and 9 (second octet) carry 1 each at column 1 -> octet sum 2; total 2^24 + 2
    row = np.array([0, 1, 1, 1, 1, 1, 1, 2], np.float32)
    W = _bf16_mat(orc, np.tile(row, (16, 1)))
    S = np.zeros((16, 8), np.float32)
    S[0, 1] = 2.0 ** 24
    S[0, 2:7] = 1.0
    S[8, 1] = 1.0
    S[9, 1] = 1.0
    cost = orc.cost_table(W, S, 16, 8, [1])
    assert cost[0, 0] == 2.0 ** 24 + 2.0


def _cost_float64(Wf, S, m, n, bits, power=2):
    """The definition written out in float64 with the textbook quantizer; the grid step is
    rounded to float32 because the stored scale, which dequantization uses, is float32."""
    R, C = Wf.shape
    out = np.zeros(((R // m) * (C // n), len(bits)))
    W = Wf.astype(np.float64)
    for I in range(R // m):
        for J in range(C // n):
            w = W[I * m:(I + 1) * m, J * n:(J + 1) * n]
            s = S[I * m:(I + 1) * m, J * n:(J + 1) * n].astype(np.float64)
            mn = w.min(axis=1, keepdims=True)
            rg = w.max(axis=1, keepdims=True) - mn
            for l, b in enumerate(bits):
                step = (rg.astype(np.float32) / np.float32(2 ** b - 1)).astype(np.float64)
                step = np.where(rg > 0, step, 1.0)
                what = np.rint((w - mn) / step) * step + mn
                out[I * (C // n) + J, l] = (s * np.abs(w - what) ** power).sum()
    return out


@pytest.mark.parametrize("m,n,bits", [(16, 16, [1, 2, 3, 4, 8]), (128, 128, [2, 3, 4]), (64, 64, [1, 2, 3, 4, 8])])
def test_cost_table_close_to_float64_definition(orc, m, n, bits):
    rng = np.random.default_rng(m + n)
    R, C = 2 * m, 3 * n
    Wb = orc.f32_to_bf16(0.02 * rng.standard_t(4, size=(R, C)))
    S = np.exp(rng.normal(size=(R, 1)) + rng.normal(size=(1, C)) + 0.5 * rng.normal(size=(R, C))).astype(np.float32)
    cost = orc.cost_table(Wb, S, m, n, bits)
    ref = _cost_float64(orc.bf16_to_f32(Wb), S, m, n, bits)
    assert np.all(cost >= 0)
    np.testing.assert_allclose(cost, ref, rtol=1e-5)


@pytest.mark.parametrize("m,n,bits", [(16, 16, [1, 2, 3, 4, 8]), (64, 128, [1, 2, 3, 4, 5, 6, 7, 8])])
def test_power_one_table_close_to_float64_definition(orc, m, n, bits):
    rng = np.random.default_rng(m + n + 1)
    R, C = 2 * m, 3 * n
    Wb = orc.f32_to_bf16(0.02 * rng.standard_t(4, size=(R, C)))
    S = np.exp(rng.normal(size=(R, 1)) + rng.normal(size=(1, C)) + 0.5 * rng.normal(size=(R, C))).astype(np.float32)
    cost = orc.cost_table(Wb, S, m, n, bits, power=1)
    ref = _cost_float64(orc.bf16_to_f32(Wb), S, m, n, bits, power=1)
    np.testing.assert_allclose(cost, ref, rtol=1e-5)
    # and it is not the squared table
    assert not np.allclose(cost, orc.cost_table(Wb, S, m, n, bits), rtol=1e-2)


def test_nested_grids_give_non_increasing_block_cost(orc):
    # 2^a - 1 divides 2^b - 1 for a | b: the 1, 2, 4, 8-bit min-max grids are nested, so the
    # nearest-point error of every element cannot grow; the block sums follow (up to rounding)
    rng = np.random.default_rng(11)
    Wb = orc.f32_to_bf16(0.02 * rng.standard_t(4, size=(128, 256)))
    S = np.exp(rng.normal(size=(128, 256))).astype(np.float32)
    cost = orc.cost_table(Wb, S, 64, 64, [1, 2, 4, 8]).astype(np.float64)
    assert np.all(cost[:, 1:] <= cost[:, :-1] * (1 + 1e-5))


def test_block_cost_decreases_with_bitwidth_on_the_workload_distribution(orc):
    # 2, 3, 4-bit grids are not nested, so monotonicity (paper App. B) is a property of the
    # block sums on realistic data, not of single elements: count violations
    rng = np.random.default_rng(12)
    Wb = orc.f32_to_bf16(0.02 * rng.standard_t(4, size=(256, 512)))
    S = np.exp(rng.normal(size=(256, 1)) + rng.normal(size=(1, 512))).astype(np.float32)
    cost = orc.cost_table(Wb, S, 128, 128, [1, 2, 3, 4])
    assert np.all(np.diff(cost, axis=1) < 0)
    # uniform-noise model of a b-bit grid: error variance ~ step^2 / 12, so one more bit
    # divides the cost by about ((2^(b+1) - 1) / (2^b - 1))^2 -> 5.4 from 2 to 3 bits, 4.6 from 3 to 4
    ratio = cost[:, 1:-1] / cost[:, 2:]
    assert np.all(ratio[:, 0] > 3.5) and np.all(ratio[:, 0] < 7.5)
    assert np.all(ratio[:, 1] > 3.0) and np.all(ratio[:, 1] < 6.5)
