"""Pins for the 0-bit candidate in the oracle: a block at 0 bits is pruned (paper Sec. 3:
b_i = 0 removes the component), i.e. its stored value is 0 everywhere, its change is the weight
itself, it takes no bytes, and Algorithm 2 treats 0 like any other candidate bitwidth.

Expected values: hand-worked blocks, the float64 definition, exhaustive search on tiny tables.
"""
import numpy as np
import pytest


def _bf16(orc, x):
    return orc.f32_to_bf16(np.asarray(x, np.float32))


def test_pruned_group_stores_nothing(orc):
    w = np.array([-1.5, 2.0, 0.25, 7.0, -3.0, 0.0, 1.0, 4.0], np.float32)
    q, scale, zero = orc.quant_group(w, 0)
    assert not q.any() and scale == 0.0 and zero == 0.0
    assert np.signbit(zero) == False        # noqa: E712  (+0, as every stored origin)


def test_pruned_cost_is_the_weighted_square_of_the_weight_itself(orc):
    # 8 x 8 block: row r = [r, 0, 0, 0, 0, 0, 0, -2]; S = 1 except S[3][0] = 10
    W = np.zeros((8, 8), np.float32)
    W[:, 0] = np.arange(8)
    W[:, 7] = -2.0
    S = np.ones((8, 8), np.float32)
    S[3, 0] = 10.0
    cost = orc.cost_table(_bf16(orc, W), S, 8, 8, [0, 1, 8])
    expect = sum(r * r for r in range(8)) + 9 * 9 + 8 * 4         # 140 + 81 + 32
    assert cost[0, 0] == expect
    # 1 bit: the row's grid is {-2, r}; only its six zeros are off it, by min(2, r): 6 * (0 + 1 + 6 * 4)
    assert cost[0, 1] == 150.0 and cost[0, 2] <= cost[0, 1]
    # first-order variant: sum s * |w|
    cost1 = orc.cost_table(_bf16(orc, W), S, 8, 8, [0], power=1)
    assert cost1[0, 0] == sum(range(8)) + 9 * 3 + 8 * 2


def test_pruned_is_not_the_one_level_grid_at_the_minimum(orc):
    # a constant block 5.0: any grid with at least one level stores it exactly; pruning loses all of it
    W = np.full((8, 8), 5.0, np.float32)
    S = np.ones((8, 8), np.float32)
    cost = orc.cost_table(_bf16(orc, W), S, 8, 8, [0, 1])
    assert cost[0, 0] == 64 * 25.0 and cost[0, 1] == 0.0


@pytest.mark.parametrize("m,n", [(16, 16), (64, 128)])
def test_pruned_column_close_to_float64_and_other_columns_unchanged(orc, m, n):
    rng = np.random.default_rng(m + n)
    R, C = 2 * m, 3 * n
    Wb = orc.f32_to_bf16(0.02 * rng.standard_t(4, size=(R, C)))
    S = np.exp(rng.normal(size=(R, 1)) + rng.normal(size=(1, C)) + 0.5 * rng.normal(size=(R, C))).astype(np.float32)
    cost = orc.cost_table(Wb, S, m, n, [0, 1, 2, 4])
    w = orc.bf16_to_f32(Wb).astype(np.float64)
    s = S.astype(np.float64)
    ref = np.array([(s[I * m:(I + 1) * m, J * n:(J + 1) * n] * w[I * m:(I + 1) * m, J * n:(J + 1) * n] ** 2).sum()
                    for I in range(R // m) for J in range(C // n)])
    np.testing.assert_allclose(cost[:, 0], ref, rtol=1e-5)
    np.testing.assert_array_equal(cost[:, 1:], orc.cost_table(Wb, S, m, n, [1, 2, 4]))
    # (heavy-tailed rows: the 1-bit min-max grid can cost MORE than dropping the block; 4 bits never do here)
    assert np.all(cost[:, 0] > cost[:, 3])


def test_surrogates_of_a_pruned_block(orc):
    rng = np.random.default_rng(5)
    m, n = 16, 16
    Wb = orc.f32_to_bf16(rng.normal(size=(m, 2 * n)))
    G = rng.normal(size=(m, 2 * n)).astype(np.float32)
    up, dn = orc.surrogates(Wb, G, m, n, [0, 2, 4], np.array([0, 1], np.uint8))
    w = orc.bf16_to_f32(Wb).astype(np.float64)
    # pruned block: what = 0, so s_up = g . w and nothing is left to lose
    np.testing.assert_allclose(up[0], (G[:, :n].astype(np.float64) * w[:, :n]).sum(), rtol=1e-4, atol=1e-5)
    assert dn[0] == 0.0
    # its neighbour at 2 bits is what it is without a 0 in the list
    up2, dn2 = orc.surrogates(Wb, G, m, n, [2, 4], np.array([0, 0], np.uint8))
    assert up[1] == up2[1] and dn[1] == dn2[1]


def test_pruned_blocks_take_no_bytes_and_dequantize_to_zero(orc):
    rng = np.random.default_rng(9)
    m, n, R, C = 8, 16, 16, 48
    Wb = orc.f32_to_bf16(rng.normal(size=(R, C)))
    bits = [0, 3, 4]
    level = np.array([1, 0, 2, 0, 0, 1], np.uint8)              # blocks (0,0) (0,1) (0,2) (1,0) (1,1) (1,2)
    off = orc.offsets(level, m, n, bits)
    np.testing.assert_array_equal(off, [0, 48, 48, 112, 112, 112, 160])
    N = 6
    codes = np.full(int(off[-1]), 0xAA, np.uint8)
    scale = np.full(N * m, 7.0, np.float32)
    zero = np.full(N * m, 7.0, np.float32)
    orc.pack(Wb, m, n, bits, level, off, 0, codes, scale, zero)
    # the same blocks packed from a list without 0: identical bytes for the kept blocks
    bits2 = [3, 4]
    Wkeep = np.concatenate([Wb[:8, 0:16], Wb[:8, 32:48], Wb[8:, 32:48]], axis=1)     # the three kept blocks side by side
    level2 = np.array([0, 1, 0], np.uint8)
    off2 = orc.offsets(level2, m, n, bits2)
    codes2 = np.zeros(int(off2[-1]), np.uint8)
    scale2, zero2 = np.zeros(3 * m, np.float32), np.zeros(3 * m, np.float32)
    orc.pack(np.ascontiguousarray(Wkeep), m, n, bits2, level2, off2, 0, codes2, scale2, zero2)
    np.testing.assert_array_equal(codes, codes2)
    kept = [0, 2, 5]
    for t, b in enumerate(kept):
        np.testing.assert_array_equal(scale[b * m:(b + 1) * m], scale2[t * m:(t + 1) * m])
        np.testing.assert_array_equal(zero[b * m:(b + 1) * m], zero2[t * m:(t + 1) * m])
    for b in (1, 3, 4):
        assert not scale[b * m:(b + 1) * m].any() and not zero[b * m:(b + 1) * m].any()
    What = orc.dequant(codes, scale, zero, level, off, 0, R, C, m, n, bits)
    assert not What[:8, 16:32].any() and not What[8:, :32].any()
    assert What[:8, :16].any() and What[8:, 32:].any()
    # the product sees zeros there
    x = orc.f32_to_bf16(rng.normal(size=(3, C)))
    y = orc.mp_gemm(codes, scale, zero, level, off, 0, R, C, m, n, bits, x)
    np.testing.assert_allclose(y, orc.bf16_to_f32(x).astype(np.float64) @ What.astype(np.float64).T, rtol=1e-12, atol=1e-12)


def _convex(rng, N, K):
    d = np.sort(rng.integers(1, 64, size=(N, K - 1)), axis=1)[:, ::-1]        # decreasing gains
    c = np.zeros((N, K))
    c[:, 0] = d.sum(1) + rng.integers(0, 8, size=N)
    for l in range(1, K):
        c[:, l] = c[:, l - 1] - d[:, l - 1]
    return c.astype(np.float32)


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("bits,avgs", [([0, 1, 2], (0.0, 0.5, 1.0, 1.4)), ([0, 1, 2, 3], (0.75, 1.5, 2.5))])
def test_search_with_a_pruned_candidate_reaches_the_exhaustive_optimum(orc, seed, bits, avgs):
    rng = np.random.default_rng(300 + seed)
    N = 8
    cost = _convex(rng, N, len(bits))
    for avg in avgs:
        opt, _ = orc.brute_force(cost, bits, avg)
        rc, level, st, _ = orc.allocate(cost, bits, avg, gamma0=0.3, gammaT=0.0)
        assert rc == 0
        assert st["bits_used"] == int(np.asarray(bits)[level].sum()) <= int(np.floor(avg * N))
        assert float(cost[np.arange(N), level].astype(np.float64).sum()) == opt, (avg, level)


def test_uneven_steps_from_zero_stay_feasible(orc):
    rng = np.random.default_rng(17)
    N, bits = 7, [0, 2, 3, 8]
    cost = rng.random((N, 4)).astype(np.float32)
    for avg in (0.0, 0.9, 2.0, 4.5):
        opt, _ = orc.brute_force(cost, bits, avg)
        rc, level, st, _ = orc.allocate(cost, bits, avg, gamma0=0.3, gammaT=0.0)
        assert rc == 0
        assert st["bits_used"] == int(np.asarray(bits)[level].sum()) <= int(np.floor(avg * N))
        assert float(cost[np.arange(N), level].astype(np.float64).sum()) >= opt - 1e-9
    # warm start: the largest candidate not above floor(B); below 2 bits that is the pruned one
    rc, level, st, tr = orc.allocate(cost, bits, 1.9, gamma0=0.0, gammaT=0.0, max_iters=1, want_trace=True)
    assert tr[0]["bits_before"] == 0
