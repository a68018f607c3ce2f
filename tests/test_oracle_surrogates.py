"""Pins of the oracle's dynamic-sensitivity surrogates (paper App. "choice of sensitivity
statistics": s_up = g^T (w - w^Q_b), s_down = 2^-b ||g . w^Q_b||_1 per block)."""
import numpy as np
import pytest


def bf16(orc, x):
    return orc.f32_to_bf16(np.asarray(x, np.float32))


def test_weights_on_the_grid_have_no_gain_and_an_exact_loss(orc):
    """Every row holds all of 0..7, so the 3-bit grid (min 0, range 7, step 1) represents the block
    exactly: s_up = 0.  With g = 1, s_down = 2^-3 * sum(w), an integer sum."""
    m = n = 8
    rng = np.random.default_rng(0)
    W = np.stack([rng.permutation(8) for _ in range(8)]).astype(np.float32)
    G = np.ones((m, n), np.float32)
    up, dn = orc.surrogates(bf16(orc, W), G, m, n, [3], np.zeros(1, np.uint8))
    assert up[0] == 0.0
    assert dn[0] == W.sum() / 8.0


def test_one_bit_hand_example(orc):
    """One row group [0, 1, 0.25, 0.75, 0.5, 0.125, 0.875, 1] at 1 bit: grid {0, 1}, codes by
    round-half-to-even = [0,1,0,1,0,0,1,1], so w - what = [0,0,.25,-.25,.5,.125,-.125,0].
    With g = [1,1,4,1,2,8,8,1]: s_up = 1 - .25 + 1 + 1 - 1 = 1.75; what = [0,1,0,1,0,0,1,1]:
    s_down = 2^-1 * (1 + 1 + 8 + 1) = 5.5.  The other seven rows are zero weights (range 0)."""
    m = n = 8
    W = np.zeros((m, n), np.float32)
    W[0] = [0, 1, 0.25, 0.75, 0.5, 0.125, 0.875, 1]
    G = np.zeros((m, n), np.float32)
    G[0] = [1, 1, 4, 1, 2, 8, 8, 1]
    G[1:] = 3.0                                   # constant groups: what = w = 0, no contribution
    up, dn = orc.surrogates(bf16(orc, W), G, m, n, [1, 2], np.zeros(1, np.uint8))
    assert up[0] == 1.75 and dn[0] == 5.5


def test_sign_and_scale_of_the_gradient(orc):
    rng = np.random.default_rng(1)
    m, n = 16, 32
    W = bf16(orc, rng.standard_normal((2 * m, 3 * n)) * 0.02)
    G = rng.standard_normal((2 * m, 3 * n)).astype(np.float32)
    level = rng.integers(0, 3, 6).astype(np.uint8)
    up, dn = orc.surrogates(W, G, m, n, [2, 3, 4], level)
    up2, dn2 = orc.surrogates(W, -G, m, n, [2, 3, 4], level)
    np.testing.assert_array_equal(up2, -up)       # signed aggregation
    np.testing.assert_array_equal(dn2, dn)        # magnitude aggregation
    up4, dn4 = orc.surrogates(W, 4 * G, m, n, [2, 3, 4], level)
    np.testing.assert_array_equal(up4, 4 * up)    # powers of two commute with every rounding
    np.testing.assert_array_equal(dn4, 4 * dn)
    assert np.all(dn >= 0)


def test_gain_with_the_error_as_gradient_is_the_cost_table_entry(orc):
    """With g = s * (w - what_b), s_up = sum s (w - what_b)^2: the cost-table entry of bitwidth b
    (pinned on its own), up to the rounding of the two ways of forming w - what."""
    rng = np.random.default_rng(2)
    m = n = 64
    bits = [2, 3, 4]
    Wf = (rng.standard_normal((m, 2 * n)) * 0.02).astype(np.float32)
    W = bf16(orc, Wf)
    Wv = orc.bf16_to_f32(W)
    S = rng.random((m, 2 * n)).astype(np.float32)
    cost = orc.cost_table(W, S, m, n, bits)
    for l, b in enumerate(bits):
        codes = np.zeros(m * 2 * n * 8, np.uint8)
        D = np.empty_like(Wv)
        for r in range(m):
            for J in range(2):
                g = Wv[r, J * n:(J + 1) * n]
                q, scale, zero = orc.quant_group(g, b)
                D[r, J * n:(J + 1) * n] = g - (q.astype(np.float32) * scale + zero)
        up, _ = orc.surrogates(W, (S * D).astype(np.float32), m, n, bits, np.full(2, l, np.uint8))
        np.testing.assert_allclose(up, cost[:, l], rtol=2e-5)


def test_loss_scales_with_the_step_size(orc):
    """s_down carries the factor 2^-b of its block's own bitwidth."""
    m = n = 8
    W = np.tile(np.arange(8, dtype=np.float32), (8, 1))          # on the 3-bit grid
    G = np.ones((m, n), np.float32)
    _, dn3 = orc.surrogates(bf16(orc, W), G, m, n, [3, 8], np.zeros(1, np.uint8))
    _, dn8 = orc.surrogates(bf16(orc, W), G, m, n, [3, 8], np.ones(1, np.uint8))
    # at 8 bits the grid step is 7/255: what differs from w by rounding only, the 2^-b factor dominates
    assert dn3[0] == W.sum() / 8
    np.testing.assert_allclose(dn8[0], W.sum() / 256, rtol=1e-6)
