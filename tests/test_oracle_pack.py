"""Pins for the oracle's byte offsets and bit-packing (uniform bitwidth per block, paper Sec. 5.3).

The unpacker below is independent numpy (np.unpackbits, little bit order); the codes it
recovers must equal the quantizer's, and dequantizing them must reproduce the weights
to within half a grid step.
"""
import numpy as np
import pytest


def unpack_block(buf, c, m, n):
    bits = np.unpackbits(np.asarray(buf, np.uint8), bitorder="little")
    assert bits.size == m * n * c
    weights = (1 << np.arange(c)).astype(np.int32)
    return (bits.reshape(m * n, c) * weights).sum(1).reshape(m, n)


def test_offsets_are_an_exclusive_scan_of_block_sizes(orc):
    rng = np.random.default_rng(0)
    bits = [1, 2, 3, 4, 8]
    level = rng.integers(0, 5, size=1000).astype(np.uint8)
    off = orc.offsets(level, 64, 64, bits)
    sizes = 64 * 64 * np.asarray(bits)[level] // 8
    np.testing.assert_array_equal(off, np.concatenate([[0], np.cumsum(sizes)]))


def test_bit_layout_lsb_first_and_three_bit_codes_cross_bytes(orc):
    # one 8x8 block whose every row is the on-grid ramp 0..7 at 3 bits: codes = 0..7
    W = orc.f32_to_bf16(np.tile(np.arange(8, dtype=np.float32), (8, 1)))
    level = np.array([0], np.uint8)
    off = orc.offsets(level, 8, 8, [3])
    assert off.tolist() == [0, 24]
    codes = np.full(24, 0xAA, np.uint8)                 # must be fully overwritten
    scale = np.zeros(8, np.float32)
    zero = np.zeros(8, np.float32)
    orc.pack(W, 8, 8, [3], level, off, 0, codes, scale, zero)
    # codes 0,1,2,...,7 -> bit stream 000 100 010 110 001 101 011 111 (LSB first)
    # bytes: 0b10001000 = 0x88, 0b11000110 = 0xC6, 0b11111010 = 0xFA
    np.testing.assert_array_equal(codes.reshape(8, 3), np.tile(np.array([0x88, 0xC6, 0xFA], np.uint8), (8, 1)))
    np.testing.assert_array_equal(scale, np.ones(8, np.float32))
    np.testing.assert_array_equal(zero, np.zeros(8, np.float32))


@pytest.mark.parametrize("m,n,bits", [(8, 8, [1, 2, 3, 4, 8]), (16, 32, [2, 3, 4]), (64, 64, [1, 2, 3, 4, 8])])
def test_round_trip_over_a_multi_block_matrix(orc, m, n, bits):
    rng = np.random.default_rng(m * n)
    R, C, base = 2 * m, 3 * n, 5                        # this matrix's blocks start at global id 5
    Wb = orc.f32_to_bf16(0.02 * rng.standard_t(4, size=(R, C)))
    Wf = orc.bf16_to_f32(Wb)
    N = base + 6 + 2
    level = rng.integers(0, len(bits), size=N).astype(np.uint8)
    off = orc.offsets(level, m, n, bits)
    codes = np.full(off[-1], 0x55, np.uint8)
    scale = np.full(N * m, -1, np.float32)
    zero = np.full(N * m, -1, np.float32)
    orc.pack(Wb, m, n, bits, level, off, base, codes, scale, zero)
    assert np.all(codes[:off[base]] == 0x55) and np.all(codes[off[base + 6]:] == 0x55)   # stays inside its range
    assert np.all(scale[:base * m] == -1) and np.all(scale[(base + 6) * m:] == -1)
    for I in range(2):
        for J in range(3):
            b = base + I * 3 + J
            c = bits[level[b]]
            q = unpack_block(codes[off[b]:off[b + 1]], c, m, n)
            blk = Wf[I * m:(I + 1) * m, J * n:(J + 1) * n]
            for r in range(m):
                q_ref, sc, ze = orc.quant_group(blk[r], c)
                np.testing.assert_array_equal(q[r], q_ref)
                assert scale[b * m + r] == sc and zero[b * m + r] == ze
            what = q * scale[b * m:(b + 1) * m, None].astype(np.float64) + zero[b * m:(b + 1) * m, None]
            assert np.all(np.abs(blk - what) <= 0.5 * scale[b * m:(b + 1) * m, None] * (1 + 1e-5))
            np.testing.assert_array_equal(zero[b * m:(b + 1) * m], blk.min(axis=1))
