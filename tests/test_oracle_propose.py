"""Pins of the oracle's single step of Algorithm 2 on caller-supplied estimates (the paper's own
loop: s_up / s_down re-estimated every iteration, acceptance by the caller's loss)."""
import numpy as np
import pytest

import oracle as orc_mod


@pytest.fixture(scope="module")
def orc():
    orc_mod.build()
    return orc_mod


def test_swap_hand_example(orc):
    """Six blocks at 3 bits, budget 3.0 (no slack), k = 4: the two largest s_up are blocks 2 and 5;
    the smallest s_down is block 2 (already raised: skipped), then blocks 1 and 4."""
    s_up = [5, 1, 7, 3, 2, 6]
    s_dn = [9, 1, 0.5, 4, 2, 8]
    kind, out, info = orc.propose(s_up, s_dn, [1] * 6, [2, 3, 4], 3.0, 4)
    assert kind == 2
    np.testing.assert_array_equal(out, [1, 0, 2, 1, 0, 2])
    assert info == dict(n_up=2, n_dn=2, bits_before=18, bits_after=18)


def test_expansion_hand_example(orc):
    """Budget 3.5 * 6 = 21 bits, 18 used: of the top 4 by s_up (blocks 2, 5, 0, 3) only three fit."""
    s_up = [5, 1, 7, 3, 2, 6]
    kind, out, info = orc.propose(s_up, [0] * 6, [1] * 6, [2, 3, 4], 3.5, 4)
    assert kind == 1
    np.testing.assert_array_equal(out, [2, 1, 2, 1, 1, 2])
    assert info == dict(n_up=3, n_dn=0, bits_before=18, bits_after=21)


def test_expansion_stops_at_the_first_non_positive_estimate(orc):
    kind, out, info = orc.propose([2, 0, -1, 3], [1] * 4, [0] * 4, [1, 2], 2.0, 4)
    assert kind == 1 and info["n_up"] == 2
    np.testing.assert_array_equal(out, [1, 0, 0, 1])
    # nothing positive: the step falls through to the swap, which needs someone to lower: none at level 0
    kind, out, info = orc.propose([0, -1, -2, 0], [1] * 4, [0] * 4, [1, 2], 2.0, 4)
    assert kind == 0
    np.testing.assert_array_equal(out, [0] * 4)


def test_wide_steps_count_their_bits(orc):
    """Candidates {2, 4, 8}: raising 4 -> 8 costs 4 bits.  Two blocks at 4 bits, one at 8; budget
    16 bits in all (used 16).  k = 2 -> h = 1: U = {0} (needs 4 bits), D = {2} (frees 4)."""
    kind, out, info = orc.propose([3, 1, 0], [5, 4, 1], [1, 1, 2], [2, 4, 8], 16 / 3 + 1e-9, 2)
    assert kind == 2
    np.testing.assert_array_equal(out, [2, 1, 1])
    assert info["bits_after"] == 16
    # lowering 4 -> 2 frees only 2 bits: the raise does not fit, nothing is proposed
    kind, out, info = orc.propose([3, 1, 0], [5, 1, 4], [1, 1, 2], [2, 4, 8], 16 / 3 + 1e-9, 2)
    assert kind == 0


def _definition(s_up, s_dn, level, bits, avg, k):
    """The step written out with Python's sort."""
    N, K = len(level), len(bits)
    T = int(np.floor(avg * N))
    used = sum(bits[l] for l in level)
    slack = T - used
    su = [np.float32(v) + np.float32(0) for v in s_up]
    sd = [np.float32(v) + np.float32(0) for v in s_dn]
    eu = sorted((i for i in range(N) if level[i] < K - 1), key=lambda i: (-su[i], i))
    ed = sorted((i for i in range(N) if level[i] > 0), key=lambda i: (sd[i], i))
    out = list(level)
    if slack > 0:
        cum, P = 0, []
        for i in eu[:k]:
            st = bits[level[i] + 1] - bits[level[i]]
            if not su[i] > 0 or cum + st > slack:
                break
            cum += st; P.append(i)
        if P:
            for i in P: out[i] += 1
            return 1, out
    h = max(1, k // 2)
    U = eu[:h]
    D = [i for i in ed if i not in U][:h]
    freed = sum(bits[level[i]] - bits[level[i] - 1] for i in D)
    cum, U2 = 0, []
    for i in U:
        st = bits[level[i] + 1] - bits[level[i]]
        if cum + st > slack + freed:
            break
        cum += st; U2.append(i)
    if U2 and D:
        for i in U2: out[i] += 1
        for i in D: out[i] -= 1
        return 2, out
    return 0, out


@pytest.mark.parametrize("seed", range(40))
def test_against_the_written_out_definition(orc, seed):
    rng = np.random.default_rng(seed)
    bits = [[1, 2, 3, 4], [2, 3, 4], [1, 2, 3, 4, 8], [2, 4, 8]][seed % 4]
    K = len(bits)
    N = int(rng.integers(1, 40))
    level = rng.integers(0, K, N).astype(np.uint8)
    s_up = rng.integers(-2, 6, N).astype(np.float32)             # many ties, some non-positive
    s_dn = rng.integers(0, 5, N).astype(np.float32)
    used = sum(bits[l] for l in level)
    avg = (used + int(rng.integers(-1, 6))) / N + 1e-9
    k = int(rng.integers(1, N + 3))
    kind, out, info = orc.propose(s_up, s_dn, level, bits, avg, k)
    wkind, wout = _definition(s_up, s_dn, list(level), bits, avg, k)
    assert kind == wkind
    np.testing.assert_array_equal(out, wout)
    d = out.astype(int) - level.astype(int)
    assert np.abs(d).max(initial=0) <= 1                          # Eq. 5: at most one step per block
    assert np.abs(d).sum() <= max(k, 2)                           # and at most k changes (h = 1 when k = 1)
    if kind:
        assert info["bits_after"] == sum(bits[l] for l in out)
        assert info["bits_after"] <= max(info["bits_before"], int(np.floor(avg * N)))


def test_loop_on_exact_gains_reproduces_the_static_search(orc):
    """Driving the step with the table's own differences as estimates and the table's fixed-point
    cost change as the caller's loss test gives the static search's allocation (contiguous bits)."""
    rng = np.random.default_rng(7)
    N, bits = 300, [1, 2, 3, 4]
    base = rng.lognormal(0, 1.5, N).astype(np.float32)
    cost = (base[:, None] * np.array([1.0, 0.3, 0.1, 0.02], np.float32) *
            rng.uniform(0.7, 1.3, (N, 4)).astype(np.float32)).astype(np.float32)
    for avg in (2.5, 3.0, 2.2):
        rc, want, st, _ = orc.allocate(cost, bits, avg, 0.05, 0.02)
        assert rc == 0
        shift = orc.cost_shift(cost)
        level = np.full(N, [b for b in range(4) if bits[b] <= int(avg)][-1], np.uint8)
        k, kmin, iters = max(1, int(0.05 * N)), max(1, int(0.02 * N)), 0
        idx = np.arange(N)
        while k >= kmin:
            iters += 1
            l = level.astype(int)
            up = np.where(l < 3, cost[idx, l] - cost[idx, np.minimum(l + 1, 3)], 0).astype(np.float32)
            dn = np.where(l > 0, cost[idx, np.maximum(l - 1, 0)] - cost[idx, l], 0).astype(np.float32)
            kind, prop, _ = orc.propose(up, dn, level, bits, avg, k)
            if kind == 1:
                level = prop
            elif kind == 2:
                raised, lowered = np.nonzero(prop > level)[0], np.nonzero(prop < level)[0]
                delta = sum(orc.fx(dn[i], shift) for i in lowered) - sum(orc.fx(up[i], shift) for i in raised)
                if delta < 0: level = prop
                else: k //= 2
            else:
                k //= 2
        np.testing.assert_array_equal(level, want)
        assert iters == st["iters"]
