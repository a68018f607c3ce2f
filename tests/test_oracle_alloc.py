"""Pins for the oracle's scalable greedy search (paper Algorithm 2 on a cost table).

What fixes the result independently of the oracle: hand-traced runs of Algorithm 2,
the exhaustive optimum of Eq. 1 on tiny instances, Algorithm 1 (classic greedy),
and the constraints of Eq. 5 (per-iteration ||db||_inf <= 1, ||db||_1 <= k) with
the budget of Eq. 1 holding exactly.  The iteration-by-iteration trajectory on
large tables has no independent pin ("parity unpinned"): it is Algorithm 2 itself.
"""
import numpy as np
import pytest

B234 = [2, 3, 4]


def convex_table(rng, N, K, integer=True):
    """Rows with positive, strictly decreasing per-step gains (monotone + diminishing returns)."""
    gains = np.sort(rng.choice(np.arange(1, 50 * K * N), size=(N, K - 1), replace=False), axis=1)[:, ::-1]
    tail = rng.integers(0, 5, size=(N, 1))
    cost = np.concatenate([gains[:, ::-1].cumsum(1)[:, ::-1] + tail, tail], axis=1)
    return cost.astype(np.float32)


# --------------------------------------------------------------- hand-traced runs

TABLE4 = np.array([[10, 4, 1],
                   [8, 5, 4.5],
                   [20, 6, 1],
                   [3, 2, 1.5]], np.float32)


def test_hand_traced_swap_phase(orc):
    # B = 3: warm start at 3 bits uses the whole budget, so only swaps happen; k = 2 -> k/2 = 1.
    # it 1: raise block 2 (gain 5), lower block 3 (loss 1): 1 - 5 < 0, accepted
    # it 2: raise block 0 (gain 3), lower block 1 (loss 3): 0 is not an improvement, rejected, k = 1
    # it 3: same proposal, rejected, k = 0 -> stop
    rc, level, st, tr = orc.allocate(TABLE4, B234, 3.0, gamma0=0.5, gammaT=0.25, want_trace=True)
    assert rc == 0
    np.testing.assert_array_equal(level, [1, 1, 2, 0])
    assert (st["iters"], st["expansions"], st["swaps_ok"], st["swaps_rej"]) == (3, 0, 1, 2)
    assert st["bits_used"] == 12 and st["bits_budget"] == 12 and st["k_final"] == 0
    assert [t["kind"] for t in tr] == [1, 2, 2]
    assert tr[0]["delta_fixed"] == orc.fx(1.0, st["cost_shift"]) - orc.fx(5.0, st["cost_shift"])
    assert tr[1]["delta_fixed"] == 0
    assert st["cost_fixed"] == orc.fx(13.0, st["cost_shift"])


def test_hand_traced_expansion_then_swap(orc):
    # B = 2.5, T = 10: warm start at 2 bits (8 used, slack 2), k = 2
    # it 1: expansion raises the two largest gains, blocks 2 (14) and 0 (6) -> budget met
    # it 2: raise 2 (gain 5) / lower 0 (loss 6): worse, rejected, k = 1;  it 3: again, k = 0
    rc, level, st, tr = orc.allocate(TABLE4, B234, 2.5, gamma0=0.5, gammaT=0.25, want_trace=True)
    assert rc == 0
    np.testing.assert_array_equal(level, [1, 0, 1, 0])
    assert (st["iters"], st["expansions"], st["swaps_ok"], st["swaps_rej"]) == (3, 1, 0, 2)
    assert st["bits_used"] == 10
    assert tr[0]["kind"] == 0 and tr[0]["n_up"] == 2 and tr[0]["bits_before"] == 8 and tr[0]["bits_after"] == 10


def test_expansion_is_capped_by_the_budget_and_by_positive_gain(orc):
    # slack 1 with k = 2: only the best block moves
    cost = np.array([[9, 1, 0], [8, 1, 0], [7, 1, 0], [6, 1, 0]], np.float32)
    rc, level, st, tr = orc.allocate(cost, B234, 2.25, gamma0=0.5, gammaT=0.25, want_trace=True)
    assert tr[0]["kind"] == 0 and tr[0]["n_up"] == 1
    assert st["bits_used"] == 9 and level[0] == 1
    # no positive gain anywhere: nothing is raised although there is slack
    flat = np.ones((4, 3), np.float32)
    rc, level, st, tr = orc.allocate(flat, B234, 2.5, gamma0=0.5, gammaT=0.25, want_trace=True)
    np.testing.assert_array_equal(level, [0, 0, 0, 0])
    assert st["expansions"] == 0 and st["bits_used"] == 8


def test_tie_break_lower_index_first(orc):
    cost = np.tile(np.array([[5, 2, 1]], np.float32), (6, 1))       # all blocks identical
    rc, level, st, _ = orc.allocate(cost, B234, 2.5, gamma0=0.34, gammaT=0.1)   # k = 2, slack 3
    # expansion 1 raises blocks 0, 1; expansion 2 raises block 2 only (slack 1)
    np.testing.assert_array_equal(level, [1, 1, 1, 0, 0, 0])


def test_infeasible_budget_and_budget_above_the_largest_candidate(orc):
    rc, *_ = orc.allocate(TABLE4, B234, 1.9)
    assert rc == -1
    rc, level, st, _ = orc.allocate(TABLE4, B234, 4.0)
    assert rc == 0 and np.all(level == 2) and st["iters"] == 0 and st["bits_used"] == 16
    rc, level, st, _ = orc.allocate(TABLE4, B234, 7.5)
    assert rc == 0 and np.all(level == 2)


def test_warm_start_uses_largest_candidate_not_above_floor_b(orc):
    # candidates {1,2,4,8}, B = 3.5: floor(B) = 3 is no candidate -> start at 2 bits
    cost = np.tile(np.array([[8, 4, 2, 1]], np.float32), (4, 1))
    rc, level, st, tr = orc.allocate(cost, [1, 2, 4, 8], 3.5, gamma0=0.5, gammaT=0.25, want_trace=True)
    assert tr[0]["bits_before"] == 8
    rc, level, st, tr = orc.allocate(cost, [1, 2, 4, 8], 3.5, gamma0=0.5, gammaT=0.25, init_mode=1, want_trace=True)
    assert tr[0]["bits_before"] == 4


def test_max_iters_status(orc):
    rng = np.random.default_rng(0)
    cost = convex_table(rng, 64, 3)
    rc, level, st, _ = orc.allocate(cost, B234, 2.5, gamma0=0.05, gammaT=0.0, max_iters=2)
    assert rc == -2 and st["iters"] == 2
    assert st["bits_used"] <= st["bits_budget"]


# ------------------------------------------------------- optimum on tiny instances

@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("avg", [2.0, 2.25, 2.5, 3.0, 3.4, 3.9])
def test_convex_tables_reach_the_exhaustive_optimum(orc, seed, avg):
    rng = np.random.default_rng(seed)
    N = 8
    cost = convex_table(rng, N, 3)
    opt, _ = orc.brute_force(cost, B234, avg)
    for init_mode in (0, 1):
        rc, level, st, _ = orc.allocate(cost, B234, avg, gamma0=0.3, gammaT=0.0, init_mode=init_mode)
        assert rc == 0
        got = float(cost[np.arange(N), level].astype(np.float64).sum())
        assert got == opt, (init_mode, level)
        assert st["bits_used"] <= int(np.floor(avg * N))
    lv1 = orc.classic_greedy(cost, B234, avg)
    assert float(cost[np.arange(N), lv1].astype(np.float64).sum()) == opt


@pytest.mark.parametrize("seed", range(4))
def test_four_candidates_convex_optimum(orc, seed):
    rng = np.random.default_rng(100 + seed)
    N, bits = 9, [1, 2, 3, 4]
    cost = convex_table(rng, N, 4)
    for avg in (1.5, 2.5, 3.0, 3.3):
        opt, _ = orc.brute_force(cost, bits, avg)
        rc, level, st, _ = orc.allocate(cost, bits, avg, gamma0=0.25, gammaT=0.0)
        assert float(cost[np.arange(N), level].astype(np.float64).sum()) == opt


@pytest.mark.parametrize("seed", range(6))
def test_never_better_than_the_optimum_and_always_feasible(orc, seed):
    # arbitrary (non-convex, non-monotone) tables and uneven candidate steps
    rng = np.random.default_rng(200 + seed)
    N, bits = 7, [1, 2, 3, 4, 8]
    cost = rng.random((N, 5)).astype(np.float32)
    for avg in (1.0, 2.25, 3.7, 5.0):
        opt, _ = orc.brute_force(cost, bits, avg)
        rc, level, st, _ = orc.allocate(cost, bits, avg, gamma0=0.3, gammaT=0.0)
        assert rc == 0
        used = int(np.asarray(bits)[level].sum())
        assert used == st["bits_used"] <= int(np.floor(avg * N))
        assert float(cost[np.arange(N), level].astype(np.float64).sum()) >= opt - 1e-9


def test_brute_force_itself_on_a_known_instance():
    # independent enumeration in Python of the 3^4 assignments of TABLE4 at 12 bits
    import itertools
    import oracle
    best = min(sum(float(TABLE4[i, l]) for i, l in enumerate(lv))
               for lv in itertools.product(range(3), repeat=4)
               if sum(B234[l] for l in lv) <= 12)
    assert best == 13.0
    opt, lv = oracle.brute_force(TABLE4, B234, 3.0)
    assert opt == 13.0 and sum(B234[l] for l in lv) <= 12


# ------------------------------------------------------------ invariants at scale

@pytest.mark.parametrize("bits,avg,N", [([2, 3, 4], 3.0, 4000), ([1, 2, 3, 4], 2.5, 5000),
                                        ([1, 2, 3, 4, 8], 2.25, 3000), ([2, 3, 4], 2.75, 2048)])
def test_trace_obeys_the_relaxed_step_constraints(orc, bits, avg, N):
    rng = np.random.default_rng(N)
    K = len(bits)
    # error ~ sens * 4^-b, the shape the quantizer produces, with noise so that rows are not exactly convex
    sens = np.exp(2.0 * rng.normal(size=(N, 1)))
    cost = (sens * 4.0 ** -np.asarray(bits, np.float64)[None, :] * np.exp(0.2 * rng.normal(size=(N, K)))).astype(np.float32)
    rc, level, st, tr = orc.allocate(cost, bits, avg, want_trace=True)
    assert rc == 0
    T = int(np.floor(avg * N))
    barr = np.asarray(bits)
    assert st["bits_budget"] == T and st["bits_used"] == int(barr[level].sum()) <= T
    assert st["iters"] == len(tr) == st["expansions"] + st["swaps_ok"] + st["swaps_rej"]
    k0, kmin = max(1, int(0.05 * N)), max(1, int(0.02 * N))
    assert tr[0]["k"] == k0 and st["k_final"] < kmin
    total = None
    for t in tr:
        assert t["bits_before"] <= T and t["bits_after"] <= T            # Eq. 1 holds at every step
        assert t["n_up"] + t["n_dn"] <= t["k"]                            # ||db||_1 <= k
        if t["kind"] == 0:
            assert t["bits_before"] < T and t["n_up"] >= 1 and t["n_dn"] == 0
        if t["kind"] == 1:
            assert t["delta_fixed"] < 0 and t["n_up"] >= 1 and t["n_dn"] >= 1
        if t["kind"] == 2:
            assert t["n_up"] == t["n_dn"] == 0 and t["bits_after"] == t["bits_before"]
    # k halves exactly on rejections
    ks = [t["k"] for t in tr]
    for a, b, t in zip(ks, ks[1:], tr):
        assert b == (a // 2 if t["kind"] == 2 else a)
    # the search lands in the tens of iterations (paper Table 3 reports 16-36)
    assert 3 <= st["iters"] <= 200
    # fixed-point total equals the sum of the chosen entries, and is order independent
    sh = st["cost_shift"]
    chosen = cost[np.arange(N), level]
    fxs = np.array([orc.fx(v, sh) for v in chosen], dtype=object)
    assert int(fxs.sum()) == st["cost_fixed"] == int(fxs[rng.permutation(N)].sum())
    assert abs(st["cost_fixed"]) < 2 ** 62


def test_mixed_precision_beats_uniform_at_equal_budget(orc):
    rng = np.random.default_rng(5)
    N = 2000
    sens = np.exp(2.0 * rng.normal(size=(N, 1)))
    cost = (sens * 4.0 ** -np.array([2.0, 3.0, 4.0])[None, :]).astype(np.float32)
    rc, level, st, _ = orc.allocate(cost, B234, 3.0)
    assert cost[np.arange(N), level].sum() < 0.8 * cost[:, 1].sum()
    # blocks with larger sensitivity get at least as many bits on average
    order = np.argsort(sens[:, 0])
    assert level[order[-200:]].mean() > level[order[:200]].mean()


def test_fixed_point_shift_cannot_overflow(orc):
    for scale in (1e-30, 1e-3, 1.0, 1e6, 1e30):
        for N in (1, 2, 3, 1000, 4177920):
            cost = np.full((min(N, 4), 3), scale, np.float32)
            sh = 61 - int(np.ceil(np.log2(N))) - (int(np.floor(np.log2(float(np.float32(scale))))) + 1)
            import ctypes
            got = orc.lib().orc_cost_shift(cost.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(N), ctypes.c_int(3)) \
                if N <= 4 else None
            if got is not None:
                assert got == sh
            assert abs(orc.fx(np.float32(scale), sh)) * N < 2 ** 62
    assert orc.cost_shift(np.zeros((4, 3), np.float32)) == 0
    assert orc.fx(1.5, 1) == 3 and orc.fx(0.75, 1) == 2 and orc.fx(1.25, 1) == 2 and orc.fx(-0.75, 1) == -2  # half to even
