"""Pins for the oracle's channel scores, permutations and reorder-gather.

Each check compares the oracle with something fixed by mathematics or by a
library routine, never with the oracle itself: exact integer sums, numpy's
stable argsort and fancy indexing, and the invariance of a linear layer's
output under consistent row/column permutation (paper Sec. 4.1: reordering must
preserve functional equivalence).
"""
import numpy as np
import pytest


def test_canon8_exact_on_integers(orc):
    # integer-valued floats below 2^24 add exactly in any order
    rng = np.random.default_rng(0)
    for L in (1, 7, 8, 9, 63, 64, 65, 1000, 1792 * 8):
        x = rng.integers(0, 100, size=L).astype(np.float32)
        assert orc.canon8(x) == float(x.astype(np.int64).sum())


def test_canon8_order_is_chunk_sequential_then_pair_tree(orc):
    big = np.float32(2.0 ** 24)
    # chunk 0 runs left to right from +0: 2^24 absorbs each following 1 (ties to even)
    x = np.array([big] + [1] * 7 + [1] * 8, np.float32)
    assert orc.canon8(x) == 2.0 ** 24 + 8.0
    # a pairwise tree inside the chunk would give 2^24 + 6 + 8; a fully sequential
    # sum would give 2^24: both differ from the canonical value
    x = np.zeros(32, np.float32)
    x[0], x[8], x[16], x[24] = big, 1, 1, 1
    # ((2^24 + 1) + (1 + 1)) = 2^24 + 2, whereas left-to-right over chunk sums gives 2^24
    assert orc.canon8(x) == 2.0 ** 24 + 2.0


def test_canon8_padding_to_power_of_two(orc):
    # 3 chunks -> padded to 4: ((c0 + c1) + (c2 + 0))
    big = np.float32(2.0 ** 24)
    x = np.zeros(24, np.float32)
    x[0], x[8], x[16] = 1, big, 1
    assert orc.canon8(x) == 2.0 ** 24                 # (1 + 2^24) -> 2^24, then + (1 + 0) -> 2^24 (ties to even)
    x[0], x[8], x[16] = 1, 1, big
    assert orc.canon8(x) == 2.0 ** 24 + 2.0          # (1 + 1) + (2^24 + 0)


def test_channel_scores_rows_vs_columns(orc):
    rng = np.random.default_rng(1)
    S = rng.integers(0, 50, size=(24, 40)).astype(np.float32)
    S[3, 5] = -7.0                                    # l1 norm: sign must not cancel
    rs, cs = orc.channel_scores(S)
    assert rs.shape == (24,) and cs.shape == (40,)
    np.testing.assert_array_equal(rs, np.abs(S).sum(axis=1))
    np.testing.assert_array_equal(cs, np.abs(S).sum(axis=0))


def test_channel_scores_close_to_float64(orc):
    rng = np.random.default_rng(2)
    S = np.exp(rng.normal(size=(136, 264))).astype(np.float32)
    rs, cs = orc.channel_scores(S)
    np.testing.assert_allclose(rs, S.astype(np.float64).sum(1), rtol=2e-6)
    np.testing.assert_allclose(cs, S.astype(np.float64).sum(0), rtol=2e-6)


def test_argsort_matches_numpy_stable_descending(orc):
    rng = np.random.default_rng(3)
    s = rng.integers(0, 20, size=500).astype(np.float32)   # many ties
    perm = orc.argsort_desc(s)
    ref = np.argsort(-s, kind="stable").astype(np.int32)
    np.testing.assert_array_equal(perm, ref)
    assert sorted(perm.tolist()) == list(range(500))        # a bijection
    assert np.all(np.diff(s[perm]) <= 0)                     # scores non-increasing
    s = rng.normal(size=1000).astype(np.float32)
    np.testing.assert_array_equal(orc.argsort_desc(s), np.argsort(-s, kind="stable"))


def test_argsort_zero_signs_tie(orc):
    s = np.array([0.0, -0.0, 0.0, 1.0, -0.0], np.float32)
    np.testing.assert_array_equal(orc.argsort_desc(s), [3, 0, 1, 2, 4])


def test_gather_is_fancy_indexing(orc):
    rng = np.random.default_rng(4)
    W = rng.integers(0, 65535, size=(16, 24)).astype(np.uint16)
    S = rng.random((16, 24)).astype(np.float32)
    rp = rng.permutation(16).astype(np.int32)
    cp = rng.permutation(24).astype(np.int32)
    Wo, So = orc.gather(W, S, rp, cp)
    np.testing.assert_array_equal(Wo, W[rp][:, cp])
    np.testing.assert_array_equal(So, S[rp][:, cp])


def test_reordered_layer_output_is_a_permutation_of_the_original(orc):
    # W' (P_c x) = P_r (W x), exact with small integers (bf16 holds them exactly)
    rng = np.random.default_rng(5)
    R, C = 32, 48
    Wf = rng.integers(-8, 9, size=(R, C)).astype(np.float32)
    S = np.exp(rng.normal(size=(R, 1)) + rng.normal(size=(1, C))).astype(np.float32)
    W = orc.f32_to_bf16(Wf)
    np.testing.assert_array_equal(orc.bf16_to_f32(W), Wf)
    rs, cs = orc.channel_scores(S)
    rp, cp = orc.argsort_desc(rs), orc.argsort_desc(cs)
    Wp, Sp = orc.gather(W, S, rp, cp)
    x = rng.integers(-5, 6, size=C).astype(np.float32)
    y = Wf @ x
    yp = orc.bf16_to_f32(Wp) @ x[cp]
    np.testing.assert_array_equal(yp, y[rp])
    # sensitive channels first: scores of the reordered matrix are non-increasing
    assert np.all(np.diff(rs[rp]) <= 0)
    assert np.all(np.diff(cs[cp]) <= 0)
    # the same channels, summed in the new element order: equal up to rounding
    rs2, cs2 = orc.channel_scores(Sp)
    np.testing.assert_allclose(rs2, rs[rp], rtol=1e-5)
    np.testing.assert_allclose(cs2, cs[cp], rtol=1e-5)


def test_bf16_helpers_round_to_nearest_even(orc):
    # 1 + 2^-8 is halfway between bf16 neighbours 1 and 1 + 2^-7: ties to even -> 1
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0], np.float32)
    h = orc.f32_to_bf16(x)
    np.testing.assert_array_equal(orc.bf16_to_f32(h), np.array([1.0, 1.0 + 2.0 ** -6, -2.5, 0.0], np.float32))


# ------------------------------------------------- coupled reordering (App. "Channel Reordering")
def test_coupled_scores_hand_example(orc):
    """Two coupled dimensions with scores [1,5,3] and [4,0,3]: the sums are [5,5,6], so channel 2
    comes first and the tie between channels 0 and 1 goes to the lower index."""
    a, b = np.array([1, 5, 3], np.float32), np.array([4, 0, 3], np.float32)
    np.testing.assert_array_equal(orc.group_scores([a, b]), np.array([5, 5, 6], np.float32))
    np.testing.assert_array_equal(orc.coupled_perm([a, b]), [2, 0, 1])


def test_coupled_scores_are_summed_member_after_member(orc):
    """fp32 addition is not associative: (1e8 + 1) + (-1e8) = 0 but 1e8 + (-1e8) + 1 = 1."""
    m = [np.array([1e8], np.float32), np.array([1.0], np.float32), np.array([-1e8], np.float32)]
    assert orc.group_scores(m)[0] == 0.0
    assert orc.group_scores([m[0], m[2], m[1]])[0] == 1.0


def test_coupled_perm_of_one_member_is_the_plain_argsort(orc):
    rng = np.random.default_rng(3)
    s = rng.random(777).astype(np.float32)
    np.testing.assert_array_equal(orc.coupled_perm([s]), orc.argsort_desc(s))


def test_pieces_keep_their_channels(orc):
    rng = np.random.default_rng(4)
    s = rng.integers(0, 5, 96).astype(np.float32)                # many ties
    perm = orc.argsort_desc_pieces(s, 32)
    for p0 in range(0, 96, 32):
        piece = perm[p0:p0 + 32]
        assert sorted(piece) == list(range(p0, p0 + 32))          # a permutation of its own piece
        np.testing.assert_array_equal(piece - p0, np.argsort(-s[p0:p0 + 32], kind="stable"))
    np.testing.assert_array_equal(orc.argsort_desc_pieces(s, 0), orc.argsort_desc(s))


def test_coupled_reordering_preserves_a_gated_mlp(orc):
    """y = Wd (relu(Wg x) * (Wu x)): the rows of Wg, Wu and the columns of Wd carry the same
    activation; the input side of Wg, Wu and the output side of Wd carry the residual stream.
    Reordered with shared permutations, the block computes the same function up to the residual
    permutation: y'[i] = y[q[i]] for x'[j] = x[q[j]].  Small integers: exact in float64."""
    rng = np.random.default_rng(5)
    H, F = 24, 40
    Wg, Wu = rng.integers(-3, 4, (F, H)), rng.integers(-3, 4, (F, H))
    Wd = rng.integers(-3, 4, (H, F))
    Sg, Su, Sd = (rng.random((F, H)).astype(np.float32), rng.random((F, H)).astype(np.float32),
                  rng.random((H, F)).astype(np.float32))
    rs_g, cs_g = orc.channel_scores(Sg)
    rs_u, cs_u = orc.channel_scores(Su)
    rs_d, cs_d = orc.channel_scores(Sd)
    p = orc.coupled_perm([rs_g, rs_u, cs_d])                      # the MLP's inner activation
    q = orc.coupled_perm([rs_d, cs_g, cs_u])                      # the residual stream
    bits = lambda M: M.astype(np.uint16)                          # gather moves 16-bit patterns
    g2 = orc.gather(bits(Wg + 8), Sg, p, q)[0].astype(np.int64) - 8
    u2 = orc.gather(bits(Wu + 8), Su, p, q)[0].astype(np.int64) - 8
    d2 = orc.gather(bits(Wd + 8), Sd, q, p)[0].astype(np.int64) - 8
    x = rng.integers(-5, 6, H)
    y = Wd @ (np.maximum(Wg @ x, 0) * (Wu @ x))
    y2 = d2 @ (np.maximum(g2 @ x[q], 0) * (u2 @ x[q]))
    np.testing.assert_array_equal(y2, y[q])


def test_fold_and_expand_hand_example(orc):
    """Group of 2 pieces x 2 channels, member with repeat 2 (8 channels): group piece 0 stands for
    member pieces 0, 1 and group piece 1 for member pieces 2, 3."""
    s = np.arange(8, dtype=np.float32)
    lo, hi = orc.fold_repeated(s, 2, 2)
    np.testing.assert_array_equal(lo, [0, 1, 4, 5])
    np.testing.assert_array_equal(hi, [2, 3, 6, 7])
    np.testing.assert_array_equal(orc.expand_perm([1, 0, 2, 3], 2, 2), [1, 0, 3, 2, 4, 5, 6, 7])


def test_coupled_reordering_preserves_grouped_query_attention(orc):
    """One token, one key position (attention weights 1): y = Wo concat_h (a_h * (Wv x)[kv(h)]) with
    kv(h) = h // rep: query head h reads the value head it shares with rep - 1 others.  The rows of
    Wv and the columns of Wo are reordered head by head from their summed scores (the r column
    pieces of Wo folded onto the value head they read); the function is unchanged.  Exact integers."""
    rng = np.random.default_rng(6)
    HD, KV, REP, H = 8, 3, 4, 16
    Wv = rng.integers(-3, 4, (KV * HD, H))
    Wo = rng.integers(-3, 4, (H, KV * REP * HD))
    Sv = rng.random(Wv.shape).astype(np.float32)
    So = rng.random(Wo.shape).astype(np.float32)
    a = rng.integers(1, 4, KV * REP)                              # per query head factor
    rs_v, _ = orc.channel_scores(Sv)
    _, cs_o = orc.channel_scores(So)
    members = [rs_v] + orc.fold_repeated(cs_o, HD, REP)
    assert len(members) == 1 + REP
    pv = orc.coupled_perm(members, HD)
    po = orc.expand_perm(pv, HD, REP)
    assert sorted(po) == list(range(KV * REP * HD))
    for h in range(KV * REP):                                     # every query head: its value head's order
        np.testing.assert_array_equal(po[h * HD:(h + 1) * HD] - h * HD,
                                      pv[(h // REP) * HD:(h // REP + 1) * HD] - (h // REP) * HD)
    ident_v, ident_h = np.arange(KV * HD, dtype=np.int32), np.arange(H, dtype=np.int32)
    bits = lambda M: M.astype(np.uint16)
    v2 = orc.gather(bits(Wv + 8), Sv, pv, ident_h)[0].astype(np.int64) - 8
    o2 = orc.gather(bits(Wo + 8), So, ident_h, po)[0].astype(np.int64) - 8

    def attn(wv, wo, x):
        v = (wv @ x).reshape(KV, HD)
        per_head = np.concatenate([a[h] * v[h // REP] for h in range(KV * REP)])
        return wo @ per_head

    x = rng.integers(-5, 6, H)
    np.testing.assert_array_equal(attn(v2, o2, x), attn(Wv, Wo, x))
    # the group's score of a value channel = its own + the REP columns that read it, in that order
    j = 5
    want = rs_v[j]
    for t in range(REP):
        want = np.float32(want + cs_o[(j // HD) * REP * HD + t * HD + j % HD])
    assert orc.group_scores(members)[j] == want
