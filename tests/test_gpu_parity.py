"""GPU parity: every stage of the HIP path against the CPU oracle, element by element,
on the same seeded inputs, through the C-ABI (binding -> libscalebits.so).

Bar: permutations, levels, statistics, offsets, packed bytes, scales and zeros bit-exact;
cost entries bit-exact as well (the summation order is part of the definition), which is
inside the 1e-5 relative bound the search is specified to.
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2602_17698_amd import binding as sb
from paper_2602_17698_amd import synth

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    sb.load()                                            # fails loudly if the library is not built
    return torch.device("cuda:0")


@pytest.fixture(scope="module")
def ctx(dev):
    c = sb.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    yield c
    c.close()


def make_plan(ctx, shapes, m, n, bits, dev):
    plan = sb.Plan(ctx, shapes, m, n, bits)
    ws = torch.empty(plan.workspace_bytes(), dtype=torch.uint8, device=dev)
    assert ws.data_ptr() % 256 == 0
    return plan, ws


def to_np_bf16(w):
    return synth.bf16_bits(w)


def shape_with_blocks(N):
    """A matrix shape with exactly N blocks of 8 x 8 inside the library's per-matrix limits."""
    b = 1
    while N % b or N // b > 4096:
        b += 1
    return (8 * (N // b), 8 * b)


# ------------------------------------------------------------------ scores + permutations

@pytest.mark.parametrize("R,C,m,n", [(8, 8, 8, 8), (40, 520, 8, 8), (264, 1032, 8, 8), (1024, 1024, 128, 128),
                                      (96, 4096, 32, 128), (2048, 64, 64, 64)])
def test_scores_and_permutations(orc, ctx, dev, R, C, m, n):
    say("scores/perm", R, C)
    g = torch.Generator().manual_seed(R * 7 + C)
    S = torch.exp(torch.randn(R, 1, generator=g) + torch.randn(1, C, generator=g) + 0.5 * torch.randn(R, C, generator=g))
    plan, ws = make_plan(ctx, [(R, C)], m, n, [2, 3, 4], dev)
    Sd = S.to(dev)
    M = sb.matrix(None, Sd)
    rs = torch.empty(R, dtype=torch.float32, device=dev)
    cs = torch.empty(C, dtype=torch.float32, device=dev)
    plan.channel_scores(0, M, rs, cs, ws)
    rp = torch.empty(R, dtype=torch.int32, device=dev)
    cp = torch.empty(C, dtype=torch.int32, device=dev)
    plan.reorder(0, M, rp, cp, ws)
    torch.cuda.synchronize()
    rs_o, cs_o = orc.channel_scores(S.numpy())
    np.testing.assert_array_equal(rs.cpu().numpy(), rs_o)
    np.testing.assert_array_equal(cs.cpu().numpy(), cs_o)
    np.testing.assert_array_equal(rp.cpu().numpy(), orc.argsort_desc(rs_o))
    np.testing.assert_array_equal(cp.cpu().numpy(), orc.argsort_desc(cs_o))
    plan.close()


def test_scores_take_absolute_values_of_signed_sensitivities(orc, ctx, dev):
    """The channel score is an l1 norm (Sec. 4.1): a sensitivity input that carries signed values (a raw
    first-order term, a gradient) must enter by magnitude -- through the single-matrix call, the
    batched call and the coupled call.  With the signs dropped on the device the scores of these
    matrices would cancel and order the channels differently."""
    say("scores of signed sensitivities")
    shapes = [(264, 1032), (1024, 520), (264, 1032)]
    g = torch.Generator().manual_seed(77)
    Ss = []
    for R, C in shapes:
        mag = torch.exp(torch.randn(R, 1, generator=g) + torch.randn(1, C, generator=g) + 0.5 * torch.randn(R, C, generator=g))
        sign = torch.where(torch.rand(R, C, generator=g) < 0.5, -1.0, 1.0)
        Ss.append(mag * sign)
    assert all((S < 0).float().mean().item() > 0.4 for S in Ss)
    plan, ws = make_plan(ctx, shapes, 8, 8, [2, 3, 4], dev)
    dS = [S.to(dev) for S in Ss]
    mats = [sb.matrix(None, s_) for s_ in dS]
    want = [orc.channel_scores(S.numpy()) for S in Ss]
    for (rs_o, cs_o), S in zip(want, Ss):                           # the oracle's scores are those of |S| ...
        rs_a, cs_a = orc.channel_scores(S.abs().numpy())
        np.testing.assert_array_equal(rs_o, rs_a)
        np.testing.assert_array_equal(cs_o, cs_a)
        rs_sgn = S.double().sum(1).abs().numpy()                    # ... and far from those of a signed sum
        assert np.median(rs_sgn / rs_o) < 0.2
    for i, (R, C) in enumerate(shapes):
        rs = torch.empty(R, dtype=torch.float32, device=dev)
        cs = torch.empty(C, dtype=torch.float32, device=dev)
        plan.channel_scores(i, mats[i], rs, cs, ws)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(rs.cpu().numpy(), want[i][0])
        np.testing.assert_array_equal(cs.cpu().numpy(), want[i][1])
    nr, nc = sum(r for r, _ in shapes), sum(c for _, c in shapes)
    rp = torch.full((nr,), -7, dtype=torch.int32, device=dev)
    cp = torch.full((nc,), -7, dtype=torch.int32, device=dev)
    plan.reorder_all(mats, rp, cp, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(rp.cpu().numpy(), np.concatenate([orc.argsort_desc(w[0]) for w in want]))
    np.testing.assert_array_equal(cp.cpu().numpy(), np.concatenate([orc.argsort_desc(w[1]) for w in want]))
    # coupled: matrices 0 and 2 share both permutations (rows group 0, columns group 1), matrix 1 is on its own
    I = sb.DIM_INDEPENDENT
    rp.fill_(-7); cp.fill_(-7)
    plan.reorder_coupled_all(mats, [0, I, 0], [1, I, 1], 2, [0, 0], rp, cp, ws)
    torch.cuda.synchronize()
    rp, cp = rp.cpu().numpy(), cp.cpu().numpy()
    pr = orc.coupled_perm([want[0][0], want[2][0]], 0)
    pc = orc.coupled_perm([want[0][1], want[2][1]], 0)
    np.testing.assert_array_equal(rp[:264], pr)
    np.testing.assert_array_equal(rp[264 + 1024:], pr)
    np.testing.assert_array_equal(cp[:1032], pc)
    np.testing.assert_array_equal(cp[1032 + 520:], pc)
    np.testing.assert_array_equal(rp[264:264 + 1024], orc.argsort_desc(want[1][0]))
    np.testing.assert_array_equal(cp[1032:1032 + 520], orc.argsort_desc(want[1][1]))
    plan.close()


def test_permutation_ties_go_to_the_lower_index(orc, ctx, dev):
    say("perm ties")
    R, C = 64, 128
    S = torch.ones(R, C)
    S[10] = 2.0
    S[:, 5] = 3.0
    S[40] = 0.0                                           # a dead channel: score 0 (+0 / -0 immaterial)
    plan, ws = make_plan(ctx, [(R, C)], 8, 8, [2, 3], dev)
    Sd = S.to(dev)
    rp = torch.empty(R, dtype=torch.int32, device=dev)
    cp = torch.empty(C, dtype=torch.int32, device=dev)
    plan.reorder(0, sb.matrix(None, Sd), rp, cp, ws)
    torch.cuda.synchronize()
    rs_o, cs_o = orc.channel_scores(S.numpy())
    np.testing.assert_array_equal(rp.cpu().numpy(), orc.argsort_desc(rs_o))
    np.testing.assert_array_equal(cp.cpu().numpy(), orc.argsort_desc(cs_o))
    assert rp[0].item() == 10 and rp[-1].item() == 40 and cp[0].item() == 5
    plan.close()


# ------------------------------------------------------------------------------- gather

@pytest.mark.parametrize("R,C", [(8, 8), (40, 520), (256, 4096), (64, 14336)])
def test_gather(orc, ctx, dev, R, C):
    say("gather", R, C)
    W, S = synth.make_matrix("student_t", R, C, seed=1, tid=R + C)
    g = torch.Generator().manual_seed(3)
    rp = torch.randperm(R, generator=g).to(torch.int32)
    cp = torch.randperm(C, generator=g).to(torch.int32)
    plan, ws = make_plan(ctx, [(R, C)], 8, 8, [2, 3, 4], dev)
    Wd, Sd = W.to(dev), S.to(dev)
    Wo = torch.empty_like(Wd)
    So = torch.empty_like(Sd)
    plan.gather(0, sb.matrix(Wd, Sd), rp.to(dev), cp.to(dev), Wo, So)
    torch.cuda.synchronize()
    Wr, Sr = orc.gather(to_np_bf16(W), S.numpy(), rp.numpy(), cp.numpy())
    np.testing.assert_array_equal(to_np_bf16(Wo), Wr)
    np.testing.assert_array_equal(So.cpu().numpy(), Sr)
    plan.close()


def test_gather_with_row_pitch(orc, ctx, dev):
    say("gather pitch")
    R, C, ld = 32, 256, 384
    W, S = synth.make_matrix("student_t", R, ld, seed=2)
    Wd, Sd = W.to(dev), S.to(dev)
    g = torch.Generator().manual_seed(4)
    rp = torch.randperm(R, generator=g).to(torch.int32)
    cp = torch.randperm(C, generator=g).to(torch.int32)
    plan, ws = make_plan(ctx, [(R, C)], 8, 8, [2], dev)
    M = sb.Matrix(Wd.data_ptr(), Sd.data_ptr(), R, C, ld, ld)
    Wo = torch.empty(R, C, dtype=torch.bfloat16, device=dev)
    So = torch.empty(R, C, dtype=torch.float32, device=dev)
    plan.gather(0, M, rp.to(dev), cp.to(dev), Wo, So)
    rs = torch.empty(R, dtype=torch.float32, device=dev)
    cs = torch.empty(C, dtype=torch.float32, device=dev)
    plan.channel_scores(0, M, rs, cs, ws)
    torch.cuda.synchronize()
    Wr, Sr = orc.gather(to_np_bf16(W)[:, :C].copy(), S.numpy()[:, :C].copy(), rp.numpy(), cp.numpy())
    np.testing.assert_array_equal(to_np_bf16(Wo), Wr)
    np.testing.assert_array_equal(So.cpu().numpy(), Sr)
    rs_o, cs_o = orc.channel_scores(S.numpy()[:, :C].copy())
    np.testing.assert_array_equal(rs.cpu().numpy(), rs_o)
    np.testing.assert_array_equal(cs.cpu().numpy(), cs_o)
    plan.close()


# --------------------------------------------------------------------------- cost table

COST_CASES = [
    # R, C, m, n, bits
    (256, 384, 128, 128, [2, 3, 4]),
    (256, 384, 128, 128, [1, 2, 3, 4]),
    (192, 320, 64, 64, [1, 2, 3, 4, 8]),
    (24, 40, 8, 8, [1, 2, 3, 4, 5, 6, 7, 8]),
    (64, 96, 16, 32, [2, 4]),
    (32, 48, 8, 16, [3]),
    (2048, 256, 1024, 256, [2, 3, 4]),
    (128, 1024, 64, 512, [1, 2, 3, 4, 8]),
    (520, 128, 8, 128, [2, 3, 4]),                        # 65 row blocks: ragged last workgroup
    (256, 384, 128, 128, [0, 2, 3, 4]),                   # 0 bits = the block is pruned
    (192, 320, 64, 64, [0, 1, 2, 3, 4, 5, 6, 7, 8]),      # nine candidates on 64-column blocks: two launches
    (24, 40, 8, 8, [0, 1, 2, 3, 4, 5, 6, 7, 8]),
    (128, 1024, 64, 512, [0, 4]),
]


@pytest.mark.parametrize("R,C,m,n,bits", COST_CASES)
def test_cost_table(orc, ctx, dev, R, C, m, n, bits):
    say("cost", R, C, m, n, bits)
    W, S = synth.make_matrix("student_t", R, C, seed=5, tid=m * n + len(bits))
    plan, ws = make_plan(ctx, [(m, n), (R, C)], m, n, bits, dev)
    N, K = plan.num_blocks(), len(bits)
    cost = torch.full((N, K), -1.0, dtype=torch.float32, device=dev)
    Wd, Sd = W.to(dev), S.to(dev)
    plan.cost_table(1, Wd, Sd, cost)                      # second matrix: rows start at its block base
    torch.cuda.synchronize()
    got = cost.cpu().numpy()
    ref = orc.cost_table(to_np_bf16(W), S.numpy(), m, n, bits)
    base = plan.block_base(1)
    assert base == 1 and np.all(got[:base] == -1.0)       # other matrices' rows untouched
    np.testing.assert_array_equal(got[base:], ref)
    np.testing.assert_allclose(got[base:], ref, rtol=1e-5)
    plan.close()


def test_cost_table_degenerate_groups(orc, ctx, dev):
    say("cost degenerate")
    m = n = 64
    R, C = 128, 128
    W, S = synth.make_matrix("gauss_outlier", R, C, seed=6)
    Wn = to_np_bf16(W).copy()
    Wn[0, :64] = Wn[0, 0]                                 # constant group: range 0
    Wn[1, :64] = 0
    Wn[1, 7] = 0x0001                                     # range = smallest subnormal: qmax / R overflows
    Wn[2, :64] = 0x8000                                   # all -0
    Wn[2, 3] = 0x0000                                     # +0 among -0: range 0
    Wn[3, :64] = 0
    Wn[3, 9] = 0x0040                                     # subnormal range whose reciprocal is finite for small qmax
    Wn[4, 64:] = 0x7F7F                                   # largest finite bf16, constant
    Wd = torch.from_numpy(Wn.view(np.int16)).view(torch.bfloat16).to(dev)
    bits = [1, 2, 3, 4, 8]
    plan, ws = make_plan(ctx, [(R, C)], m, n, bits, dev)
    cost = torch.empty(plan.num_blocks(), len(bits), dtype=torch.float32, device=dev)
    plan.cost_table(0, Wd, S.to(dev), cost)
    torch.cuda.synchronize()
    ref = orc.cost_table(Wn, S.numpy(), m, n, bits)
    np.testing.assert_array_equal(cost.cpu().numpy(), ref)
    plan.close()


# ------------------------------------------------------------------------ coupled reordering
def test_coupled_reordering(orc, ctx, dev):
    """A toy decoder layer: the residual stream (hidden = 256) couples the columns of q, v, up, gate
    and the rows of o, down; the MLP activation (512) couples the rows of up, gate and the columns of
    down; the value/output activation couples the rows of v and the columns of o inside heads of 64;
    the rows of q stay fixed.  One independent matrix rides along."""
    say("coupled reordering")
    H, F, HD = 256, 512, 64
    names = ["q", "v", "o", "up", "gate", "down", "free"]
    shapes = [(H, H), (H, H), (H, H), (F, H), (F, H), (H, F), (128, 384)]
    RES, MLP, ATT = 0, 1, 2
    I, FX = sb.DIM_INDEPENDENT, sb.DIM_FIXED
    row_group = [FX, ATT, RES, MLP, MLP, RES, I]
    col_group = [RES, RES, ATT, RES, RES, MLP, I]
    segment = [0, 0, HD]
    mats = [synth.make_matrix("student_t", r, c, seed=21, tid=i) for i, (r, c) in enumerate(shapes)]
    plan, ws = make_plan(ctx, shapes, 64, 64, [2, 3, 4], dev)
    dS = [S.to(dev) for _, S in mats]
    rp = torch.full((sum(r for r, _ in shapes),), -7, dtype=torch.int32, device=dev)
    cp = torch.full((sum(c for _, c in shapes),), -7, dtype=torch.int32, device=dev)
    plan.reorder_coupled_all([sb.matrix(None, s_) for s_ in dS], row_group, col_group, 3, segment, rp, cp, ws)
    torch.cuda.synchronize()
    rp, cp = rp.cpu().numpy(), cp.cpu().numpy()

    scores = [orc.channel_scores(S.numpy()) for _, S in mats]       # (row scores, column scores) per matrix
    members = {g: [] for g in (RES, MLP, ATT)}
    for i, g in enumerate(row_group):                               # member order: all rows, then all columns
        if g >= 0:
            members[g].append(scores[i][0])
    for i, g in enumerate(col_group):
        if g >= 0:
            members[g].append(scores[i][1])
    gperm = {g: orc.coupled_perm(members[g], segment[g]) for g in members}
    ro = co = 0
    for i, (r, c) in enumerate(shapes):
        got_r, got_c = rp[ro:ro + r], cp[co:co + c]
        for got, g, own, n in ((got_r, row_group[i], scores[i][0], r), (got_c, col_group[i], scores[i][1], c)):
            if g == FX:
                want = np.arange(n, dtype=np.int32)
            elif g == I:
                want = orc.argsort_desc(own)
            else:
                want = gperm[g]
            np.testing.assert_array_equal(got, want, err_msg="%s group %d" % (names[i], g))
        ro, co = ro + r, co + c
    # the attention permutation stays inside its heads
    att = gperm[ATT]
    assert all(att[h * HD:(h + 1) * HD].min() == h * HD and att[h * HD:(h + 1) * HD].max() == (h + 1) * HD - 1
               for h in range(H // HD))
    plan.close()


def test_coupled_reordering_grouped_query_heads(orc, ctx, dev):
    """Value rows (3 heads of 64) coupled with output columns (12 heads of 64, 4 per value head)."""
    say("coupled reordering: grouped-query heads")
    HD, KV, REP, H = 64, 3, 4, 256
    shapes = [(KV * HD, H), (H, KV * REP * HD)]                     # v, o
    mats = [synth.make_matrix("student_t", r, c, seed=22, tid=i) for i, (r, c) in enumerate(shapes)]
    plan, ws = make_plan(ctx, shapes, 64, 64, [2, 3, 4], dev)
    dS = [S.to(dev) for _, S in mats]
    rp = torch.full((sum(r for r, _ in shapes),), -7, dtype=torch.int32, device=dev)
    cp = torch.full((sum(c for _, c in shapes),), -7, dtype=torch.int32, device=dev)
    I = sb.DIM_INDEPENDENT
    plan.reorder_coupled_all([sb.matrix(None, s_) for s_ in dS], [0, I], [I, 0], 1, [HD], rp, cp, ws,
                             row_repeat=[1, 1], col_repeat=[1, REP])
    torch.cuda.synchronize()
    rp, cp = rp.cpu().numpy(), cp.cpu().numpy()
    (rs_v, cs_v), (rs_o, cs_o) = [orc.channel_scores(S.numpy()) for _, S in mats]
    pv = orc.coupled_perm([rs_v] + orc.fold_repeated(cs_o, HD, REP), HD)
    np.testing.assert_array_equal(rp[:KV * HD], pv)
    np.testing.assert_array_equal(cp[H:], orc.expand_perm(pv, HD, REP))
    np.testing.assert_array_equal(rp[KV * HD:], orc.argsort_desc(rs_o))
    np.testing.assert_array_equal(cp[:H], orc.argsort_desc(cs_v))
    # a repeated member cannot lead its group, and repeats need pieces
    for args, kw, status in ((([0, I], [I, 0]), dict(row_repeat=[REP, 1], col_repeat=[1, 1]), sb.ERR_INVALID_ARG),
                             (([0, I], [I, 0]), dict(row_repeat=[1, 1], col_repeat=[1, 2]), sb.ERR_BAD_SHAPE)):
        with pytest.raises(sb.SbitsError) as e:
            plan.reorder_coupled_all([sb.matrix(None, s_) for s_ in dS], args[0], args[1], 1, [HD],
                                     torch.empty_like(torch.from_numpy(rp)).to(dev),
                                     torch.empty_like(torch.from_numpy(cp)).to(dev), ws, **kw)
        assert e.value.status == status
    plan.close()


def test_coupled_reordering_rejects_unequal_members(ctx, dev):
    say("coupled reordering: unequal members")
    shapes = [(128, 256), (256, 128)]
    plan, ws = make_plan(ctx, shapes, 64, 64, [2, 4], dev)
    dS = [torch.ones(r, c, dtype=torch.float32, device=dev) for r, c in shapes]
    rp = torch.empty(384, dtype=torch.int32, device=dev)
    cp = torch.empty(384, dtype=torch.int32, device=dev)
    with pytest.raises(sb.SbitsError) as e:                         # rows of both: 128 vs 256
        plan.reorder_coupled_all([sb.matrix(None, s_) for s_ in dS], [0, 0], [-1, -1], 1, None, rp, cp, ws)
    assert e.value.status == sb.ERR_BAD_SHAPE
    plan.reorder_coupled_all([sb.matrix(None, s_) for s_ in dS], [0, -1], [-1, 0], 1, [32], rp, cp, ws)   # 128 and 128
    torch.cuda.synchronize()
    np.testing.assert_array_equal(rp[:128].cpu().numpy(), cp[256:].cpu().numpy())
    np.testing.assert_array_equal(rp[:128].cpu().numpy(), np.arange(128))   # all scores equal: ties to the lower index
    plan.close()


# ------------------------------------------------- reordering and cost table in one pass
ONE_PASS_CASES = [
    # shapes, m, n, bits
    ([(256, 384), (128, 1024)], 128, 128, [1, 2, 3, 4]),          # one chunk per lane, two rows per step
    ([(192, 320), (64, 4096)], 64, 64, [1, 2, 3, 4, 8]),          # ragged run of octets (192 rows), K = 5
    ([(128, 4224), (256, 8192)], 128, 128, [2, 3, 4]),            # two chunks per lane, ragged and full
    ([(64, 14336), (64, 16384), (64, 8320)], 64, 128, [1, 2, 3, 4]),   # four chunks per lane
    ([(24, 192), (2048, 128)], 8, 64, [1, 2, 3, 4, 5, 6, 7, 8]),  # one octet per block; 16 runs
    ([(2048, 256)], 1024, 128, [3]),                              # 128 octets per block
    ([(64, 14336)], 64, 64, [1, 2, 3, 4, 8]),                     # four chunks per lane, K = 5
    ([(64, 14336), (128, 256)], 64, 128, [1, 2, 3, 4, 5, 6, 7, 8]),  # four chunks per lane, K = 8: two launches of 4 candidates
    ([(64, 8320)], 64, 64, [1, 2, 3, 4, 5, 6, 8]),                # K = 7: 4 + 3 candidates
    ([(256, 384), (128, 1024)], 128, 128, [0, 1, 2, 3, 4]),       # with the pruned candidate (0 bits)
    ([(64, 14336), (128, 256)], 64, 128, [0, 1, 2, 3, 4, 5, 6, 7, 8]),   # nine candidates; four chunks per lane: 5 + 4
    ([(64, 8320), (192, 320)], 64, 64, [0, 2, 4]),
]

# rows wider than the cost kernel stages (16384): those matrices go through a reordered copy in the
# workspace, the others of the same plan through the one-pass kernel; the packing kernel stages every row
WIDE_ROW_CASES = [
    ([(64, 28672), (128, 4096), (64, 14336)], 64, 128, [2, 3, 4]),
    ([(128, 20480), (64, 1024)], 64, 64, [1, 2, 3, 4, 8]),
    ([(64, 32768)], 64, 128, [0, 1, 2, 3, 4]),
]


def _random_one_pass_cases(count, seed):
    """Seeded shapes around the kernels' boundaries: block-column counts next to the chunk limits of the
    instances (512, 1024, 2048 chunks of 8 columns), row counts that leave ragged runs of octets, every
    number of candidates, with and without the 0-bit one."""
    rng = np.random.default_rng(seed)
    edge_cols = {64: [1, 3, 8, 9, 63, 64, 65, 66, 127, 128, 129, 130, 200, 255, 256],
                 128: [1, 2, 5, 31, 32, 33, 34, 63, 64, 65, 66, 100, 127, 128]}
    cases = []
    for i in range(count):
        n = int(rng.choice([64, 128]))
        m = int(rng.choice([8, 16, 64, 128, 256]))
        K = int(rng.integers(1, 9))
        bits = sorted(int(b) for b in rng.choice(np.arange(1, 9), size=K, replace=False))
        if i % 5 == 4:
            bits = [0] + bits
        shapes = []
        for _ in range(int(rng.integers(1, 4))):
            nbc = int(rng.choice(edge_cols[n]))
            nbr = int(rng.integers(1, max(2, 320 // m)))
            shapes.append((m * nbr, n * nbc))
        cases.append((shapes, m, n, bits))
    return cases


RANDOM_ONE_PASS_CASES = _random_one_pass_cases(24, 20260217)


@pytest.mark.parametrize("shapes,m,n,bits", ONE_PASS_CASES + WIDE_ROW_CASES + RANDOM_ONE_PASS_CASES)
def test_gather_cost_one_pass(orc, ctx, dev, shapes, m, n, bits):
    say("one-pass gather+cost", shapes, m, n, bits)
    plan, ws = make_plan(ctx, shapes, m, n, bits, dev)
    assert plan.gather_cost_supported()
    N, K = plan.num_blocks(), len(bits)
    mats = [synth.make_matrix("student_t", r, c, seed=11, tid=i) for i, (r, c) in enumerate(shapes)]
    g = torch.Generator().manual_seed(17)
    rps = [torch.randperm(r, generator=g).to(torch.int32) for r, _ in shapes]
    cps = [torch.randperm(c, generator=g).to(torch.int32) for _, c in shapes]
    dW = [W.to(dev) for W, _ in mats]
    dS = [S.to(dev) for _, S in mats]
    nel = sum(r * c for r, c in shapes)
    w_re = torch.zeros(nel, dtype=torch.bfloat16, device=dev)
    cost = torch.full((N, K), -1.0, dtype=torch.float32, device=dev)
    plan.gather_cost_all([sb.matrix(w, s_) for w, s_ in zip(dW, dS)], torch.cat(rps).to(dev), torch.cat(cps).to(dev),
                         w_re, cost, ws)
    torch.cuda.synchronize()
    eo = 0
    refs = []
    for (R, C), (W, S), rp, cp in zip(shapes, mats, rps, cps):
        Wp, Sp = orc.gather(to_np_bf16(W), S.numpy(), rp.numpy(), cp.numpy())
        np.testing.assert_array_equal(to_np_bf16(w_re[eo:eo + R * C]).reshape(R, C), Wp)
        refs.append(orc.cost_table(Wp, Sp, m, n, bits))
        eo += R * C
    np.testing.assert_array_equal(cost.cpu().numpy(), np.concatenate(refs, 0))
    plan.close()


@pytest.mark.parametrize("shapes,m,n,bits", ONE_PASS_CASES + WIDE_ROW_CASES + RANDOM_ONE_PASS_CASES)
def test_gather_pack_one_pass(orc, ctx, dev, shapes, m, n, bits):
    """Packing straight from the original weights and the permutations == oracle gather + pack."""
    say("one-pass gather+pack", shapes, m, n, bits)
    plan, ws = make_plan(ctx, shapes, m, n, bits, dev)
    N = plan.num_blocks()
    mats = [synth.make_matrix("student_t", r, c, seed=12, tid=i) for i, (r, c) in enumerate(shapes)]
    g = torch.Generator().manual_seed(19)
    rps = [torch.randperm(r, generator=g).to(torch.int32) for r, _ in shapes]
    cps = [torch.randperm(c, generator=g).to(torch.int32) for _, c in shapes]
    rng = np.random.default_rng(N)
    level = rng.integers(0, len(bits), size=N).astype(np.uint8)
    off = orc.offsets(level, m, n, bits)
    total = int(off[-1])
    dW = [W.to(dev) for W, _ in mats]
    codes_d = torch.full((total,), 0x55, dtype=torch.uint8, device=dev)
    scale_d = torch.full((N * m,), -1.0, dtype=torch.float32, device=dev)
    zero_d = torch.full((N * m,), -1.0, dtype=torch.float32, device=dev)
    plan.gather_pack_all([sb.matrix(w, None) for w in dW], torch.cat(rps).to(dev), torch.cat(cps).to(dev),
                         torch.from_numpy(level).to(dev), torch.from_numpy(off).to(dev), codes_d, scale_d, zero_d, ws)
    torch.cuda.synchronize()
    codes = np.full(total, 0x55, np.uint8)
    scale = np.full(N * m, -1.0, np.float32)
    zero = np.full(N * m, -1.0, np.float32)
    base = 0
    for (R, C), (W, S), rp, cp in zip(shapes, mats, rps, cps):
        Wp, _ = orc.gather(to_np_bf16(W), S.numpy(), rp.numpy(), cp.numpy())
        orc.pack(Wp, m, n, bits, level, off, base, codes, scale, zero)
        base += (R // m) * (C // n)
    np.testing.assert_array_equal(codes_d.cpu().numpy(), codes)
    np.testing.assert_array_equal(scale_d.cpu().numpy(), scale)
    np.testing.assert_array_equal(zero_d.cpu().numpy().view(np.uint32), zero.view(np.uint32))
    plan.close()


@pytest.mark.parametrize("shapes,m,n,bits", ONE_PASS_CASES)
def test_surrogates_one_pass(orc, ctx, dev, shapes, m, n, bits):
    """Dynamic-sensitivity surrogates from the original weights, a signed gradient, the
    permutations and the current levels == oracle gather + surrogates, bit for bit."""
    say("surrogates", shapes, m, n, bits)
    plan, ws = make_plan(ctx, shapes, m, n, bits, dev)
    N = plan.num_blocks()
    mats = [synth.make_matrix("student_t", r, c, seed=13, tid=i) for i, (r, c) in enumerate(shapes)]
    g = torch.Generator().manual_seed(23)
    grads = [torch.randn(r, c, generator=g) * torch.exp(torch.randn(r, 1, generator=g)) for r, c in shapes]
    rps = [torch.randperm(r, generator=g).to(torch.int32) for r, _ in shapes]
    cps = [torch.randperm(c, generator=g).to(torch.int32) for _, c in shapes]
    level = np.random.default_rng(N).integers(0, len(bits), size=N).astype(np.uint8)
    dW = [W.to(dev) for W, _ in mats]
    dG = [G.to(dev) for G in grads]
    s_up = torch.full((N,), -7.0, dtype=torch.float32, device=dev)
    s_dn = torch.full((N,), -7.0, dtype=torch.float32, device=dev)
    plan.surrogates_all([sb.matrix(w, g_) for w, g_ in zip(dW, dG)], torch.cat(rps).to(dev), torch.cat(cps).to(dev),
                        torch.from_numpy(level).to(dev), s_up, s_dn, ws)
    torch.cuda.synchronize()
    ups, dns, base = [], [], 0
    for (R, C), (W, _), G, rp, cp in zip(shapes, mats, grads, rps, cps):
        Wp, Gp = orc.gather(to_np_bf16(W), G.numpy(), rp.numpy(), cp.numpy())
        nb = (R // m) * (C // n)
        u, d_ = orc.surrogates(Wp, Gp, m, n, bits, level[base:base + nb])
        ups.append(u); dns.append(d_); base += nb
    np.testing.assert_array_equal(s_up.cpu().numpy(), np.concatenate(ups))
    np.testing.assert_array_equal(s_dn.cpu().numpy(), np.concatenate(dns))
    assert np.any(np.concatenate(ups) < 0) and np.all(np.concatenate(dns) >= 0)
    plan.close()


def test_one_pass_degenerate_groups(orc, ctx, dev):
    """Constant groups, ranges so small that qmax / R overflows, signed zeros and the largest finite
    bf16 through the one-pass cost, packing and surrogate kernels (identity and random permutations).
    Every group's max - min stays finite in fp32: beyond that the library's results are unspecified
    (NaN arithmetic, which the kernels are compiled not to honour)."""
    say("one-pass degenerate groups")
    m = n = 64
    R, C = 128, 192
    W, S = synth.make_matrix("gauss_outlier", R, C, seed=6)
    Wn = to_np_bf16(W).copy()
    Wn[0, :64] = Wn[0, 0]                                 # constant group: range 0
    Wn[1, :64] = 0
    Wn[1, 7] = 0x0001                                     # range = smallest subnormal: qmax / R overflows
    Wn[2, :64] = 0x8000                                   # all -0
    Wn[2, 3] = 0x0000                                     # +0 among -0: range 0
    Wn[3, :64] = 0
    Wn[3, 9] = 0x0040                                     # subnormal range whose reciprocal is finite for small qmax
    Wn[4, 64:128] = 0x7F7F                                # largest finite bf16, constant
    Wn[5, 128:] = 0xFEFF                                  # -1.69e38 ...
    Wn[5, 130] = 0x7EFF                                   # ... and +1.69e38: the widest range that is finite in fp32
    Wd = torch.from_numpy(Wn.view(np.int16)).view(torch.bfloat16).to(dev)
    Sd = S.to(dev)
    Gs = (S * torch.sign(torch.randn(R, C, generator=torch.Generator().manual_seed(1)))).contiguous()
    bits = [1, 2, 3, 4, 8]
    plan, ws = make_plan(ctx, [(R, C)], m, n, bits, dev)
    N, K = plan.num_blocks(), len(bits)
    g = torch.Generator().manual_seed(2)
    for rp, cp in ((torch.arange(R), torch.arange(C)), (torch.randperm(R, generator=g), torch.randperm(C, generator=g))):
        rp, cp = rp.to(torch.int32), cp.to(torch.int32)
        Wp, Sp = orc.gather(Wn, S.numpy(), rp.numpy(), cp.numpy())
        _, Gp = orc.gather(Wn, Gs.numpy(), rp.numpy(), cp.numpy())
        cost = torch.empty(N, K, dtype=torch.float32, device=dev)
        plan.gather_cost_all([sb.matrix(Wd, Sd)], rp.to(dev), cp.to(dev), None, cost, ws)
        level = np.arange(N, dtype=np.uint8) % K
        off = orc.offsets(level, m, n, bits)
        codes_d = torch.zeros(int(off[-1]), dtype=torch.uint8, device=dev)
        scale_d = torch.empty(N * m, dtype=torch.float32, device=dev)
        zero_d = torch.empty(N * m, dtype=torch.float32, device=dev)
        plan.gather_pack_all([sb.matrix(Wd, None)], rp.to(dev), cp.to(dev), torch.from_numpy(level).to(dev),
                             torch.from_numpy(off).to(dev), codes_d, scale_d, zero_d, ws)
        s_up = torch.empty(N, dtype=torch.float32, device=dev)
        s_dn = torch.empty(N, dtype=torch.float32, device=dev)
        Gd = Gs.to(dev)
        plan.surrogates_all([sb.matrix(Wd, Gd)], rp.to(dev), cp.to(dev), torch.from_numpy(level).to(dev),
                            s_up, s_dn, ws)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(cost.cpu().numpy().view(np.uint32), orc.cost_table(Wp, Sp, m, n, bits).view(np.uint32))
        codes = np.zeros(int(off[-1]), np.uint8)
        scale = np.zeros(N * m, np.float32)
        zero = np.zeros(N * m, np.float32)
        orc.pack(Wp, m, n, bits, level, off, 0, codes, scale, zero)
        np.testing.assert_array_equal(codes_d.cpu().numpy(), codes)
        np.testing.assert_array_equal(scale_d.cpu().numpy().view(np.uint32), scale.view(np.uint32))
        np.testing.assert_array_equal(zero_d.cpu().numpy().view(np.uint32), zero.view(np.uint32))
        u, d_ = orc.surrogates(Wp, Gp, m, n, bits, level)
        np.testing.assert_array_equal(s_up.cpu().numpy().view(np.uint32), u.view(np.uint32))
        np.testing.assert_array_equal(s_dn.cpu().numpy().view(np.uint32), d_.view(np.uint32))
    plan.close()


def test_gather_cost_one_pass_refuses_other_shapes(ctx, dev):
    say("one-pass refuses")
    plan, ws = make_plan(ctx, [(64, 256)], 32, 256, [2, 4], dev)     # 256-column blocks: two-pass route only
    assert not plan.gather_cost_supported()
    W, S = synth.make_matrix("student_t", 64, 256, seed=1)
    Wd, Sd = W.to(dev), S.to(dev)
    rp = torch.arange(64, dtype=torch.int32, device=dev)
    cp = torch.arange(256, dtype=torch.int32, device=dev)
    w_re = torch.zeros(64 * 256, dtype=torch.bfloat16, device=dev)
    cost = torch.zeros(plan.num_blocks(), 2, dtype=torch.float32, device=dev)
    with pytest.raises(sb.SbitsError) as e:
        plan.gather_cost_all([sb.matrix(Wd, Sd)], rp, cp, w_re, cost, ws)
    assert e.value.status == sb.ERR_UNIMPLEMENTED
    plan.close()


def test_surrogates_refuse_rows_too_wide_to_stage(ctx, dev):
    say("surrogates refuse wide rows")
    plan, ws = make_plan(ctx, [(64, 20480)], 64, 128, [2, 4], dev)
    assert plan.gather_cost_supported()                              # the cost table has a route for it
    W, G = synth.make_matrix("student_t", 64, 20480, seed=1)
    Wd, Gd = W.to(dev), G.to(dev)
    rp = torch.arange(64, dtype=torch.int32, device=dev)
    cp = torch.arange(20480, dtype=torch.int32, device=dev)
    N = plan.num_blocks()
    level = torch.zeros(N, dtype=torch.uint8, device=dev)
    up = torch.zeros(N, dtype=torch.float32, device=dev)
    down = torch.zeros(N, dtype=torch.float32, device=dev)
    with pytest.raises(sb.SbitsError) as e:
        plan.surrogates_all([sb.matrix(Wd, Gd)], rp, cp, level, up, down, ws)
    assert e.value.status == sb.ERR_UNIMPLEMENTED
    plan.close()


# --------------------------------------------------------------------------- allocation

def synthetic_cost(N, bits, seed, noise=0.2):
    rng = np.random.default_rng(seed)
    sens = np.exp(2.0 * rng.normal(size=(N, 1)))
    c = sens * 4.0 ** -np.asarray(bits, np.float64)[None, :] * np.exp(noise * rng.normal(size=(N, len(bits))))
    return c.astype(np.float32)


ALLOC_CASES = [
    ([2, 3, 4], 3.0, 64, 0.05, 0.02, 0),
    ([2, 3, 4], 3.0, 4000, 0.05, 0.02, 0),
    ([1, 2, 3, 4], 2.5, 5000, 0.05, 0.02, 0),
    ([1, 2, 3, 4], 3.0, 5000, 0.05, 0.02, 0),
    ([1, 2, 3, 4, 8], 2.25, 3000, 0.05, 0.02, 0),
    ([2, 3, 4], 2.75, 2048, 0.05, 0.02, 0),
    ([2, 3, 4], 2.6, 1000, 0.3, 0.0, 1),                  # cold start, runs down to k = 0
    ([1, 2, 4, 8], 3.5, 777, 0.1, 0.01, 0),               # floor(B) is no candidate
    ([2, 3, 4], 3.999, 300, 0.05, 0.02, 0),
    ([2, 3, 4], 2.0, 300, 0.05, 0.02, 0),                 # no slack at the lowest level
    ([3], 3.0, 100, 0.05, 0.02, 0),                       # a single candidate
    ([2, 3, 4], 5.0, 100, 0.05, 0.02, 0),                 # budget above the largest candidate
    ([2, 3, 4], 3.0, 70000, 0.05, 0.02, 0),               # several workgroups and histogram flushes
    ([0, 1, 2, 3, 4], 1.5, 5000, 0.05, 0.02, 0),          # with the pruned candidate
    ([0, 2, 4, 8], 0.9, 3000, 0.05, 0.02, 0),             # warm start at 0 bits, uneven steps
    ([0, 1, 2, 3, 4, 5, 6, 7, 8], 3.0, 4000, 0.05, 0.02, 0),   # nine candidates
]


@pytest.mark.parametrize("bits,avg,N,g0,gT,init", ALLOC_CASES)
def test_allocate_matches_oracle_step_by_step(orc, ctx, dev, bits, avg, N, g0, gT, init):
    say("alloc", bits, avg, N, g0, gT, init)
    cost = synthetic_cost(N, bits, seed=N + len(bits))
    plan, ws = make_plan(ctx, [shape_with_blocks(N)], 8, 8, bits, dev)
    assert plan.num_blocks() == N
    level = torch.full((N,), 255, dtype=torch.uint8, device=dev)
    rc, st, tr = plan.allocate(torch.from_numpy(cost).to(dev), avg, level, ws, gamma0=g0, gammaT=gT,
                               init_mode=init, max_iters=5000, trace_cap=5000)
    rc_o, level_o, st_o, tr_o = orc.allocate(cost, bits, avg, gamma0=g0, gammaT=gT, init_mode=init,
                                             max_iters=5000, want_trace=True)
    assert rc == 0 and rc_o == 0
    assert st == st_o
    assert tr == tr_o
    np.testing.assert_array_equal(level.cpu().numpy(), level_o)
    plan.close()


def test_allocate_ties_and_flat_tables(orc, ctx, dev):
    say("alloc ties")
    for cost, bits, avg in [
        (np.tile(np.array([[5, 2, 1]], np.float32), (600, 1)), [2, 3, 4], 2.5),      # all blocks identical
        (np.ones((300, 3), np.float32), [2, 3, 4], 2.5),                              # no gain anywhere
        (np.zeros((300, 3), np.float32), [2, 3, 4], 3.0),                             # all-zero table: shift 0
        (np.tile(np.array([[1, 2, 3]], np.float32), (128, 1)), [2, 3, 4], 2.5),      # cost grows with bits
    ]:
        N = cost.shape[0]
        plan, ws = make_plan(ctx, [shape_with_blocks(N)], 8, 8, bits, dev)
        level = torch.empty(N, dtype=torch.uint8, device=dev)
        rc, st, tr = plan.allocate(torch.from_numpy(cost).to(dev), avg, level, ws, trace_cap=1000)
        rc_o, level_o, st_o, tr_o = orc.allocate(cost, bits, avg, want_trace=True)
        assert (rc, st, tr) == (rc_o, st_o, tr_o)
        np.testing.assert_array_equal(level.cpu().numpy(), level_o)
        plan.close()


def test_allocate_max_iters_status(orc, ctx, dev):
    say("alloc max_iters")
    N, bits = 2000, [2, 3, 4]
    cost = synthetic_cost(N, bits, seed=9)
    plan, ws = make_plan(ctx, [shape_with_blocks(N)], 8, 8, bits, dev)
    level = torch.empty(N, dtype=torch.uint8, device=dev)
    rc, st, _ = plan.allocate(torch.from_numpy(cost).to(dev), 2.5, level, ws, max_iters=3)
    rc_o, level_o, st_o, _ = orc.allocate(cost, bits, 2.5, max_iters=3)
    assert rc == sb.ERR_MAX_ITERS and rc_o == -2 and st == st_o
    np.testing.assert_array_equal(level.cpu().numpy(), level_o)
    plan.close()


# ---------------------------------------------------------------------- offsets and pack

@pytest.mark.parametrize("R,C,m,n,bits", [(256, 384, 128, 128, [2, 3, 4]), (192, 320, 64, 64, [1, 2, 3, 4, 8]),
                                           (24, 40, 8, 8, [1, 2, 3, 4, 5, 6, 7, 8]), (64, 96, 16, 32, [1, 3, 5]),
                                           (64, 1024, 32, 512, [1, 2, 3, 4, 8]), (4096, 16, 8, 16, [3, 4])])
def test_offsets_and_pack(orc, ctx, dev, R, C, m, n, bits):
    say("pack", R, C, m, n, bits)
    W, _ = synth.make_matrix("student_t", R, C, seed=7, tid=m + n)
    plan, ws = make_plan(ctx, [(m, n), (R, C), (m, 2 * n)], m, n, bits, dev)
    N, base = plan.num_blocks(), plan.block_base(1)
    rng = np.random.default_rng(R + C)
    level = rng.integers(0, len(bits), size=N).astype(np.uint8)
    level_d = torch.from_numpy(level).to(dev)
    off_d = torch.empty(N + 1, dtype=torch.int64, device=dev)
    plan.offsets(level_d, off_d, ws)
    off = orc.offsets(level, m, n, bits)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(off_d.cpu().numpy(), off)
    total = int(off[-1])
    codes_d = torch.full((total,), 0x55, dtype=torch.uint8, device=dev)
    scale_d = torch.full((N * m,), -1.0, dtype=torch.float32, device=dev)
    zero_d = torch.full((N * m,), -1.0, dtype=torch.float32, device=dev)
    plan.pack(1, W.to(dev), level_d, off_d, codes_d, scale_d, zero_d)
    torch.cuda.synchronize()
    codes = np.full(total, 0x55, np.uint8)
    scale = np.full(N * m, -1.0, np.float32)
    zero = np.full(N * m, -1.0, np.float32)
    orc.pack(to_np_bf16(W), m, n, bits, level, off, base, codes, scale, zero)
    np.testing.assert_array_equal(codes_d.cpu().numpy(), codes)
    np.testing.assert_array_equal(scale_d.cpu().numpy(), scale)
    np.testing.assert_array_equal(zero_d.cpu().numpy().view(np.uint32), zero.view(np.uint32))
    plan.close()


def test_offsets_many_tiles(orc, ctx, dev):
    say("offsets large")
    N, bits = 601000, [1, 2, 3, 4, 8]
    plan, ws = make_plan(ctx, [(8000, 4808)], 8, 8, bits, dev)
    assert plan.num_blocks() == N
    level = np.random.default_rng(1).integers(0, 5, size=N).astype(np.uint8)
    off_d = torch.empty(N + 1, dtype=torch.int64, device=dev)
    plan.offsets(torch.from_numpy(level).to(dev), off_d, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(off_d.cpu().numpy(), orc.offsets(level, 8, 8, bits))
    plan.close()


# --------------------------------------------------------------------------- end to end

def oracle_search(orc, mats, m, n, bits, avg, power=2, **kw):
    """The whole path on the CPU oracle: returns every output the library produces."""
    perms, W2, S2, costs = [], [], [], []
    for W, S in mats:
        Wn, Sn = to_np_bf16(W), S.numpy()
        rs, cs = orc.channel_scores(Sn)
        rp, cp = orc.argsort_desc(rs), orc.argsort_desc(cs)
        Wp, Sp = orc.gather(Wn, Sn, rp, cp)
        perms.append((rp, cp)); W2.append(Wp); S2.append(Sp)
        costs.append(orc.cost_table(Wp, Sp, m, n, bits, power=power))
    cost = np.concatenate(costs, 0)
    rc, level, st, _ = orc.allocate(cost, bits, avg, **kw)
    off = orc.offsets(level, m, n, bits)
    N = cost.shape[0]
    codes = np.zeros(int(off[-1]), np.uint8)
    scale = np.zeros(N * m, np.float32)
    zero = np.zeros(N * m, np.float32)
    base = 0
    for Wp in W2:
        orc.pack(Wp, m, n, bits, level, off, base, codes, scale, zero)
        base += (Wp.shape[0] // m) * (Wp.shape[1] // n)
    return dict(perms=perms, W2=W2, S2=S2, cost=cost, level=level, stats=st, off=off, codes=codes,
                scale=scale, zero=zero, rc=rc)


def gpu_search(ctx, dev, mats, m, n, bits, avg, **kw):
    shapes = [tuple(W.shape) for W, _ in mats]
    plan, ws = make_plan(ctx, shapes, m, n, bits, dev)
    N, K = plan.num_blocks(), len(bits)
    dW = [W.to(dev) for W, _ in mats]
    dS = [S.to(dev) for _, S in mats]
    nel = sum(r * c for r, c in shapes)
    o = dict(
        row_perm=torch.empty(sum(r for r, _ in shapes), dtype=torch.int32, device=dev),
        col_perm=torch.empty(sum(c for _, c in shapes), dtype=torch.int32, device=dev),
        w_re=torch.empty(nel, dtype=torch.bfloat16, device=dev),
        s_re=torch.empty(nel, dtype=torch.float32, device=dev),
        cost=torch.empty(N, K, dtype=torch.float32, device=dev),
        level=torch.empty(N, dtype=torch.uint8, device=dev),
        byte_off=torch.empty(N + 1, dtype=torch.int64, device=dev),
        codes=torch.zeros(plan.codes_bytes_bound(avg), dtype=torch.uint8, device=dev),
        scale=torch.empty(N * m, dtype=torch.float32, device=dev),
        zero=torch.empty(N * m, dtype=torch.float32, device=dev),
    )
    out = sb.Outputs(o["row_perm"].data_ptr(), o["col_perm"].data_ptr(), o["w_re"].data_ptr(), o["s_re"].data_ptr(),
                     o["cost"].data_ptr(), o["level"].data_ptr(), o["byte_off"].data_ptr(), o["codes"].data_ptr(),
                     o["codes"].numel(), o["scale"].data_ptr(), o["zero"].data_ptr())
    o["one_pass"] = plan.gather_cost_supported()         # then the reordered sensitivities are never written
    rc, st = plan.search([sb.matrix(w, s) for w, s in zip(dW, dS)], avg, out, ws, **kw)
    torch.cuda.synchronize()
    plan.close()
    return rc, st, o, shapes


def compare_search(orc, ref, rc, st, o, shapes, m):
    assert rc == ref["rc"] and st == ref["stats"]
    ro = co = eo = 0
    for (R, C), (rp, cp), Wp, Sp in zip(shapes, ref["perms"], ref["W2"], ref["S2"]):
        np.testing.assert_array_equal(o["row_perm"][ro:ro + R].cpu().numpy(), rp)
        np.testing.assert_array_equal(o["col_perm"][co:co + C].cpu().numpy(), cp)
        np.testing.assert_array_equal(to_np_bf16(o["w_re"][eo:eo + R * C]).reshape(R, C), Wp)
        if not o["one_pass"]:
            np.testing.assert_array_equal(o["s_re"][eo:eo + R * C].cpu().numpy().reshape(R, C), Sp)
        ro, co, eo = ro + R, co + C, eo + R * C
    np.testing.assert_array_equal(o["cost"].cpu().numpy(), ref["cost"])
    np.testing.assert_array_equal(o["level"].cpu().numpy(), ref["level"])
    np.testing.assert_array_equal(o["byte_off"].cpu().numpy(), ref["off"])
    total = int(ref["off"][-1])
    np.testing.assert_array_equal(o["codes"][:total].cpu().numpy(), ref["codes"])
    np.testing.assert_array_equal(o["scale"].cpu().numpy(), ref["scale"])
    np.testing.assert_array_equal(o["zero"].cpu().numpy().view(np.uint32), ref["zero"].view(np.uint32))


def test_search_single_matrix_config(orc, ctx, dev):
    """One 1024 x 1024 matrix, N(0, 0.02) weights with 0.1 % outliers x50, squared-normal
    sensitivity, 128 x 128 blocks, {2,3,4} bits, budget 3.0, seed 0."""
    say("search config 1")
    mats = [synth.make_matrix("gauss_outlier", 1024, 1024, seed=0, tid=0)]
    ref = oracle_search(orc, mats, 128, 128, [2, 3, 4], 3.0)
    rc, st, o, shapes = gpu_search(ctx, dev, mats, 128, 128, [2, 3, 4], 3.0)
    compare_search(orc, ref, rc, st, o, shapes, 128)
    assert st["bits_used"] <= st["bits_budget"] == 192


@pytest.mark.parametrize("m,n,bits,avg,recipe", [(64, 64, [1, 2, 3, 4, 8], 2.25, "outlier_chan"),
                                                  (128, 128, [1, 2, 3, 4], 2.5, "student_t"),
                                                  (32, 256, [2, 3, 4], 2.75, "student_t")])
def test_search_several_matrices(orc, ctx, dev, m, n, bits, avg, recipe):
    say("search multi", m, n, bits, avg, recipe)
    shapes = [(512, 512), (256, 1024), (1024, 256), (256, 512)]
    mats = [synth.make_matrix(recipe, r, c, seed=3, tid=i) for i, (r, c) in enumerate(shapes)]
    ref = oracle_search(orc, mats, m, n, bits, avg)
    rc, st, o, shp = gpu_search(ctx, dev, mats, m, n, bits, avg)
    compare_search(orc, ref, rc, st, o, shp, m)


def test_search_with_rows_too_wide_to_stage(orc, ctx, dev):
    """One call over a plan that mixes matrices the one-pass cost kernel stages with one it cannot (20480 columns):
    that one is scored from a reordered copy, here written straight into the caller's w_re."""
    say("search with a wide-row matrix")
    shapes = [(128, 20480), (256, 1024), (128, 4096)]
    mats = [synth.make_matrix("student_t", r, c, seed=5, tid=i) for i, (r, c) in enumerate(shapes)]
    ref = oracle_search(orc, mats, 64, 128, [1, 2, 3, 4], 2.5)
    rc, st, o, shp = gpu_search(ctx, dev, mats, 64, 128, [1, 2, 3, 4], 2.5)
    assert o["one_pass"]
    compare_search(orc, ref, rc, st, o, shp, 64)


def test_search_with_a_pruned_candidate(orc, ctx, dev):
    """{0, 1, 2, 3, 4} bits at 1.5 bits per weight: blocks at 0 bits are pruned (no bytes, zero scale / zero)."""
    say("search with 0 bits")
    shapes = [(512, 512), (256, 1024), (1024, 256)]
    mats = [synth.make_matrix("student_t", r, c, seed=6, tid=i) for i, (r, c) in enumerate(shapes)]
    bits = [0, 1, 2, 3, 4]
    ref = oracle_search(orc, mats, 64, 128, bits, 1.5)
    rc, st, o, shp = gpu_search(ctx, dev, mats, 64, 128, bits, 1.5)
    compare_search(orc, ref, rc, st, o, shp, 64)
    pruned = ref["level"] == 0
    assert pruned.any() and not pruned.all()
    assert not ref["scale"].reshape(-1, 64)[pruned].any()


@pytest.mark.parametrize("bits,avg", [([2, 4, 8], 8.0), ([0, 2, 4], 0.0), ([0, 2, 4], 0.3)])
def test_search_at_the_ends_of_the_budget_range(orc, ctx, dev, bits, avg):
    """Budget = the largest candidate (everything at the top level, 8-bit codes), budget 0 with a 0-bit candidate
    (everything pruned: an empty code stream, no buffer) and a budget that keeps only a few blocks."""
    say("search, budget", avg, "of", bits)
    shapes = [(256, 512), (128, 1024)]
    mats = [synth.make_matrix("student_t", r, c, seed=8, tid=i) for i, (r, c) in enumerate(shapes)]
    ref = oracle_search(orc, mats, 64, 128, bits, avg)
    rc, st, o, shp = gpu_search(ctx, dev, mats, 64, 128, bits, avg)
    compare_search(orc, ref, rc, st, o, shp, 64)
    assert st["bits_used"] <= st["bits_budget"]
    if avg == 0.0:
        assert o["codes"].numel() == 0 and not ref["level"].any()


def test_search_is_deterministic(ctx, dev):
    say("determinism")
    mats = [synth.make_matrix("student_t", 512, 1024, seed=11, tid=i) for i in range(3)]
    a = gpu_search(ctx, dev, mats, 64, 64, [1, 2, 3, 4], 2.5)
    b = gpu_search(ctx, dev, mats, 64, 64, [1, 2, 3, 4], 2.5)
    assert a[1] == b[1]
    for key in a[2]:
        if key == "one_pass" or (key == "s_re" and a[2]["one_pass"]):     # s_re: not written on the one-pass route
            continue
        assert torch.equal(a[2][key].view(torch.uint8), b[2][key].view(torch.uint8)), key


# ------------------------------------------------------------------------ one step on caller-supplied estimates
def _blocks_plan(ctx, N, bits, dev):
    """A plan with exactly N blocks (8 x 8 blocks of one matrix, or the 8B-shaped model)."""
    if N == 425984:
        shapes = [(r, c) for _ in range(32) for _, r, c in synth.layer_shapes(synth.LLAMA3_8B)]
        return make_plan(ctx, shapes, 128, 128, bits, dev)
    if N == 50000:
        return make_plan(ctx, [(1600, 2000)], 8, 8, bits, dev)
    return make_plan(ctx, [(8, 8 * N)], 8, 8, bits, dev)


@pytest.mark.parametrize("N,bits", [(1, [2, 3, 4]), (37, [1, 2, 3, 4]), (4096, [1, 2, 3, 4, 8]), (50000, [2, 4, 8]),
                                    (425984, [1, 2, 3, 4]), (4096, [0, 1, 2, 3, 4, 5, 6, 7, 8]), (1000, [0, 2, 4])])
def test_propose_matches_oracle(orc, ctx, dev, N, bits):
    say("propose", N, bits)
    plan, ws = _blocks_plan(ctx, N, bits, dev)
    assert plan.num_blocks() == N
    K = len(bits)
    rng = np.random.default_rng(N)
    for case in range(8):
        level = rng.integers(0, K, N).astype(np.uint8)
        if case == 6: level[:] = K - 1                             # nobody can be raised
        if case == 7: level[:] = 0                                 # nobody can be lowered
        if case % 2:                                               # many ties, some non-positive
            s_up = rng.integers(-2, 6, N).astype(np.float32)
            s_dn = rng.integers(0, 4, N).astype(np.float32)
        else:
            s_up = rng.standard_normal(N).astype(np.float32) * np.float32(3)
            s_dn = np.abs(rng.standard_normal(N)).astype(np.float32)
        used = int(np.asarray(bits)[level].sum())
        slack = [0, 0, max(1, N // 50), 3 * N, -1, 1, 0, N][case]
        avg = (used + slack) / N + 1e-9
        if avg < bits[0]:
            continue
        k = [max(1, N // 20), 1, max(1, N // 20), N + 5, max(1, N // 10), 2, 4, max(1, N // 3)][case]
        d_out = torch.full((N,), 77, dtype=torch.uint8, device=dev)
        info = plan.propose(torch.from_numpy(s_up).to(dev), torch.from_numpy(s_dn).to(dev),
                            torch.from_numpy(level).to(dev), avg, k, d_out, ws)
        kind, want, winfo = orc.propose(s_up, s_dn, level, bits, avg, k)
        assert info["kind"] == kind, (case, info, winfo)
        np.testing.assert_array_equal(d_out.cpu().numpy(), want, err_msg="case %d" % case)
        for f in ("n_up", "n_dn", "bits_before", "bits_after"):
            assert info[f] == winfo[f], (case, f, info, winfo)
        assert info["bits_budget"] == int(np.floor(avg * N))
    # in place, and without the host read-back
    lv = torch.from_numpy(level).to(dev)
    plan.propose(torch.from_numpy(s_up).to(dev), torch.from_numpy(s_dn).to(dev), lv, avg, k, lv, ws, want_info=False)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(lv.cpu().numpy(), want)
    plan.close()


def test_propose_loop_on_exact_differences_reproduces_allocate(orc, ctx, dev):
    """The caller-driven loop (propose, the caller's fixed-point loss test, halve k on rejection) fed with
    the cost table's own differences ends at the allocation of sbits_allocate (contiguous bitwidths)."""
    say("propose loop == allocate")
    N, bits = 4096, [1, 2, 3, 4]
    plan, ws = _blocks_plan(ctx, N, bits, dev)
    rng = np.random.default_rng(3)
    base = rng.lognormal(0, 1.5, N).astype(np.float32)
    cost = (base[:, None] * np.array([1.0, 0.3, 0.1, 0.02], np.float32) *
            rng.uniform(0.7, 1.3, (N, 4)).astype(np.float32)).astype(np.float32)
    dcost = torch.from_numpy(cost).to(dev)
    idx = torch.arange(N, device=dev)
    shift = orc.cost_shift(cost)
    for avg in (2.5, 3.0):
        want = torch.empty(N, dtype=torch.uint8, device=dev)
        _, st, _ = plan.allocate(dcost, avg, want, ws)
        level = torch.full((N,), int(avg) - 1, dtype=torch.uint8, device=dev)
        prop = torch.empty_like(level)
        k, kmin, iters = max(1, int(0.05 * N)), max(1, int(0.02 * N)), 0
        while k >= kmin:
            iters += 1
            l = level.long()
            up = torch.where(l < 3, dcost[idx, l] - dcost[idx, (l + 1).clamp(max=3)], torch.zeros((), device=dev))
            dn = torch.where(l > 0, dcost[idx, (l - 1).clamp(min=0)] - dcost[idx, l], torch.zeros((), device=dev))
            info = plan.propose(up, dn, level, avg, k, prop, ws)
            if info["kind"] == 1:
                level, prop = prop, level
            elif info["kind"] == 2:
                fxs = lambda v: torch.round(v.double() * 2.0 ** shift).long().sum().item()   # exact: |v| 2^shift < 2^53
                delta = fxs(dn[prop < level]) - fxs(up[prop > level])
                if delta < 0: level, prop = prop, level
                else: k //= 2
            else:
                k //= 2
        np.testing.assert_array_equal(level.cpu().numpy(), want.cpu().numpy())
        assert iters == st["iters"]
    plan.close()


# ------------------------------------------------------------------------ product with the stored weights
def _packed_matrix(orc, R, C, m, n, bits, seed, base_blocks=3, levels=None):
    """A random matrix packed by the oracle at random levels, its blocks starting at global id base_blocks."""
    rng = np.random.default_rng(seed)
    Wb = orc.f32_to_bf16(0.02 * rng.standard_t(4, size=(R, C)))
    nb = (R // m) * (C // n)
    N = base_blocks + nb
    level = rng.integers(0, len(bits), size=N).astype(np.uint8) if levels is None else levels(rng, N)
    off = orc.offsets(level, m, n, bits)
    codes = np.zeros(int(off[-1]) , np.uint8)
    scale = np.zeros(N * m, np.float32)
    zero = np.zeros(N * m, np.float32)
    orc.pack(Wb, m, n, bits, level, off, base_blocks, codes, scale, zero)
    return level, off, codes, scale, zero


def _mp_gemm_check(orc, y, packed, base, R, C, m, n, bits, xb):
    level, off, codes, scale, zero = packed
    ref = orc.mp_gemm(codes, scale, zero, level, off, base, R, C, m, n, bits, xb)
    What = orc.dequant(codes, scale, zero, level, off, base, R, C, m, n, bits).astype(np.float64)
    # scale of every element's block row, for the bound: the kernel sums (128 + q) * x and takes 128 * sum x out again
    nbc = C // n
    srow = scale.reshape(-1, m)[base:base + (R // m) * nbc].reshape(R // m, nbc, m).transpose(0, 2, 1).reshape(R, nbc)
    xa = np.abs(orc.bf16_to_f32(xb).astype(np.float64))
    bound = xa @ np.abs(What).T + 128.0 * (xa.reshape(xa.shape[0], nbc, n).sum(2) @ np.abs(srow.astype(np.float64)).T)
    err = np.abs(y.astype(np.float64) - ref)
    assert np.all(err <= bound * 2.0 ** -18 + 1e-30), float((err / (bound + 1e-300)).max())
    assert np.sqrt((err ** 2).mean()) <= 2.0 ** -22 * np.sqrt((bound ** 2).mean())       # typical error: far below the bound
    return ref


@pytest.mark.parametrize("R,C,m,n,bits,batch", [
    (64, 256, 32, 128, [1, 2, 3, 4, 5, 6, 7, 8], 16),       # every bitwidth, one workgroup
    (160, 128 * 40, 32, 128, [2, 4, 8], 5),                 # three column splits, ragged rows and batch
    (256, 128 * 17, 128, 128, [1, 2, 3, 4], 32),            # two batch tiles, a split with one block column
    (128, 192, 64, 64, [1, 2, 3, 4, 5, 6, 7, 8], 17),       # group size 64
    (192, 64 * 33, 64, 64, [2, 3, 4, 8], 1),                # group size 64, three splits, a single row of x
    (128, 128 * 18, 64, 128, [2, 4], 70),                   # more than 32 rows of x: three launches
    (160, 128 * 20, 32, 128, [0, 2, 4, 8], 16),             # pruned blocks among the others
    (128, 192, 64, 64, [0, 1, 2, 3, 4, 5, 6, 7, 8], 9),     # nine candidates, group size 64
])
def test_mp_gemm(orc, ctx, dev, R, C, m, n, bits, batch):
    say("mixed-precision product", R, C, m, n, bits, batch)
    base = 3
    shapes = [(m, 3 * n), (R, C)]                           # a first matrix of 3 blocks, so this one's base is 3
    plan, ws = make_plan(ctx, shapes, m, n, bits, dev)
    assert plan.block_base(1) == base
    packed = _packed_matrix(orc, R, C, m, n, bits, seed=R + C)
    level, off, codes, scale, zero = packed
    rng = np.random.default_rng(batch)
    xb = orc.f32_to_bf16(rng.standard_normal((batch, C)))
    xd = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).to(dev)
    y = torch.full((batch, R), 7.0, dtype=torch.float32, device=dev)
    dcodes = torch.from_numpy(codes).to(dev)
    args = (torch.from_numpy(level).to(dev), torch.from_numpy(off).to(dev), dcodes,
            torch.from_numpy(scale).to(dev), torch.from_numpy(zero).to(dev))
    plan.mp_gemm(1, xd, *args, y, ws)
    torch.cuda.synchronize()
    _mp_gemm_check(orc, y.cpu().numpy(), packed, base, R, C, m, n, bits, xb)
    # a strided x (ld_x > cols) gives the same bits
    xw = torch.zeros(batch, C + 8, dtype=torch.bfloat16, device=dev)
    xw[:, :C] = xd
    y2 = torch.empty_like(y)
    plan.mp_gemm(1, xw[:, :C], *args, y2, ws)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    plan.close()


def test_mp_gemm_exact_on_integer_weights(orc, ctx, dev):
    """Integer weights stored exactly at 8 bits and at 4 bits (0..15), integer x: the exact integer product."""
    say("mixed-precision product: exact integers")
    m, n, R, C = 32, 128, 64, 256
    rng = np.random.default_rng(1)
    plan, ws = make_plan(ctx, [(R, C)], m, n, [4, 8], dev)
    Wi = np.empty((R, C), np.int64)
    level = np.array([0, 1, 1, 0], np.uint8)                         # blocks (0,0) 4-bit, (0,1) 8-bit, (1,0) 8-bit, (1,1) 4-bit
    for I in range(2):
        for J in range(2):
            hi = 16 if level[I * 2 + J] == 0 else 256
            blk = rng.integers(0, hi, (m, n)); blk[:, 0] = 0; blk[:, 1] = hi - 1
            Wi[I * m:(I + 1) * m, J * n:(J + 1) * n] = blk
    off = orc.offsets(level, m, n, [4, 8])
    codes = np.zeros(int(off[-1]), np.uint8); scale = np.zeros(4 * m, np.float32); zero = np.zeros(4 * m, np.float32)
    orc.pack(orc.f32_to_bf16(Wi.astype(np.float32)), m, n, [4, 8], level, off, 0, codes, scale, zero)
    assert np.all(scale == 1) and np.all(zero == 0)
    xi = rng.integers(-8, 9, (16, C))
    xd = torch.from_numpy(xi.astype(np.float32)).to(torch.bfloat16).to(dev)
    y = torch.empty(16, R, dtype=torch.float32, device=dev)
    plan.mp_gemm(0, xd, torch.from_numpy(level).to(dev), torch.from_numpy(off).to(dev), torch.from_numpy(codes).to(dev),
                 torch.from_numpy(scale).to(dev), torch.from_numpy(zero).to(dev), y, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(y.cpu().numpy(), (xi @ Wi.T).astype(np.float32))
    plan.close()


def test_mp_gemm_refuses_other_shapes(ctx, dev):
    plan, ws = make_plan(ctx, [(64, 512)], 16, 256, [2, 4], dev)
    t = torch.zeros(4096, dtype=torch.uint8, device=dev)
    x = torch.zeros(16, 512, dtype=torch.bfloat16, device=dev)
    with pytest.raises(sb.SbitsError) as e:
        plan.mp_gemm(0, x, t, t, t, t, t, t, ws)
    assert e.value.status == sb.ERR_UNIMPLEMENTED
    plan.close()


def test_search_then_inference_preserves_the_layer_function(orc, ctx, dev):
    """The whole chain on one matrix: search (reorder, allocate, pack), then the product with the
    stored weights.  With x in the permuted input order the result is the permuted output of the layer
    computed with the dequantized weights; against the unquantized layer it differs by the
    quantization error only (more bits, smaller difference)."""
    say("search -> inference")
    R, C, m, n, bits = 256, 512, 64, 128, [2, 3, 4, 8]
    W, S = synth.make_matrix("student_t", R, C, seed=5, tid=0)
    rng = np.random.default_rng(8)
    x = torch.from_numpy(rng.standard_normal((16, C)).astype(np.float32)).to(torch.bfloat16)
    y_full = x.float().numpy().astype(np.float64) @ W.float().numpy().astype(np.float64).T      # unquantized, original order
    errs = []
    for avg in (2.5, 4.0, 8.0):
        rc, st, o, _ = gpu_search(ctx, dev, [(W, S)], m, n, bits, avg)
        assert rc == 0
        plan, ws = make_plan(ctx, [(R, C)], m, n, bits, dev)
        rp, cp = o["row_perm"].cpu().numpy(), o["col_perm"].cpu().numpy()
        xp = x[:, torch.from_numpy(cp).long()].contiguous().to(dev)                               # permuted input channels
        y = torch.empty(16, R, dtype=torch.float32, device=dev)
        plan.mp_gemm(0, xp, o["level"], o["byte_off"], o["codes"], o["scale"], o["zero"], y, ws)
        torch.cuda.synchronize()
        level, off = o["level"].cpu().numpy(), o["byte_off"].cpu().numpy()
        ref = orc.mp_gemm(o["codes"][:int(off[-1])].cpu().numpy(), o["scale"].cpu().numpy(), o["zero"].cpu().numpy(),
                          level, off, 0, R, C, m, n, bits, to_np_bf16(xp.cpu()))
        yh = y.cpu().numpy().astype(np.float64)
        assert np.abs(yh - ref).max() <= 1e-4 * np.abs(ref).max()
        errs.append(float(np.linalg.norm(yh - y_full[:, rp]) / np.linalg.norm(y_full)))           # permuted output channels
        plan.close()
    say("  relative difference to the unquantized layer at 2.5 / 4 / 8 bits:", errs)
    assert errs[0] > errs[1] > errs[2] and errs[2] < 0.02


@pytest.mark.parametrize("R,C,m,n,bits", [(16, 24, 8, 8, [1, 2, 3, 4, 5, 6, 7, 8]), (128, 384, 64, 128, [1, 2, 3, 4, 8]),
                                          (96, 1024, 32, 512, [3, 5, 7]), (2048, 2056 - 8, 1024, 8, [2, 4]),
                                          (128, 384, 64, 128, [0, 1, 2, 3, 4, 5, 6, 7, 8]), (64, 96, 8, 16, [0, 3])])
def test_dequant(orc, ctx, dev, R, C, m, n, bits):
    """The stored matrix as fp32 (bit for bit the format's value) and as bf16 (nearest even)."""
    say("dequant", R, C, m, n, bits)
    base = 3
    plan, ws = make_plan(ctx, [(m, 3 * n), (R, C)], m, n, bits, dev)
    packed = _packed_matrix(orc, R, C, m, n, bits, seed=R + C)
    level, off, codes, scale, zero = packed
    args = (torch.from_numpy(level).to(dev), torch.from_numpy(off).to(dev), torch.from_numpy(codes).to(dev),
            torch.from_numpy(scale).to(dev), torch.from_numpy(zero).to(dev))
    want = orc.dequant(codes, scale, zero, level, off, base, R, C, m, n, bits)
    out = torch.full((R, C + 8), -3.0, dtype=torch.float32, device=dev)          # a pitch wider than the matrix
    plan.dequant(1, *args, out[:, :C])
    ob = torch.zeros(R, C, dtype=torch.bfloat16, device=dev)
    plan.dequant(1, *args, ob)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out[:, :C].cpu().numpy().view(np.uint32), want.view(np.uint32))
    assert torch.all(out[:, C:] == -3.0)
    np.testing.assert_array_equal(to_np_bf16(ob.cpu()), orc.f32_to_bf16(want))
    plan.close()


def test_search_coupled_equals_the_stages(orc, ctx, dev):
    """The one-call coupled search = coupled reordering, then the stages, each against the oracle."""
    say("search, coupled")
    model = dict(hidden=256, ffn=512, kv=128, layers=2)
    mats, shapes = [], []
    for layer in range(2):
        for name, r, c in synth.layer_shapes(model):
            mats.append(synth.make_matrix("student_t", r, c, seed=9, tid=synth.tensor_id(layer, name)))
            shapes.append((r, c))
    coupling = synth.llama_coupling(model, 2, head_dim=64)
    rg, cg, ng, seg, rrep, crep = coupling
    m = n = 64
    bits, avg = [2, 3, 4], 3.0
    plan, ws = make_plan(ctx, shapes, m, n, bits, dev)
    N, K = plan.num_blocks(), len(bits)
    dW = [W.to(dev) for W, _ in mats]
    dS = [S.to(dev) for _, S in mats]
    o = dict(row_perm=torch.empty(sum(r for r, _ in shapes), dtype=torch.int32, device=dev),
             col_perm=torch.empty(sum(c for _, c in shapes), dtype=torch.int32, device=dev),
             cost=torch.empty(N, K, dtype=torch.float32, device=dev), level=torch.empty(N, dtype=torch.uint8, device=dev),
             byte_off=torch.empty(N + 1, dtype=torch.int64, device=dev),
             codes=torch.zeros(plan.codes_bytes_bound(avg), dtype=torch.uint8, device=dev),
             scale=torch.empty(N * m, dtype=torch.float32, device=dev), zero=torch.empty(N * m, dtype=torch.float32, device=dev))
    out = sb.Outputs(o["row_perm"].data_ptr(), o["col_perm"].data_ptr(), None, None, o["cost"].data_ptr(),
                     o["level"].data_ptr(), o["byte_off"].data_ptr(), o["codes"].data_ptr(), o["codes"].numel(),
                     o["scale"].data_ptr(), o["zero"].data_ptr())
    assert plan.gather_cost_supported()
    rc, st = plan.search_coupled([sb.matrix(w, s) for w, s in zip(dW, dS)], coupling, avg, out, ws)
    torch.cuda.synchronize()
    # oracle: group scores -> shared permutations -> per-matrix stages -> global allocation -> packing
    scores = [orc.channel_scores(S.numpy()) for _, S in mats]
    members = {}
    for which, groups, reps in ((0, rg, rrep), (1, cg, crep)):
        for i, g in enumerate(groups):
            if g >= 0:
                sc = scores[i][which]
                members.setdefault(g, []).extend([sc] if reps[i] == 1 else orc.fold_repeated(sc, seg[g], reps[i]))
    gperm = {g: orc.coupled_perm(ms, seg[g]) for g, ms in members.items()}
    def perm_of(i, which):
        g = (rg if which == 0 else cg)[i]
        rep = (rrep if which == 0 else crep)[i]
        if g == sb.DIM_FIXED:
            return np.arange(shapes[i][which], dtype=np.int32)
        return gperm[g] if rep == 1 else orc.expand_perm(gperm[g], seg[g], rep)
    costs, Wps, ro, co = [], [], 0, 0
    for i, ((W, S), (R, C)) in enumerate(zip(mats, shapes)):
        rp, cp = perm_of(i, 0), perm_of(i, 1)
        np.testing.assert_array_equal(o["row_perm"][ro:ro + R].cpu().numpy(), rp)
        np.testing.assert_array_equal(o["col_perm"][co:co + C].cpu().numpy(), cp)
        Wp, Sp = orc.gather(to_np_bf16(W), S.numpy(), rp, cp)
        Wps.append(Wp); costs.append(orc.cost_table(Wp, Sp, m, n, bits))
        ro, co = ro + R, co + C
    cost = np.concatenate(costs)
    np.testing.assert_array_equal(o["cost"].cpu().numpy(), cost)
    rc_o, level, st_o, _ = orc.allocate(cost, bits, avg)
    assert rc == rc_o and st == st_o
    np.testing.assert_array_equal(o["level"].cpu().numpy(), level)
    off = orc.offsets(level, m, n, bits)
    codes = np.zeros(int(off[-1]), np.uint8); scale = np.zeros(N * m, np.float32); zero = np.zeros(N * m, np.float32)
    for i, Wp in enumerate(Wps):
        orc.pack(Wp, m, n, bits, level, off, plan.block_base(i), codes, scale, zero)
    np.testing.assert_array_equal(o["codes"][:int(off[-1])].cpu().numpy(), codes)
    np.testing.assert_array_equal(o["scale"].cpu().numpy(), scale)
    np.testing.assert_array_equal(o["zero"].cpu().numpy().view(np.uint32), zero.view(np.uint32))
    plan.close()


# ------------------------------------------ build variant: cost = sum s * |d| (first-order form of Eq. 3)

@pytest.fixture()
def ctx_l1(dev):
    """A context of libscalebits_l1.so; the default library is back in place afterwards."""
    import os
    prev = sb.LIB_PATH
    path = sb.variant_path("l1")
    assert os.path.exists(path), "build the variant first: python -m paper_2602_17698_amd.build"
    sb.use_library(path)
    try:
        assert sb.cost_power() == 1
        c = sb.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
        yield c
        c.close()
    finally:
        sb.use_library(prev)
        assert sb.cost_power() == 2


def test_power_one_variant_cost_tables(orc, ctx_l1, dev):
    say("l1 variant: cost tables, both routes")
    shapes, m, n, bits = [(256, 384), (128, 1024), (64, 14336)], 64, 128, [0, 1, 2, 3, 4, 8]
    plan, ws = make_plan(ctx_l1, shapes, m, n, bits, dev)
    N, K = plan.num_blocks(), len(bits)
    mats = [synth.make_matrix("student_t", r, c, seed=21, tid=i) for i, (r, c) in enumerate(shapes)]
    g = torch.Generator().manual_seed(23)
    rps = [torch.randperm(r, generator=g).to(torch.int32) for r, _ in shapes]
    cps = [torch.randperm(c, generator=g).to(torch.int32) for _, c in shapes]
    dW = [W.to(dev) for W, _ in mats]
    dS = [S.to(dev) for _, S in mats]
    dm = [sb.matrix(w, s_) for w, s_ in zip(dW, dS)]
    nel = sum(r * c for r, c in shapes)
    w_re = torch.zeros(nel, dtype=torch.bfloat16, device=dev)
    s_re = torch.zeros(nel, dtype=torch.float32, device=dev)
    cost1 = torch.full((N, K), -1.0, dtype=torch.float32, device=dev)
    cost2 = torch.full((N, K), -1.0, dtype=torch.float32, device=dev)
    rp, cp = torch.cat(rps).to(dev), torch.cat(cps).to(dev)
    plan.gather_cost_all(dm, rp, cp, None, cost1, ws)
    plan.gather_all(dm, rp, cp, w_re, s_re, ws)
    plan.cost_table_all(w_re, s_re, cost2, ws)
    torch.cuda.synchronize()
    refs = []
    for (W, S), r_, c_ in zip(mats, rps, cps):
        Wp, Sp = orc.gather(to_np_bf16(W), S.numpy(), r_.numpy(), c_.numpy())
        refs.append(orc.cost_table(Wp, Sp, m, n, bits, power=1))
    ref = np.concatenate(refs, 0)
    np.testing.assert_array_equal(cost1.cpu().numpy(), ref)
    np.testing.assert_array_equal(cost2.cpu().numpy(), ref)
    plan.close()


def test_power_one_variant_search(orc, ctx_l1, dev):
    say("l1 variant: whole search")
    shapes = [(512, 512), (256, 1024), (1024, 256)]
    mats = [synth.make_matrix("student_t", r, c, seed=4, tid=i) for i, (r, c) in enumerate(shapes)]
    ref = oracle_search(orc, mats, 64, 128, [1, 2, 3, 4, 8], 2.5, power=1)
    rc, st, o, shp = gpu_search(ctx_l1, dev, mats, 64, 128, [1, 2, 3, 4, 8], 2.5)
    compare_search(orc, ref, rc, st, o, shp, 64)
    ref2 = oracle_search(orc, mats, 64, 128, [1, 2, 3, 4, 8], 2.5)
    assert not np.array_equal(ref["level"], ref2["level"])          # the two costs do allocate differently
