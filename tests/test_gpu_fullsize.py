"""GPU parity at the workload sizes, in the launch configuration bench.py times (the batched
entry points through sbits_search).

* one Llama-3-8B-shaped decoder layer (7 matrices, 218 M weights): every output against the
  oracle, element by element;
* the full 32-layer 8B-shaped model (224 matrices, 6.98 G weights, as in bench.py): every
  matrix through the per-matrix stages of the oracle (one process per matrix over the host's
  cores), the allocation and the offsets on the whole cost table, the packed output of every
  matrix.
"""
import os
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


def run_search(dev, mats_dev, shapes, m, n, bits, avg):
    ctx = sb.Context(0, torch.cuda.current_stream().cuda_stream)
    plan = sb.Plan(ctx, shapes, m, n, bits)
    N, K = plan.num_blocks(), len(bits)
    nel = sum(r * c for r, c in shapes)
    ws = torch.empty(plan.workspace_bytes(), dtype=torch.uint8, device=dev)
    one_pass = plan.gather_cost_supported()              # then the reordered sensitivities are never written
    o = dict(
        row_perm=torch.empty(sum(r for r, _ in shapes), dtype=torch.int32, device=dev),
        col_perm=torch.empty(sum(c for _, c in shapes), dtype=torch.int32, device=dev),
        w_re=torch.empty(nel, dtype=torch.bfloat16, device=dev),
        s_re=None if one_pass else torch.empty(nel, dtype=torch.float32, device=dev),
        cost=torch.empty(N, K, dtype=torch.float32, device=dev),
        level=torch.empty(N, dtype=torch.uint8, device=dev),
        byte_off=torch.empty(N + 1, dtype=torch.int64, device=dev),
        codes=torch.zeros(plan.codes_bytes_bound(avg), dtype=torch.uint8, device=dev),
        scale=torch.empty(N * m, dtype=torch.float32, device=dev),
        zero=torch.empty(N * m, dtype=torch.float32, device=dev),
    )
    out = sb.Outputs(o["row_perm"].data_ptr(), o["col_perm"].data_ptr(), o["w_re"].data_ptr(),
                     None if one_pass else o["s_re"].data_ptr(),
                     o["cost"].data_ptr(), o["level"].data_ptr(), o["byte_off"].data_ptr(), o["codes"].data_ptr(),
                     o["codes"].numel(), o["scale"].data_ptr(), o["zero"].data_ptr())
    rc, st = plan.search([sb.matrix(w, s) for w, s in mats_dev], avg, out, ws)
    torch.cuda.synchronize()
    bases = [plan.block_base(i) for i in range(len(shapes))]
    plan.close()
    ctx.close()
    return rc, st, o, bases


def check_matrix(orc, o, shapes, bases, idx, W, S, m, n, bits, level, off):
    """Per-matrix stages of matrix `idx` against the oracle; level/off are the global arrays."""
    R, C = shapes[idx]
    ro = sum(r for r, _ in shapes[:idx])
    co = sum(c for _, c in shapes[:idx])
    eo = sum(r * c for r, c in shapes[:idx])
    Wn, Sn = synth.bf16_bits(W), S.cpu().numpy()
    rs, cs = orc.channel_scores(Sn)
    rp, cp = orc.argsort_desc(rs), orc.argsort_desc(cs)
    np.testing.assert_array_equal(o["row_perm"][ro:ro + R].cpu().numpy(), rp)
    np.testing.assert_array_equal(o["col_perm"][co:co + C].cpu().numpy(), cp)
    Wp, Sp = orc.gather(Wn, Sn, rp, cp)
    np.testing.assert_array_equal(synth.bf16_bits(o["w_re"][eo:eo + R * C]).reshape(R, C), Wp)
    if o["s_re"] is not None:
        np.testing.assert_array_equal(o["s_re"][eo:eo + R * C].cpu().numpy().reshape(R, C), Sp)
    cost = orc.cost_table(Wp, Sp, m, n, bits)
    nb = cost.shape[0]
    b0 = bases[idx]
    np.testing.assert_array_equal(o["cost"][b0:b0 + nb].cpu().numpy(), cost)
    # pack this matrix with the global levels / offsets into a private copy of its byte range
    lo, hi = int(off[b0]), int(off[b0 + nb])
    codes = np.zeros(int(off[-1]), np.uint8) if int(off[-1]) < (1 << 28) else None
    if codes is None:                                    # large stream: pack into a window
        shifted = off - lo
        codes = np.zeros(hi - lo, np.uint8)
        scale = np.zeros(level.size * m, np.float32)
        zero = np.zeros(level.size * m, np.float32)
        orc.pack(Wp, m, n, bits, level, shifted, b0, codes, scale, zero)
        ref_codes = codes
    else:
        scale = np.zeros(level.size * m, np.float32)
        zero = np.zeros(level.size * m, np.float32)
        orc.pack(Wp, m, n, bits, level, off, b0, codes, scale, zero)
        ref_codes = codes[lo:hi]
    np.testing.assert_array_equal(o["codes"][lo:hi].cpu().numpy(), ref_codes)
    np.testing.assert_array_equal(o["scale"][b0 * m:(b0 + nb) * m].cpu().numpy(), scale[b0 * m:(b0 + nb) * m])
    np.testing.assert_array_equal(o["zero"][b0 * m:(b0 + nb) * m].cpu().numpy().view(np.uint32),
                                  zero[b0 * m:(b0 + nb) * m].view(np.uint32))


def test_one_decoder_layer(orc):
    """One Llama-3-8B-shaped decoder layer: q/o 4096x4096, k/v 1024x4096, gate/up 14336x4096,
    down 4096x14336; Student-t(4) weights x0.02, log-normal sensitivity; 128x128 blocks; {2,3,4}; budget 3.0."""
    say("config 2: one decoder layer")
    dev = torch.device("cuda:0")
    m = n = 128
    bits, avg = [2, 3, 4], 3.0
    layer = synth.make_layer(synth.LLAMA3_8B, 0, "student_t", seed=0, device=dev)
    shapes = [tuple(w.shape) for _, w, _ in layer]
    rc, st, o, bases = run_search(dev, [(w, s) for _, w, s in layer], shapes, m, n, bits, avg)
    cost = o["cost"].cpu().numpy()
    rc_o, level, st_o, _ = orc.allocate(cost, bits, avg)
    assert rc == rc_o and st == st_o
    np.testing.assert_array_equal(o["level"].cpu().numpy(), level)
    off = orc.offsets(level, m, n, bits)
    np.testing.assert_array_equal(o["byte_off"].cpu().numpy(), off)
    for idx in range(len(shapes)):                       # every matrix of the layer
        say("  matrix", layer[idx][0], shapes[idx])
        check_matrix(orc, o, shapes, bases, idx, layer[idx][1], layer[idx][2], m, n, bits, level, off)
    assert st["bits_used"] <= st["bits_budget"] == int(avg * cost.shape[0])


def _bounded(tasks, sem):
    """Hands tasks to a pool's feeder thread, at most as many ahead of the results as the semaphore allows."""
    for t in tasks:
        sem.acquire()
        yield t


def test_full_model_every_matrix(orc):
    """Full 32-layer 8B-shaped model, {1,2,3,4} bits, global budgets 2.5 and 3.0, all on the device -- and
    EVERY one of its 224 matrices through the oracle: one single-threaded oracle call chain per matrix, spread
    over the host's cores (oracle/parallel.py).  Compared element by element: both permutations and the cost
    rows of every matrix, levels and offsets on the whole table, scales and zeros of every matrix; the packed
    codes of every matrix by a digest of their bytes."""
    import threading
    from oracle import parallel as par
    dev = torch.device("cuda:0")
    m = n = 128
    bits = [1, 2, 3, 4]
    names, mats, shapes = [], [], []
    for layer in range(32):
        for name, r, c in synth.layer_shapes(synth.LLAMA3_8B):
            w, s = synth.make_matrix("student_t", r, c, seed=0, tid=synth.tensor_id(layer, name), device=dev)
            names.append((layer, name)); mats.append((w, s)); shapes.append((r, c))
    nm = len(shapes)
    ro = np.concatenate([[0], np.cumsum([r for r, _ in shapes])])
    co = np.concatenate([[0], np.cumsum([c for _, c in shapes])])
    workers = par.cores()
    say("config 3: full model, %d matrices, oracle on %d host cores (os.cpu_count() = %s)" % (nm, workers, os.cpu_count()))

    runs = {}
    for avg in (2.5, 3.0):
        rc, st, o, bases = run_search(dev, mats, shapes, m, n, bits, avg)
        o.pop("w_re"); o.pop("s_re")
        runs[avg] = (rc, st, {k: (v.cpu().numpy() if k != "codes" else v) for k, v in o.items()}, bases)
    o25, bases = runs[2.5][2], runs[2.5][3]
    cost = o25["cost"]
    assert cost.shape == (425984, 4) and np.all(np.isfinite(cost)) and np.all(cost >= 0)
    assert np.all(np.diff(cost, axis=1) < 0)             # more bits, less error, on this distribution
    for key in ("row_perm", "col_perm", "cost"):         # the stages before the allocation do not see the budget
        np.testing.assert_array_equal(runs[3.0][2][key].view(np.uint32), o25[key].view(np.uint32))

    shm = par.SharedInputs()
    sem = threading.Semaphore(2 * workers)
    pool = par.pool(workers)
    try:
        # ---- stage A: permutations and cost rows of every matrix
        def tasks_a():
            for i, (r, c) in enumerate(shapes):
                wn = shm.put(("w", i), synth.bf16_bits(mats[i][0]))
                sn = shm.put(("s", i), mats[i][1].cpu().numpy())
                yield (i, wn, sn, r, c, m, n, bits, 2)
        perms = [None] * nm
        done = 0
        for i, rp, cp, rows in pool.imap_unordered(par.stage_a, _bounded(tasks_a(), sem)):
            shm.free(("w", i)); shm.free(("s", i)); sem.release()
            r, c = shapes[i]
            np.testing.assert_array_equal(o25["row_perm"][ro[i]:ro[i] + r], rp, err_msg="row_perm of %s" % (names[i],))
            np.testing.assert_array_equal(o25["col_perm"][co[i]:co[i] + c], cp, err_msg="col_perm of %s" % (names[i],))
            np.testing.assert_array_equal(cost[bases[i]:bases[i] + rows.shape[0]].view(np.uint32), rows.view(np.uint32),
                                          err_msg="cost rows of %s" % (names[i],))
            perms[i] = (rp, cp)
            done += 1
            if done % 56 == 0:
                say("  stage A: %d of %d matrices equal" % (done, nm))
        assert done == nm
        # ---- per budget: allocation and offsets on the whole table, then stage B for every matrix
        for avg in (2.5, 3.0):
            rc, st, o, _ = runs[avg]
            rc_o, level, st_o, _ = orc.allocate(cost, bits, avg)
            assert rc == rc_o == 0 and st == st_o
            np.testing.assert_array_equal(o["level"], level)
            assert st["bits_used"] <= st["bits_budget"] == int(avg * 425984)
            off = orc.offsets(level, m, n, bits)
            np.testing.assert_array_equal(o["byte_off"], off)

            def tasks_b():
                for i, (r, c) in enumerate(shapes):
                    wn = shm.put(("w", i), synth.bf16_bits(mats[i][0]))
                    nb = (r // m) * (c // n)
                    yield (i, wn, r, c, m, n, bits, perms[i][0], perms[i][1], level[bases[i]:bases[i] + nb])
            done = 0
            for i, dg, nbytes, scale, zero in pool.imap_unordered(par.stage_b, _bounded(tasks_b(), sem)):
                shm.free(("w", i)); sem.release()
                r, c = shapes[i]
                b0, nb = bases[i], (r // m) * (c // n)
                lo, hi = int(off[b0]), int(off[b0 + nb])
                assert hi - lo == nbytes
                assert par.digest(o["codes"][lo:hi].cpu().numpy()) == dg, "codes of %s at budget %s" % (names[i], avg)
                np.testing.assert_array_equal(o["scale"][b0 * m:(b0 + nb) * m].view(np.uint32), scale.view(np.uint32))
                np.testing.assert_array_equal(o["zero"][b0 * m:(b0 + nb) * m].view(np.uint32), zero.view(np.uint32))
                done += 1
            assert done == nm
            say("  budget %.1f: levels, offsets and the packed output of all %d matrices equal" % (avg, nm))
    finally:
        pool.terminate()
        pool.join()
        shm.free_all()


def test_outlier_channel_model_small_blocks(orc):
    """8B-shaped model, 64x64 blocks (group 64), {1,2,3,4,8} bits, Student-t(3) weights with rare x100
    outlier channels scattered per matrix, budget 2.25: uneven candidate steps, K = 5."""
    say("config 5: 64x64 blocks, K = 5, outlier channels")
    dev = torch.device("cuda:0")
    m = n = 64
    bits, avg = [1, 2, 3, 4, 8], 2.25
    names, mats, shapes = [], [], []
    for layer in range(32):
        for name, r, c in synth.layer_shapes(synth.LLAMA3_8B):
            w, s = synth.make_matrix("outlier_chan", r, c, seed=0, tid=synth.tensor_id(layer, name), device=dev)
            names.append((layer, name)); mats.append((w, s)); shapes.append((r, c))
    rc, st, o, bases = run_search(dev, mats, shapes, m, n, bits, avg)
    cost = o["cost"].cpu().numpy()
    assert cost.shape == (1703936, 5) and np.all(np.isfinite(cost)) and np.all(cost >= 0)
    rc_o, level, st_o, _ = orc.allocate(cost, bits, avg)
    assert rc == rc_o == 0 and st == st_o
    np.testing.assert_array_equal(o["level"].cpu().numpy(), level)
    assert st["bits_used"] <= st["bits_budget"] == int(avg * 1703936)
    off = orc.offsets(level, m, n, bits)
    np.testing.assert_array_equal(o["byte_off"].cpu().numpy(), off)
    # reordering moves the outlier channels to the top-left: the first block row / column of a
    # matrix gets more bits than the rest
    idx = names.index((3, "q"))
    lv = level[bases[idx]:bases[idx] + 64 * 64].reshape(64, 64).astype(np.float64)
    assert lv[0].mean() > lv[1:].mean() and lv[:, 0].mean() > lv[:, 1:].mean()
    for layer, name in [(0, "v"), (16, "o"), (31, "k")]:
        idx = names.index((layer, name))
        say("  sampled", layer, name, shapes[idx])
        check_matrix(orc, o, shapes, bases, idx, mats[idx][0], mats[idx][1], m, n, bits, level, off)


def test_streamed_70b_shaped_model(orc):
    """80-layer Llama-3-70B-shaped model (hidden 8192, ffn 28672, 8 KV heads of 128): 410 GB of inputs
    do not fit, so weights and sensitivities are regenerated per layer on the device from the seed;
    128x128 blocks, {2,3,4} bits, budget 2.75.  One per-layer plan serves the per-matrix stages of
    every layer (pointer offsets place its outputs in the global arrays) through the calls the search
    itself uses (sbits_gather_cost_all, sbits_gather_pack_all); only permutations and
    the cost table are kept, the global allocation runs on the full table, and a second streaming
    pass packs.  Layers 0, 40 and 79 are checked against the oracle."""
    say("config 4: streamed 70B-shaped model")
    dev = torch.device("cuda:0")
    m = n = 128
    bits, avg = [2, 3, 4], 2.75
    K = len(bits)
    model = synth.LLAMA3_70B
    lshapes = [(r, c) for _, r, c in synth.layer_shapes(model)]
    L = model["layers"]
    ctx = sb.Context(0, torch.cuda.current_stream().cuda_stream)
    lplan = sb.Plan(ctx, lshapes, m, n, bits)                    # one layer
    gplan = sb.Plan(ctx, lshapes * L, m, n, bits)                # the whole model: allocation, offsets
    NL, N = lplan.num_blocks(), gplan.num_blocks()
    assert NL == 52224 and N == 4177920
    lws = torch.empty(lplan.workspace_bytes(), dtype=torch.uint8, device=dev)
    gws = torch.empty(gplan.workspace_bytes(), dtype=torch.uint8, device=dev)
    nel = sum(r * c for r, c in lshapes)
    sum_r, sum_c = sum(r for r, _ in lshapes), sum(c for _, c in lshapes)
    row_perm = torch.empty(L * sum_r, dtype=torch.int32, device=dev)
    col_perm = torch.empty(L * sum_c, dtype=torch.int32, device=dev)
    cost = torch.empty(N, K, dtype=torch.float32, device=dev)
    w_re = torch.empty(nel, dtype=torch.bfloat16, device=dev)
    s_re = torch.empty(nel, dtype=torch.float32, device=dev)
    check_layers = (0, 40, 79)
    kept = {}

    def gen(layer):
        return [synth.make_matrix("student_t", r, c, seed=0, tid=synth.tensor_id(layer, nm), device=dev)
                for nm, r, c in synth.layer_shapes(model)]

    for layer in range(L):                                       # pass 1: permutations + cost rows
        mats = gen(layer)
        dm = [sb.matrix(w, s) for w, s in mats]
        rp = row_perm[layer * sum_r:(layer + 1) * sum_r]
        cp = col_perm[layer * sum_c:(layer + 1) * sum_c]
        lplan.reorder_all(dm, rp, cp, lws)
        lcost = cost[layer * NL:(layer + 1) * NL]
        # the product's route: one pass over the originals for the six matrices whose rows fit in LDS,
        # the reordered copy in the workspace for `down` (28672 columns)
        lplan.gather_cost_all(dm, rp, cp, None, lcost, lws)
        if layer in check_layers:
            # ... and the two-pass route beside it: the same table, and the reordered copies for the oracle check
            cost2 = torch.empty_like(lcost)
            lplan.gather_all(dm, rp, cp, w_re, s_re, lws)
            lplan.cost_table_all(w_re, s_re, cost2, lws)
            torch.cuda.synchronize()
            assert torch.equal(cost2.view(torch.int32), lcost.view(torch.int32))
            kept[layer] = dict(w_re=w_re.clone(), s_re=s_re.clone())
            del cost2
        torch.cuda.synchronize()
        del mats, dm
        if layer % 10 == 0:
            say("  pass 1 layer", layer)
    level = torch.empty(N, dtype=torch.uint8, device=dev)
    rc, st, _ = gplan.allocate(cost, avg, level, gws)
    byte_off = torch.empty(N + 1, dtype=torch.int64, device=dev)
    gplan.offsets(level, byte_off, gws)
    torch.cuda.synchronize()
    cost_h = cost.cpu().numpy()
    say("  oracle allocation on", N, "blocks")
    rc_o, level_o, st_o, _ = orc.allocate(cost_h, bits, avg)
    assert rc == rc_o == 0 and st == st_o
    np.testing.assert_array_equal(level.cpu().numpy(), level_o)
    off = orc.offsets(level_o, m, n, bits)
    np.testing.assert_array_equal(byte_off.cpu().numpy(), off)
    assert st["bits_used"] <= st["bits_budget"] == 11489280

    codes = torch.zeros(int(off[-1]), dtype=torch.uint8, device=dev)
    scale = torch.empty(N * m, dtype=torch.float32, device=dev)
    zero = torch.empty(N * m, dtype=torch.float32, device=dev)
    for layer in range(L):                                       # pass 2: regenerate, reorder, pack
        mats = gen(layer)
        dm = [sb.matrix(w, s) for w, s in mats]
        rp = row_perm[layer * sum_r:(layer + 1) * sum_r]
        cp = col_perm[layer * sum_c:(layer + 1) * sum_c]
        b0 = layer * NL
        lplan.gather_pack_all(dm, rp, cp, level[b0:], byte_off[b0:], codes, scale[b0 * m:], zero[b0 * m:], lws)
        torch.cuda.synchronize()
        if layer in check_layers:
            say("  checking layer", layer)
            o = dict(row_perm=rp, col_perm=cp, w_re=kept[layer]["w_re"], s_re=kept[layer]["s_re"],
                     cost=cost[b0:b0 + NL], codes=codes, scale=scale[b0 * m:], zero=zero[b0 * m:])
            lbases = [lplan.block_base(i) for i in range(7)]
            # the layer's slice of the global levels / offsets, as the layer plan sees them
            lvl = level_o[b0:b0 + NL]
            loff = off[b0:b0 + NL + 1]
            for idx in (1, 3, 6):                                # k (1024x8192), o (8192x8192), down (8192x28672)
                check_matrix(orc, o, lshapes, lbases, idx, mats[idx][0], mats[idx][1], m, n, bits, lvl, loff)
        del mats, dm
    lplan.close(); gplan.close(); ctx.close()


def test_coupled_reordering_four_layers(orc):
    """Four 8B-shaped decoder layers with the Llama coupling: the residual stream couples 28
    dimensions of 4096 channels, each MLP 3 dimensions of 14336, each attention block the 1024 value
    rows with the 4096 output columns head by head (4 query heads per value head); against the
    oracle's summed scores."""
    say("coupled reordering, 4 layers of the 8B shape")
    dev = torch.device("cuda:0")
    L = 4
    model = synth.LLAMA3_8B
    shapes, mats = [], []
    for layer in range(L):
        for name, r, c in synth.layer_shapes(model):
            _, s = synth.make_matrix("student_t", r, c, seed=0, tid=synth.tensor_id(layer, name), device=dev)
            shapes.append((r, c)); mats.append(s)
    rg, cg, ng, seg, rrep, crep = synth.llama_coupling(model, L)
    ctx = sb.Context(0, torch.cuda.current_stream().cuda_stream)
    plan = sb.Plan(ctx, shapes, 128, 128, [2, 3, 4])
    ws = torch.empty(plan.workspace_bytes(), dtype=torch.uint8, device=dev)
    rp = torch.empty(sum(r for r, _ in shapes), dtype=torch.int32, device=dev)
    cp = torch.empty(sum(c for _, c in shapes), dtype=torch.int32, device=dev)
    dm = [sb.matrix(None, s) for s in mats]
    plan.reorder_coupled_all(dm, rg, cg, ng, seg, rp, cp, ws, rrep, crep)
    torch.cuda.synchronize()
    t0 = torch.cuda.Event(enable_timing=True); t1 = torch.cuda.Event(enable_timing=True)
    t0.record(); plan.reorder_coupled_all(dm, rg, cg, ng, seg, rp, cp, ws, rrep, crep); t1.record()
    torch.cuda.synchronize()
    say("  coupled reorder of 4 layers: %.2f ms" % t0.elapsed_time(t1))
    rp, cp = rp.cpu().numpy(), cp.cpu().numpy()
    scores = [orc.channel_scores(s.cpu().numpy()) for s in mats]
    members = {}
    for which, groups, reps in ((0, rg, rrep), (1, cg, crep)):
        for i, g in enumerate(groups):
            if g < 0: continue
            sc = scores[i][which]
            members.setdefault(g, []).extend([sc] if reps[i] == 1 else orc.fold_repeated(sc, seg[g], reps[i]))
    assert len(members[0]) == 7 * L
    assert all(len(members[1 + 2 * l]) == 3 and len(members[2 + 2 * l]) == 1 + 4 for l in range(L))
    gperm = {g: orc.coupled_perm(m, seg[g]) for g, m in members.items()}
    ro = co = 0
    for i, (r, c) in enumerate(shapes):
        for got, g, n, rep in ((rp[ro:ro + r], rg[i], r, rrep[i]), (cp[co:co + c], cg[i], c, crep[i])):
            if g == -2:
                want = np.arange(n, dtype=np.int32)
            else:
                want = gperm[g] if rep == 1 else orc.expand_perm(gperm[g], seg[g], rep)
            np.testing.assert_array_equal(got, want)
        ro, co = ro + r, co + c
    plan.close(); ctx.close()


@pytest.mark.parametrize("bits,avg", [([1, 2, 3, 4, 5, 6, 7, 8], 3.0), ([0, 1, 2, 3, 4, 5, 6, 7, 8], 2.0)])
def test_paper_default_search_space(orc, bits, avg):
    """Two 8B-shaped decoder layers in the paper's own search space (Sec. 5 "Implementation"):
    64 x 128 blocks, group size 128, bitwidths {1,...,8}, budget 3.0; and the widest space of the
    search-space ablation (App. "impact of precision search space"): {0,...,8}, 0 = pruned, budget 2.0."""
    say("paper-default search space: 64x128 blocks, bits", bits)
    dev = torch.device("cuda:0")
    m, n = 64, 128
    K = len(bits)
    mats, shapes = [], []
    for layer in range(2):
        for name, r, c in synth.layer_shapes(synth.LLAMA3_8B):
            w, s = synth.make_matrix("student_t", r, c, seed=0, tid=synth.tensor_id(layer, name), device=dev)
            mats.append((w, s)); shapes.append((r, c))
    rc, st, o, bases = run_search(dev, mats, shapes, m, n, bits, avg)
    cost = o["cost"].cpu().numpy()
    real = cost[:, 1:] if bits[0] == 0 else cost             # (a heavy-tailed row's 1-bit grid may cost more than pruning)
    assert cost.shape == (2 * 26624, K) and np.all(np.isfinite(cost)) and np.all(np.diff(real, axis=1) < 0)
    rc_o, level, st_o, _ = orc.allocate(cost, bits, avg)
    assert rc == rc_o == 0 and st == st_o
    np.testing.assert_array_equal(o["level"].cpu().numpy(), level)
    off = orc.offsets(level, m, n, bits)
    np.testing.assert_array_equal(o["byte_off"].cpu().numpy(), off)
    assert st["bits_used"] <= st["bits_budget"] == int(avg * cost.shape[0])
    assert len(np.unique(level)) >= 4                         # a real mixture of bitwidths
    for idx in (1, 3, 13):                                    # k of layer 0, o of layer 0, down of layer 1
        say("  matrix", idx, shapes[idx])
        check_matrix(orc, o, shapes, bases, idx, mats[idx][0], mats[idx][1], m, n, bits, level, off)


def test_dynamic_iteration_full_model(orc):
    """One iteration of the paper's own loop on the 8B-shaped model (Alg. 2 lines 4-10 with fresh
    estimates): surrogates from a signed gradient at the current levels, then the proposal.  Sampled
    matrices' surrogates against the oracle; the proposal against the oracle's step on the (GPU-made)
    full surrogate arrays; both an expansion and a swap."""
    say("dynamic iteration, full 8B-shaped model")
    dev = torch.device("cuda:0")
    m = n = 128
    bits = [1, 2, 3, 4]
    names, mats, shapes = [], [], []
    for layer in range(32):
        for name, r, c in synth.layer_shapes(synth.LLAMA3_8B):
            w, s = synth.make_matrix("student_t", r, c, seed=0, tid=synth.tensor_id(layer, name), device=dev)
            names.append((layer, name)); mats.append((w, s)); shapes.append((r, c))
    ctx = sb.Context(0, torch.cuda.current_stream().cuda_stream)
    plan = sb.Plan(ctx, shapes, m, n, bits)
    N = plan.num_blocks()
    ws = torch.empty(plan.workspace_bytes(), dtype=torch.uint8, device=dev)
    rp = torch.empty(sum(r for r, _ in shapes), dtype=torch.int32, device=dev)
    cp = torch.empty(sum(c for _, c in shapes), dtype=torch.int32, device=dev)
    dm = [sb.matrix(w, s) for w, s in mats]
    plan.reorder_all(dm, rp, cp, ws)
    torch.cuda.synchronize()
    for _, s in mats:                                    # the "gradient": the sensitivity with a sign per element
        r, c = s.shape
        sign = ((torch.arange(r, device=dev)[:, None] * 7 + torch.arange(c, device=dev)[None, :] * 13) % 5 < 2)
        s.mul_(torch.where(sign, -1.0, 1.0))
    rng = np.random.default_rng(5)
    level_h = rng.integers(0, 4, N).astype(np.uint8)
    level = torch.from_numpy(level_h).to(dev)
    s_up = torch.empty(N, dtype=torch.float32, device=dev)
    s_dn = torch.empty(N, dtype=torch.float32, device=dev)
    prop = torch.empty_like(level)
    used = int(np.asarray(bits)[level_h].sum())
    k = int(0.05 * N)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for avg, want_kind in ((used / N + 1e-9, 2), ((used + 3 * k) / N + 1e-9, 1)):
        for rep in range(2):                             # second round timed
            ev[0].record()
            plan.surrogates_all(dm, rp, cp, level, s_up, s_dn, ws)
            ev[1].record()
            info = plan.propose(s_up, s_dn, level, avg, k, prop, ws)
            ev[2].record()
            torch.cuda.synchronize()
        say("  surrogates %.2f ms, proposal %.2f ms (kind %d, %d up, %d down)" % (
            ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2]), info["kind"], info["n_up"], info["n_dn"]))
        su, sd = s_up.cpu().numpy(), s_dn.cpu().numpy()
        assert np.all(np.isfinite(su)) and np.all(sd >= 0)
        kind, want, winfo = orc.propose(su, sd, level_h, bits, avg, k)
        assert kind == info["kind"] == want_kind
        np.testing.assert_array_equal(prop.cpu().numpy(), want)
        assert all(info[f] == winfo[f] for f in winfo)
        assert info["bits_after"] <= max(info["bits_budget"], used)
        # the same iteration without asking for the outcome: both calls only enqueue (the proposal does not wait
        # for the stream, hence not for the estimate pass before it), the host is back long before the device
        # is done, and the levels proposed are the same
        import time
        prop2 = torch.full_like(prop, 255)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev[0].record()
        plan.surrogates_all(dm, rp, cp, level, s_up, s_dn, ws)
        assert plan.propose(s_up, s_dn, level, avg, k, prop2, ws, want_info=False) is None
        ev[2].record()
        host_ms = (time.perf_counter() - t0) * 1e3
        torch.cuda.synchronize()
        dev_ms = ev[0].elapsed_time(ev[2])
        say("  back to back without a read-back: host returns after %.2f ms, device busy %.2f ms" % (host_ms, dev_ms))
        assert host_ms < 0.5 * dev_ms
        np.testing.assert_array_equal(prop2.cpu().numpy(), want)
    rph, cph = rp.cpu().numpy(), cp.cpu().numpy()
    for layer, name in [(0, "k"), (15, "v"), (31, "k")]:
        idx = names.index((layer, name))
        say("  sampled surrogates", layer, name)
        R, C = shapes[idx]
        ro, co = sum(r for r, _ in shapes[:idx]), sum(c for _, c in shapes[:idx])
        Wp, Gp = orc.gather(synth.bf16_bits(mats[idx][0]), mats[idx][1].cpu().numpy(), rph[ro:ro + R], cph[co:co + C])
        b0, nb = plan.block_base(idx), (R // m) * (C // n)
        u, d = orc.surrogates(Wp, Gp, m, n, bits, level_h[b0:b0 + nb])
        np.testing.assert_array_equal(su[b0:b0 + nb], u)
        np.testing.assert_array_equal(sd[b0:b0 + nb], d)
    plan.close(); ctx.close()


@pytest.mark.parametrize("mix", [(0.0, 1.0, 0.0), (0.4, 0.4, 0.2)])
def test_mp_gemm_llm_scale_projection(orc, mix):
    """The paper's kernel workload (Sec. 5.3, kernel-latency table): an 8192 x 8192 projection at 4 bits on
    average, all INT4 or 40 % INT2 / 40 % INT4 / 20 % INT8 tiles, batch 16 and 32.  Packed on the device by
    the library's own packing kernel; sampled output channels against the oracle's float64 product."""
    say("mixed-precision product, 8192 x 8192, mix", mix)
    dev = torch.device("cuda:0")
    R = C = 8192
    m = n = 128
    bits = [2, 4, 8]
    ctx = sb.Context(0, torch.cuda.current_stream().cuda_stream)
    plan = sb.Plan(ctx, [(R, C)], m, n, bits)
    N = plan.num_blocks()
    ws = torch.empty(plan.workspace_bytes(), dtype=torch.uint8, device=dev)
    W, _ = synth.make_matrix("student_t", R, C, seed=0, tid=0, device=dev)
    rng = np.random.default_rng(0)
    counts = [int(round(f * N)) for f in mix]
    counts[1] += N - sum(counts)
    level_h = rng.permutation(np.repeat(np.arange(3, dtype=np.uint8), counts))
    assert abs(float(np.asarray(bits)[level_h].mean()) - 4.0) < 1e-3
    level = torch.from_numpy(level_h).to(dev)
    off = torch.empty(N + 1, dtype=torch.int64, device=dev)
    plan.offsets(level, off, ws)
    torch.cuda.synchronize()
    total = int(off[-1].item())
    codes = torch.zeros(total, dtype=torch.uint8, device=dev)
    scale = torch.empty(N * m, dtype=torch.float32, device=dev)
    zero = torch.empty(N * m, dtype=torch.float32, device=dev)
    plan.pack_all(W.reshape(-1), level, off, codes, scale, zero, ws)
    torch.cuda.synchronize()
    packed_bytes = total + 2 * 4 * N * m
    # the stored matrix as numbers: every output of the product is checked against a dense fp32 product with it
    What = torch.empty(R, C, dtype=torch.float32, device=dev)
    plan.dequant(0, level, off, codes, scale, zero, What)
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(5):
        plan.dequant(0, level, off, codes, scale, zero, What)
    t1.record()
    torch.cuda.synchronize()
    us = t0.elapsed_time(t1) / 5 * 1e3
    say("  dequantization to fp32: %.0f us (%.2f TB/s written)" % (us, R * C * 4 / us * 1e-6))
    for batch in (16, 32):
        x = torch.randn(batch, C, device=dev).to(torch.bfloat16)
        y = torch.empty(batch, R, dtype=torch.float32, device=dev)
        for _ in range(3):
            plan.mp_gemm(0, x, level, off, codes, scale, zero, y, ws)
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 50
        t0.record()
        for _ in range(reps):
            plan.mp_gemm(0, x, level, off, codes, scale, zero, y, ws)
        t1.record()
        torch.cuda.synchronize()
        us = t0.elapsed_time(t1) / reps * 1e3
        say("  batch %d: %.1f us per product, %.2f TB/s of packed weights (%.1f MB)" % (
            batch, us, packed_bytes / us * 1e-6, packed_bytes * 1e-6))
        # every output against a dense float64 product with the stored matrix, PER ELEMENT, with the bound of the
        # small cases: 2^-18 * sum_j (|what_ij| + 128 * scale of the element's block row) * |x_bj|  (the kernel sums
        # (128 + q) * x in fp32 and takes 128 * sum x out again)
        xd = x.double()
        dense = xd @ What.double().t()
        nbc = C // n
        srow = scale.view(R // m, nbc, m).permute(0, 2, 1).reshape(R, nbc).double().abs()     # [row][block column]
        bound = xd.abs() @ What.double().abs().t() + 128.0 * (xd.abs().view(batch, nbc, n).sum(2) @ srow.t())
        err = (y.double() - dense).abs()
        assert bool((err <= bound * 2.0 ** -18 + 1e-30).all()), float((err / (bound + 1e-300)).max())
        assert float((err ** 2).mean().sqrt()) <= 2.0 ** -22 * float((bound ** 2).mean().sqrt())
        # sampled block rows through the oracle: the oracle dequantizes whole matrices, so hand it the
        # sampled block rows as a matrix of their own (their blocks are consecutive in the global order)
        yh = y.cpu().numpy()
        xb = synth.bf16_bits(x)
        lv, of = level_h, off.cpu().numpy()
        nbc = C // n
        for I in (0, 37, 63):
            b0 = I * nbc
            sub_off = of[b0:b0 + nbc + 1] - of[b0]
            sub_codes = codes[int(of[b0]):int(of[b0 + nbc])].cpu().numpy()
            ref = orc.mp_gemm(sub_codes, scale[b0 * m:(b0 + nbc) * m].cpu().numpy(), zero[b0 * m:(b0 + nbc) * m].cpu().numpy(),
                              lv[b0:b0 + nbc], sub_off, 0, m, C, m, n, bits, xb)
            got = yh[:, I * m:(I + 1) * m].astype(np.float64)
            bnd = bound[:, I * m:(I + 1) * m].cpu().numpy()
            assert np.all(np.abs(got - ref) <= bnd * 2.0 ** -18 + 1e-30), (I, float((np.abs(got - ref) / (bnd + 1e-300)).max()))
    plan.close(); ctx.close()


def test_sweeps_of_the_search_space_behave_as_the_ablations_say(capsys):
    """`python -m paper_2602_17698_amd.sweep` on one decoder layer: every search meets its budget, and the
    orderings the paper's ablations report hold for the search's own objective: mixed precision beats uniform
    at the same budget, a wider candidate set is never worse, the update rate hardly matters on a static table."""
    say("sweep, one layer")
    from paper_2602_17698_amd import sweep
    import json
    assert sweep.main(["--layers", "1", "--json"]) == 0
    rows = [json.loads(l) for l in capsys.readouterr().out.splitlines() if l.startswith("{")]
    assert len(rows) >= 20 and all(r["status"] == 0 and r["bits_used"] <= r["bits_budget"] for r in rows)
    uni = next(r for r in rows if r["sweep"] == "uniform")["objective"]
    space = {tuple(r["bits"]): r["objective"] for r in rows if r["sweep"] == "space"}
    full, low4 = space[tuple(range(1, 9))], space[(1, 2, 3, 4)]
    assert full < low4 < uni                                   # capping the candidates at 4 bits costs
    assert space[tuple(range(0, 9))] <= full * 1.001           # adding 0 bits does not
    assert space[(3, 4, 5, 6, 7, 8)] == uni                    # nothing below 3 bits at budget 3: uniform
    g = [r["objective"] for r in rows if r["sweep"] == "gamma0"]
    assert max(g) <= min(g) * 1.01
