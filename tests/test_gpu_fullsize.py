"""GPU parity at the workload sizes, in the launch configuration bench.py times (the batched
entry points through sbits_search).

* one Llama-3-8B-shaped decoder layer (7 matrices, 218 M weights): every output against the
  oracle, element by element;
* the full 32-layer 8B-shaped model (224 matrices, 6.98 G weights, as in bench.py): sampled
  matrices through the per-matrix stages of the oracle, the allocation and the offsets on the
  whole (GPU-produced) cost table, packed codes of the sampled matrices.
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


def run_search(dev, mats_dev, shapes, m, n, bits, avg):
    ctx = sb.Context(0, torch.cuda.current_stream().cuda_stream)
    plan = sb.Plan(ctx, shapes, m, n, bits)
    N, K = plan.num_blocks(), len(bits)
    nel = sum(r * c for r, c in shapes)
    ws = torch.empty(plan.workspace_bytes(), dtype=torch.uint8, device=dev)
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


@pytest.mark.parametrize("avg", [2.5, 3.0])
def test_full_model_sampled(orc, avg):
    """Full 32-layer 8B-shaped model, {1,2,3,4} bits, global budget 2.5 / 3.0, all on the device."""
    say("config 3: full model, budget", avg)
    dev = torch.device("cuda:0")
    m = n = 128
    bits = [1, 2, 3, 4]
    names, mats, shapes = [], [], []
    for layer in range(32):
        for name, r, c in synth.layer_shapes(synth.LLAMA3_8B):
            w, s = synth.make_matrix("student_t", r, c, seed=0, tid=synth.tensor_id(layer, name), device=dev)
            names.append((layer, name)); mats.append((w, s)); shapes.append((r, c))
    rc, st, o, bases = run_search(dev, mats, shapes, m, n, bits, avg)
    cost = o["cost"].cpu().numpy()
    assert cost.shape == (425984, 4) and np.all(np.isfinite(cost)) and np.all(cost >= 0)
    # properties that hold at any size
    assert np.all(np.diff(cost, axis=1) < 0)             # more bits, less error, on this distribution
    rc_o, level, st_o, _ = orc.allocate(cost, bits, avg)
    assert rc == rc_o == 0 and st == st_o
    np.testing.assert_array_equal(o["level"].cpu().numpy(), level)
    assert st["bits_used"] <= st["bits_budget"] == int(avg * 425984)
    off = orc.offsets(level, m, n, bits)
    np.testing.assert_array_equal(o["byte_off"].cpu().numpy(), off)
    # permutations are bijections everywhere (cheap, on the device)
    ro = 0
    for R, _ in shapes[:14]:
        p = o["row_perm"][ro:ro + R]
        assert torch.equal(torch.sort(p).values, torch.arange(R, dtype=torch.int32, device=dev))
        ro += R
    # sampled matrices through the oracle: first / middle / last layer, small and large shapes
    for layer, name in [(0, "k"), (0, "q"), (15, "v"), (31, "down"), (31, "k")]:
        idx = names.index((layer, name))
        say("  sampled", layer, name, shapes[idx])
        check_matrix(orc, o, shapes, bases, idx, mats[idx][0], mats[idx][1], m, n, bits, level, off)
