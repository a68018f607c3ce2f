"""The entry point that allocates nothing (sbits_offsets_static) against sbits_offsets, through the
C-ABI: two calls in a row on one GPU, the second on a smaller plan, so that whatever the first call
left in the library's fixed scratch array must not show.  Bar: int64 offsets bit-exact; the oracle's
offsets are compared as well."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2602_17698_amd import binding as sb

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


def _one(ctx, dev, orc, shapes, m, n, bits, seed):
    plan = sb.Plan(ctx, shapes, m, n, bits)
    N = plan.num_blocks()
    say("offsets_static", shapes[0], "x", len(shapes), "blocks", N, "bits", bits)
    ws = torch.empty(plan.workspace_bytes(), dtype=torch.uint8, device=dev)
    level = np.random.default_rng(seed).integers(0, len(bits), size=N).astype(np.uint8)
    level_d = torch.from_numpy(level).to(dev)
    ref_d = torch.full((N + 1,), -1, dtype=torch.int64, device=dev)
    out_d = torch.full((N + 1,), -2, dtype=torch.int64, device=dev)
    plan.offsets(level_d, ref_d, ws)
    free_before = torch.cuda.mem_get_info()[0]
    plan.offsets_static(level_d, out_d)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before          # nothing was allocated on the device
    ref, out = ref_d.cpu().numpy(), out_d.cpu().numpy()
    np.testing.assert_array_equal(out, ref)
    np.testing.assert_array_equal(out, orc.offsets(level, m, n, bits))
    plan.close()


def test_offsets_static_matches_offsets_twice_in_a_row(orc):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    sb.load()
    dev = torch.device("cuda:0")
    ctx = sb.Context(device=0, stream=torch.cuda.current_stream().cuda_stream)
    try:
        # 1,048,576 blocks = 512 scan tiles (several rounds of the middle kernel), then 1,500 blocks
        # (one ragged tile) on the same GPU's array
        _one(ctx, dev, orc, [(8192, 8192)] * 1, 8, 8, [0, 1, 2, 3, 4, 8], seed=1)
        _one(ctx, dev, orc, [(8 * 60, 8 * 25)], 8, 8, [2, 3, 4], seed=2)
    finally:
        ctx.close()


def test_offsets_static_rejects_plans_beyond_its_array(orc):
    sb.load()
    host = sb.Context(device=-1)
    try:
        # 9,437,184 blocks: a valid plan (limit 2^24), beyond the fixed array's 8,388,608
        plan = sb.Plan(host, [(8 * 1536, 8 * 768)] * 8, 8, 8, [2, 4])
        assert plan.num_blocks() > sb.OFFSETS_STATIC_MAX_BLOCKS
        with pytest.raises(sb.SbitsError) as e:
            plan.offsets_static(1 << 20, 1 << 21)                # never dereferenced
        assert e.value.status == sb.ERR_WORKSPACE
        plan.close()
    finally:
        host.close()
