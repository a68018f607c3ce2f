"""Host-only checks of the C-ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching a device (device = -1 context)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2602_17698_amd import binding as sb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sb.LIB_PATH):
        from paper_2602_17698_amd import build
        build.build()
    return sb.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "scalebits.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sbits_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert set(names) == set(sb.EXPORTS)
    for name in names:
        assert hasattr(lib, name), name


def test_build_variants_export_the_same_symbols_and_name_their_cost(lib):
    from paper_2602_17698_amd import build
    assert sb.cost_power() == 2
    path = sb.variant_path("l1")
    if not os.path.exists(path):
        build.build(variant="l1")
    l1 = C.CDLL(path)
    for name in declared_symbols():
        assert hasattr(l1, name), name
    assert l1.sbits_cost_power() == 1


def test_strerror_covers_all_codes(lib):
    for code in range(0, -11, -1):
        assert sb.strerror(code) != "unknown status"
    assert sb.strerror(-99) == "unknown status"


@pytest.fixture()
def ctx(lib):
    c = sb.Context(device=-1)
    yield c
    c.close()


def test_plan_numbers_blocks_matrix_after_matrix(ctx):
    p = sb.Plan(ctx, [(4096, 4096), (1024, 4096), (4096, 14336)], 128, 128, [2, 3, 4])
    assert p.num_blocks(0) == 1024 and p.num_blocks(1) == 256 and p.num_blocks(2) == 32 * 112
    assert p.num_blocks() == 1024 + 256 + 3584
    assert [p.block_base(i) for i in range(3)] == [0, 1024, 1280]
    assert p.workspace_bytes() > 0 and p.workspace_bytes() % 256 == 0
    assert p.codes_bytes_bound(3.0) == int(3.0 * p.num_blocks()) * 128 * 128 // 8
    assert p.codes_bytes_bound(9.0) == 4 * p.num_blocks() * 128 * 128 // 8
    p.close()


@pytest.mark.parametrize("shape,m,n,bits,err", [
    ((1024, 1024), 128, 100, [2, 3, 4], sb.ERR_BAD_SHAPE),       # not a power of two
    ((1024, 1024), 4, 128, [2, 3, 4], sb.ERR_BAD_SHAPE),         # block rows < 8
    ((1024, 1024), 128, 1024, [2, 3, 4], sb.ERR_BAD_SHAPE),      # block cols > 512
    ((1000, 1024), 128, 128, [2, 3, 4], sb.ERR_BAD_SHAPE),       # rows not divisible
    ((1024, 1024), 128, 128, [], sb.ERR_BAD_BITWIDTHS),
    ((1024, 1024), 128, 128, [2, 2, 4], sb.ERR_BAD_BITWIDTHS),   # not strictly increasing
    ((1024, 1024), 128, 128, [4, 3, 2], sb.ERR_BAD_BITWIDTHS),
    ((1024, 1024), 128, 128, [0], sb.ERR_BAD_BITWIDTHS),         # pruning alone is no search space
    ((1024, 1024), 128, 128, [-1, 2], sb.ERR_BAD_BITWIDTHS),
    ((1024, 1024), 128, 128, [0, 0, 2], sb.ERR_BAD_BITWIDTHS),
    ((1024, 1024), 128, 128, [2, 3, 9], sb.ERR_BAD_BITWIDTHS),
    ((1024, 1024), 128, 128, list(range(1, 9)) + [8], sb.ERR_BAD_BITWIDTHS),
])
def test_plan_rejects_bad_partitions(ctx, shape, m, n, bits, err):
    with pytest.raises(sb.SbitsError) as e:
        sb.Plan(ctx, [shape], m, n, bits)
    assert e.value.status == err


def test_plan_takes_zero_bits_and_nine_candidates(ctx):
    p = sb.Plan(ctx, [(256, 256)], 128, 128, list(range(9)))      # 0 (pruned), 1, ..., 8
    assert p.num_blocks() == 4
    assert p.codes_bytes_bound(0.5) == 2 * 128 * 128 // 8
    assert p.codes_bytes_bound(0.0) == 0
    p.close()
    sb.Plan(ctx, [(256, 256)], 128, 128, [0, 4]).close()


def test_calls_validate_before_touching_the_device(ctx, lib):
    p = sb.Plan(ctx, [(256, 256)], 128, 128, [2, 3, 4])
    ws = 256 * 1024                                    # fake, aligned, never dereferenced
    cost = np.zeros((4, 3), np.float32)
    level = np.zeros(4, np.uint8)
    prm = sb.Params(0.05, 0.02, 0, 100)
    call = lambda *a: lib.sbits_allocate(p.h, *a)
    args = lambda avg, prm_, ws_: (sb._ptr(cost), C.c_double(avg), C.byref(prm_), sb._ptr(level), None, None,
                                   C.c_int64(0), C.c_void_p(ws_))
    assert call(*args(1.5, prm, ws)) == sb.ERR_INFEASIBLE_BUDGET
    assert call(*args(3.0, prm, ws + 8)) == sb.ERR_INVALID_ARG          # misaligned workspace
    assert call(*args(3.0, sb.Params(0.05, 0.02, 0, 0), ws)) == sb.ERR_INVALID_ARG
    assert call(*args(3.0, sb.Params(0.05, 0.02, 7, 10), ws)) == sb.ERR_INVALID_ARG
    assert call(*args(float("nan"), prm, ws)) == sb.ERR_INVALID_ARG
    assert call(*args(3.0, prm, ws)) == sb.ERR_HIP                       # host-only context: no device
    # null pointers and wrong matrix index
    assert lib.sbits_cost_table(p.h, C.c_int(0), None, None, None) == sb.ERR_INVALID_ARG
    assert lib.sbits_cost_table(p.h, C.c_int(3), C.c_void_p(256), C.c_void_p(256), C.c_void_p(256)) == sb.ERR_INVALID_ARG
    M = sb.Matrix(256, 256, 128, 256, 256, 256)                          # shape differs from the plan
    assert lib.sbits_reorder(p.h, C.c_int(0), C.byref(M), C.c_void_p(256), C.c_void_p(256), C.c_void_p(ws)) == sb.ERR_BAD_SHAPE
    M = sb.Matrix(256, 256, 256, 256, 256, 250)                          # pitch not a multiple of 4
    assert lib.sbits_reorder(p.h, C.c_int(0), C.byref(M), C.c_void_p(256), C.c_void_p(256), C.c_void_p(ws)) == sb.ERR_INVALID_ARG
    assert lib.sbits_num_blocks(p.h, C.c_int(5)) == sb.ERR_INVALID_ARG
    p.close()


def test_a_declared_workspace_that_is_too_small_is_refused_on_the_host(ctx, lib):
    """Every call that uses the workspace checks the size the caller declared for it, before any device work."""
    p = sb.Plan(ctx, [(256, 256), (128, 512)], 128, 128, [2, 3, 4])
    need = p.workspace_bytes()
    ws, ptr = C.c_void_p(256 * 1024), C.c_void_p(4096)                   # aligned, never dereferenced
    level, off = np.zeros(8, np.uint8), np.zeros(9, np.int64)
    prm = sb.Params(0.05, 0.02, 0, 100)
    mats = (sb.Matrix * 2)(sb.Matrix(4096, 4096, 256, 256, 256, 256), sb.Matrix(4096, 4096, 128, 512, 512, 512))
    calls = {
        "offsets": lambda: lib.sbits_offsets(p.h, sb._ptr(level), sb._ptr(off), ws),
        "allocate": lambda: lib.sbits_allocate(p.h, ptr, C.c_double(3.0), C.byref(prm), sb._ptr(level), None, None,
                                               C.c_int64(0), ws),
        "reorder_all": lambda: lib.sbits_reorder_all(p.h, mats, ptr, ptr, ws),
        "gather_cost_all": lambda: lib.sbits_gather_cost_all(p.h, mats, ptr, ptr, None, ptr, ws),
        "cost_table_all": lambda: lib.sbits_cost_table_all(p.h, ptr, ptr, ptr, ws),
        "pack_all": lambda: lib.sbits_pack_all(p.h, ptr, sb._ptr(level), sb._ptr(off), ptr, ptr, ptr, ws),
    }
    for name, call in calls.items():                                     # size not declared: not checked
        assert call() == sb.ERR_HIP, name
    assert p.set_workspace_size(need - 1) == sb.ERR_WORKSPACE
    for name, call in calls.items():
        assert call() == sb.ERR_WORKSPACE, name
    assert p.set_workspace_size(need) == sb.OK
    for name, call in calls.items():
        assert call() == sb.ERR_HIP, name                                # past the check: host-only context has no device
    assert lib.sbits_set_workspace_size(None, C.c_size_t(1)) == sb.ERR_INVALID_ARG
    p.close()


def test_one_pass_and_coupled_entry_points_validate_on_the_host(ctx, lib):
    """Argument and shape errors are reported before any device work (host-only context)."""
    ws = 256 * 1024
    ptr = C.c_void_p(4096)                                               # aligned, never dereferenced
    p = sb.Plan(ctx, [(256, 256), (256, 512)], 64, 128, [2, 3, 4])
    assert lib.sbits_gather_cost_supported(p.h) == 1
    mats = (sb.Matrix * 2)(sb.Matrix(4096, 4096, 256, 256, 256, 256), sb.Matrix(4096, 4096, 256, 512, 512, 512))
    assert lib.sbits_gather_cost_all(p.h, mats, ptr, ptr, None, None, C.c_void_p(ws)) == sb.ERR_INVALID_ARG   # no table
    assert lib.sbits_gather_cost_all(p.h, mats, ptr, ptr, None, ptr, C.c_void_p(ws)) == sb.ERR_HIP            # valid: needs a device
    assert lib.sbits_gather_pack_all(p.h, mats, ptr, ptr, ptr, ptr, C.c_void_p(4100), ptr, ptr,
                                     C.c_void_p(ws)) == sb.ERR_INVALID_ARG                                   # codes not 8-byte aligned
    assert lib.sbits_surrogates_all(p.h, mats, ptr, ptr, None, ptr, ptr, C.c_void_p(ws)) == sb.ERR_INVALID_ARG
    i32 = lambda *v: (C.c_int32 * len(v))(*v)
    call = lambda rg, cg, ng, seg, rr=None, cr=None: lib.sbits_reorder_coupled_all(
        p.h, mats, rg, cg, C.c_int(ng), seg, rr, cr, ptr, ptr, C.c_void_p(ws))
    assert call(i32(0, 0), i32(-1, -1), 1, None) == sb.ERR_HIP           # rows 256 and 256: a valid group
    assert call(i32(0, -1), i32(-1, 0), 1, None) == sb.ERR_BAD_SHAPE     # 256 rows with 512 columns
    assert call(i32(1, -1), i32(-1, -1), 1, None) == sb.ERR_INVALID_ARG  # group id out of range
    assert call(i32(0, 0), i32(-1, -1), 1, i32(96)) == sb.ERR_BAD_SHAPE  # piece length does not divide 256
    assert call(i32(-2, -2), i32(-2, -2), 0, None) == sb.ERR_HIP         # everything fixed: valid
    # rows of matrix 0 (256) lead; the 512 columns of matrix 1 are two pieces per piece of 64
    assert call(i32(0, -1), i32(-1, 0), 1, i32(64), i32(1, 1), i32(1, 2)) == sb.ERR_HIP
    assert call(i32(0, -1), i32(-1, 0), 1, None, i32(1, 1), i32(1, 2)) == sb.ERR_BAD_SHAPE       # repeat without pieces
    assert call(i32(0, -1), i32(-1, 0), 1, i32(64), i32(1, 1), i32(1, 4)) == sb.ERR_BAD_SHAPE    # 4 * 256 != 512
    assert call(i32(0, -1), i32(-1, 0), 1, i32(64), i32(1, 1), i32(1, 0)) == sb.ERR_INVALID_ARG  # repeat < 1
    assert call(i32(0, -1), i32(-1, -1), 1, i32(64), i32(2, 1), None) == sb.ERR_INVALID_ARG      # a repeated leader
    assert call(i32(-1, -1), i32(-1, -1), 0, None, i32(2, 1), None) == sb.ERR_INVALID_ARG        # repeat on an independent dimension
    p.close()
    q = sb.Plan(ctx, [(256, 512)], 64, 256, [2, 3, 4])                   # 256-column blocks: two-pass route only
    assert lib.sbits_gather_cost_supported(q.h) == 0
    m1 = (sb.Matrix * 1)(sb.Matrix(4096, 4096, 256, 512, 512, 512))
    assert lib.sbits_gather_cost_all(q.h, m1, ptr, ptr, None, ptr, C.c_void_p(ws)) == sb.ERR_UNIMPLEMENTED
    assert lib.sbits_gather_pack_all(q.h, m1, ptr, ptr, ptr, ptr, ptr, ptr, ptr, C.c_void_p(ws)) == sb.ERR_UNIMPLEMENTED
    assert lib.sbits_surrogates_all(q.h, m1, ptr, ptr, ptr, ptr, ptr, C.c_void_p(ws)) == sb.ERR_UNIMPLEMENTED
    q.close()


def test_propose_validates_on_the_host(ctx, lib):
    ptr = C.c_void_p(4096)
    p = sb.Plan(ctx, [(256, 256)], 64, 128, [2, 3, 4])
    call = lambda su, lv, avg, k: lib.sbits_propose(p.h, su, ptr, lv, C.c_double(avg), C.c_int64(k), ptr, None,
                                                    C.c_void_p(256 * 1024))
    assert call(None, ptr, 3.0, 4) == sb.ERR_INVALID_ARG
    assert call(ptr, None, 3.0, 4) == sb.ERR_INVALID_ARG
    assert call(ptr, ptr, 3.0, 0) == sb.ERR_INVALID_ARG                 # k >= 1
    assert call(ptr, ptr, float("nan"), 4) == sb.ERR_INVALID_ARG
    assert call(ptr, ptr, 1.5, 4) == sb.ERR_INFEASIBLE_BUDGET           # below the smallest candidate
    assert call(ptr, ptr, 3.0, 4) == sb.ERR_HIP                         # valid: needs a device
    p.close()


def test_mp_gemm_validates_on_the_host(ctx, lib):
    ptr = C.c_void_p(4096)
    ws = C.c_void_p(256 * 1024)
    p = sb.Plan(ctx, [(256, 256)], 64, 128, [2, 3, 4])
    call = lambda pl, mat, x, ld, batch: lib.sbits_mp_gemm(pl.h, C.c_int(mat), x, C.c_int64(ld), C.c_int(batch), ptr, ptr,
                                                            ptr, ptr, ptr, ptr, ws)
    assert call(p, 0, None, 256, 16) == sb.ERR_INVALID_ARG
    assert call(p, 1, ptr, 256, 16) == sb.ERR_INVALID_ARG                # no such matrix
    assert call(p, 0, ptr, 248, 16) == sb.ERR_INVALID_ARG                # ld_x below the column count
    assert call(p, 0, ptr, 260, 16) == sb.ERR_INVALID_ARG                # ld_x not a multiple of 8
    assert call(p, 0, C.c_void_p(4100), 256, 16) == sb.ERR_INVALID_ARG   # x not 16-byte aligned
    assert call(p, 0, ptr, 256, 0) == sb.ERR_INVALID_ARG
    assert call(p, 0, ptr, 256, 32) == sb.ERR_HIP                        # valid: needs a device
    p.close()
    q = sb.Plan(ctx, [(64, 512)], 16, 256, [2, 4])                       # 16-row blocks, 256 columns wide
    assert call(q, 0, ptr, 512, 16) == sb.ERR_UNIMPLEMENTED
    q.close()


def test_dequant_validates_on_the_host(ctx, lib):
    ptr = C.c_void_p(4096)
    p = sb.Plan(ctx, [(256, 256)], 64, 128, [2, 3, 4])
    call = lambda mat, out, ld, bf: lib.sbits_dequant(p.h, C.c_int(mat), ptr, ptr, ptr, ptr, ptr, out, C.c_int64(ld), C.c_int(bf))
    assert call(0, None, 256, 0) == sb.ERR_INVALID_ARG
    assert call(2, ptr, 256, 0) == sb.ERR_INVALID_ARG                    # no such matrix
    assert call(0, ptr, 248, 0) == sb.ERR_INVALID_ARG                    # pitch below the column count
    assert call(0, C.c_void_p(4100), 256, 0) == sb.ERR_INVALID_ARG       # out not 16-byte aligned
    assert call(0, ptr, 256, 2) == sb.ERR_INVALID_ARG                    # 0 = fp32, 1 = bf16
    assert call(0, ptr, 264, 1) == sb.ERR_HIP                            # valid: needs a device
    p.close()


def test_plan_limits(ctx):
    """At most 32768 rows / columns per matrix and 2^24 blocks per plan."""
    sb.Plan(ctx, [(32768, 32768)], 8, 8, [2]).close()                    # 2^24 blocks: the limit itself
    for shapes, m, n in (([(32768 + 8, 8)], 8, 8), ([(8, 32768 + 8)], 8, 8),
                         ([(32768, 32768), (8, 8)], 8, 8)):              # one block too many
        with pytest.raises(sb.SbitsError) as e:
            sb.Plan(ctx, shapes, m, n, [2])
        assert e.value.status == sb.ERR_BAD_SHAPE
