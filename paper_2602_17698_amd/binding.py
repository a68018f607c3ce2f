"""Thin ctypes binding over the C-ABI of libscalebits.so (see include/scalebits.h).

Argument marshalling only: every step of the search runs in the library's HIP
kernels.  PyTorch supplies device memory and the stream.  There is no fallback:
if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SBITS_LIB") or os.path.join(_HERE, "libscalebits.so")

OK = 0
ERR_INVALID_ARG, ERR_BAD_SHAPE, ERR_BAD_BITWIDTHS, ERR_INFEASIBLE_BUDGET = -1, -2, -3, -4
DIM_INDEPENDENT, DIM_FIXED = -1, -2
ERR_WORKSPACE, ERR_MAX_ITERS, ERR_HIP, ERR_UNIMPLEMENTED, ERR_CAPACITY, ERR_INTERNAL = -5, -6, -7, -8, -9, -10
OFFSETS_STATIC_MAX_BLOCKS = 8388608          # SBITS_OFFSETS_STATIC_MAX_BLOCKS of the header

EXPORTS = [
    "sbits_create", "sbits_destroy", "sbits_last_hip_error", "sbits_strerror",
    "sbits_plan_create", "sbits_plan_destroy", "sbits_num_blocks", "sbits_block_base",
    "sbits_workspace_bytes", "sbits_set_workspace_size", "sbits_codes_bytes_bound",
    "sbits_reorder", "sbits_reorder_all", "sbits_channel_scores", "sbits_gather", "sbits_gather_all",
    "sbits_cost_table", "sbits_cost_table_all", "sbits_cost_power", "sbits_pack_all",
    "sbits_gather_cost_supported", "sbits_gather_cost_all", "sbits_gather_pack_all",
    "sbits_reorder_coupled_all", "sbits_surrogates_all",
    "sbits_allocate", "sbits_propose", "sbits_offsets", "sbits_offsets_static", "sbits_pack", "sbits_search", "sbits_search_coupled", "sbits_mp_gemm", "sbits_dequant",
]


class Matrix(C.Structure):
    _fields_ = [("w_bf16", C.c_void_p), ("sens", C.c_void_p),
                ("rows", C.c_int64), ("cols", C.c_int64), ("ld_w", C.c_int64), ("ld_s", C.c_int64)]


class Params(C.Structure):
    _fields_ = [("gamma0", C.c_double), ("gammaT", C.c_double),
                ("init_mode", C.c_int32), ("max_iters", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [("iters", C.c_int32), ("expansions", C.c_int32), ("swaps_ok", C.c_int32),
                ("swaps_rej", C.c_int32), ("k_final", C.c_int64), ("bits_used", C.c_int64),
                ("bits_budget", C.c_int64), ("cost_fixed", C.c_int64), ("cost_shift", C.c_int32),
                ("pad_", C.c_int32)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_ if f != "pad_"}


class Trace(C.Structure):
    _fields_ = [("kind", C.c_int32), ("pad_", C.c_int32), ("k", C.c_int64), ("n_up", C.c_int64),
                ("n_dn", C.c_int64), ("p_up", C.c_int64), ("p_dn", C.c_int64),
                ("bits_before", C.c_int64), ("bits_after", C.c_int64), ("delta_fixed", C.c_int64)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_ if f != "pad_"}


class Proposal(C.Structure):
    _fields_ = [("kind", C.c_int32), ("pad_", C.c_int32), ("n_up", C.c_int64), ("n_dn", C.c_int64),
                ("bits_before", C.c_int64), ("bits_after", C.c_int64), ("bits_budget", C.c_int64)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_ if f != "pad_"}


class Outputs(C.Structure):
    _fields_ = [("row_perm", C.c_void_p), ("col_perm", C.c_void_p), ("w_re_bf16", C.c_void_p),
                ("s_re", C.c_void_p), ("cost", C.c_void_p), ("level", C.c_void_p),
                ("byte_off", C.c_void_p), ("codes", C.c_void_p), ("codes_capacity", C.c_int64),
                ("scale", C.c_void_p), ("zero", C.c_void_p)]


class SbitsError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, strerror(status), status))


_lib = None
_loaded = {}                    # path -> CDLL (a library is opened once per process)


def load():
    """Loads libscalebits.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if LIB_PATH not in _loaded:
            if not os.path.exists(LIB_PATH):
                raise FileNotFoundError(
                    "%s is missing: build it with `python -m paper_2602_17698_amd.build`" % LIB_PATH)
            lib = C.CDLL(LIB_PATH)
            lib.sbits_strerror.restype = C.c_char_p
            lib.sbits_num_blocks.restype = C.c_int64
            lib.sbits_block_base.restype = C.c_int64
            lib.sbits_workspace_bytes.restype = C.c_size_t
            lib.sbits_codes_bytes_bound.restype = C.c_int64
            lib.sbits_codes_bytes_bound.argtypes = [C.c_void_p, C.c_double]
            _loaded[LIB_PATH] = lib
        _lib = _loaded[LIB_PATH]
    return _lib


def variant_path(variant: str = "") -> str:
    """In-tree path of a build variant: "" = sum s*d^2 (default), "l1" = sum s*|d|."""
    return os.path.join(_HERE, "libscalebits%s.so" % ("_" + variant if variant else ""))


def use_library(path: str) -> None:
    """Routes all later calls to another build of the library (see variant_path).  Contexts and
    plans belong to the library that created them: close them before switching, or switch back
    before using them again."""
    global _lib, LIB_PATH
    LIB_PATH = path
    _lib = None
    load()


def cost_power() -> int:
    """Power of the quantization change in the block cost of the loaded build (2 or 1)."""
    return int(load().sbits_cost_power())


def strerror(status: int) -> str:
    return load().sbits_strerror(C.c_int(status)).decode()


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return C.c_void_p(None)
    if isinstance(t, int):
        return C.c_void_p(t)
    if hasattr(t, "data_ptr"):
        return C.c_void_p(t.data_ptr())
    return C.c_void_p(t.ctypes.data)


def _check(rc, where, allow=()):
    if rc != OK and rc not in allow:
        raise SbitsError(rc, where)
    return rc


def matrix(w, s) -> Matrix:
    """Descriptor of one weight matrix (bf16 tensor) and its sensitivity (fp32 tensor)."""
    rows, cols = (w.shape if w is not None else s.shape)
    d = Matrix(_ptr(w).value, _ptr(s).value, rows, cols,
               w.stride(0) if w is not None else cols, s.stride(0) if s is not None else cols)
    d._keep = (w, s)            # the descriptor holds raw addresses: keep the tensors alive as long as it lives
    return d


class Context:
    def __init__(self, device: int = 0, stream: int = 0):
        self.h = C.c_void_p()
        _check(load().sbits_create(C.byref(self.h), C.c_int(device), C.c_void_p(stream)), "sbits_create")

    def close(self):
        if self.h:
            load().sbits_destroy(self.h)
            self.h = C.c_void_p()

    def last_hip_error(self) -> int:
        return load().sbits_last_hip_error(self.h)


class Plan:
    """The partition: matrices, block shape, candidate bitwidths (sbits_plan_create)."""

    def __init__(self, ctx: Context, shapes, block_rows: int, block_cols: int, bitwidths):
        self.ctx = ctx
        self.shapes = [(int(r), int(c)) for r, c in shapes]
        self.m, self.n = block_rows, block_cols
        self.bitwidths = [int(b) for b in bitwidths]
        n = len(self.shapes)
        rows = (C.c_int64 * n)(*[r for r, _ in self.shapes])
        cols = (C.c_int64 * n)(*[c for _, c in self.shapes])
        bw = (C.c_int32 * len(self.bitwidths))(*self.bitwidths)
        self.h = C.c_void_p()
        _check(load().sbits_plan_create(ctx.h, rows, cols, C.c_int(n), C.c_int(block_rows), C.c_int(block_cols),
                                        bw, C.c_int(len(self.bitwidths)), C.byref(self.h)), "sbits_plan_create")

    def close(self):
        if self.h:
            load().sbits_plan_destroy(self.h)
            self.h = C.c_void_p()

    @property
    def K(self):
        return len(self.bitwidths)

    def num_blocks(self, mat: int = -1) -> int:
        return int(load().sbits_num_blocks(self.h, C.c_int(mat)))

    def block_base(self, mat: int) -> int:
        return int(load().sbits_block_base(self.h, C.c_int(mat)))

    def workspace_bytes(self) -> int:
        return int(load().sbits_workspace_bytes(self.h))

    def set_workspace_size(self, nbytes: int) -> int:
        """Declares the size of the workspace later calls receive; calls fail with ERR_WORKSPACE while it is too small."""
        return int(load().sbits_set_workspace_size(self.h, C.c_size_t(nbytes)))

    def codes_bytes_bound(self, avg_bits: float) -> int:
        return int(load().sbits_codes_bytes_bound(self.h, C.c_double(avg_bits)))

    # ---- the calls of the path; tensors are caller-allocated device tensors -------------
    def reorder(self, mat, M: Matrix, row_perm, col_perm, ws):
        return _check(load().sbits_reorder(self.h, C.c_int(mat), C.byref(M), _ptr(row_perm), _ptr(col_perm),
                                           _ptr(ws)), "sbits_reorder")

    def channel_scores(self, mat, M: Matrix, row_score, col_score, ws):
        return _check(load().sbits_channel_scores(self.h, C.c_int(mat), C.byref(M), _ptr(row_score),
                                                  _ptr(col_score), _ptr(ws)), "sbits_channel_scores")

    def gather(self, mat, M: Matrix, row_perm, col_perm, w_out, s_out):
        return _check(load().sbits_gather(self.h, C.c_int(mat), C.byref(M), _ptr(row_perm), _ptr(col_perm),
                                          _ptr(w_out), _ptr(s_out)), "sbits_gather")

    def cost_table(self, mat, w_re, s_re, cost):
        return _check(load().sbits_cost_table(self.h, C.c_int(mat), _ptr(w_re), _ptr(s_re), _ptr(cost)),
                      "sbits_cost_table")

    def reorder_all(self, mats, row_perm, col_perm, ws):
        arr = (Matrix * len(mats))(*mats)
        return _check(load().sbits_reorder_all(self.h, arr, _ptr(row_perm), _ptr(col_perm), _ptr(ws)),
                      "sbits_reorder_all")

    def reorder_coupled_all(self, mats, row_group, col_group, n_groups, group_segment, row_perm, col_perm, ws,
                            row_repeat=None, col_repeat=None):
        """row_group / col_group / group_segment / row_repeat / col_repeat: host sequences of ints
        (see scalebits.h)."""
        arr = (Matrix * len(mats))(*mats)
        rg = (C.c_int32 * len(row_group))(*row_group)
        cg = (C.c_int32 * len(col_group))(*col_group)
        gs = (C.c_int32 * max(len(group_segment), 1))(*group_segment) if group_segment is not None else None
        rr = (C.c_int32 * len(row_repeat))(*row_repeat) if row_repeat is not None else None
        cr = (C.c_int32 * len(col_repeat))(*col_repeat) if col_repeat is not None else None
        return _check(load().sbits_reorder_coupled_all(self.h, arr, rg, cg, C.c_int(n_groups), gs, rr, cr,
                                                       _ptr(row_perm), _ptr(col_perm), _ptr(ws)),
                      "sbits_reorder_coupled_all")

    def gather_all(self, mats, row_perm, col_perm, w_re, s_re, ws):
        arr = (Matrix * len(mats))(*mats)
        return _check(load().sbits_gather_all(self.h, arr, _ptr(row_perm), _ptr(col_perm), _ptr(w_re),
                                              _ptr(s_re), _ptr(ws)), "sbits_gather_all")

    def gather_cost_supported(self):
        return bool(load().sbits_gather_cost_supported(self.h))

    def gather_cost_all(self, mats, row_perm, col_perm, w_re, cost, ws):
        arr = (Matrix * len(mats))(*mats)
        return _check(load().sbits_gather_cost_all(self.h, arr, _ptr(row_perm), _ptr(col_perm), _ptr(w_re),
                                                   _ptr(cost), _ptr(ws)), "sbits_gather_cost_all")

    def surrogates_all(self, mats, row_perm, col_perm, level, s_up, s_down, ws):
        """mats: matrix(w, g) with the gradient in the place of the sensitivity."""
        arr = (Matrix * len(mats))(*mats)
        return _check(load().sbits_surrogates_all(self.h, arr, _ptr(row_perm), _ptr(col_perm), _ptr(level),
                                                  _ptr(s_up), _ptr(s_down), _ptr(ws)), "sbits_surrogates_all")

    def gather_pack_all(self, mats, row_perm, col_perm, level, byte_off, codes, scale, zero, ws):
        arr = (Matrix * len(mats))(*mats)
        return _check(load().sbits_gather_pack_all(self.h, arr, _ptr(row_perm), _ptr(col_perm), _ptr(level),
                                                   _ptr(byte_off), _ptr(codes), _ptr(scale), _ptr(zero), _ptr(ws)),
                      "sbits_gather_pack_all")

    def pack_all(self, w_re, level, byte_off, codes, scale, zero, ws):
        return _check(load().sbits_pack_all(self.h, _ptr(w_re), _ptr(level), _ptr(byte_off), _ptr(codes),
                                            _ptr(scale), _ptr(zero), _ptr(ws)), "sbits_pack_all")

    def cost_table_all(self, w_re, s_re, cost, ws):
        return _check(load().sbits_cost_table_all(self.h, _ptr(w_re), _ptr(s_re), _ptr(cost), _ptr(ws)),
                      "sbits_cost_table_all")

    def allocate(self, cost, avg_bits, level, ws, gamma0=0.05, gammaT=0.02, init_mode=0,
                 max_iters=100000, trace_cap=0):
        """Returns (status, stats dict, trace list); status is OK or ERR_MAX_ITERS."""
        prm = Params(gamma0, gammaT, init_mode, max_iters)
        st = Stats()
        tr = (Trace * max(trace_cap, 1))()
        rc = load().sbits_allocate(self.h, _ptr(cost), C.c_double(avg_bits), C.byref(prm), _ptr(level),
                                   C.byref(st), tr if trace_cap else None, C.c_int64(trace_cap), _ptr(ws))
        _check(rc, "sbits_allocate", allow=(ERR_MAX_ITERS,))
        n = min(st.iters, trace_cap)
        return rc, st.as_dict(), [tr[i].as_dict() for i in range(n)]

    def propose(self, s_up, s_down, level_in, avg_bits, k, level_out, ws, want_info=True):
        """One step of Algorithm 2 on caller-supplied estimates; returns the proposal's dict
        (kind 0 none, 1 expansion, 2 swap) or None without waiting when want_info is False."""
        pr = Proposal()
        _check(load().sbits_propose(self.h, _ptr(s_up), _ptr(s_down), _ptr(level_in), C.c_double(avg_bits),
                                    C.c_int64(k), _ptr(level_out), C.byref(pr) if want_info else None, _ptr(ws)),
               "sbits_propose")
        return pr.as_dict() if want_info else None

    def offsets(self, level, byte_off, ws):
        return _check(load().sbits_offsets(self.h, _ptr(level), _ptr(byte_off), _ptr(ws)), "sbits_offsets")

    def offsets_static(self, level, byte_off):
        """sbits_offsets on the library's fixed per-GPU scratch array: no workspace, no allocation."""
        return _check(load().sbits_offsets_static(self.h, _ptr(level), _ptr(byte_off)), "sbits_offsets_static")

    def pack(self, mat, w_re, level, byte_off, codes, scale, zero):
        return _check(load().sbits_pack(self.h, C.c_int(mat), _ptr(w_re), _ptr(level), _ptr(byte_off),
                                        _ptr(codes), _ptr(scale), _ptr(zero)), "sbits_pack")

    def dequant(self, mat, level, byte_off, codes, scale, zero, out):
        """out[i][j] = code * scale + zero of the stored (reordered) matrix; out: fp32 or bf16 [rows, cols]."""
        import torch
        return _check(load().sbits_dequant(self.h, C.c_int(mat), _ptr(level), _ptr(byte_off), _ptr(codes), _ptr(scale),
                                           _ptr(zero), _ptr(out), C.c_int64(out.stride(0)),
                                           C.c_int(1 if out.dtype == torch.bfloat16 else 0)), "sbits_dequant")

    def mp_gemm(self, mat, x, level, byte_off, codes, scale, zero, y, ws):
        """y[b][i] = sum_j What[i][j] x[b][j] from the packed arrays; x: bf16 [batch, cols], y: fp32 [batch, rows]."""
        return _check(load().sbits_mp_gemm(self.h, C.c_int(mat), _ptr(x), C.c_int64(x.stride(0)), C.c_int(x.shape[0]),
                                           _ptr(level), _ptr(byte_off), _ptr(codes), _ptr(scale), _ptr(zero),
                                           _ptr(y), _ptr(ws)), "sbits_mp_gemm")

    def search(self, mats, avg_bits, out: Outputs, ws, gamma0=0.05, gammaT=0.02, init_mode=0,
               max_iters=100000):
        arr = (Matrix * len(mats))(*mats)
        prm = Params(gamma0, gammaT, init_mode, max_iters)
        st = Stats()
        rc = load().sbits_search(self.h, arr, C.c_double(avg_bits), C.byref(prm), C.byref(out),
                                 C.byref(st), _ptr(ws))
        _check(rc, "sbits_search", allow=(ERR_MAX_ITERS,))
        return rc, st.as_dict()

    def search_coupled(self, mats, coupling, avg_bits, out: Outputs, ws, gamma0=0.05, gammaT=0.02, init_mode=0,
                       max_iters=100000):
        """coupling = (row_group, col_group, n_groups, group_segment, row_repeat, col_repeat), host
        sequences as for reorder_coupled_all (the last three may be None)."""
        rg, cg, ng, seg, rrep, crep = coupling
        i32 = lambda v: (C.c_int32 * max(len(v), 1))(*v) if v is not None else None
        arr = (Matrix * len(mats))(*mats)
        prm = Params(gamma0, gammaT, init_mode, max_iters)
        st = Stats()
        rc = load().sbits_search_coupled(self.h, arr, i32(rg), i32(cg), C.c_int(ng), i32(seg), i32(rrep), i32(crep),
                                         C.c_double(avg_bits), C.byref(prm), C.byref(out), C.byref(st), _ptr(ws))
        _check(rc, "sbits_search_coupled", allow=(ERR_MAX_ITERS,))
        return rc, st.as_dict()
