"""CPU oracle for the ScaleBITS bitwidth-allocation search (test infrastructure).

numpy-facing ctypes wrappers around ``sbits_oracle.c``.  Only tests, the smoke
check and the benchmark's ``cpu_baseline`` leg may import this package; the GPU
library and its binding never do, and this package never imports them.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sbits_oracle.c")
_HDR = os.path.join(_HERE, "sbits_oracle.h")
_LIB = os.path.join(_HERE, "liboracle.so")

CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math",
          "-D_DEFAULT_SOURCE", "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no contraction)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class Params(C.Structure):
    _fields_ = [("gamma0", C.c_double), ("gammaT", C.c_double),
                ("init_mode", C.c_int32), ("max_iters", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [("iters", C.c_int32), ("expansions", C.c_int32),
                ("swaps_ok", C.c_int32), ("swaps_rej", C.c_int32),
                ("k_final", C.c_int64), ("bits_used", C.c_int64),
                ("bits_budget", C.c_int64), ("cost_fixed", C.c_int64),
                ("cost_shift", C.c_int32), ("pad_", C.c_int32)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_ if f != "pad_"}


class Trace(C.Structure):
    _fields_ = [("kind", C.c_int32), ("pad_", C.c_int32), ("k", C.c_int64),
                ("n_up", C.c_int64), ("n_dn", C.c_int64),
                ("p_up", C.c_int64), ("p_dn", C.c_int64),
                ("bits_before", C.c_int64), ("bits_after", C.c_int64),
                ("delta_fixed", C.c_int64)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_ if f != "pad_"}


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_canon8.restype = C.c_float
        _lib.orc_brute_force.restype = C.c_double
        _lib.orc_fx.restype = C.c_int64
        _lib.orc_fx.argtypes = [C.c_float, C.c_int32]
        _lib.orc_cost_shift.restype = C.c_int32
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "bf16 data travels as raw uint16"
    return a


def f32_to_bf16(x) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even), returned as raw uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_to_f32(h) -> np.ndarray:
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def canon8(x) -> float:
    x = _f32(x)
    return float(lib().orc_canon8(_p(x), C.c_int64(x.size), C.c_int64(1)))


def channel_scores(S):
    S = _f32(S)
    R, Cc = S.shape
    rs = np.empty(R, np.float32)
    cs = np.empty(Cc, np.float32)
    lib().orc_channel_scores(_p(S), C.c_int64(R), C.c_int64(Cc), C.c_int64(Cc), _p(rs), _p(cs))
    return rs, cs


def argsort_desc(score):
    score = _f32(score)
    perm = np.empty(score.size, np.int32)
    lib().orc_argsort_desc(_p(score), C.c_int64(score.size), _p(perm))
    return perm


def group_scores(member_scores):
    """Summed channel scores of coupled dimensions, member after member (fp32)."""
    ms = [_f32(m) for m in member_scores]
    n = ms[0].size
    assert all(m.size == n for m in ms)
    ptrs = (C.c_void_p * len(ms))(*[m.ctypes.data for m in ms])
    out = np.empty(n, np.float32)
    lib().orc_group_scores(ptrs, C.c_int(len(ms)), C.c_int64(n), _p(out))
    return out


def argsort_desc_pieces(score, piece=0):
    score = _f32(score)
    perm = np.empty(score.size, np.int32)
    lib().orc_argsort_desc_pieces(_p(score), C.c_int64(score.size), C.c_int64(piece), _p(perm))
    return perm


def coupled_perm(member_scores, piece=0):
    """The one permutation shared by coupled dimensions (App. "Channel Reordering")."""
    return argsort_desc_pieces(group_scores(member_scores), piece)


def fold_repeated(score, piece, repeat):
    """A member whose dimension is `repeat` times the group's (one value head feeding several query
    heads): group piece p stands for the member's pieces repeat*p .. repeat*p + repeat - 1.
    Returns the `repeat` score arrays of the group's length that the member contributes to the
    group sum, lower piece first."""
    score = _f32(score)
    v = score.reshape(-1, repeat, piece)             # [group piece][which of the member's pieces][channel]
    return [np.ascontiguousarray(v[:, t, :]).reshape(-1) for t in range(repeat)]


def expand_perm(perm, piece, repeat):
    """The member's permutation from the group's: every one of the member's pieces takes the
    within-piece order of the group piece it belongs to."""
    perm = _i32(perm)
    within = perm.reshape(-1, piece) - (np.arange(perm.size // piece, dtype=np.int32) * piece)[:, None]
    out = np.empty(perm.size * repeat, np.int32)
    for pc in range(perm.size // piece * repeat):
        out[pc * piece:(pc + 1) * piece] = pc * piece + within[pc // repeat]
    return out


def gather(W_u16, S, rp, cp):
    W_u16 = _u16(W_u16)
    S = _f32(S)
    rp, cp = _i32(rp), _i32(cp)
    R, Cc = W_u16.shape
    Wo = np.empty_like(W_u16)
    So = np.empty_like(S)
    lib().orc_gather_bf16(_p(W_u16), C.c_int64(R), C.c_int64(Cc), C.c_int64(Cc), _p(rp), _p(cp), _p(Wo))
    lib().orc_gather_f32(_p(S), C.c_int64(R), C.c_int64(Cc), C.c_int64(Cc), _p(rp), _p(cp), _p(So))
    return Wo, So


def quant_group(w, bits):
    w = _f32(w)
    q = np.empty(w.size, np.int32)
    sc = C.c_float()
    ze = C.c_float()
    lib().orc_quant_group(_p(w), C.c_int(w.size), C.c_int(bits), _p(q), C.byref(sc), C.byref(ze))
    return q, np.float32(sc.value), np.float32(ze.value)


def surrogates(Wp_u16, Gp, m, n, bits, level):
    """(s_up, s_down) per block of one reordered matrix at the blocks' current levels."""
    Wp_u16 = _u16(Wp_u16)
    Gp = _f32(Gp)
    R, Cc = Wp_u16.shape
    b = np.ascontiguousarray(bits, np.int32)
    lv = np.ascontiguousarray(level, np.uint8)
    nb = (R // m) * (Cc // n)
    assert lv.size == nb
    up, dn = np.empty(nb, np.float32), np.empty(nb, np.float32)
    lib().orc_surrogates(_p(Wp_u16), _p(Gp), C.c_int64(R), C.c_int64(Cc), C.c_int(m), C.c_int(n), _p(b), _p(lv),
                         _p(up), _p(dn))
    return up, dn


def cost_table(Wp_u16, Sp, m, n, bits, power=2):
    Wp_u16 = _u16(Wp_u16)
    Sp = _f32(Sp)
    bits = _i32(bits)
    R, Cc = Wp_u16.shape
    assert R % m == 0 and Cc % n == 0
    cost = np.empty(((R // m) * (Cc // n), bits.size), np.float32)
    assert power in (1, 2)
    lib().orc_cost_table_pow(_p(Wp_u16), _p(Sp), C.c_int64(R), C.c_int64(Cc), C.c_int(m), C.c_int(n),
                             _p(bits), C.c_int(bits.size), C.c_int(power), _p(cost))
    return cost


def allocate(cost, bits, avg_bits, gamma0=0.05, gammaT=0.02, init_mode=0,
             max_iters=100000, want_trace=False):
    cost = _f32(cost)
    bits = _i32(bits)
    N, K = cost.shape
    assert K == bits.size
    level = np.zeros(N, np.uint8)
    prm = Params(gamma0, gammaT, init_mode, max_iters)
    st = Stats()
    cap = max_iters if want_trace else 0
    tr = (Trace * max(cap, 1))()
    ntr = C.c_int64(0)
    rc = lib().orc_allocate(_p(cost), C.c_int64(N), _p(bits), C.c_int(K), C.c_double(avg_bits),
                            C.byref(prm), _p(level), C.byref(st),
                            tr if want_trace else None, C.c_int64(cap), C.byref(ntr))
    trace = [tr[i].as_dict() for i in range(min(ntr.value, cap))] if want_trace else None
    return rc, level, st.as_dict(), trace


def propose(s_up, s_down, level, bits, avg_bits, k):
    """One step of Algorithm 2 on caller-supplied estimates: (kind, level_out, info);
    kind 0 none, 1 expansion, 2 swap proposal."""
    s_up, s_down = _f32(s_up), _f32(s_down)
    level = np.ascontiguousarray(level, np.uint8)
    bits = _i32(bits)
    out = np.empty_like(level)
    nu, nd, bb, ba = C.c_int64(0), C.c_int64(0), C.c_int64(0), C.c_int64(0)
    kind = lib().orc_propose(_p(s_up), _p(s_down), _p(level), C.c_int64(level.size), _p(bits), C.c_int(bits.size),
                             C.c_double(avg_bits), C.c_int64(k), _p(out), C.byref(nu), C.byref(nd), C.byref(bb),
                             C.byref(ba))
    return kind, out, dict(n_up=nu.value, n_dn=nd.value, bits_before=bb.value, bits_after=ba.value)


def cost_shift(cost) -> int:
    cost = _f32(cost)
    N, K = cost.shape
    return int(lib().orc_cost_shift(_p(cost), C.c_int64(N), C.c_int(K)))


def fx(v, shift) -> int:
    return int(lib().orc_fx(C.c_float(float(v)), C.c_int32(shift)))


def classic_greedy(cost, bits, avg_bits):
    cost = _f32(cost)
    bits = _i32(bits)
    N, K = cost.shape
    level = np.zeros(N, np.uint8)
    lib().orc_classic_greedy(_p(cost), C.c_int64(N), _p(bits), C.c_int(K), C.c_double(avg_bits), _p(level))
    return level


def brute_force(cost, bits, avg_bits):
    cost = _f32(cost)
    bits = _i32(bits)
    N, K = cost.shape
    level = np.zeros(N, np.uint8)
    best = lib().orc_brute_force(_p(cost), C.c_int(N), _p(bits), C.c_int(K), C.c_double(avg_bits), _p(level))
    return float(best), level


def offsets(level, m, n, bits):
    level = np.ascontiguousarray(level, dtype=np.uint8)
    bits = _i32(bits)
    off = np.empty(level.size + 1, np.int64)
    lib().orc_offsets(_p(level), C.c_int64(level.size), C.c_int(m), C.c_int(n), _p(bits), _p(off))
    return off


def pack(Wp_u16, m, n, bits, level, byte_off, block_base, codes, scale, zero):
    """Packs one matrix into the global codes/scale/zero arrays (in place)."""
    Wp_u16 = _u16(Wp_u16)
    bits = _i32(bits)
    R, Cc = Wp_u16.shape
    assert level.dtype == np.uint8 and byte_off.dtype == np.int64
    assert codes.dtype == np.uint8 and scale.dtype == np.float32 and zero.dtype == np.float32
    lib().orc_pack(_p(Wp_u16), C.c_int64(R), C.c_int64(Cc), C.c_int(m), C.c_int(n), _p(bits),
                   C.c_int(bits.size), _p(level), _p(byte_off), C.c_int64(block_base),
                   _p(codes), _p(scale), _p(zero))


def dequant(codes, scale, zero, level, byte_off, block_base, R, Cc, m, n, bits):
    """The stored matrix (fp32 [R, Cc]) from the packed arrays."""
    bits = _i32(bits)
    out = np.empty((R, Cc), np.float32)
    lib().orc_dequant(_p(codes), _p(scale), _p(zero), _p(level), _p(byte_off), C.c_int64(block_base),
                      C.c_int64(R), C.c_int64(Cc), C.c_int(m), C.c_int(n), _p(bits), _p(out))
    return out


def mp_gemm(codes, scale, zero, level, byte_off, block_base, R, Cc, m, n, bits, x_u16):
    """y[b][i] = sum_j What[i][j] x[b][j] (float64); x_u16: bf16 patterns [batch, Cc]."""
    bits = _i32(bits)
    x_u16 = _u16(x_u16)
    assert x_u16.shape[1] == Cc
    y = np.empty((x_u16.shape[0], R), np.float64)
    lib().orc_mp_gemm(_p(codes), _p(scale), _p(zero), _p(level), _p(byte_off), C.c_int64(block_base),
                      C.c_int64(R), C.c_int64(Cc), C.c_int(m), C.c_int(n), _p(bits), _p(x_u16),
                      C.c_int(x_u16.shape[0]), _p(y))
    return y
