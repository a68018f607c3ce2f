"""The oracle's per-matrix stages on several host cores (test infrastructure, like the rest of this package).

The oracle itself is single-threaded; a model is many matrices whose stages before and after the
global allocation are independent of each other (paper Sec. 4.1: reordering and partition are per
matrix; Sec. 5: the quantizer works on a block row).  This module runs one plain oracle call chain
per matrix in a pool of worker processes (spawned: the parent may hold a GPU context) and hands
the inputs over in shared memory.  Nothing of the method's arithmetic lives here.

  stage A, per matrix: channel scores -> permutations -> reordered copy -> cost rows
  (the caller runs the global allocation and the offsets on the concatenated rows)
  stage B, per matrix: reordered copy again -> packed codes (as a digest), scales, zeros
"""
from __future__ import annotations

import hashlib
import multiprocessing as mp
import os
from multiprocessing import shared_memory

import numpy as np


def _attach(name, shape, dtype):
    shm = shared_memory.SharedMemory(name=name)
    return shm, np.ndarray(shape, dtype=dtype, buffer=shm.buf)


def stage_a(task):
    """(idx, shm names of W (uint16 bf16 bits) and S (float32), R, C, m, n, bits, power)
    -> (idx, row_perm, col_perm, cost rows)."""
    import oracle
    idx, wname, sname, R, Cc, m, n, bits, power = task
    wshm, W = _attach(wname, (R, Cc), np.uint16)
    sshm, S = _attach(sname, (R, Cc), np.float32)
    try:
        rs, cs = oracle.channel_scores(S)
        rp, cp = oracle.argsort_desc(rs), oracle.argsort_desc(cs)
        Wp, Sp = oracle.gather(W, S, rp, cp)
        cost = oracle.cost_table(Wp, Sp, m, n, bits, power=power)
    finally:
        del W, S
        wshm.close()
        sshm.close()
    return idx, rp, cp, cost


def digest(a) -> bytes:
    return hashlib.blake2b(np.ascontiguousarray(a).view(np.uint8).reshape(-1), digest_size=16).digest()


def stage_b(task):
    """(idx, shm name of W, R, C, m, n, bits, row_perm, col_perm, levels of the matrix's blocks)
    -> (idx, digest of the matrix's code bytes, number of code bytes, scale, zero)."""
    import oracle
    idx, wname, R, Cc, m, n, bits, rp, cp, level = task
    wshm, W = _attach(wname, (R, Cc), np.uint16)
    try:
        Wp = np.ascontiguousarray(W[rp][:, cp])          # the reordered weights (plain fancy indexing)
        off = oracle.offsets(level, m, n, bits)          # offsets inside the matrix's own byte range
        codes = np.zeros(int(off[-1]), np.uint8)
        scale = np.zeros(level.size * m, np.float32)
        zero = np.zeros(level.size * m, np.float32)
        oracle.pack(Wp, m, n, bits, level, off, 0, codes, scale, zero)
    finally:
        del W
        wshm.close()
    return idx, digest(codes), int(codes.size), scale, zero


class SharedInputs:
    """Copies of matrices in shared memory, by name; freed explicitly."""

    def __init__(self):
        self._live = {}

    def put(self, key, arr):
        arr = np.ascontiguousarray(arr)
        shm = shared_memory.SharedMemory(create=True, size=max(arr.nbytes, 1))
        np.ndarray(arr.shape, dtype=arr.dtype, buffer=shm.buf)[...] = arr
        self._live[key] = shm
        return shm.name

    def free(self, key):
        shm = self._live.pop(key, None)
        if shm is not None:
            shm.close()
            shm.unlink()

    def free_all(self):
        for k in list(self._live):
            self.free(k)


def cores(limit=16) -> int:
    """Worker processes to use: the host's cores, at most `limit` (a one-GPU machine's share is 16)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(limit, n))


def pool(workers):
    """A pool of freshly started interpreters (no fork: the parent may have initialised the GPU)."""
    import oracle
    oracle.lib()                                         # built before the workers load it
    return mp.get_context("spawn").Pool(workers)
