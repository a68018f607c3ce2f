"""oracle/parallel.py (the oracle's per-matrix stages in worker processes, used by the full-model GPU
test and by the benchmark's cpu_baseline) returns what the same oracle calls return in this process."""
import numpy as np

from oracle import parallel as par


def test_worker_stages_equal_direct_oracle_calls(orc):
    rng = np.random.default_rng(0)
    shapes = [(256, 384), (128, 512), (384, 256)]
    m = n = 128
    bits = [1, 2, 3, 4]
    Wb = [orc.f32_to_bf16((rng.standard_normal((r, c)) * 0.02).astype(np.float32)) for r, c in shapes]
    Ss = [np.exp(rng.standard_normal((r, c))).astype(np.float32) for r, c in shapes]
    shm = par.SharedInputs()
    pool = par.pool(2)
    try:
        tasks = [(i, shm.put(("w", i), Wb[i]), shm.put(("s", i), Ss[i]), r, c, m, n, bits, 2)
                 for i, (r, c) in enumerate(shapes)]
        res = sorted(pool.imap_unordered(par.stage_a, tasks), key=lambda t: t[0])
        costs = []
        for i, rp, cp, rows in res:
            rs, cs = orc.channel_scores(Ss[i])
            np.testing.assert_array_equal(rp, orc.argsort_desc(rs))
            np.testing.assert_array_equal(cp, orc.argsort_desc(cs))
            Wp, Sp = orc.gather(Wb[i], Ss[i], rp, cp)
            np.testing.assert_array_equal(rows, orc.cost_table(Wp, Sp, m, n, bits))
            costs.append(rows)
        cost = np.concatenate(costs)
        _, level, _, _ = orc.allocate(cost, bits, 2.5)
        off = orc.offsets(level, m, n, bits)
        N = cost.shape[0]
        codes = np.zeros(int(off[-1]), np.uint8)
        scale = np.zeros(N * m, np.float32)
        zero = np.zeros(N * m, np.float32)
        bases, b0 = [], 0
        for i, (r, c) in enumerate(shapes):
            Wp, _ = orc.gather(Wb[i], Ss[i], res[i][1], res[i][2])
            orc.pack(Wp, m, n, bits, level, off, b0, codes, scale, zero)
            bases.append(b0)
            b0 += (r // m) * (c // n)
        tb = [(i, tasks[i][1], r, c, m, n, bits, res[i][1], res[i][2], level[bases[i]:bases[i] + (r // m) * (c // n)])
              for i, (r, c) in enumerate(shapes)]
        seen = 0
        for i, dg, nbytes, sc, ze in pool.imap_unordered(par.stage_b, tb):
            r, c = shapes[i]
            nb = (r // m) * (c // n)
            lo, hi = int(off[bases[i]]), int(off[bases[i] + nb])
            assert hi - lo == nbytes and par.digest(codes[lo:hi]) == dg
            np.testing.assert_array_equal(sc, scale[bases[i] * m:(bases[i] + nb) * m])
            np.testing.assert_array_equal(ze.view(np.uint32), zero[bases[i] * m:(bases[i] + nb) * m].view(np.uint32))
            seen += 1
        assert seen == len(shapes)
        assert par.digest(codes[:7]) != par.digest(codes[:8])
    finally:
        pool.terminate()
        pool.join()
        shm.free_all()
