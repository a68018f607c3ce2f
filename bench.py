#!/usr/bin/env python3
"""Benchmark of the bitwidth-allocation search on one MI355X.

One "step" = one pass of the whole hot path over the full 32-layer Llama-3-8B-shaped
synthetic model (224 matrices, 6.98 G weights, bf16 weights + fp32 sensitivities resident
in HBM): channel scores + argsort, reorder-gather, block x bitwidth cost table, scalable
greedy allocation to the budget, offsets + bit-packing.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--layers L] [--budget B]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes of the cost stage of ONE step of the default workload (32 layers, 128 x 128 blocks, four
# candidates) from rocprofv3 counters of that very workload: FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000 in KiB
# (factors from a plain 1 GiB copy in the same runs), summed over the stage's dispatches
# (profiles/cost_stage_8b_shaped_hbm_traffic_pmc.md).  Other workloads: null.
ONE_PASS_TRAFFIC_KIB_32L = 41162492        # both gather_cost launches + octet_finish
TWO_PASS_TRAFFIC_KIB_32L = 40924660        # cost_kernel


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--layers", type=int, default=32, help="decoder layers (32 = the full 8B-shaped model)")
    ap.add_argument("--budget", type=float, default=2.5, help="average bits per weight")
    ap.add_argument("--block", type=int, default=128, help="block rows = block columns")
    ap.add_argument("--block-rows", type=int, default=0, help="block rows if different from --block")
    ap.add_argument("--bits", type=str, default="1,2,3,4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-route-check", action="store_true",
                    help="skip the untimed comparison run of the two-pass route (needs 56 GB more HBM)")
    ap.add_argument("--coupled", action="store_true",
                    help="coupled reordering (residual stream and MLP groups share permutations) instead of "
                         "per-matrix reordering")
    ap.add_argument("--two-pass", action="store_true",
                    help="separate gather and cost launches instead of the fused one-pass kernel")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cost-power", type=int, default=2, choices=(1, 2),
                    help="1: the build variant whose block cost is sum s*|d| (libscalebits_l1.so)")
    ap.add_argument("--only-mp-gemm", action="store_true",
                    help="run only the inference-product probe and print its object (for profiling that kernel)")
    ap.add_argument("--no-mp-gemm", action="store_true",
                    help="skip the untimed probe of the inference product on the paper's 8192 x 8192 workload")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy first (calibrates rocprofv3 byte counters)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the untimed runs of the other workloads (budget 3.0, 64 x 64 blocks with five "
                         "candidates, one 70B-shaped layer)")
    return ap.parse_args()


def _oracle_search(oracle, par, mats, m, n, bits, avg, power, pool, workers):
    """The whole path of the oracle on `mats` = [(W bf16 bits, S fp32)]: per-matrix stages in `pool` (or in
    this process when pool is None), the allocation on the sample's own table, offsets, packing.
    Returns seconds of wall time."""
    import threading
    import numpy as np
    shapes = [w.shape for w, _ in mats]
    t0 = time.perf_counter()
    if pool is None:
        rows, packed = [], []
        for Wn, Sn in mats:
            rs, cs = oracle.channel_scores(Sn)
            rp, cp = oracle.argsort_desc(rs), oracle.argsort_desc(cs)
            Wp, Sp = oracle.gather(Wn, Sn, rp, cp)
            rows.append(oracle.cost_table(Wp, Sp, m, n, bits, power=power))
            packed.append(Wp)
        cost = np.concatenate(rows, 0)
        rc, level, st, _ = oracle.allocate(cost, bits, avg)
        off = oracle.offsets(level, m, n, bits)
        N = cost.shape[0]
        codes = np.zeros(int(off[-1]), np.uint8)
        scale = np.zeros(N * m, np.float32)
        zero = np.zeros(N * m, np.float32)
        base = 0
        for Wp in packed:
            oracle.pack(Wp, m, n, bits, level, off, base, codes, scale, zero)
            base += (Wp.shape[0] // m) * (Wp.shape[1] // n)
        return time.perf_counter() - t0
    shm = par.SharedInputs()
    try:
        names = [(shm.put(("w", i), w), shm.put(("s", i), s_)) for i, (w, s_) in enumerate(mats)]
        t0 = time.perf_counter()                       # (the copies into shared memory are hand-over, not oracle work)
        order = sorted(range(len(mats)), key=lambda i: -mats[i][0].size)          # large matrices first
        res = {}
        for i, rp, cp, rows in pool.imap_unordered(
                par.stage_a, [(i, names[i][0], names[i][1], shapes[i][0], shapes[i][1], m, n, bits, power) for i in order]):
            res[i] = (rp, cp, rows)
        cost = np.concatenate([res[i][2] for i in range(len(mats))], 0)
        rc, level, st, _ = oracle.allocate(cost, bits, avg)
        bases, b = [], 0
        for r, c in shapes:
            bases.append(b)
            b += (r // m) * (c // n)
        nb = lambda i: (shapes[i][0] // m) * (shapes[i][1] // n)
        for _ in pool.imap_unordered(
                par.stage_b, [(i, names[i][0], shapes[i][0], shapes[i][1], m, n, bits, res[i][0], res[i][1],
                               level[bases[i]:bases[i] + nb(i)]) for i in order]):
            pass
        return time.perf_counter() - t0
    finally:
        shm.free_all()


def cpu_baseline(synth, Ws, Ss, shapes, layers_all, m, n, bits, avg, power=2):
    """The oracle as it stands (single-threaded C, one call chain per matrix) on a bounded sample of the same
    workload: (a) on all host cores, one process per matrix (`value`), (b) on one core, one decoder layer
    (`one_core`).  The sample's tensors are the benchmark's own, copied to the host."""
    import oracle
    from oracle import parallel as par
    oracle.lib()
    workers = par.cores()
    per_layer = len(shapes) // max(1, len({l for l, _, _, _ in shapes}))
    def host(layer_ids):
        idx = [i for i, (l, _, _, _) in enumerate(shapes) if l in layer_ids]
        return [(synth.bf16_bits(Ws[i]), Ss[i].cpu().numpy()) for i in idx]
    sample_layers = list(range(min(layers_all, 4)))
    mats = host(sample_layers)
    nw = sum(w.size for w, _ in mats)
    pool = par.pool(workers)
    try:
        dt = _oracle_search(oracle, par, mats, m, n, bits, avg, power, pool, workers)
    finally:
        pool.terminate()
        pool.join()
    one = mats[:per_layer]
    nw1 = sum(w.size for w, _ in one)
    dt1 = _oracle_search(oracle, par, one, m, n, bits, avg, power, None, 1)
    return {"value": nw / dt, "unit": "weights/s", "cores": workers, "kind": "oracle",
            "sample": "decoder layers %s, all 7 projections each (%d weights): per-matrix stages one process per "
                      "matrix on %d cores, allocation on the sample's own table in one, %.1f s wall"
                      % (sample_layers, nw, workers, dt),
            "one_core": {"value": nw1 / dt1, "unit": "weights/s", "cores": 1,
                         "sample": "decoder layer 0 (%d weights), whole path in one process, %.1f s" % (nw1, dt1),
                         "whole_model_extrapolated_s": None}}


def mp_gemm_probe(torch, sb, synth, dev, copy_probe=False):
    """The paper's kernel workload beside the search (outside the timed region): an 8192 x 8192
    projection at 4 bits on average, all INT4 tiles or 40 % INT2 / 40 % INT4 / 20 % INT8, batch 16 and
    32 (Sec. 5.3, kernel-latency table).  Latency per call over 200 back-to-back calls; bytes = the
    packed codes plus scales and zeros."""
    import numpy as np
    R = C = 8192
    m = n = 128
    bits = [2, 4, 8]
    ctx = sb.Context(0, torch.cuda.current_stream().cuda_stream)
    plan = sb.Plan(ctx, [(R, C)], m, n, bits)
    N = plan.num_blocks()
    ws = torch.empty(plan.workspace_bytes(), dtype=torch.uint8, device=dev)
    W, _ = synth.make_matrix("student_t", R, C, seed=0, tid=0, device=dev)
    res = {"workload": "8192 x 8192 projection, 128 x 128 tiles, 4 bits per weight on average", "cases": []}
    for name, mix in (("all INT4", (0.0, 1.0, 0.0)), ("40% INT2 / 40% INT4 / 20% INT8", (0.4, 0.4, 0.2))):
        counts = [int(round(f * N)) for f in mix]
        counts[1] += N - sum(counts)
        lv = np.random.default_rng(0).permutation(np.repeat(np.arange(3, dtype=np.uint8), counts))
        level = torch.from_numpy(lv).to(dev)
        off = torch.empty(N + 1, dtype=torch.int64, device=dev)
        plan.offsets(level, off, ws)
        torch.cuda.synchronize()
        codes = torch.zeros(int(off[-1].item()), dtype=torch.uint8, device=dev)
        scale = torch.empty(N * m, dtype=torch.float32, device=dev)
        zero = torch.empty(N * m, dtype=torch.float32, device=dev)
        plan.pack_all(W.reshape(-1), level, off, codes, scale, zero, ws)
        nbytes = codes.numel() + 8 * N * m
        for batch in (16, 32):
            x = torch.randn(batch, C, device=dev).to(torch.bfloat16)
            y = torch.empty(batch, R, dtype=torch.float32, device=dev)
            for _ in range(10):
                plan.mp_gemm(0, x, level, off, codes, scale, zero, y, ws)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 200
            e0.record()
            for _ in range(reps):
                plan.mp_gemm(0, x, level, off, codes, scale, zero, y, ws)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / reps * 1e3
            ref = x.float() @ (W.float().t())                 # the unquantized product, for scale only
            res["cases"].append({"tiles": name, "batch": batch, "latency_us": us, "packed_bytes": nbytes,
                                 "GBs": nbytes / us * 1e-3, "frac_of_hbm_peak": nbytes / us * 1e-3 / HBM_PEAK_GBS,
                                 "rel_diff_to_unquantized": float((y - ref).norm() / ref.norm())})
    if copy_probe:                                   # a copy of known size, to scale the byte counters by
        a = torch.empty(1 << 28, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
    plan.close()
    ctx.close()
    return res


class Search:
    """One workload resident on the device: a plan over its matrices and the output buffers of a step."""

    STAGES = ["reorder", "gather", "cost", "allocate", "offsets_pack"]

    def __init__(self, torch, sb, dev, shapes, Ws, Ss, m, n, bits, budget, two_pass=False, coupling=None):
        self.torch, self.sb = torch, sb
        self.shapes, self.m, self.n, self.bits, self.budget = shapes, m, n, bits, budget
        self.K = len(bits)
        self.ctx = sb.Context(0, torch.cuda.current_stream().cuda_stream)
        self.plan = sb.Plan(self.ctx, [(r, c) for _, _, r, c in shapes], m, n, bits)
        self.N = self.plan.num_blocks()
        self.nw = sum(r * c for _, _, r, c in shapes)
        self.ws = torch.empty(self.plan.workspace_bytes(), dtype=torch.uint8, device=dev)
        self.mats = [sb.matrix(w, s_) for w, s_ in zip(Ws, Ss)]
        self.row_perm = torch.empty(sum(r for _, _, r, _ in shapes), dtype=torch.int32, device=dev)
        self.col_perm = torch.empty(sum(c for _, _, _, c in shapes), dtype=torch.int32, device=dev)
        self.one_pass = bool(self.plan.gather_cost_supported()) and not two_pass
        # reordered matrices, concatenated: only the two-pass route materialises them
        self.w_re = None if self.one_pass else torch.empty(self.nw, dtype=torch.bfloat16, device=dev)
        self.s_re = None if self.one_pass else torch.empty(self.nw, dtype=torch.float32, device=dev)
        self.cost = torch.empty(self.N, self.K, dtype=torch.float32, device=dev)
        self.level = torch.empty(self.N, dtype=torch.uint8, device=dev)
        self.byte_off = torch.empty(self.N + 1, dtype=torch.int64, device=dev)
        self.codes = torch.empty(self.plan.codes_bytes_bound(budget), dtype=torch.uint8, device=dev)
        self.scale = torch.empty(self.N * m, dtype=torch.float32, device=dev)
        self.zero = torch.empty(self.N * m, dtype=torch.float32, device=dev)
        self.coupling = coupling

    def step(self, ev):
        p, ws = self.plan, self.ws
        ev[0].record()
        if self.coupling:
            c = self.coupling
            p.reorder_coupled_all(self.mats, c[0], c[1], c[2], c[3], self.row_perm, self.col_perm, ws, c[4], c[5])
        else:
            p.reorder_all(self.mats, self.row_perm, self.col_perm, ws)
        ev[1].record()
        if self.one_pass:                            # the reorder-gather is fused into the cost pass
            ev[2].record()
            p.gather_cost_all(self.mats, self.row_perm, self.col_perm, self.w_re, self.cost, ws)
        else:
            p.gather_all(self.mats, self.row_perm, self.col_perm, self.w_re, self.s_re, ws)
            ev[2].record()
            p.cost_table_all(self.w_re, self.s_re, self.cost, ws)
        ev[3].record()
        rc, st, _ = p.allocate(self.cost, self.budget, self.level, ws)
        ev[4].record()
        p.offsets(self.level, self.byte_off, ws)
        if self.one_pass:
            p.gather_pack_all(self.mats, self.row_perm, self.col_perm, self.level, self.byte_off, self.codes,
                              self.scale, self.zero, ws)
        else:
            p.pack_all(self.w_re, self.level, self.byte_off, self.codes, self.scale, self.zero, ws)
        ev[5].record()
        return rc, st

    def run(self, steps, warmup):
        """W untimed steps, then K timed ones between two device synchronisations; stage times from HIP
        events on the library's stream (torch's current stream: the context was created on it)."""
        torch = self.torch
        new_events = lambda: [torch.cuda.Event(enable_timing=True) for _ in range(6)]
        for _ in range(warmup):
            self.step(new_events())
        torch.cuda.synchronize()
        evs = []
        t0 = time.perf_counter()
        for _ in range(steps):
            ev = new_events()
            rc, st = self.step(ev)
            evs.append(ev)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        stage_ms = {nm_: sum(e[i].elapsed_time(e[i + 1]) for e in evs) / steps for i, nm_ in enumerate(self.STAGES)}
        return {"ms_per_step": wall * 1e3 / steps, "stage_ms": stage_ms, "stats": st, "status": rc}

    def cost_stage(self, cost_ms):
        """Algorithmic bytes of the cost stage: each weight once as bf16 (2 B) with its fp32 sensitivity (4 B),
        the table (4K B per block); the one-pass kernel also reads both permutations."""
        b = self.nw * 6 + self.N * self.K * 4
        if self.one_pass:
            b += 4 * (self.row_perm.numel() + self.col_perm.numel())
        gbs = b / (cost_ms * 1e-3) / 1e9
        return {"kernel": "gather_cost_kernel" if self.one_pass else "cost_kernel", "algorithmic_bytes": b,
                "GBs": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}

    def path_bytes(self):
        """What the route has to move per step: S once for the scores, W and S once for the table, W once
        more and the packed output for the codes (two-pass: the reordered copies written and read as well)."""
        packed = int(self.byte_off[-1].item()) + 8 * self.N * self.m
        perms = 4 * (self.row_perm.numel() + self.col_perm.numel())
        nw, tab = self.nw, self.N * self.K * 4
        if self.one_pass:
            return (nw * 4) + (nw * 6 + tab + perms) + (nw * 2 + packed + perms)
        return (nw * 4) + (nw * 12 + perms) + (nw * 6 + tab) + (nw * 2 + packed)

    def close(self):
        self.plan.close()
        self.ctx.close()


def model_shapes(synth, model, layers):
    return [(layer, name, r, c) for layer in range(layers) for name, r, c in synth.layer_shapes(model)]


def generate(torch, synth, dev, shapes, recipe, seed):
    Ws, Ss = [], []
    for layer, name, r, c in shapes:
        W, S = synth.make_matrix(recipe, r, c, seed=seed, tid=synth.tensor_id(layer, name), device=dev)
        Ws.append(W)
        Ss.append(S)
    torch.cuda.synchronize()
    return Ws, Ss


def extra_run(torch, sb, dev, what, shapes, Ws, Ss, m, n, bits, budget):
    """One more workload beside the headline one, outside its timed region: 2 warm-ups + 4 steps."""
    srch = Search(torch, sb, dev, shapes, Ws, Ss, m, n, bits, budget)
    r = srch.run(4, 2)
    out = {"workload": what, "route": "one-pass" if srch.one_pass else "two-pass", "ms_per_step": r["ms_per_step"],
           "stage_ms": r["stage_ms"], "cost_stage": srch.cost_stage(r["stage_ms"]["cost"]),
           "iterations": r["stats"]["iters"], "search_status": r["status"], "blocks": srch.N, "weights": srch.nw}
    srch.close()
    del srch
    torch.cuda.empty_cache()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding "
              "in this library; see DESIGN.md for how the path would shard)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_17698_amd import binding as sb
    from paper_2602_17698_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.cost_power == 1:
        sb.use_library(sb.variant_path("l1"))
    sb.load()
    assert sb.cost_power() == args.cost_power
    if args.only_mp_gemm:
        print(json.dumps({"mp_gemm": mp_gemm_probe(torch, sb, synth, dev, copy_probe=args.copy_probe)}))
        return
    bits = [int(b) for b in args.bits.split(",")]
    n = args.block
    m = args.block_rows or args.block
    K = len(bits)
    model = dict(synth.LLAMA3_8B)
    shapes = model_shapes(synth, model, args.layers)

    # ---- synthetic inputs, generated on the device, resident before any timing ----
    t_gen = time.perf_counter()
    Ws, Ss = generate(torch, synth, dev, shapes, "student_t", args.seed)
    t_gen = time.perf_counter() - t_gen

    coupling = synth.llama_coupling(model, args.layers) if args.coupled else None
    srch = Search(torch, sb, dev, shapes, Ws, Ss, m, n, bits, args.budget, two_pass=args.two_pass, coupling=coupling)
    N, nw, nm, one_pass = srch.N, srch.nw, len(shapes), srch.one_pass

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    r = srch.run(args.steps, args.warmup)
    ms_per_step, stage_ms, st, rc = r["ms_per_step"], r["stage_ms"], r["stats"], r["status"]
    cost_ms = stage_ms["cost"]
    cs = srch.cost_stage(cost_ms)
    default_workload = args.layers == 32 and m == 128 and n == 128 and bits == [1, 2, 3, 4] and not args.coupled
    kib = (ONE_PASS_TRAFFIC_KIB_32L if one_pass else TWO_PASS_TRAFFIC_KIB_32L) if default_workload else None
    launches = 1            # the stage covers all matrices (one-pass: one launch per column-count class)

    out = {
        "metric": "weights scored/s through the whole search path (8B-shaped, all bitwidths)",
        "value": nw / (ms_per_step * 1e-3),
        "unit": "weights/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "Llama-3-8B-shaped, %d layers, %d matrices, %d weights (bf16) + fp32 sensitivity, "
                               "%dx%d blocks (%d), bitwidths %s, budget %.2f%s"
                               % (args.layers, nm, nw, m, n, N, bits, args.budget,
                                  (", coupled reordering" if args.coupled else "")
                                  + (", cost = sum s*|d|" if args.cost_power == 1 else ""))},
        "full_search_ms": ms_per_step,
        "stage_ms": stage_ms,
        "cost_pass_weights_per_s": nw / (cost_ms * 1e-3),
        "search_stats": st, "search_status": rc,
        "gen_s": t_gen,
        "roofline": {"kernel": cs["kernel"], "bound": "hbm", "achieved": cs["GBs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": cs["frac_of_hbm_peak"],
                     "traffic": kib * 1024.0 if kib else None,
                     "launches_per_step": launches, "avg_launch_ms": cost_ms / launches,
                     "algorithmic_bytes_per_launch": cs["algorithmic_bytes"] / launches},
    }
    path_bytes = srch.path_bytes()
    out["whole_path"] = {"algorithmic_bytes_per_step": path_bytes, "GBs": path_bytes / (ms_per_step * 1e-3) / 1e9,
                         "frac_of_hbm_peak": path_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "bytes_per_weight": path_bytes / nw}
    if one_pass and not args.no_route_check:
        # the two-pass route beside it, outside the timed region: its cost kernel alone (a5 as a
        # separate pass over reordered copies) and the bit-equality of the two tables
        plan, ws, mats, cost = srch.plan, srch.ws, srch.mats, srch.cost
        w2 = torch.empty(nw, dtype=torch.bfloat16, device=dev)
        s2 = torch.empty(nw, dtype=torch.float32, device=dev)
        cost2 = torch.empty_like(cost)
        plan.reorder_all(mats, srch.row_perm, srch.col_perm, ws)
        plan.gather_cost_all(mats, srch.row_perm, srch.col_perm, None, cost, ws)
        e = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
        e[0].record()
        plan.gather_all(mats, srch.row_perm, srch.col_perm, w2, s2, ws)
        e[1].record()
        for i in range(3):
            plan.cost_table_all(w2, s2, cost2, ws)
            e[2 + i].record()
        torch.cuda.synchronize()
        t_cost = sorted(e[1 + i].elapsed_time(e[2 + i]) for i in range(3))[1]
        b2 = nw * 6 + N * K * 4
        out["two_pass_route"] = {"gather_ms": e[0].elapsed_time(e[1]), "cost_kernel_ms": t_cost,
                                 "cost_kernel_GBs": b2 / (t_cost * 1e-3) / 1e9,
                                 "cost_kernel_frac_of_hbm_peak": b2 / (t_cost * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                 "cost_kernel_weights_per_s": nw / (t_cost * 1e-3),
                                 "tables_bit_equal": bool(torch.equal(cost.view(torch.int32), cost2.view(torch.int32)))}
        del w2, s2, cost2
    srch.close()
    del srch
    torch.cuda.empty_cache()
    if not args.no_mp_gemm:
        out["mp_gemm"] = mp_gemm_probe(torch, sb, synth, dev)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(synth, Ws, Ss, shapes, args.layers, m, n, bits, args.budget,
                                           power=args.cost_power)
        one = out["cpu_baseline"]["one_core"]
        one["whole_model_extrapolated_s"] = nw / one["value"]
    if not args.no_extras and default_workload and args.cost_power == 2 and not args.two_pass:
        # the other workloads the search is specified on, each one run outside the headline's timed region
        ex = {}
        ex["budget_3.0"] = extra_run(torch, sb, dev, "the same model and candidates, budget 3.00 (the warm start is on "
                                     "budget: swaps only)", shapes, Ws, Ss, m, n, bits, 3.0)
        ex["paper_default_space"] = extra_run(torch, sb, dev, "the same model, the paper's default search space: 64x128 "
                                              "blocks (group 128), bitwidths [1 .. 8], budget 3.00", shapes, Ws, Ss,
                                              64, 128, [1, 2, 3, 4, 5, 6, 7, 8], 3.0)
        del Ws, Ss
        torch.cuda.empty_cache()
        W5, S5 = generate(torch, synth, dev, shapes, "outlier_chan", args.seed)
        ex["blocks_64x64_five_candidates"] = extra_run(
            torch, sb, dev, "8B-shaped, Student-t(3) weights with rare x100 outlier channels, 64x64 blocks "
            "(group 64), bitwidths [1, 2, 3, 4, 8], budget 2.25", shapes, W5, S5, 64, 64, [1, 2, 3, 4, 8], 2.25)
        del W5, S5
        torch.cuda.empty_cache()
        s70 = model_shapes(synth, dict(synth.LLAMA3_70B), 1)
        W7, S7 = generate(torch, synth, dev, s70, "student_t", args.seed)
        ex["one_70b_shaped_layer"] = extra_run(
            torch, sb, dev, "one decoder layer of the 70B-shaped model (7 matrices, hidden 8192, ffn 28672; the model "
            "itself is streamed layer by layer), 128x128 blocks, bitwidths [2, 3, 4], budget 2.75 on the layer's "
            "own table; the six matrices with rows of 8192 elements take the one-pass kernels, the 28672-column one "
            "a reordered copy in the workspace for the cost stage", s70, W7, S7, 128, 128, [2, 3, 4], 2.75)
        del W7, S7
        out["extras"] = ex
    print(json.dumps(out))


if __name__ == "__main__":
    main()
