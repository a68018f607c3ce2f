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
# HBM bytes per weight of the cost kernel from rocprofv3 counters (FETCH_SIZE x 2.000 and WRITE_SIZE
# x 1.000 after calibration against a plain 1 GiB copy; profiles/hbm_traffic_8_layers_pmc.md)
COST_TRAFFIC_B_PER_WEIGHT = (5114570 * 2.0 + 1664) * 1024 / 1744830464
# the same for the one-pass stage: both gather_cost launches + octet_finish
ONE_PASS_TRAFFIC_B_PER_WEIGHT = ((3739368 + 1378226 + 13328) * 2.0 + 20405 + 7594 + 1664) * 1024 / 1744830464


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
    return ap.parse_args()


def cpu_baseline(torch, synth, shapes_sample, m, n, bits, avg, seed, power=2):
    """The oracle as it stands, single-threaded, on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    oracle.lib()
    mats = []
    for layer, name, r, c in shapes_sample:
        W, S = synth.make_matrix("student_t", r, c, seed=seed, tid=synth.tensor_id(layer, name))
        mats.append((synth.bf16_bits(W), S.numpy()))
    nw = sum(w.size for w, _ in mats)
    t0 = time.perf_counter()
    costs, packed = [], []
    for Wn, Sn in mats:
        rs, cs = oracle.channel_scores(Sn)
        rp, cp = oracle.argsort_desc(rs), oracle.argsort_desc(cs)
        Wp, Sp = oracle.gather(Wn, Sn, rp, cp)
        costs.append(oracle.cost_table(Wp, Sp, m, n, bits, power=power))
        packed.append(Wp)
    cost = np.concatenate(costs, 0)
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
    dt = time.perf_counter() - t0
    return {"value": nw / dt, "unit": "weights/s", "cores": 1, "kind": "oracle",
            "sample": "decoder layers %s, all 7 projections each (%d weights), whole path incl. allocation on "
                      "the sample's own table, %.1f s" % (sorted({l for l, _, _, _ in shapes_sample}), nw, dt)}


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
    shapes = []
    for layer in range(args.layers):
        for name, r, c in synth.layer_shapes(model):
            shapes.append((layer, name, r, c))

    # ---- synthetic inputs, generated on the device, resident before any timing ----
    t_gen = time.perf_counter()
    Ws, Ss = [], []
    for layer, name, r, c in shapes:
        W, S = synth.make_matrix("student_t", r, c, seed=args.seed, tid=synth.tensor_id(layer, name), device=dev)
        Ws.append(W)
        Ss.append(S)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    ctx = sb.Context(0, torch.cuda.current_stream().cuda_stream)
    plan = sb.Plan(ctx, [(r, c) for _, _, r, c in shapes], m, n, bits)
    N = plan.num_blocks()
    nw = sum(r * c for _, _, r, c in shapes)
    ws = torch.empty(plan.workspace_bytes(), dtype=torch.uint8, device=dev)
    mats = [sb.matrix(w, s) for w, s in zip(Ws, Ss)]
    row_perm = torch.empty(sum(r for _, _, r, _ in shapes), dtype=torch.int32, device=dev)
    col_perm = torch.empty(sum(c for _, _, _, c in shapes), dtype=torch.int32, device=dev)
    one_pass = plan.gather_cost_supported() and not args.two_pass
    # reordered matrices, concatenated: only the two-pass route materialises them
    w_re = None if one_pass else torch.empty(nw, dtype=torch.bfloat16, device=dev)
    s_re = None if one_pass else torch.empty(nw, dtype=torch.float32, device=dev)
    cost = torch.empty(N, K, dtype=torch.float32, device=dev)
    level = torch.empty(N, dtype=torch.uint8, device=dev)
    byte_off = torch.empty(N + 1, dtype=torch.int64, device=dev)
    codes = torch.empty(plan.codes_bytes_bound(args.budget), dtype=torch.uint8, device=dev)
    scale = torch.empty(N * m, dtype=torch.float32, device=dev)
    zero = torch.empty(N * m, dtype=torch.float32, device=dev)
    nm = len(shapes)

    # one_pass: the reorder-gather is fused into the cost pass (stage "gather" is then empty)
    stage_names = ["reorder", "gather", "cost", "allocate", "offsets_pack"]

    coupling = synth.llama_coupling(model, args.layers) if args.coupled else None

    def step(ev):
        ev[0].record()
        if coupling:
            plan.reorder_coupled_all(mats, coupling[0], coupling[1], coupling[2], coupling[3], row_perm, col_perm, ws,
                                     coupling[4], coupling[5])
        else:
            plan.reorder_all(mats, row_perm, col_perm, ws)
        ev[1].record()
        if one_pass:
            ev[2].record()
            plan.gather_cost_all(mats, row_perm, col_perm, w_re, cost, ws)
        else:
            plan.gather_all(mats, row_perm, col_perm, w_re, s_re, ws)
            ev[2].record()
            plan.cost_table_all(w_re, s_re, cost, ws)
        ev[3].record()
        rc, st, _ = plan.allocate(cost, args.budget, level, ws)
        ev[4].record()
        plan.offsets(level, byte_off, ws)
        if one_pass:
            plan.gather_pack_all(mats, row_perm, col_perm, level, byte_off, codes, scale, zero, ws)
        else:
            plan.pack_all(w_re, level, byte_off, codes, scale, zero, ws)
        ev[5].record()
        return rc, st

    def new_events():
        return [torch.cuda.Event(enable_timing=True) for _ in range(6)]

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step(new_events())
    torch.cuda.synchronize()

    evs = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ev = new_events()
        rc, st = step(ev)
        evs.append(ev)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    stage_ms = {nm_: sum(e[i].elapsed_time(e[i + 1]) for e in evs) / args.steps for i, nm_ in enumerate(stage_names)}
    cost_ms = stage_ms["cost"]
    # cost-table pass: each weight is read once as bf16 (2 B) with its fp32 sensitivity (4 B);
    # the table written is K*4 bytes per m*n weights.  The one-pass kernel also reads both
    # permutations.
    if one_pass:
        cost_bytes = nw * 6 + N * K * 4 + 4 * (row_perm.numel() + col_perm.numel())
        kernel = "gather_cost_kernel"
        traffic = ONE_PASS_TRAFFIC_B_PER_WEIGHT * nw if (m == 128 and K == 4 and ONE_PASS_TRAFFIC_B_PER_WEIGHT) else None
    else:
        cost_bytes = nw * 6 + N * K * 4
        kernel = "cost_kernel"
        traffic = COST_TRAFFIC_B_PER_WEIGHT * nw if (m == 128 and K == 4) else None
    launches = 1            # the stage covers all matrices (one-pass: one launch per column-count class)
    achieved = cost_bytes / (cost_ms * 1e-3) / 1e9

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
        "roofline": {"kernel": kernel, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "launches_per_step": launches, "avg_launch_ms": cost_ms / launches,
                     "algorithmic_bytes_per_launch": cost_bytes / launches},
    }
    # the whole step against the same roofline: what the route has to move (S once for the scores, W and S
    # once for the table, W once more and the packed output for the codes; two-pass: the reordered copies
    # written and read as well) over the wall time of a step
    packed = int(byte_off[-1].item()) + 8 * N * m
    perms = 4 * (row_perm.numel() + col_perm.numel())
    path_bytes = (nw * 4) + (nw * 6 + N * K * 4 + perms) + (nw * 2 + packed + perms) if one_pass else \
                 (nw * 4) + (nw * 12 + perms) + (nw * 6 + N * K * 4) + (nw * 2 + packed)
    out["whole_path"] = {"algorithmic_bytes_per_step": path_bytes, "GBs": path_bytes / (ms_per_step * 1e-3) / 1e9,
                         "frac_of_hbm_peak": path_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "bytes_per_weight": path_bytes / nw}
    if one_pass and not args.no_route_check:
        # the two-pass route beside it, outside the timed region: its cost kernel alone (a5 as a
        # separate pass over reordered copies) and the bit-equality of the two tables
        w2 = torch.empty(nw, dtype=torch.bfloat16, device=dev)
        s2 = torch.empty(nw, dtype=torch.float32, device=dev)
        cost2 = torch.empty_like(cost)
        plan.reorder_all(mats, row_perm, col_perm, ws)
        plan.gather_cost_all(mats, row_perm, col_perm, None, cost, ws)
        e = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
        e[0].record()
        plan.gather_all(mats, row_perm, col_perm, w2, s2, ws)
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
    if not args.no_mp_gemm:
        out["mp_gemm"] = mp_gemm_probe(torch, sb, synth, dev)
    if not args.no_cpu_baseline:
        # two full decoder layers: 436 M weights, 10-20 s of single-threaded oracle time
        sample = [(l, nm_, r, c) for l in (0, 1) for nm_, r, c in synth.layer_shapes(model)]
        out["cpu_baseline"] = cpu_baseline(torch, synth, sample, m, n, bits, args.budget, args.seed, power=args.cost_power)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
