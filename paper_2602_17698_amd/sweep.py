"""Sweeps of the search's own hyper-parameters on the synthetic 8B-shaped model, mirroring the
paper's ablations (App. "impact of batch size k", "impact of precision search space", "impact of
block size"): update rate gamma_0, candidate set, block shape.

The paper plots perplexity; without a model to evaluate, the figure of merit here is the search's
own objective, the total sensitivity-weighted quantization error of the chosen allocation
(sum over blocks of cost[i][level[i]]), which is comparable across all three sweeps because it is a
sum over the same weights.  Printed relative to uniform quantization at floor(budget) bits on
128-column groups, next to the search time and the iterations of Algorithm 2.

    python -m paper_2602_17698_amd.sweep [--layers 32] [--budget 3.0] [--json]

Runs on one GPU through libscalebits.so; every line is one full search (reordering, cost table,
allocation).  Inputs as in bench.py (seeded, generated on the device).
"""
from __future__ import annotations

import argparse
import json
import sys
import time


def run(torch, sb, synth, dev, Ws, Ss, shapes, m, n, bits, avg, gamma0, gammaT):
    ctx = sb.Context(0, torch.cuda.current_stream().cuda_stream)
    plan = sb.Plan(ctx, shapes, m, n, bits)
    N, K = plan.num_blocks(), len(bits)
    ws = torch.empty(plan.workspace_bytes(), dtype=torch.uint8, device=dev)
    mats = [sb.matrix(w, s) for w, s in zip(Ws, Ss)]
    row_perm = torch.empty(sum(r for r, _ in shapes), dtype=torch.int32, device=dev)
    col_perm = torch.empty(sum(c for _, c in shapes), dtype=torch.int32, device=dev)
    cost = torch.empty(N, K, dtype=torch.float32, device=dev)
    level = torch.empty(N, dtype=torch.uint8, device=dev)
    one_pass = plan.gather_cost_supported()               # 64- and 128-column blocks; else gather, then score
    if not one_pass:
        nel = sum(r * c for r, c in shapes)
        w_re = torch.empty(nel, dtype=torch.bfloat16, device=dev)
        s_re = torch.empty(nel, dtype=torch.float32, device=dev)
    out = None
    for rep in range(2):                                  # the second pass is the timed one
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        plan.reorder_all(mats, row_perm, col_perm, ws)
        if one_pass:
            plan.gather_cost_all(mats, row_perm, col_perm, None, cost, ws)
        else:
            plan.gather_all(mats, row_perm, col_perm, w_re, s_re, ws)
            plan.cost_table_all(w_re, s_re, cost, ws)
        rc, st, _ = plan.allocate(cost, avg, level, ws, gamma0=gamma0, gammaT=gammaT)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3
        out = (rc, st, ms)
    rc, st, ms = out
    total = float(cost.double().gather(1, level.long().unsqueeze(1)).sum().item())
    lv = level.long()
    hist = torch.bincount(lv, minlength=K).tolist()
    plan.close()
    ctx.close()
    return {"block": [m, n], "bits": bits, "budget": avg, "gamma0": gamma0, "gammaT": gammaT, "status": rc,
            "objective": total, "search_ms": ms, "iters": st["iters"], "bits_used": st["bits_used"],
            "bits_budget": st["bits_budget"], "blocks": N, "blocks_per_level": hist,
            "effective_bits": avg + 64.0 / n}            # fp32 scale and zero per group of n weights


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--budget", type=float, default=3.0)
    ap.add_argument("--json", action="store_true", help="one JSON object per line instead of the table")
    args = ap.parse_args(argv)

    import torch
    from . import binding as sb
    from . import synth
    assert torch.cuda.is_available(), "the sweep needs a GPU"
    dev = torch.device("cuda:0")
    sb.load()

    model = dict(synth.LLAMA3_8B)
    shapes, Ws, Ss = [], [], []
    for layer in range(args.layers):
        for name, r, c in synth.layer_shapes(model):
            W, S = synth.make_matrix("student_t", r, c, seed=0, tid=synth.tensor_id(layer, name), device=dev)
            shapes.append((r, c)); Ws.append(W); Ss.append(S)
    torch.cuda.synchronize()
    B = args.budget
    full = list(range(1, 9))

    def go(tag, m, n, bits, g0, gT, avg=B):
        r = run(torch, sb, synth, dev, Ws, Ss, shapes, m, n, bits, avg, g0, gT)
        r["sweep"] = tag
        return r

    # the reference point: uniform quantization at floor(B) bits, group size 128
    uni = go("uniform", 64, 128, [int(B)], 0.05, 0.02, avg=float(int(B)))
    rows = [uni]
    for g0 in (0.01, 0.02, 0.05, 0.10, 0.20):             # App. "impact of batch size k"
        rows.append(go("gamma0", 64, 128, full, g0, min(0.02, g0)))
    for bits in ([1, 2, 3, 4], [2, 3, 4], [1, 2, 3, 4, 5, 6], full, [0] + full, [2, 3, 4, 5, 6, 7, 8], [3, 4, 5, 6, 7, 8]):
        if bits[0] <= B:                                  # App. "impact of precision search space"
            rows.append(go("space", 64, 128, bits, 0.05, 0.02))
    for m, n in ((32, 128), (64, 128), (128, 128), (256, 128), (64, 64), (128, 64), (64, 256), (128, 256)):
        rows.append(go("block", m, n, full, 0.05, 0.02))  # App. "impact of block size"

    if args.json:
        for r in rows:
            print(json.dumps(r))
        return 0
    base = uni["objective"]
    print("8B-shaped, %d layers, budget %.2f bits; objective relative to uniform %d-bit (group 128) = 1.000"
          % (args.layers, B, int(B)))
    print("%-8s %-9s %-22s %6s %6s  %9s %6s %9s %8s" % ("sweep", "block", "bits", "g0", "gT", "objective", "iters",
                                                         "search ms", "eff.bits"))
    for r in rows:
        print("%-8s %-9s %-22s %6.2f %6.2f  %9.4f %6d %9.2f %8.3f"
              % (r["sweep"], "%dx%d" % tuple(r["block"]), ",".join(map(str, r["bits"])), r["gamma0"], r["gammaT"],
                 r["objective"] / base, r["iters"], r["search_ms"], r["effective_bits"]))
    return 0


if __name__ == "__main__":
    sys.exit(main())
