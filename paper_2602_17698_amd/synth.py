"""Seeded synthetic inputs for the bitwidth-allocation search.

This module holds no arithmetic of the method: it only draws weights and
sensitivities with the shapes and value distributions of the workloads the
search is measured on (Llama-3-8B / 70B shaped projection matrices).  The same
tensors are handed to the GPU library and, copied to the host, to the CPU
oracle, so generator differences between devices never matter.

Recipes
  "gauss_outlier"  W = 0.02*Z, each element x50 with probability 0.001;
                   S = Z'^2                                   (small single matrix)
  "student_t"      W = 0.02*t_nu (Student-t, nu degrees of freedom);
                   S = exp(sr*a_i + sc*b_j + se*z_ij): log-normal with a rank-one
                   row x column structure, as the paper's element sensitivity
                   |g_i||x_j||dW_ij| has (Sec. 3.2)
  "outlier_chan"   student_t with nu = 3 plus max(1, round(0.005*dim)) outlier
                   rows and as many outlier columns at scattered positions:
                   weights x100 there, sensitivity row/column factor x100
"""
from __future__ import annotations

import torch

LLAMA3_8B = dict(hidden=4096, ffn=14336, kv=1024, layers=32)
LLAMA3_70B = dict(hidden=8192, ffn=28672, kv=1024, layers=80)
PROJ = ("q", "k", "v", "o", "gate", "up", "down")


def layer_shapes(model: dict):
    """(name, rows = d_out, cols = d_in) of the seven projections of one decoder layer."""
    h, f, kv = model["hidden"], model["ffn"], model["kv"]
    return [("q", h, h), ("k", kv, h), ("v", kv, h), ("o", h, h),
            ("gate", f, h), ("up", f, h), ("down", h, f)]


def llama_coupling(model: dict, layers: int, head_dim: int = 128):
    """Permutation groups of a Llama-shaped decoder stack, matrices in layer_shapes() order per layer
    (paper App. "Channel Reordering"): group 0 = the residual stream (columns of q, k, v, gate, up and
    rows of o, down of every layer); per layer one group for the MLP activation (rows of gate, up,
    columns of down) and one for the attention values (rows of v, columns of o), reordered inside
    each head only.  With grouped-query attention one value head serves hidden / kv query heads: the
    columns of o are that many times the rows of v (repeat).  Rows of q and k stay fixed (rotary
    embeddings).
    Returns (row_group, col_group, n_groups, group_segment, row_repeat, col_repeat) for
    sbits_reorder_coupled_all."""
    FIXED = -2
    rep = model["hidden"] // model["kv"]
    row_group, col_group, row_repeat, col_repeat = [], [], [], []
    segment = [0]
    for layer in range(layers):
        mlp, att = 1 + 2 * layer, 2 + 2 * layer
        row_group += [FIXED, FIXED, att, 0, mlp, mlp, 0]            # q k v o gate up down
        col_group += [0, 0, 0, att, 0, 0, mlp]
        row_repeat += [1] * 7
        col_repeat += [1, 1, 1, rep, 1, 1, 1]
        segment += [0, head_dim]
    return row_group, col_group, 1 + 2 * layers, segment, row_repeat, col_repeat


def tensor_id(layer: int, proj: str) -> int:
    return layer * 16 + PROJ.index(proj) * 2


def _gen(seed: int, tid: int, device):
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + tid * 7919 + 12345) & 0x7FFFFFFFFFFFFFFF)
    return g


def _student_t(rows, cols, nu, g, device, row_chunk=2048):
    out = torch.empty(rows, cols, dtype=torch.float32, device=device)
    for r0 in range(0, rows, row_chunk):
        r1 = min(rows, r0 + row_chunk)
        z = torch.randn(r1 - r0, cols, generator=g, device=device)
        chi = torch.zeros_like(z)
        for _ in range(nu):
            chi += torch.randn(r1 - r0, cols, generator=g, device=device) ** 2
        out[r0:r1] = z / torch.sqrt(chi / nu)
    return out


def make_matrix(recipe: str, rows: int, cols: int, seed: int = 0, tid: int = 0,
                device="cpu", nu: int = 4, sr: float = 1.0, sc: float = 1.0, se: float = 0.5):
    """Returns (W bf16 [rows, cols], S fp32 [rows, cols]) on `device`."""
    g = _gen(seed, tid, device)
    if recipe == "gauss_outlier":
        w = 0.02 * torch.randn(rows, cols, generator=g, device=device)
        hit = torch.rand(rows, cols, generator=g, device=device) < 0.001
        w = torch.where(hit, w * 50.0, w)
        s = torch.randn(rows, cols, generator=g, device=device) ** 2
        return w.to(torch.bfloat16).contiguous(), s.contiguous()
    if recipe in ("student_t", "outlier_chan"):
        if recipe == "outlier_chan":
            nu = 3
        w = 0.02 * _student_t(rows, cols, nu, g, device)
        a = sr * torch.randn(rows, 1, generator=g, device=device)
        b = sc * torch.randn(1, cols, generator=g, device=device)
        if recipe == "outlier_chan":
            nro = max(1, round(0.005 * rows))
            nco = max(1, round(0.005 * cols))
            ri = torch.randperm(rows, generator=g, device=device)[:nro]
            ci = torch.randperm(cols, generator=g, device=device)[:nco]
            w[ri, :] *= 100.0
            w[:, ci] *= 100.0
            a[ri, 0] += 4.605170185988092   # log(100)
            b[0, ci] += 4.605170185988092
        s = torch.empty(rows, cols, dtype=torch.float32, device=device)
        chunk = 2048
        for r0 in range(0, rows, chunk):
            r1 = min(rows, r0 + chunk)
            z = torch.randn(r1 - r0, cols, generator=g, device=device)
            s[r0:r1] = torch.exp(a[r0:r1] + b + se * z)
        return w.to(torch.bfloat16).contiguous(), s.contiguous()
    raise ValueError("unknown recipe %r" % recipe)


def make_layer(model: dict, layer: int, recipe: str = "student_t", seed: int = 0,
               device="cpu", **kw):
    """The seven projections of one decoder layer: list of (name, W, S)."""
    out = []
    for name, r, c in layer_shapes(model):
        w, s = make_matrix(recipe, r, c, seed=seed, tid=tensor_id(layer, name), device=device, **kw)
        out.append((name, w, s))
    return out


def bf16_bits(w: torch.Tensor):
    """Raw uint16 view (numpy) of a CPU bf16 tensor, for the oracle."""
    return w.detach().cpu().contiguous().view(torch.int16).numpy().view("uint16")
