"""Seeded synthetic inputs with the shapes of the five benchmark configurations.

Input generation only: no arithmetic of the method lives here.  The same
tensors are handed to the HIP path (on the GPU) and, copied to the host, to the
CPU oracle.  They stand in for the paper's Llama-2 / OPT runs on WMT18-DeEn,
XSum and Dolly, which need model weights and datasets that are not available.

Logits are indexed by tree node: row (b, i) holds the next-token logits of the
model after the token sequence that ends in node i of sequence b, so "running
the draft or target model" on a tree is a row lookup.
"""
import math

import torch

CONFIGS = [
    dict(name="cfg0_tiny", B=1, V=64, sampler="gumbel", branching=(2, 2), N=7,
         Hq=1, Hkv=1, D=64, P=32, dtype="f32", logits="normal"),
    dict(name="cfg1_llama2_7b", B=1, V=32000, sampler="gumbel", branching=(3, 2, 2, 1), N=34,
         Hq=32, Hkv=32, D=128, P=1024, dtype="bf16", logits="zipf"),
    dict(name="cfg2_opt_13b_sbs", B=8, V=50272, sampler="sbs", width=6, depth=6, N=37,
         Hq=40, Hkv=40, D=128, P=2048, dtype="bf16", logits="zipf"),
    dict(name="cfg3_llama2_70b_gqa", B=16, V=32000, sampler="gumbel", branching=(4, 3, 2, 1), N=65,
         Hq=64, Hkv=8, D=128, P=4096, dtype="bf16", logits="zipf"),
    dict(name="cfg4_stress", B=64, V=32000, sampler="gumbel", branching=(8, 4, 2), N=64,
         random_subtree=True, Hq=32, Hkv=32, D=128, P=8192, dtype="bf16", logits="zipf"),
]


def config(index_or_name):
    for i, c in enumerate(CONFIGS):
        if index_or_name == i or index_or_name == c["name"]:
            return dict(c)
    raise KeyError(index_or_name)


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def make_logits(kind, B, N, V, seed, device="cpu", chunk_rows=1024):
    """(target_logits, draft_logits), each [B,N,V] fp32.

    kind "normal": target ~ N(0, 2^2).  kind "zipf": target = -1.1 * log(rank) + N(0,1)
    with rank an independent random permutation of 1..V per row.  In both cases
    draft = target + N(0,1).
    """
    g = _gen(seed, device)
    rows = B * N
    zt = torch.empty((rows, V), dtype=torch.float32, device=device)
    zd = torch.empty((rows, V), dtype=torch.float32, device=device)
    for lo in range(0, rows, chunk_rows):
        hi = min(rows, lo + chunk_rows)
        n = hi - lo
        if kind == "normal":
            t = 2.0 * torch.randn((n, V), generator=g, device=device)
        elif kind == "zipf":
            perm = torch.rand((n, V), generator=g, device=device).argsort(dim=1)
            rank = torch.empty_like(perm)
            rank.scatter_(1, perm, torch.arange(1, V + 1, device=device).expand(n, V))
            t = -1.1 * torch.log(rank.to(torch.float32)) + torch.randn((n, V), generator=g, device=device)
        else:
            raise ValueError(kind)
        zt[lo:hi] = t
        zd[lo:hi] = t + torch.randn((n, V), generator=g, device=device)
    return zt.view(B, N, V), zd.view(B, N, V)


def make_qkv(B, Hq, Hkv, N, D, P, dtype, seed, device="cpu"):
    """q [B,Hq,N,D], k_prefix/v_prefix [B,Hkv,P,D], k_tree/v_tree [B,Hkv,N,D], all ~ N(0,1)
    rounded to `dtype` ("bf16" or "f32")."""
    g = _gen(seed, device)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32

    def rnd(*shape):
        out = torch.empty(shape, dtype=td, device=device)
        flat = out.view(-1)
        step = 1 << 26
        for lo in range(0, flat.numel(), step):
            hi = min(flat.numel(), lo + step)
            flat[lo:hi] = torch.randn(hi - lo, generator=g, device=device).to(td)
        return out

    return (rnd(B, Hq, N, D), rnd(B, Hkv, P, D), rnd(B, Hkv, P, D),
            rnd(B, Hkv, N, D), rnd(B, Hkv, N, D))


def full_tree_child_counts(branching):
    """Per-level child counts of the complete tree with the given branching factors."""
    counts, n = [], 1
    for b in branching:
        counts.append([b] * n)
        n *= b
    return counts


def random_subtree_child_counts(branching, n_keep, seed):
    """Child counts, per level in level order, of a random n_keep-node (root included)
    subtree of the complete `branching` tree that is closed under parents and under
    earlier siblings: grown one node at a time, each time uniformly among the nodes whose
    parent and previous sibling are already kept."""
    g = torch.Generator()
    g.manual_seed(int(seed))
    kept = {()}
    frontier = [(0,)] if branching else []
    while len(kept) < n_keep and frontier:
        pick = frontier.pop(int(torch.randint(len(frontier), (1,), generator=g)))
        kept.add(pick)
        if pick[-1] + 1 < branching[len(pick) - 1]:
            frontier.append(pick[:-1] + (pick[-1] + 1,))
        if len(pick) < len(branching):
            frontier.append(pick + (0,))
    counts = []
    for level in range(len(branching)):
        nodes = sorted(p for p in kept if len(p) == level)
        if not nodes:
            break
        counts.append([sum(1 for c in range(branching[level]) if p + (c,) in kept) for p in nodes])
    return counts


def tree_child_counts(cfg, seed):
    """Per-sequence child-count tables for a Gumbel-Top-k configuration."""
    if cfg.get("random_subtree"):
        return [random_subtree_child_counts(cfg["branching"], cfg["N"], seed * 1000003 + b)
                for b in range(cfg["B"])]
    return [full_tree_child_counts(cfg["branching"]) for _ in range(cfg["B"])]


def attention_scale(D):
    return 1.0 / math.sqrt(D)
