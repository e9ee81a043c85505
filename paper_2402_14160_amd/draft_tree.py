"""Host-side glue that grows draft trees with the HIP samplers.

The level loop of draft-tree construction (Alg. 3 for constant branching,
Alg. 8 for Stochastic Beam Search) is bookkeeping around one sampler call per
level; the sampling itself runs in rsd_gumbel_topk / rsd_sbs_step.  With
node-indexed synthetic logits, "running the draft model on the newest level"
is a row gather.
"""
import torch

from . import binding


def create_draft_tree_const(draft_logits, child_counts, seed=0, step=0, inv_temperature=1.0,
                            seq_id=None):
    """draft_logits [B,N_cap,V] on the GPU; child_counts[b][level][i] = number of children of
    the i-th node of `level` in sequence b.  Returns dict(tokens, parent, n_nodes) as int32
    GPU tensors ([B,N_cap], padded with -1) plus `level_off` (host lists)."""
    B, n_cap, V = draft_logits.shape
    dev = draft_logits.device
    tokens = [[-1] for _ in range(B)]
    parent = [[-1] for _ in range(B)]
    level_off = [[0, 1] for _ in range(B)]
    seqs = list(range(B)) if seq_id is None else [int(s) for s in seq_id]
    level = 0
    while True:
        rb, rn, ks = [], [], []
        for b in range(B):
            if level + 1 >= len(level_off[b]) or level >= len(child_counts[b]):
                continue
            lo, hi = level_off[b][level], level_off[b][level + 1]
            for i in range(lo, hi):
                rb.append(b); rn.append(i); ks.append(int(child_counts[b][level][i - lo]))
        if not ks or sum(ks) == 0:
            break
        rows = draft_logits[torch.tensor(rb, device=dev), torch.tensor(rn, device=dev)].contiguous()
        out = binding.gumbel_topk(rows, max(ks),
                                  k_per_row=torch.tensor(ks, dtype=torch.int32, device=dev),
                                  inv_temperature=inv_temperature,
                                  seq_id=torch.tensor([seqs[b] for b in rb], dtype=torch.int32, device=dev),
                                  node_id=torch.tensor(rn, dtype=torch.int32, device=dev),
                                  seed=seed, step=step, want_scores=False)
        toks, cnt = out["tokens"].cpu(), out["count"].cpu()
        grown = set()
        for r, (b, i) in enumerate(zip(rb, rn)):
            for c in range(int(cnt[r])):
                if len(tokens[b]) >= n_cap:
                    raise ValueError("tree does not fit the node capacity of the logits tensor")
                tokens[b].append(int(toks[r, c])); parent[b].append(i)
            grown.add(b)
        for b in grown:
            level_off[b].append(len(tokens[b]))
        level += 1
    return _pack(tokens, parent, level_off, n_cap, dev)


def create_draft_tree_sbs(draft_logits, width, depth, seed=0, step=0, inv_temperature=1.0,
                          seq_id=None):
    """`depth` Stochastic Beam Search levels of beam width `width` for every sequence."""
    B, n_cap, V = draft_logits.shape
    dev = draft_logits.device
    tokens = [[-1] for _ in range(B)]
    parent = [[-1] for _ in range(B)]
    level_off = [[0, 1] for _ in range(B)]
    sigma = torch.zeros((B, 1), dtype=torch.float32, device=dev)
    gamma = torch.zeros((B, 1), dtype=torch.float32, device=dev)
    n_in = torch.ones(B, dtype=torch.int32, device=dev)
    seq = None if seq_id is None else torch.as_tensor(seq_id, dtype=torch.int32, device=dev)
    for level in range(depth):
        w_in = sigma.shape[1]
        lo = torch.tensor([level_off[b][level] for b in range(B)], device=dev)
        node = (lo[:, None] + torch.arange(w_in, device=dev)[None, :]).clamp(max=n_cap - 1)
        rows = draft_logits[torch.arange(B, device=dev)[:, None], node].contiguous()
        out = binding.sbs_step(rows, sigma.contiguous(), gamma.contiguous(), n_in, width,
                               inv_temperature=inv_temperature, seq_id=seq,
                               node_id=node.to(torch.int32).contiguous(), seed=seed, step=step)
        toks, par, n_out = out["tokens"].cpu(), out["parent"].cpu(), out["n_out"].cpu()
        for b in range(B):
            for c in range(int(n_out[b])):
                if len(tokens[b]) >= n_cap:
                    raise ValueError("tree does not fit the node capacity of the logits tensor")
                tokens[b].append(int(toks[b, c])); parent[b].append(level_off[b][level] + int(par[b, c]))
            level_off[b].append(len(tokens[b]))
        sigma, gamma, n_in = out["sum_logprob"], out["trunc_gumbel"], out["n_out"]
    res = _pack(tokens, parent, level_off, n_cap, dev)
    res["sum_logprob"], res["trunc_gumbel"] = sigma, gamma
    return res


def _pack(tokens, parent, level_off, n_cap, dev):
    B = len(tokens)
    tok = torch.full((B, n_cap), -1, dtype=torch.int32)
    par = torch.full((B, n_cap), -1, dtype=torch.int32)
    for b in range(B):
        n = len(tokens[b])
        tok[b, :n] = torch.tensor(tokens[b], dtype=torch.int32)
        par[b, :n] = torch.tensor(parent[b], dtype=torch.int32)
    n_nodes = torch.tensor([len(t) for t in tokens], dtype=torch.int32)
    return dict(tokens=tok.to(dev), parent=par.to(dev), n_nodes=n_nodes.to(dev), level_off=level_off)
