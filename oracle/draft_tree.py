"""Draft-tree construction drivers on node-indexed synthetic logits.

TEST INFRASTRUCTURE (CPU oracle) -- not part of the product path.

Alg. 3 (CreateDraftTreeConst) and Alg. 8 (CreateDraftTreeStochasticBeamSearch)
grow the tree level by level: run the draft model on the newest level, sample
children with Alg. 4 resp. Alg. 9, append tokens and parent ids.  There is no
draft model here: `draft_logits[i]` stands for the draft model's next-token
logits after the sequence ending in node i, so "running the model on a level"
is a row lookup.

Trees are returned flattened in level order: tokens[N], parent[N] with global
node indices (root = node 0, parent[0] = -1), level_off[l] = first node of
level l.  The per-level parent ids of the paper (index within the previous
level) are parent[j] - level_off[l-1].
"""
import numpy as np

from .gumbel_topk import gumbel_topk
from .sbs import sbs_step


def create_draft_tree_const(draft_logits, child_count, seq=0, seed=0, step=0,
                            inv_temperature=1.0, n_cap=None):
    """Alg. 3 with per-node child counts.

    draft_logits [n_cap,V]; child_count(level, index_in_level, node) -> number of
    children that node drafts (a constant b_l reproduces RSD-C).  Children of
    one parent are contiguous and ordered by decreasing perturbed log-prob.
    """
    n_cap = draft_logits.shape[0] if n_cap is None else n_cap
    tokens, parent, level_off = [-1], [-1], [0, 1]
    level = 0
    while True:
        lo, hi = level_off[level], level_off[level + 1]
        ks = [int(child_count(level, i - lo, i)) for i in range(lo, hi)]
        if sum(ks) == 0:
            break
        assert len(tokens) + sum(ks) <= n_cap
        nodes = np.arange(lo, hi)
        res = gumbel_topk(draft_logits[lo:hi], max(ks), k_per_row=ks,
                          inv_temperature=inv_temperature,
                          seq_id=np.full(hi - lo, seq), node_id=nodes,
                          seed=seed, step=step)
        for r, i in enumerate(nodes):
            for c in range(int(res["count"][r])):
                tokens.append(int(res["tokens"][r, c]))
                parent.append(int(i))
        level_off.append(len(tokens))
        level += 1
    return dict(tokens=np.array(tokens), parent=np.array(parent),
                level_off=np.array(level_off))


def create_draft_tree_sbs(draft_logits, width, depth, seq=0, seed=0, step=0,
                          inv_temperature=1.0):
    """Alg. 8: `depth` Stochastic Beam Search levels of beam width `width`.

    The root beam has sum log-prob 0 and truncated Gumbel 0.  Returns the tree
    plus per-node sum_logprob and trunc_gumbel.
    """
    V = draft_logits.shape[1]
    tokens, parent, level_off = [-1], [-1], [0, 1]
    sigma, gamma = [0.0], [0.0]
    for level in range(depth):
        lo, hi = level_off[level], level_off[level + 1]
        n = hi - lo
        if n == 0:
            break
        res = sbs_step(draft_logits[None, lo:hi], np.array([sigma[lo:hi]]),
                       np.array([gamma[lo:hi]]), [n], width,
                       inv_temperature=inv_temperature, seq_id=[seq],
                       node_id=np.arange(lo, hi)[None], seed=seed, step=step)
        m = int(res["n_out"][0])
        for c in range(m):
            tokens.append(int(res["tokens"][0, c]))
            parent.append(lo + int(res["parent"][0, c]))
            sigma.append(float(res["sum_logprob"][0, c]))
            gamma.append(float(res["trunc_gumbel"][0, c]))
        level_off.append(len(tokens))
    return dict(tokens=np.array(tokens), parent=np.array(parent),
                level_off=np.array(level_off), sum_logprob=np.array(sigma),
                trunc_gumbel=np.array(gamma))
