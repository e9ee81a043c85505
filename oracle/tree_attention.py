"""Tree-masked attention of the draft-tree tokens, dense fp64 definition.

TEST INFRASTRUCTURE (CPU oracle) -- not part of the product path.

The target model evaluates all tree tokens in one pass "with appropriate
attention masking" (Sec. 3.2.1 after Eq. (6); Sec. 3.2.2, tree evaluation;
Alg. 2 step 2): every tree token attends the cached prefix plus its own tree
ancestors.  The mask over draft nodes is built level by level in Alg. 5
(BuildAttentionMask): a child's row is a copy of its parent's row, and the
diagonal is set to one; it occupies the bottom-right corner of the attention
weights, the part to its left (the already-known tokens) is unmasked.

Node layout used here: node 0 is the root (the last known token, whose
target distribution is level 0 of the verification), nodes 1..N-1 are the
draft tokens in level order, parent[i] < i, parent[0] = -1.  Row i therefore
sees: all prefix keys, the root, and the draft nodes on its root path
including itself.

Readings: the softmax scale is an explicit argument (callers use 1/sqrt(D));
positional encoding is applied by the caller before Q and K get here.
"""
import numpy as np


def ancestor_or_self(parent, n_nodes):
    """Boolean [n,n]: vis[i,j] iff j is i or an ancestor of i (root included)."""
    n = int(n_nodes)
    vis = np.zeros((n, n), dtype=bool)
    for i in range(n):
        j = i
        while j >= 0:
            vis[i, j] = True
            j = int(parent[j]) if j > 0 else -1
    return vis


def build_attention_mask_by_levels(level_parent_ids):
    """Alg. 5 applied level after level, as Alg. 3 / Alg. 8 call it.

    level_parent_ids: one integer array per draft level; entry i of level l is
    the index, *within level l-1*, of the parent of the i-th node of level l
    (for the first draft level the parent is the root and the ids are unused).
    Returns the 0/1 matrix over draft nodes (root excluded).
    """
    mask = None
    n_prev, n_curr = 0, 0
    for ids in level_parent_ids:
        n_new = len(ids)
        if mask is None:
            mask = np.zeros((n_new, n_new), dtype=np.int64)
        else:
            mask = np.pad(mask, ((0, n_new), (0, n_new)))
            for i in range(n_new):
                mask[n_curr + i, :] = mask[n_prev + int(ids[i]), :]
        np.fill_diagonal(mask, 1)
        n_prev, n_curr = n_curr, n_curr + n_new
    return mask


def tree_attention(q, k_prefix, v_prefix, k_tree, v_tree, prefix_len, n_nodes,
                   parent, scale):
    """Dense masked attention in fp64.

    q [B,Hq,N,D]; k_prefix,v_prefix [B,Hkv,P,D]; k_tree,v_tree [B,Hkv,N,D];
    prefix_len [B]; n_nodes [B]; parent [B,N].  Query head h uses KV head
    h // (Hq // Hkv).  Returns (out [B,Hq,N,D], lse [B,Hq,N]); rows at or
    beyond n_nodes[b] are zero.
    """
    q = np.asarray(q, dtype=np.float64)
    k_prefix = np.asarray(k_prefix, dtype=np.float64)
    v_prefix = np.asarray(v_prefix, dtype=np.float64)
    k_tree = np.asarray(k_tree, dtype=np.float64)
    v_tree = np.asarray(v_tree, dtype=np.float64)
    B, Hq, N, D = q.shape
    Hkv = k_prefix.shape[1]
    group = Hq // Hkv
    out = np.zeros((B, Hq, N, D))
    lse = np.zeros((B, Hq, N))
    for b in range(B):
        P, n = int(prefix_len[b]), int(n_nodes[b])
        if n == 0:
            continue
        vis = ancestor_or_self(parent[b], n)
        allowed = np.concatenate([np.ones((n, P), dtype=bool), vis], axis=1)
        for h in range(Hq):
            g = h // group
            keys = np.concatenate([k_prefix[b, g, :P], k_tree[b, g, :n]], axis=0)
            vals = np.concatenate([v_prefix[b, g, :P], v_tree[b, g, :n]], axis=0)
            s = scale * (q[b, h, :n] @ keys.T)
            s = np.where(allowed, s, -np.inf)
            m = np.max(s, axis=1, keepdims=True)
            e = np.exp(s - m)
            l = np.sum(e, axis=1, keepdims=True)
            out[b, h, :n] = (e / l) @ vals
            lse[b, h, :n] = (m + np.log(l))[:, 0]
    return out, lse
