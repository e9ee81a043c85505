"""Pins for the oracle's tree-masked attention and tree mask (Alg. 5)."""
import numpy as np
import torch
from scipy import special

from oracle.tree_attention import (ancestor_or_self, build_attention_mask_by_levels,
                                   tree_attention)


def random_level_tree(rng, level_sizes):
    """Level-ordered tree with arbitrary (interleaved) parents per level."""
    parent, level_off, per_level = [-1], [0, 1], []
    for n_new in level_sizes:
        lo, hi = level_off[-2], level_off[-1]
        ids = rng.integers(0, hi - lo, size=n_new)
        per_level.append(ids)
        parent.extend((lo + ids).tolist())
        level_off.append(len(parent))
    return np.array(parent), per_level


def test_ancestor_mask_equals_the_level_by_level_construction():
    rng = np.random.default_rng(0)
    for sizes in ([3, 6, 12, 12], [6, 6, 6, 6, 6, 6], [2, 4], [1], [8, 32, 23]):
        parent, per_level = random_level_tree(rng, sizes)
        n = len(parent)
        lit = build_attention_mask_by_levels(per_level)       # draft nodes only
        vis = ancestor_or_self(parent, n)
        assert np.array_equal(vis[1:, 1:].astype(np.int64), lit)
        assert np.all(vis[:, 0])                              # root visible to all
        assert np.array_equal(vis[0], np.eye(n, dtype=bool)[0])


def test_alg5_small_example_by_hand():
    # b = (2, 1): nodes A, B children of the root; C child of A; D child of B.
    lit = build_attention_mask_by_levels([[0, 0], [0, 1]])
    assert lit.tolist() == [[1, 0, 0, 0], [0, 1, 0, 0], [1, 0, 1, 0], [0, 1, 0, 1]]


def _rand_inputs(rng, B, Hq, Hkv, N, D, P):
    q = rng.normal(size=(B, Hq, N, D))
    kp = rng.normal(size=(B, Hkv, P, D))
    vp = rng.normal(size=(B, Hkv, P, D))
    kt = rng.normal(size=(B, Hkv, N, D))
    vt = rng.normal(size=(B, Hkv, N, D))
    return q, kp, vp, kt, vt


def test_chain_tree_is_causal_attention_library_check():
    rng = np.random.default_rng(1)
    B, H, N, D, P = 2, 3, 6, 16, 0
    q, kp, vp, kt, vt = _rand_inputs(rng, B, H, H, N, D, P)
    parent = np.tile(np.arange(-1, N - 1), (B, 1))
    out, _ = tree_attention(q, kp, vp, kt, vt, [0] * B, [N] * B, parent, 1 / np.sqrt(D))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q), torch.from_numpy(kt), torch.from_numpy(vt), is_causal=True)
    assert np.allclose(out, ref.numpy(), atol=1e-12)


def test_random_tree_with_prefix_and_gqa_matches_library_sdpa_with_boolean_mask():
    rng = np.random.default_rng(2)
    B, Hq, Hkv, N, D, P = 2, 4, 2, 9, 8, 11
    q, kp, vp, kt, vt = _rand_inputs(rng, B, Hq, Hkv, N, D, P)
    parents, n_nodes, plens = [], [9, 7], [11, 5]
    for b in range(B):
        par, _ = random_level_tree(rng, [2, 3, 3])
        parents.append(par)
    parent = np.stack(parents)
    out, lse = tree_attention(q, kp, vp, kt, vt, plens, n_nodes, parent, 0.37)
    for b in range(B):
        n, pl = n_nodes[b], plens[b]
        vis = ancestor_or_self(parent[b], n)
        mask = torch.from_numpy(np.concatenate([np.ones((n, pl), bool), vis], 1))
        k = torch.from_numpy(np.concatenate([kp[b, :, :pl], kt[b, :, :n]], 1)).repeat_interleave(2, 0)
        v = torch.from_numpy(np.concatenate([vp[b, :, :pl], vt[b, :, :n]], 1)).repeat_interleave(2, 0)
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q[b, :, :n]), k, v, attn_mask=mask, scale=0.37)
        assert np.allclose(out[b, :, :n], ref.numpy(), atol=1e-12)
        assert np.all(out[b, :, n:] == 0)
        s = 0.37 * np.einsum("hnd,hkd->hnk", q[b, :, :n], k.numpy())
        s = np.where(mask.numpy()[None], s, -np.inf)
        assert np.allclose(lse[b, :, :n], special.logsumexp(s, axis=-1), atol=1e-12)


def test_single_node_is_plain_decode_attention():
    rng = np.random.default_rng(3)
    q, kp, vp, kt, vt = _rand_inputs(rng, 1, 2, 2, 1, 8, 20)
    out, _ = tree_attention(q, kp, vp, kt, vt, [20], [1], [[-1]], 0.5)
    for h in range(2):
        keys = np.concatenate([kp[0, h], kt[0, h]], 0)
        vals = np.concatenate([vp[0, h], vt[0, h]], 0)
        w = special.softmax(0.5 * keys @ q[0, h, 0])
        assert np.allclose(out[0, h, 0], w @ vals, atol=1e-12)


def test_identical_keys_give_the_mean_of_visible_values():
    rng = np.random.default_rng(4)
    B, H, N, D, P = 1, 1, 7, 4, 3
    q, kp, vp, kt, vt = _rand_inputs(rng, B, H, H, N, D, P)
    kp[:] = kp[0, 0, 0]
    kt[:] = kp[0, 0, 0]
    parent = np.array([[-1, 0, 0, 1, 1, 2, 4]])
    out, _ = tree_attention(q, kp, vp, kt, vt, [P], [N], parent, 1.0)
    vis = ancestor_or_self(parent[0], N)
    for i in range(N):
        want = (vp[0, 0].sum(0) + vt[0, 0][vis[i]].sum(0)) / (P + vis[i].sum())
        assert np.allclose(out[0, 0, i], want, atol=1e-12)
    # sibling subtrees do not see each other: changing node 2's value leaves node 3 alone
    vt2 = vt.copy()
    vt2[0, 0, 2] += 100
    out2, _ = tree_attention(q, kp, vp, kt, vt2, [P], [N], parent, 1.0)
    assert np.allclose(out2[0, 0, 3], out[0, 0, 3]) and not np.allclose(out2[0, 0, 5], out[0, 0, 5])
