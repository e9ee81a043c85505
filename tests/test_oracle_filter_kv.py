"""Pins for the FilterKVCache oracle (Alg. 2 / Alg. 7 step 4): the filtered cache must be the cache a
plain left-to-right decoder would hold, which is checked through attention results, not by re-stating
the copy."""
import numpy as np

from oracle import filter_kv as o_filter
from oracle import tree_attention as o_attn


def _case(seed, B=2, H=2, N=9, D=8, P=5, cap=16):
    rng = np.random.default_rng(seed)
    k_cache = rng.standard_normal((B, H, cap, D))
    v_cache = rng.standard_normal((B, H, cap, D))
    k_tree = rng.standard_normal((B, H, N, D))
    v_tree = rng.standard_normal((B, H, N, D))
    q = rng.standard_normal((B, H, N, D))
    parent = np.array([[-1, 0, 0, 1, 1, 2, 3, 3, 6]] * B, dtype=np.int32)
    return q, k_cache, v_cache, k_tree, v_tree, parent


def _root_path(parent, leaf):
    path = []
    j = leaf
    while j > 0:
        path.append(j)
        j = int(parent[j])
    return path[::-1]


def test_filtered_cache_reproduces_tree_attention_of_the_accepted_leaf():
    """A node's tree-attention output (prefix + its ancestors-or-self) equals ordinary attention of the same
    query over the filtered cache when the accepted path is that node's root path."""
    q, kc, vc, kt, vt, parent = _case(0)
    B, H, N, D = q.shape
    P = 5
    plen = np.array([P, 3], dtype=np.int32)
    n_nodes = np.full(B, N, dtype=np.int32)
    ref, _ = o_attn.tree_attention(q, kc[:, :, :P], vc[:, :, :P], kt, vt, plen, n_nodes, parent, 0.3)
    for leaf in (8, 4, 5, 0):
        path = _root_path(parent[0], leaf)
        acc = -np.ones((B, 4), dtype=np.int32)
        acc[:, :len(path)] = path
        n_acc = np.full(B, len(path), dtype=np.int32)
        k2, v2, new_len, flags = o_filter.filter_kv_cache(kc, vc, kt, vt, plen, acc, n_acc)
        assert not flags.any()
        for b in range(B):
            L = int(new_len[b])
            assert L == int(plen[b]) + 1 + len(path)
            for h in range(H):
                s = 0.3 * (k2[b, h, :L] @ q[b, h, leaf])
                p = np.exp(s - s.max())
                out = (p / p.sum()) @ v2[b, h, :L]
                assert np.allclose(out, ref[b, h, leaf], rtol=0, atol=1e-12)


def test_rows_before_the_prefix_and_beyond_the_new_length_are_untouched():
    q, kc, vc, kt, vt, parent = _case(1)
    plen = np.array([5, 0], dtype=np.int32)
    acc = np.array([[2, 5, -1, -1], [-1, -1, -1, -1]], dtype=np.int32)
    n_acc = np.array([2, 0], dtype=np.int32)
    k2, v2, new_len, flags = o_filter.filter_kv_cache(kc, vc, kt, vt, plen, acc, n_acc)
    assert list(new_len) == [8, 1] and not flags.any()
    assert np.array_equal(k2[0, :, :5], kc[0, :, :5]) and np.array_equal(k2[0, :, 8:], kc[0, :, 8:])
    assert np.array_equal(v2[1, :, 1:], vc[1, :, 1:])
    assert np.array_equal(k2[1, :, 0], kt[1, :, 0]) and np.array_equal(v2[0, :, 7], vt[0, :, 5])
    assert np.array_equal(kc, _case(1)[1])  # the inputs are not modified


def test_capacity_overflow_saturates_and_flags():
    q, kc, vc, kt, vt, parent = _case(2, cap=7)
    plen = np.array([5, 6], dtype=np.int32)
    acc = np.array([[1, 3, 6, -1], [2, -1, -1, -1]], dtype=np.int32)
    n_acc = np.array([3, 1], dtype=np.int32)
    k2, v2, new_len, flags = o_filter.filter_kv_cache(kc, vc, kt, vt, plen, acc, n_acc)
    assert list(new_len) == [7, 7] and list(flags) == [1, 1]
    assert np.array_equal(k2[0, :, 5], kt[0, :, 0]) and np.array_equal(k2[0, :, 6], kt[0, :, 1])
    assert np.array_equal(k2[1, :, 6], kt[1, :, 0])
