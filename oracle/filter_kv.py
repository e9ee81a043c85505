"""FilterKVCache: keep the verified path's keys and values in the cache.

TEST INFRASTRUCTURE (CPU oracle) -- not part of the product path.

Step 4 of the decoding loop (Alg. 2 for RSD-C, Alg. 7 for RSD-S) keeps, of
the key/value rows the tree evaluation produced, only those of the accepted
nodes, appended after the rows of the tokens that were already known, so that
the next iteration starts from a cache that holds exactly the sequence decoded
so far.  The paper calls the routine (FilterKVCache(cache_draft, cache_target,
l_in, accepted flat node ids)) but never prints its body; the reading used
here:

* the cache of one (sequence, KV head) is a row array with `prefix_len` valid
  rows (the tokens before the root); the tree evaluation produced one row per
  tree node (node 0 = root = the last known token, which had no cache row yet);
* after verification the decoded sequence grew by the root's row followed by
  the rows of the accepted nodes in path order, so these 1 + n_accepted rows
  are appended at positions prefix_len, prefix_len + 1, ... and the new valid
  length is prefix_len + 1 + n_accepted;
* the freshly sampled last token becomes the next root and has no row yet;
* rows that would land at or beyond the cache capacity are dropped, the
  length saturates at the capacity and flag bit 0 of the sequence is set.

The same routine serves the draft and the target cache (call it once each).
"""
import numpy as np


def filter_kv_cache(k_cache, v_cache, k_tree, v_tree, prefix_len, accepted_nodes, n_accepted):
    """Returns (k_cache', v_cache', new_len[B], flags[B]); inputs are not modified.

    k_cache, v_cache : [B, H, P_cap, D]   k_tree, v_tree : [B, H, N, D]
    prefix_len       : [B] valid cache rows before the call
    accepted_nodes   : [B, L_max] accepted node ids in path order (-1 padding)
    n_accepted       : [B]
    """
    k_out = np.array(k_cache, copy=True)
    v_out = np.array(v_cache, copy=True)
    B, _, cap, _ = k_out.shape
    new_len = np.zeros(B, dtype=np.int32)
    flags = np.zeros(B, dtype=np.int32)
    for b in range(B):
        path = [0] + [int(accepted_nodes[b, j]) for j in range(int(n_accepted[b]))]
        pos = int(prefix_len[b])
        for node in path:
            if pos >= cap:
                flags[b] |= 1
                break
            k_out[b, :, pos, :] = k_tree[b, :, node, :]
            v_out[b, :, pos, :] = v_tree[b, :, node, :]
            pos += 1
        new_len[b] = min(int(prefix_len[b]) + len(path), cap)
    return k_out, v_out, new_len, flags
