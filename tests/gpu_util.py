"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

from oracle import draft_tree as o_tree
from oracle import gumbel_topk as o_topk

NEAR_TIE = 1e-5      # decisions may differ only when the deciding gap is below this
LOGP_TOL = 1e-5      # |delta log-prob| <=> 1e-5 relative on the probability


def dev():
    return torch.device("cuda:0")


def to_np(t):
    return t.detach().cpu().numpy()


def say(msg):
    print(msg, flush=True)


PSI_TOL = 2e-5       # truncated Gumbels of Eq. (11), absolute


def check_topk_against_oracle(logits_np, gpu, k_per_row, inv_t, seq_id, node_id, seed, step,
                              k_max):
    """Element-by-element comparison of one rsd_gumbel_topk call with the oracle.
    Returns the number of near-tie rows (whose token lists are not compared)."""
    ref = o_topk.gumbel_topk(logits_np, k_max, k_per_row=k_per_row, inv_temperature=inv_t,
                             seq_id=seq_id, node_id=node_id, seed=seed, step=step)
    near = o_topk.near_tie_rows(logits_np, np.minimum(k_per_row, k_max), inv_t, seq_id, node_id,
                                seed, step, tol=NEAR_TIE)
    tok, cnt = to_np(gpu["tokens"]), to_np(gpu["count"])
    pert, logp, lse = to_np(gpu["perturbed"]), to_np(gpu["logprob"]), to_np(gpu["lse"])
    assert np.array_equal(cnt, ref["count"])
    finite_rows = np.isfinite(ref["lse"])
    assert np.allclose(lse[finite_rows], ref["lse"][finite_rows], rtol=0, atol=LOGP_TOL)
    for r in range(logits_np.shape[0]):
        n = int(ref["count"][r])
        assert np.all(tok[r, n:] == -1)
        if near[r]:
            # same multiset is not guaranteed either; check validity instead
            assert len(set(tok[r, :n].tolist())) == n
            continue
        assert np.array_equal(tok[r, :n], ref["tokens"][r, :n]), (r, tok[r], ref["tokens"][r])
        assert np.allclose(pert[r, :n], ref["perturbed"][r, :n], rtol=0, atol=2e-5)
        assert np.allclose(logp[r, :n], ref["logprob"][r, :n], rtol=0, atol=LOGP_TOL)
    return int(near.sum())


def oracle_tree_const(zd_np, counts, seq, seed, step, inv_t=1.0):
    return o_tree.create_draft_tree_const(
        zd_np, lambda l, i, node: counts[l][i] if l < len(counts) and i < len(counts[l]) else 0,
        seq=seq, seed=seed, step=step, inv_temperature=inv_t)
