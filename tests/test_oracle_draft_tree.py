"""Pins for the oracle's draft-tree drivers (Alg. 3, Alg. 8) on node-indexed logits."""
import numpy as np
from scipy import special

from oracle import philox
from oracle.draft_tree import create_draft_tree_const, create_draft_tree_sbs


def test_rsd_c_level_sizes_are_products_of_branching_factors():
    rng = np.random.default_rng(0)
    z = rng.normal(size=(40, 50)).astype(np.float32)
    for b in ([2, 2], [3, 2, 2, 1], [4, 1, 1], [2, 2, 2, 2]):
        t = create_draft_tree_const(z, lambda l, i, node: b[l] if l < len(b) else 0, seed=1)
        sizes = np.diff(t["level_off"])
        assert list(sizes) == [int(np.prod(b[:l])) for l in range(len(b) + 1)]
        par = t["parent"]
        assert par[0] == -1 and np.all(par[1:] < np.arange(1, len(par)))
        assert np.all(np.diff(par[1:]) >= 0)             # children grouped by parent, in order
        # children of node i are its row's Gumbel-Top-k in decreasing perturbed order
        phi = special.log_softmax(z.astype(np.float64), axis=1)
        for i in range(t["level_off"][-2]):
            kids = np.where(par == i)[0]
            pt = phi[i] + philox.gumbel_row(1, 0, 0, 0, i, 50)
            assert list(t["tokens"][kids]) == list(np.argsort(-pt)[:len(kids)])
            assert len(set(t["tokens"][kids])) == len(kids)   # without replacement


def test_rsd_s_levels_have_beam_width_nodes_and_carry_sequence_log_probs():
    rng = np.random.default_rng(1)
    z = rng.normal(size=(40, 30)).astype(np.float32)
    W, L = 6, 5
    t = create_draft_tree_sbs(z, W, L, seq=2, seed=3)
    assert list(np.diff(t["level_off"])) == [1] + [W] * L
    phi = special.log_softmax(z.astype(np.float64), axis=1)
    for j in range(1, len(t["tokens"])):
        p = t["parent"][j]
        assert abs(t["sum_logprob"][j] - (t["sum_logprob"][p] + phi[p, t["tokens"][j]])) < 1e-12
        assert t["trunc_gumbel"][j] <= t["trunc_gumbel"][p] + 1e-15
    for l in range(1, L + 1):
        lo, hi = t["level_off"][l], t["level_off"][l + 1]
        assert np.all(np.diff(t["trunc_gumbel"][lo:hi]) <= 0)
        assert np.all((t["parent"][lo:hi] >= t["level_off"][l - 1]) & (t["parent"][lo:hi] < lo))
        # (parent, token) pairs are distinct: sequences are sampled without replacement
        assert len({(int(a), int(b)) for a, b in zip(t["parent"][lo:hi], t["tokens"][lo:hi])}) == hi - lo
