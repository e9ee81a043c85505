"""Pins for the oracle's Gumbel-Top-k sampler (Alg. 4)."""
import itertools

import numpy as np
import pytest
from scipy import special, stats

from oracle import philox
from oracle.gumbel_topk import (gumbel_topk, gumbel_topk_from_noise,
                                log_softmax_rows, top_k_desc)


def without_replacement_law(p, k):
    """Probability of each ordered k-tuple when drawing without replacement:
    prod_i p(x_i) / (1 - sum_{j<i} p(x_j)) -- the law that zeroing the drawn
    token and renormalising (Alg. 6) encodes."""
    law = {}
    for tup in itertools.permutations(range(len(p)), k):
        pr, rem = 1.0, 1.0
        for x in tup:
            pr *= p[x] / rem
            rem -= p[x]
        law[tup] = pr
    return law


def philox_noise(rows, V, seed, step=0, seq=0):
    node = np.arange(rows)[:, None]
    return philox.gumbel_from_word(
        philox.words(seed, step, philox.TAG_DRAFT_GUMBEL, seq, node, np.arange(V)[None, :]))


@pytest.mark.parametrize("V,k,seed", [(5, 2, 0), (8, 3, 1), (4, 3, 2), (3, 1, 3)])
def test_ordered_tuples_follow_sampling_without_replacement(V, k, seed):
    rng = np.random.default_rng(seed)
    logits = rng.normal(0, 1.5, size=V).astype(np.float32)
    p = special.softmax(logits.astype(np.float64))
    law = without_replacement_law(p, k)
    assert abs(sum(law.values()) - 1) < 1e-12
    R = 1 << 17
    g = philox_noise(R, V, seed=1000 + seed)
    toks, _, _, _ = gumbel_topk_from_noise(np.tile(logits, (R, 1)), g, np.full(R, k))
    counts = {}
    for t in toks:
        counts[tuple(int(x) for x in t)] = counts.get(tuple(int(x) for x in t), 0) + 1
    keys = sorted(law)
    obs = np.array([counts.get(key, 0) for key in keys], dtype=np.float64)
    exp = np.array([law[key] for key in keys]) * R
    assert set(counts) <= set(keys)
    big = exp >= 5
    chi2 = np.sum((obs[big] - exp[big]) ** 2 / exp[big])
    assert stats.chi2.sf(chi2, big.sum() - 1) > 1e-4
    # every single tuple within 5 sigma as well
    sd = np.sqrt(exp * (1 - exp / R))
    assert np.all(np.abs(obs - exp) <= 5 * sd + 1)


def test_public_entry_uses_documented_philox_coordinates_and_is_categorical_for_k1():
    V, R = 6, 1 << 14
    logits = np.array([0.3, -1.0, 2.0, 0.0, 1.1, -0.4], dtype=np.float32)
    out = gumbel_topk(np.tile(logits, (R, 1)), 1, seq_id=np.full(R, 3),
                      node_id=np.arange(R), seed=99, step=4)
    assert np.all(out["count"] == 1)
    freq = np.bincount(out["tokens"][:, 0], minlength=V)
    p = special.softmax(logits.astype(np.float64))
    assert stats.chisquare(freq, p * R).pvalue > 1e-4
    # same tokens as the noise-passing form with noise taken at (seq 3, node r, step 4)
    g = philox.gumbel_from_word(philox.words(99, 4, 0, 3, np.arange(R)[:, None],
                                             np.arange(V)[None, :]))
    toks, pert, _, _ = gumbel_topk_from_noise(np.tile(logits, (R, 1)), g, np.ones(R, int))
    assert np.array_equal(np.array([t[0] for t in toks]), out["tokens"][:, 0])
    assert np.allclose(np.array([x[0] for x in pert]), out["perturbed"][:, 0])


def test_log_softmax_matches_library():
    rng = np.random.default_rng(0)
    z = rng.normal(0, 4, size=(7, 100)).astype(np.float32)
    phi, lse = log_softmax_rows(z, 1 / 0.3)
    assert np.allclose(lse, special.logsumexp(z.astype(np.float64) / 0.3, axis=1), atol=1e-12)
    assert np.allclose(phi, special.log_softmax(z.astype(np.float64) / 0.3, axis=1), atol=1e-12)


def test_outputs_sorted_values_consistent_and_brute_force():
    rng = np.random.default_rng(5)
    z = rng.normal(0, 2, size=(9, 50)).astype(np.float32)
    out = gumbel_topk(z, 4, k_per_row=[4, 3, 2, 1, 0, 4, 4, 4, 4], seed=3)
    phi = special.log_softmax(z.astype(np.float64), axis=1)
    for r in range(9):
        n = out["count"][r]
        assert n == [4, 3, 2, 1, 0, 4, 4, 4, 4][r]
        g = philox.gumbel_row(3, 0, 0, 0, r, 50)
        pt = phi[r] + g
        brute = sorted(range(50), key=lambda x: -pt[x])[:n]
        assert list(out["tokens"][r, :n]) == brute
        assert np.all(np.diff(out["perturbed"][r, :n]) <= 0)
        assert np.allclose(out["perturbed"][r, :n], pt[brute])
        assert np.allclose(out["logprob"][r, :n], phi[r, brute])
        assert np.all(out["tokens"][r, n:] == -1)


def test_permutation_equivariance():
    rng = np.random.default_rng(8)
    z = rng.normal(size=(1, 40)).astype(np.float32)
    g = rng.gumbel(size=(1, 40))
    perm = rng.permutation(40)
    a, _, _, _ = gumbel_topk_from_noise(z, g, [5])
    b, _, _, _ = gumbel_topk_from_noise(z[:, perm], g[:, perm], [5])
    assert np.array_equal(perm[b[0]], a[0])


def test_minus_inf_entries_are_dropped_and_ties_go_to_lower_index():
    z = np.array([[0.0, -np.inf, 1.0, -np.inf, -np.inf]], dtype=np.float32)
    out = gumbel_topk(z, 4, seed=0)
    assert out["count"][0] == 2
    assert set(out["tokens"][0, :2]) == {0, 2} and np.all(out["tokens"][0, 2:] == -1)
    assert list(top_k_desc(np.array([1.0, 3.0, 3.0, 2.0, 3.0]), 3)) == [1, 2, 4]


def test_temperature_scales_logits_before_softmax():
    rng = np.random.default_rng(2)
    z = rng.normal(size=(3, 30)).astype(np.float32)
    a = gumbel_topk(z, 3, inv_temperature=1 / 0.3, seed=5)
    b = gumbel_topk((z.astype(np.float64) / 0.3), 3, seed=5)
    assert np.array_equal(a["tokens"], b["tokens"])
    assert np.allclose(a["logprob"], b["logprob"])
