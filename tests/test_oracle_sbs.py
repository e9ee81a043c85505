"""Pins for the oracle's Stochastic Beam Search step (Alg. 9, Eqs. (10)-(12))."""
import itertools

import mpmath
import numpy as np
import pytest
from scipy import special, stats

from oracle import philox
from oracle.gumbel_topk import gumbel_topk_from_noise
from oracle.sbs import sbs_step, sbs_step_from_noise, truncated_gumbel


def test_stable_form_equals_the_printed_mapping_in_high_precision():
    # Eq. (11): T(u, phi) = -log(exp(-u) - exp(-max phi) + exp(-phi)), evaluated with
    # 80 significant digits, against the oracle's stable evaluation.
    mpmath.mp.dps = 80
    rng = np.random.default_rng(0)
    for _ in range(300):
        gamma = float(rng.normal(0, 3))
        z = float(rng.normal(0, 30))
        phi = z - float(rng.exponential(10.0 ** rng.integers(-6, 2)))
        direct = -mpmath.log(mpmath.e ** (-mpmath.mpf(gamma)) - mpmath.e ** (-mpmath.mpf(z))
                             + mpmath.e ** (-mpmath.mpf(phi)))
        got = float(truncated_gumbel(gamma, np.array([phi]), z)[0])
        assert abs(got - float(direct)) <= 1e-12 * max(1.0, abs(float(direct)))


def test_row_maximum_maps_to_parent_value_and_map_is_monotone_and_bounded():
    rng = np.random.default_rng(1)
    phi_tilde = rng.normal(-20, 5, size=200)
    z = phi_tilde.max()
    for gamma in (-3.0, 0.0, 2.5):
        psi = truncated_gumbel(gamma, phi_tilde, z)
        assert psi.max() == gamma and np.argmax(psi) == np.argmax(phi_tilde)
        assert np.all(psi <= gamma)
        order = np.argsort(phi_tilde)
        assert np.all(np.diff(psi[order]) >= 0)
    assert truncated_gumbel(0.0, np.array([-np.inf]), 0.0)[0] == -np.inf


def _toy(V, seed):
    rng = np.random.default_rng(seed)
    root = rng.normal(0, 1, size=V).astype(np.float32)
    nxt = rng.normal(0, 1, size=(V, V)).astype(np.float32)   # logits after token x
    return root, nxt


def test_first_level_equals_gumbel_topk_on_the_same_noise():
    rng = np.random.default_rng(3)
    z = rng.normal(size=(1, 50)).astype(np.float32)
    g = rng.gumbel(size=(1, 50))
    r = sbs_step_from_noise(z, [0.0], [0.0], g, 6)
    toks, pert, logp, _ = gumbel_topk_from_noise(z, g, [6])
    assert np.array_equal(r["tokens"], toks[0]) and np.all(r["parent"] == 0)
    assert np.allclose(r["sum_logprob"], logp[0])
    # first selected entry is the row argmax, whose truncated value is the root's 0
    assert r["trunc_gumbel"][0] == 0.0 and np.all(np.diff(r["trunc_gumbel"]) <= 0)


def test_invariants_on_a_deeper_step():
    rng = np.random.default_rng(4)
    n, V, W = 5, 300, 6
    z = rng.normal(0, 2, size=(n, V)).astype(np.float32)
    sigma = -rng.exponential(3, size=n)
    gamma = np.sort(rng.normal(0, 1, size=n))[::-1]
    g = rng.gumbel(size=(n, V))
    r = sbs_step_from_noise(z, sigma, gamma, g, W)
    phi = special.log_softmax(z.astype(np.float64), axis=1) + sigma[:, None]
    # per-row maximum of psi is the parent's truncated Gumbel
    assert np.allclose(r["psi_all"].max(axis=1), gamma, atol=1e-12)
    # outputs sorted by decreasing psi, values gathered from the right cells
    assert np.all(np.diff(r["trunc_gumbel"]) <= 0)
    assert np.allclose(r["sum_logprob"], phi[r["parent"], r["tokens"]])
    assert np.allclose(r["trunc_gumbel"], r["psi_all"][r["parent"], r["tokens"]])
    # brute-force top-W of psi over all (row, token) cells
    flat = r["psi_all"].reshape(-1)
    brute = np.argsort(-flat, kind="stable")[:W]
    assert np.array_equal(brute // V, r["parent"]) and np.array_equal(brute % V, r["tokens"])
    # Theorem 3.2: within one parent the selected tokens are that parent's own
    # Gumbel-Top-k prefix, in order
    pt = phi + g
    for k in range(n):
        mine = r["tokens"][r["parent"] == k]
        own = np.argsort(-pt[k], kind="stable")[:len(mine)]
        assert np.array_equal(mine, own)


def test_two_levels_sample_sequences_without_replacement():
    # Sec. 3.2.1 (RSD-S): the step is equivalent to drawing the top-W length-(l+1)
    # sequences without replacement from the sequence distribution.
    V, W, draws = 3, 2, 1 << 14
    root, nxt = _toy(V, 11)
    p_root = special.softmax(root.astype(np.float64))
    p_next = special.softmax(nxt.astype(np.float64), axis=1)
    seqs = list(itertools.product(range(V), range(V)))
    p_seq = {s: p_root[s[0]] * p_next[s[0], s[1]] for s in seqs}
    law = {}
    for a, b in itertools.permutations(seqs, 2):
        law[(a, b)] = p_seq[a] * p_seq[b] / (1 - p_seq[a])
    counts = {}
    for d in range(draws):
        l0 = sbs_step(root[None, None, :], np.zeros((1, 1)), np.zeros((1, 1)), [1], W,
                      seq_id=[d], node_id=[[0]], seed=5)
        t0, s0, g0 = l0["tokens"][0], l0["sum_logprob"][0], l0["trunc_gumbel"][0]
        l1 = sbs_step(nxt[t0][None], s0[None], g0[None], [W], W,
                      seq_id=[d], node_id=[[1, 2]], seed=5)
        out = tuple((int(t0[l1["parent"][0, i]]), int(l1["tokens"][0, i])) for i in range(W))
        counts[out] = counts.get(out, 0) + 1
        for i in range(W):                       # carried sum log-prob = log P(sequence)
            assert abs(l1["sum_logprob"][0, i] - np.log(p_seq[out[i]])) < 1e-9
    keys = sorted(law)
    obs = np.array([counts.get(k, 0) for k in keys], dtype=np.float64)
    exp = np.array([law[k] for k in keys]) * draws
    assert set(counts) <= set(keys)
    big = exp >= 5
    assert stats.chi2.sf(np.sum((obs[big] - exp[big]) ** 2 / exp[big]), big.sum() - 1) > 1e-4


def test_batched_entry_padding_and_dead_rows():
    rng = np.random.default_rng(6)
    B, W_in, V, W = 3, 4, 40, 6
    z = rng.normal(size=(B, W_in, V)).astype(np.float32)
    z[2, 0, 5:] = -np.inf          # only 5 finite entries in the single live row
    sigma = -rng.exponential(1, size=(B, W_in))
    gamma = -np.sort(rng.exponential(1, size=(B, W_in)), axis=1)
    out = sbs_step(z, sigma, gamma, [4, 2, 1], W, seed=8)
    assert list(out["n_out"]) == [6, 6, 5]
    assert np.all(out["parent"][1, :6] < 2) and np.all(out["parent"][2, :5] == 0)
    assert np.all(out["tokens"][2, 5:] == -1) and np.all(out["tokens"][2, :5] < 5)
    # noise coordinates: row (b, w) uses seq b, node w
    g = philox.gumbel_row(8, 0, 0, 1, 0, V)
    one = sbs_step_from_noise(z[1, :1], sigma[1, :1], gamma[1, :1], g[None], 1)
    own_best = out["tokens"][1][out["parent"][1] == 0]
    if len(own_best):
        assert own_best[0] == one["tokens"][0]


def test_min_gap_reports_the_closest_call_among_the_top_width_plus_one():
    """Hand-built step: one parent with Gamma = 0 and noise that is cancelled by the logits, so that
    the perturbed scores are chosen values; at the single parent psi = T(0, phi~) is increasing in
    phi~, and the two entries placed `gap` apart in phi~ map to psi values whose distance follows
    from Eq. (11) in closed form."""
    V, width = 6, 2
    g = np.array([0.3, -1.0, 2.0, 0.1, -0.4, 1.5])
    for gap in (3e-6, 0.4):
        target = np.array([-1.0, -3.0, -3.0 - gap, -6.0, -7.0, -8.0])      # phi~ up to a common shift
        logits = (target - g)[None, :]
        r = sbs_step_from_noise(logits, [0.0], [0.0], g[None, :], width)
        assert r["tokens"].tolist() == [0, 1]
        pt = np.sort(r["psi_all"][0])[::-1]
        # closest pair among the top three: ranks 2 and 3 (the cut) when gap is tiny
        assert r["min_gap"] == pytest.approx(min(pt[0] - pt[1], pt[1] - pt[2]), rel=1e-12)
        lse = r["lse"][0]
        psi = lambda t: -np.log(np.exp(0.0) - np.exp(-(target[0] - lse)) + np.exp(-(t - lse)))   # Eq. (11)
        assert pt[1] - pt[2] == pytest.approx(psi(target[1]) - psi(target[2]), rel=1e-6, abs=1e-12)
        assert (r["min_gap"] < 1e-5) == (gap < 1e-5)
    # a single candidate: nothing to compare
    r = sbs_step_from_noise(np.array([[0.0, -np.inf]]), [0.0], [0.0], np.zeros((1, 2)), 1)
    assert r["min_gap"] == np.inf
