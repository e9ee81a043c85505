"""Pins of the baseline verifiers (K-SEQ of SpecTr, multi-round rejection sampling of SpecInfer; Sec. 2)
against what the paper and the mathematics fix:

* both recover the target distribution -- checked by exact enumeration of every tuple of K drafts drawn
  with replacement and every accept/reject pattern on small vocabularies;
* K = 1 is ordinary speculative sampling: acceptance sum_x min(p, q), residual Norm[(q - p)^+];
* the Bernoulli toy example of Sec. 3.1 (K = 2): closed-form acceptance rates of the two baselines, and
  the ordering the text describes (recursive rejection sampling accepts with certainty, the baselines
  lose acceptance as the two models drift apart).
"""
import itertools

import numpy as np
import pytest

from oracle import baselines as o_base
from oracle import philox
from oracle import rrs as o_rrs


def _output_law(q, p, K, method, gamma, allow_flag=False):
    """Exact law of the emitted token: sum over draft tuples (i.i.d. from p) and accept patterns."""
    V = len(q)
    out = np.zeros(V)
    accept_mass = 0.0
    for drafts in itertools.product(range(V), repeat=K):
        w = np.prod([p[x] for x in drafts])
        if w == 0:
            continue
        if method == o_base.METHOD_KSEQ:
            theta, final, flag = o_base.kseq_thresholds(q, p, drafts, gamma)
        else:
            theta, final, flag = o_base.multiround_thresholds(q, p, drafts)
        assert allow_flag or not flag
        reach = w
        for k, x in enumerate(drafts):
            out[x] += reach * theta[k]
            accept_mass += reach * theta[k]
            reach *= 1.0 - theta[k]
        out += reach * final
    return out, accept_mass


@pytest.mark.parametrize("V,K", [(2, 1), (2, 2), (3, 2), (3, 3), (4, 2)])
def test_both_baselines_recover_the_target_distribution(V, K):
    rng = np.random.default_rng(V * 10 + K)
    for _ in range(6):
        q = rng.dirichlet(np.ones(V))
        p = rng.dirichlet(np.ones(V))
        law, _ = _output_law(q, p, K, o_base.METHOD_MULTIROUND, None)
        assert np.allclose(law, q, atol=1e-12)
        law, _ = _output_law(q, p, K, o_base.METHOD_KSEQ, float(K))      # gamma = K is always admissible
        assert np.allclose(law, q, atol=1e-12)


def test_kseq_with_gamma_one_and_one_draft_is_speculative_sampling():
    rng = np.random.default_rng(3)
    q, p = rng.dirichlet(np.ones(5)), rng.dirichlet(np.ones(5))
    for method, gamma in ((o_base.METHOD_KSEQ, 1.0), (o_base.METHOD_MULTIROUND, None)):
        law, acc = _output_law(q, p, 1, method, gamma)
        assert np.allclose(law, q, atol=1e-12)
        assert acc == pytest.approx(np.minimum(p, q).sum(), rel=1e-12)
        if method == o_base.METHOD_KSEQ:
            _, final, _ = o_base.kseq_thresholds(q, p, [0], 1.0)
        else:
            _, final, _ = o_base.multiround_thresholds(q, p, [0])
        res = np.maximum(q - p, 0)
        assert np.allclose(final, res / res.sum(), atol=1e-12)


def test_kseq_flags_a_gamma_that_is_too_small():
    q = np.array([0.9, 0.1])
    p = np.array([0.5, 0.5])
    # K = 3, gamma = 1: min(p, q) * (1 - (1 - beta)^3) / beta exceeds q at the second symbol
    _, _, flag = o_base.kseq_thresholds(q, p, [0, 1, 0], 1.0)
    assert flag
    _, _, flag = o_base.kseq_thresholds(q, p, [0, 1, 0], 3.0)
    assert not flag


@pytest.mark.parametrize("a,b", [(0.5, 0.5), (0.3, 0.7), (0.1, 0.9), (0.9, 0.2)])
def test_bernoulli_toy_acceptance_rates(a, b):
    """Two symbols, K = 2, draft p = (a, 1 - a), target q = (b, 1 - b).  Multi-round: the first draft is
    accepted with probability sum min(p, q) = 1 - |a - b|; after a rejection the residual sits entirely on
    the symbol with q > p, and the second draft (again from p) hits it with that symbol's p.  Recursive
    rejection sampling (without replacement) always accepts its second draft."""
    q = np.array([b, 1 - b])
    p = np.array([a, 1 - a])
    # (identical models: the residual after the first draft has no mass, which the chain flags; that
    # stage is never reached because the first draft is accepted with certainty)
    _, acc = _output_law(q, p, 2, o_base.METHOD_MULTIROUND, None, allow_flag=(a == b))
    d = abs(a - b)
    heavy = 0 if b > a else 1                         # symbol the residual sits on (when d > 0)
    expect = (1 - d) + d * min(1.0, 1.0 / p[heavy]) * p[heavy] if d > 0 else 1.0
    # second stage: residual q^(2) = point mass at `heavy`; a draft from p equals it with probability
    # p[heavy] and is then accepted with min(1, 1 / p[heavy]) = 1
    assert acc == pytest.approx((1 - d) + d * p[heavy], rel=1e-12)
    assert expect == pytest.approx((1 - d) + d * p[heavy])
    _, acc_kseq = _output_law(q, p, 2, o_base.METHOD_KSEQ, 2.0)
    beta = np.minimum(p, q / 2.0).sum()
    assert acc_kseq == pytest.approx(1 - (1 - beta) ** 2, rel=1e-12)      # K independent tries at rate beta
    # recursive rejection sampling on the same pair: drafts without replacement -> both symbols
    th, _, _ = o_rrs.sibling_chain(q, p, [0, 1])
    th2, _, _ = o_rrs.sibling_chain(q, p, [1, 0])
    for t in (th, th2):
        assert t[0] == 1.0 or t[1] == pytest.approx(1.0)
    if d > 0.05:
        assert acc < 1.0 and acc_kseq < 1.0


def test_verify_draws_its_uniforms_and_final_noise_by_position():
    """The batched entry: uniforms of draft k at (seq, node, vocab index k) of the accept stream, final
    Gumbel noise at (seq, node) of the last-token stream; the decision follows them."""
    rng = np.random.default_rng(5)
    V, K, R = 12, 3, 4
    zt = rng.standard_normal((R, V)).astype(np.float32)
    zd = (zt + rng.standard_normal((R, V))).astype(np.float32)
    drafts = rng.integers(0, V, size=(R, K))
    seq, node = np.array([3, 3, 9, 1]), np.array([0, 5, 5, 2])
    for method, gamma in ((o_base.METHOD_KSEQ, 2.0), (o_base.METHOD_MULTIROUND, 1.0)):
        out = o_base.verify(zt, zd, drafts, method, gamma=gamma, seq_id=seq, node_id=node, seed=11, step=2)
        for r in range(R):
            u = philox.uniform_from_word(philox.words(11, 2, philox.TAG_ACCEPT_UNIFORM, int(seq[r]), int(node[r]), np.arange(K)))
            assert np.array_equal(out["uniforms"][r], u)
            q, p = o_rrs.softmax_row(zt[r]), o_rrs.softmax_row(zd[r])
            th = (o_base.kseq_thresholds(q, p, drafts[r], gamma) if method == o_base.METHOD_KSEQ
                  else o_base.multiround_thresholds(q, p, drafts[r]))[0]
            assert np.allclose(out["theta"][r], th)
            hits = np.nonzero(u < th)[0]
            if len(hits):
                assert out["accepted"][r] == hits[0] and out["token"][r] == drafts[r, hits[0]]
            else:
                assert out["accepted"][r] == -1
    # different rows with the same (seq, node) coordinates share their random numbers
    out2 = o_base.verify(zt[[0, 0]], zd[[0, 0]], drafts[[0, 0]], o_base.METHOD_MULTIROUND, seq_id=[7, 7], node_id=[4, 4])
    assert np.array_equal(out2["uniforms"][0], out2["uniforms"][1])
