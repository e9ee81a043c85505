"""Pins for the probability-filter oracle: brute force over subsets on tiny rows, the minimality and
coverage properties that define a nucleus, and the trivial special cases."""
import itertools

import numpy as np

from oracle import prob_filter as o_filter


def _probs(z, inv_t=1.0):
    x = z.astype(np.float64) * inv_t
    e = np.exp(x - x.max())
    return e / e.sum()


def test_nucleus_is_the_smallest_top_set_by_brute_force():
    """Among all subsets with mass >= p the kept set has the fewest elements, and among those of that size
    the largest mass (rows with distinct probabilities, so no tie rule is involved)."""
    rng = np.random.default_rng(0)
    for trial in range(40):
        V = int(rng.integers(2, 9))
        z = rng.standard_normal(V).astype(np.float32) * 2
        p = float(rng.uniform(0.05, 0.999))
        prob = _probs(z)
        best = None
        for size in range(1, V + 1):
            cands = [(sum(prob[list(s)]), s) for s in itertools.combinations(range(V), size)]
            ok = [c for c in cands if c[0] >= p]
            if ok:
                best = set(max(ok)[1])
                break
        out, margin = o_filter.filter_row(z, top_p=p)
        assert set(np.flatnonzero(np.isfinite(out))) == best
        assert np.array_equal(out[np.isfinite(out)], z[np.isfinite(out)])   # kept logits unchanged
        assert margin >= 0


def test_nucleus_covers_p_and_is_minimal():
    rng = np.random.default_rng(1)
    for V, p, inv_t in [(1000, 0.95, 1.0), (32000, 0.95, 1.0), (5000, 0.5, 1.0 / 0.3), (777, 0.999, 1.0)]:
        z = (-1.1 * np.log(rng.permutation(V) + 1.0) + rng.standard_normal(V)).astype(np.float32)
        out, _ = o_filter.filter_row(z, inv_temperature=inv_t, top_p=p)
        prob = _probs(z, np.float64(np.float32(inv_t)))
        kept = np.isfinite(out)
        assert prob[kept].sum() >= p
        assert prob[kept].sum() - prob[kept].min() < p            # dropping the least kept entry falls short
        assert prob[kept].min() > prob[~kept].max()               # a top set


def test_top_k_and_special_cases():
    rng = np.random.default_rng(2)
    z = rng.standard_normal(50).astype(np.float32)
    out, _ = o_filter.filter_row(z, top_k=1)
    assert np.flatnonzero(np.isfinite(out)).tolist() == [int(np.argmax(z))]
    out, _ = o_filter.filter_row(z, top_k=7)
    assert set(np.flatnonzero(np.isfinite(out))) == set(np.argsort(-z)[:7])
    out, margin = o_filter.filter_row(z)                           # both filters off
    assert np.array_equal(out, z) and margin == np.inf
    out, _ = o_filter.filter_row(z, top_k=500)                     # k beyond the row keeps everything
    assert np.array_equal(out, z)
    z2 = z.copy(); z2[[3, 9]] = -np.inf
    out, _ = o_filter.filter_row(z2, top_p=0.9999999)
    assert not np.isfinite(out[[3, 9]]).any()                      # -inf stays out
    out, _ = o_filter.filter_row(np.full(5, -np.inf, dtype=np.float32), top_p=0.9)
    assert not np.isfinite(out).any()


def test_ties_at_the_cut_are_kept_together_and_filters_compose():
    z = np.log(np.array([0.4, 0.2, 0.2, 0.1, 0.1], dtype=np.float64)).astype(np.float32)
    out, _ = o_filter.filter_row(z, top_p=0.5)                     # 0.4 + 0.2 reaches 0.5: both 0.2 stay
    assert np.isfinite(out).tolist() == [True, True, True, False, False]
    out, _ = o_filter.filter_row(z, top_k=2)
    assert np.isfinite(out).tolist() == [True, True, True, False, False]
    # top-k first (0.4, 0.2, 0.2 -> 0.5, 0.25, 0.25), then top-p 0.7 on the renormalised row
    out, _ = o_filter.filter_row(z, top_k=3, top_p=0.7)
    assert np.isfinite(out).tolist() == [True, True, True, False, False]
    out, _ = o_filter.filter_row(z, top_k=3, top_p=0.45)
    assert np.isfinite(out).tolist() == [True, False, False, False, False]


def test_rows_are_independent():
    rng = np.random.default_rng(3)
    z = rng.standard_normal((4, 200)).astype(np.float32)
    out, kept, margin = o_filter.filter_logits(z, top_p=0.8)
    for r in range(4):
        one, m = o_filter.filter_row(z[r], top_p=0.8)
        assert np.array_equal(out[r], one) and kept[r] == np.isfinite(one).sum() and margin[r] == m
