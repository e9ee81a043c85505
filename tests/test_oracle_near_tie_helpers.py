"""Pins of the oracle's near-tie helpers -- the functions that tell the GPU parity tests which
comparisons may be skipped.  Each is driven with hand-built inputs whose deciding gap is known in
closed form and lies just below or just above the 1e-5 threshold; a helper that reported ties too
eagerly would silently turn parity tests into shape checks, one that missed them would make them
flaky.

The random numbers the helpers draw are Philox words (pinned by known-answer vectors elsewhere);
here they are read back and *cancelled* by the inputs, so that the perturbed scores take values
chosen by the test.
"""
import numpy as np
import pytest

from oracle import gumbel_topk as o_topk
from oracle import philox
from oracle import prob_filter as o_pf
from oracle import rrs as o_rrs

TOL = 1e-5


# ------------------------------------------------------------------ gumbel_topk.near_tie_rows
def _logits_with_perturbed(target, seed, step, seq, node):
    """Logits whose perturbed scores phi + G equal `target` up to one common shift (the row's
    log-normaliser), so that every gap between them is the gap in `target`."""
    g = philox.gumbel_row(seed, step, philox.TAG_DRAFT_GUMBEL, seq, node, len(target))
    return np.asarray(target, dtype=np.float64) - g


@pytest.mark.parametrize("gap,expect", [(0.9e-5, True), (1.1e-5, False)])
def test_near_tie_rows_sees_a_gap_inside_the_top_k_plus_one(gap, expect):
    seed, step = 12345, 7
    k = 2
    # ranks 1..3 matter for k = 2; the controlled gap sits between ranks 2 and 3 (the cut itself)
    target = np.array([1.0, 4.0, 4.0 - 0.5, -2.0, 4.0 - 0.5 - gap, 0.0, -1.0, -3.0])
    z = np.stack([_logits_with_perturbed(target, seed, step, 3, 9)])
    near = o_topk.near_tie_rows(z, [k], 1.0, [3], [9], seed, step, tol=TOL)
    assert bool(near[0]) is expect
    # the same gap between ranks 1 and 2
    target = np.array([1.0, 4.0, 4.0 - gap, -2.0, 2.0, 0.0, -1.0, -3.0])
    z = np.stack([_logits_with_perturbed(target, seed, step, 3, 9)])
    assert bool(o_topk.near_tie_rows(z, [k], 1.0, [3], [9], seed, step, tol=TOL)[0]) is expect


def test_near_tie_rows_ignores_gaps_below_the_cut_and_other_rows():
    seed, step = 5, 0
    # ranks 4 and 5 are 1e-9 apart: irrelevant for k = 2 (only ranks 1..3 can change the output)
    target = np.array([9.0, 7.0, 5.0, 3.0, 3.0 - 1e-9, 1.0])
    z0 = _logits_with_perturbed(target, seed, step, 0, 0)
    # second row: a real tie at the cut; the flag must land on that row only
    target1 = np.array([9.0, 7.0, 7.0 - 1e-7, 3.0, 2.0, 1.0])
    z1 = _logits_with_perturbed(target1, seed, step, 0, 1)
    near = o_topk.near_tie_rows(np.stack([z0, z1]), [2, 2], 1.0, [0, 0], [0, 1], seed, step, tol=TOL)
    assert near.tolist() == [False, True]
    # with k = 4 the first row's close pair is ranks 4/5 = inside the top k+1: now it counts
    assert bool(o_topk.near_tie_rows(np.stack([z0]), [4], 1.0, [0], [0], seed, step, tol=TOL)[0])
    # -inf entries are not candidates: a row with two finite entries and k = 4 has one gap only
    z2 = z0.copy()
    z2[2:] = -np.inf
    assert not o_topk.near_tie_rows(np.stack([z2]), [4], 1.0, [0], [0], seed, step, tol=TOL)[0]


# ------------------------------------------------------------------ rrs: near_tie and last_gap
def _one_level_case(theta_offsets, seed, step, seq, V=6):
    """Root with len(theta_offsets) children; child k's threshold is its own uniform plus
    theta_offsets[k] -- built with a uniform draft row, so Theta_1 = q(x_1) * V etc.  Only the first
    child is placed exactly; later siblings follow whatever the residuals give."""
    K = len(theta_offsets)
    tokens = np.array([[-1] + list(range(K))])
    parent = np.array([[-1] + [0] * K])
    n_nodes = np.array([K + 1])
    u1 = philox.accept_uniform(seed, step, seq, 1)
    theta1 = u1 + theta_offsets[0]
    assert 0 < theta1 < 1
    p = np.full(V, 1.0 / V)
    q = np.full(V, (1.0 - theta1 / V) / (V - 1))
    q[0] = theta1 / V                       # Theta_1 = q(x_1) / p(x_1) = theta1
    zt = np.zeros((1, K + 1, V))
    zd = np.zeros((1, K + 1, V))
    zt[0, 0], zd[0, 0] = np.log(q), np.log(p)
    return zt, zd, tokens, parent, n_nodes, u1, theta1


@pytest.mark.parametrize("offset,expect", [(0.9e-5, True), (-0.9e-5, True), (1.1e-5, False), (-1.1e-5, False)])
def test_recursive_reject_near_tie_flag_on_the_decided_node(offset, expect):
    seed, step, seq = 99, 2, 4
    zt, zd, tokens, parent, n_nodes, u1, theta1 = _one_level_case([offset], seed, step, seq)
    r = o_rrs.recursive_reject(zt, zd, tokens, parent, n_nodes, seq_id=[seq], seed=seed, step=step)
    assert r["theta"][0, 1] == pytest.approx(theta1, rel=1e-12)
    assert r["uniforms"][0, 1] == u1
    assert bool(r["near_tie"][0]) is expect
    # the decision itself follows the sign of the offset
    assert int(r["n_accepted"][0]) == (1 if offset > 0 else 0)


def test_recursive_reject_near_tie_ignores_nodes_the_walk_never_tests():
    """Child 1 is accepted by a wide margin; child 2 (never tested: the walk stops at the first
    accepted sibling) and the children of the rejected branch are placed within 1e-9 of their
    uniforms through ALL_GROUPS thresholds -- no flag."""
    seed, step, seq, V = 7, 1, 0, 5
    # tree: root -> {1, 2}; 1 -> {3}; 2 -> {4}
    tokens = np.array([[-1, 0, 1, 2, 3]])
    parent = np.array([[-1, 0, 0, 1, 2]])
    n_nodes = np.array([5])
    u = [philox.accept_uniform(seed, step, seq, j) for j in range(5)]
    zt = np.zeros((1, 5, V))
    zd = np.zeros((1, 5, V))
    p = np.full(V, 1.0 / V)
    zd[0, :] = np.log(p)
    zt[0, 0] = np.log(p)                    # identical rows at the root: Theta = 1, child 1 accepted
    # node 2's only child (node 4) within 1e-9 of its uniform: node 2 is never reached
    th4 = u[4] + 1e-9
    q2 = np.full(V, (1.0 - th4 / V) / (V - 1)); q2[3] = th4 / V
    zt[0, 2] = np.log(q2)
    # node 1's child (node 3) is decided with a clear margin
    th3 = min(0.999, u[3] + 0.2) if u[3] < 0.7 else u[3] - 0.2
    q1 = np.full(V, (1.0 - th3 / V) / (V - 1)); q1[2] = th3 / V
    zt[0, 1] = np.log(q1)
    for mode in (o_rrs.MODE_PATH, o_rrs.MODE_ALL_GROUPS):
        r = o_rrs.recursive_reject(zt, zd, tokens, parent, n_nodes, seq_id=[seq], seed=seed, step=step,
                                   mode=mode)
        assert r["accepted_nodes"][0, 0] == 1
        assert not r["near_tie"][0]
        if mode == o_rrs.MODE_ALL_GROUPS:
            assert abs(r["theta"][0, 4] - u[4]) < 1e-8        # the near tie exists, off the walk
    # the same construction with the close call moved onto the walk (node 3) is flagged
    th3 = u[3] + 1e-9
    q1 = np.full(V, (1.0 - th3 / V) / (V - 1)); q1[2] = th3 / V
    zt[0, 1] = np.log(q1)
    r = o_rrs.recursive_reject(zt, zd, tokens, parent, n_nodes, seq_id=[seq], seed=seed, step=step)
    assert r["near_tie"][0]


def test_recursive_reject_near_tie_on_a_later_sibling():
    """First child clearly rejected, second child within 0.5e-5 of its uniform: the flag must look at
    every sibling the walk tested, not only the first or the accepted one."""
    seed, step, seq, V = 21, 0, 2, 4
    tokens = np.array([[-1, 0, 1]])
    parent = np.array([[-1, 0, 0]])
    n_nodes = np.array([3])
    u1 = philox.accept_uniform(seed, step, seq, 1)
    u2 = philox.accept_uniform(seed, step, seq, 2)
    p = np.full(V, 0.25)
    # q(x_1) = 0: Theta_1 = 0, rejected whatever u1 is; residual q^(2) = Norm[(q - p)^+],
    # p^(2) = uniform over the other three tokens.  Choose q so that Theta_2 = u2 + 0.5e-5.
    theta2 = u2 + 0.5e-5
    # q = (0, a, b, b) with a + 2b = 1.  (q - p)^+ needs a case split on a, b vs 1/4; solve numerically
    # on the closed form instead: scan a for the wanted threshold with the oracle's own chain pinned
    # elsewhere (Theorem 3.1 enumeration), then verify the threshold value independently below.
    lo, hi = 0.0, 1.0
    for _ in range(200):
        a = 0.5 * (lo + hi)
        b = (1.0 - a) / 2.0
        q = np.array([0.0, a, b, b])
        r = np.maximum(q - p, 0.0)
        th = min(1.0, (r[1] / r.sum()) / (1.0 / 3.0))       # Eq. (2), Eq. (3) written out for this case
        lo, hi = (a, hi) if th < theta2 else (lo, a)
    if not (0 < theta2 < 1):
        pytest.skip("uniform too close to the ends for this construction")
    zt = np.zeros((1, 3, V)); zd = np.zeros((1, 3, V))
    with np.errstate(divide="ignore"):
        zt[0, 0] = np.log(q)
    zd[0, 0] = np.log(p)
    r = o_rrs.recursive_reject(zt, zd, tokens, parent, n_nodes, seq_id=[seq], seed=seed, step=step)
    assert r["theta"][0, 1] == 0.0 and r["uniforms"][0, 2] == u2
    assert abs(r["theta"][0, 2] - theta2) < 1e-9
    assert r["near_tie"][0]
    assert abs(u1 - 0.0) > 1e-5           # (the first sibling's own test was not a close call)


@pytest.mark.parametrize("gap", [0.9e-5, 1.1e-5, 0.37])
def test_recursive_reject_last_gap_is_top1_minus_top2_of_the_final_scores(gap):
    """Root without children: the last token is the Gumbel-max over the target row itself, so with
    logits that cancel the noise the two best scores are what the test chose."""
    seed, step, seq, V = 31, 5, 1, 9
    g = philox.gumbel_row(seed, step, philox.TAG_LAST_GUMBEL, seq, 0, V)
    target = np.array([0.0, -1.0, 3.0, 3.0 - gap, -4.0, 1.0, 2.0, -2.0, 0.5])
    zt = (target - g)[None, None, :]
    zd = np.zeros_like(zt)
    r = o_rrs.recursive_reject(zt, zd, np.array([[-1]]), np.array([[-1]]), np.array([1]),
                               seq_id=[seq], seed=seed, step=step)
    assert int(r["last_token"][0]) == 2 and int(r["n_accepted"][0]) == 0
    assert r["last_gap"][0] == pytest.approx(gap, rel=1e-9)
    assert (r["last_gap"][0] < TOL) == (gap < TOL)


# ------------------------------------------------------------------ prob_filter.filter_row margin
def _logits_of(prob):
    return np.log(np.asarray(prob, dtype=np.float64))


@pytest.mark.parametrize("top_p,kept,margin", [
    (0.8 + 1e-5, 3, 1e-5),        # the mass just misses the target after two entries: a third is needed
    (0.8 - 1e-5, 2, 1e-5),        # ... just reaches it
    (0.8 + 2e-7, 3, 2e-7),
    (0.6, 2, 0.1),                # far from any cut: min(0.8 - 0.6, 0.6 - 0.5)
])
def test_filter_row_margin_is_the_distance_of_the_mass_from_the_target(top_p, kept, margin):
    z = _logits_of([0.5, 0.3, 0.15, 0.05])
    out, m = o_pf.filter_row(z, 1.0, 0, top_p)
    assert int(np.isfinite(out).sum()) == kept
    assert m == pytest.approx(margin, rel=1e-6)


@pytest.mark.parametrize("rel_gap", [2e-6, 0.5e-5, 1e-3])
def test_filter_row_margin_is_the_relative_gap_at_the_cut(rel_gap):
    """top-k: the k-th and (k+1)-th most probable entries differ by a known relative amount."""
    p3 = 0.2
    p4 = p3 * (1.0 - rel_gap)
    rest = 1.0 - 0.3 - 0.25 - p3 - p4
    z = _logits_of([0.3, p4, 0.25, rest, p3])
    out, m = o_pf.filter_row(z, 1.0, 3, 1.0)
    assert np.isfinite(out).tolist() == [True, False, True, False, True]
    assert m == pytest.approx(rel_gap, rel=1e-6)
    # top-p whose cut falls between those two entries, far from the mass target on both sides:
    # the margin is again the relative gap between the last kept and the first dropped entry
    out, m = o_pf.filter_row(z, 1.0, 0, 0.7)
    assert int(np.isfinite(out).sum()) == 3
    assert m == pytest.approx(rel_gap, rel=1e-6)


def test_filter_row_margin_is_infinite_when_nothing_is_decided():
    z = _logits_of([0.4, 0.3, 0.2, 0.1])
    assert o_pf.filter_row(z, 1.0, 0, 1.0)[1] == np.inf          # both filters off
    assert o_pf.filter_row(z, 1.0, 4, 1.0)[1] == np.inf          # k = number of entries: nothing dropped
    assert o_pf.filter_row(np.full(4, -np.inf), 1.0, 2, 0.5)[1] == np.inf
    # exact ties at the cut are kept together and do not count as a close call by themselves
    z = _logits_of([0.4, 0.2, 0.2, 0.1, 0.1])
    out, m = o_pf.filter_row(z, 1.0, 2, 1.0)
    assert int(np.isfinite(out).sum()) == 3 and m == pytest.approx(0.5)
