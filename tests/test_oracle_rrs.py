"""Pins for the oracle's recursive rejection sampling (Sec. 3.1, Alg. 1, Alg. 6)."""
import itertools

import numpy as np
import pytest
from scipy import special, stats

from oracle import philox
from oracle.rrs import (MODE_ALL_GROUPS, MODE_PATH, recursive_reject,
                        recursive_reject_core, sibling_chain)


def ordered_draft_law(p, K):
    """Probability of each ordered K-tuple drawn without replacement from p."""
    law = {}
    for tup in itertools.permutations(range(len(p)), K):
        pr, rem = 1.0, 1.0
        for x in tup:
            pr *= p[x] / rem
            rem -= p[x]
        law[tup] = pr
    return law


@pytest.mark.parametrize("V,K,seed", [(2, 1, 0), (3, 2, 1), (4, 3, 2), (4, 2, 3), (3, 3, 4)])
def test_theorem_3_1_output_law_equals_target_by_exact_enumeration(V, K, seed):
    rng = np.random.default_rng(seed)
    q = rng.dirichlet(np.ones(V))
    p = rng.dirichlet(np.ones(V))
    out = np.zeros(V)
    for tup, pr in ordered_draft_law(p, K).items():
        theta, residuals, deg = sibling_chain(q, p, tup)
        reach = 1.0                       # probability all earlier drafts were rejected
        for k, x in enumerate(tup):
            out[x] += pr * reach * theta[k]
            reach *= 1 - theta[k]
            assert reach < 1e-12 or not deg[k]   # a residual that can be reached exists
        out += pr * reach * residuals[K]
    assert np.allclose(out, q, atol=1e-12)


def test_single_draft_reduces_to_speculative_sampling():
    # K = 1 (Sec. 2, step 3): accept w.p. min(1, q/p); residual Norm[(q-p)^+];
    # overall acceptance probability sum_x min(p, q).
    rng = np.random.default_rng(5)
    q, p = rng.dirichlet(np.ones(6)), rng.dirichlet(np.ones(6))
    acc = 0.0
    for x in range(6):
        theta, residuals, _ = sibling_chain(q, p, [x])
        assert theta[0] == min(1.0, q[x] / p[x])
        want = np.maximum(q - p, 0)
        assert np.allclose(residuals[1], want / want.sum(), atol=1e-15)
        acc += p[x] * theta[0]
    assert abs(acc - np.minimum(p, q).sum()) < 1e-14
    # per-stage mass balance: accepted mass + residual mass = 1
    assert abs(acc + np.maximum(q - p, 0).sum() - 1) < 1e-14


def test_two_symbol_toy_second_draft_is_always_accepted():
    # Sec. 3.1, toy example: Bernoulli draft/target, K = 2 without replacement.
    for a in np.linspace(0.02, 0.98, 25):
        for b in np.linspace(0.02, 0.98, 25):
            q, p = np.array([a, 1 - a]), np.array([b, 1 - b])
            for first in (0, 1):
                theta, residuals, _ = sibling_chain(q, p, [first, 1 - first])
                if theta[0] < 1:          # first draft can be rejected
                    assert theta[1] == 1.0


def test_toy_example_acceptance_rate_matches_the_paper():
    """tests/golden/toy_bernoulli_acceptance.txt holds what the paper's toy example states; the rate is
    computed here by exact enumeration over both orders in which the two tokens can be drafted."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "toy_bernoulli_acceptance.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert rows == [["recursive_rejection_sampling", "2", "1.0"]]
    K, want = int(rows[0][1]), float(rows[0][2])
    for a in np.linspace(0.03, 0.97, 17):
        for b in np.linspace(0.03, 0.97, 17):
            q, p = np.array([a, 1 - a]), np.array([b, 1 - b])
            rate = 0.0
            for first in (0, 1):
                order = [first, 1 - first][:K]
                theta, _, _ = sibling_chain(q, p, order)
                draw = p[first]                       # the second token is then certain (without replacement)
                rate += draw * (theta[0] + (1 - theta[0]) * theta[1])
            assert abs(rate - want) < 1e-12


def test_second_stage_uses_without_replacement_conditional():
    # after rejecting x1 the draft conditional is p with x1 removed and renormalised,
    # and the threshold of x2 is q2(x2)/p2(x2) with q2 = Norm[(q-p)^+]
    q = np.array([0.1, 0.2, 0.3, 0.4])
    p = np.array([0.4, 0.3, 0.2, 0.1])
    theta, residuals, _ = sibling_chain(q, p, [0, 3])
    q2 = np.array([0, 0, 0.1, 0.3]) / 0.4
    p2 = np.array([0, 0.3, 0.2, 0.1]) / 0.6
    assert np.allclose(residuals[1], q2)
    assert theta[0] == 0.25 and theta[1] == min(1.0, q2[3] / p2[3])
    q3 = np.maximum(q2 - p2, 0)
    assert np.allclose(residuals[2], q3 / q3.sum())


# ---------- whole-tree enumeration on a tabulated toy model ----------

def _toy_model(V, seed):
    rng = np.random.default_rng(seed)
    def table():
        return {(): rng.normal(0, 1, V), **{(x,): rng.normal(0, 1, V) for x in range(V)},
                **{(x, y): rng.normal(0, 1, V) for x in range(V) for y in range(V)}}
    return table(), table()          # target logits, draft logits by token history


def _enumerate_trees(V, branching, draft):
    """All RSD-C trees with their probabilities (children of a node are an ordered
    without-replacement draw from the draft distribution after that node)."""
    trees = [(dict(tokens=[-1], parent=[-1], hist=[()], level=[0]), 1.0)]
    for l, b in enumerate(branching):
        nxt = []
        for tree, pr in trees:
            nodes = [i for i in range(len(tree["tokens"])) if tree["level"][i] == l]
            options = []
            for i in nodes:
                law = ordered_draft_law(special.softmax(draft[tree["hist"][i]]), b)
                options.append([(i, tup, w) for tup, w in law.items()])
            for combo in itertools.product(*options):
                t = {k: list(v) for k, v in tree.items()}
                w_all = pr
                for i, tup, w in combo:
                    w_all *= w
                    for x in tup:
                        t["tokens"].append(x); t["parent"].append(i)
                        t["hist"].append(tree["hist"][i] + (x,)); t["level"].append(l + 1)
                nxt.append((t, w_all))
        trees = nxt
    return trees


@pytest.mark.parametrize("mode", [MODE_PATH, MODE_ALL_GROUPS])
def test_tree_walk_recovers_target_sequence_law_by_exact_enumeration(mode):
    V, branching = 3, (2, 1)
    target, draft = _toy_model(V, 7)
    trees = _enumerate_trees(V, branching, draft)
    assert abs(sum(w for _, w in trees) - 1) < 1e-12
    first = np.zeros(V)                       # law of the first emitted token
    second = np.zeros((V, V))                 # joint law (first accepted draft x, next emitted y)
    first_accepted = np.zeros(V)
    for tree, w_tree in trees:
        n = len(tree["tokens"])
        zt = np.stack([target[h] for h in tree["hist"]])
        zd = np.stack([draft[h] for h in tree["hist"]])
        seen = {}
        for pattern in itertools.product((0.0, 1.0), repeat=n - 1):
            u = np.array((0.5,) + pattern)    # u=0 forces accept (theta>0), u=1 forces reject
            r = recursive_reject_core(zt, zd, tree["tokens"], tree["parent"], n, u,
                                      lambda node: np.zeros(V), mode=mode)
            # probability of this decision path: product over the tested nodes
            tested, cur = [], 0
            path = list(r["accepted_nodes"])
            for j in path + [None]:
                for c in [c for c in range(1, n) if tree["parent"][c] == cur]:
                    tested.append((c, c == j))
                    if c == j:
                        break
                if j is None:
                    break
                cur = j
            key = tuple(tested)
            if key in seen:
                continue
            seen[key] = True
            w = w_tree
            for c, took in tested:
                w *= r["theta"][c] if took else 1 - r["theta"][c]
            if w == 0:
                continue
            toks = [tree["tokens"][j] for j in path]
            if not toks:
                first += w * r["final_dist"]
            else:
                first[toks[0]] += w
                first_accepted[toks[0]] += w
                if len(toks) >= 2:
                    second[toks[0], toks[1]] += w
                else:
                    second[toks[0]] += w * r["final_dist"]
        assert len(seen) >= 2
    q_root = special.softmax(target[()])
    assert np.allclose(first, q_root, atol=1e-12)
    for x in range(V):
        assert np.allclose(second[x] / first_accepted[x], special.softmax(target[(x,)]), atol=1e-12)


def test_modes_agree_and_all_groups_fills_every_threshold():
    rng = np.random.default_rng(9)
    B, N, V = 4, 8, 20
    zt = rng.normal(0, 2, size=(B, N, V)).astype(np.float32)
    zd = (zt + rng.normal(0, 1, size=(B, N, V))).astype(np.float32)
    parent = np.tile(np.array([-1, 0, 0, 0, 1, 1, 2, 4]), (B, 1))
    tokens = np.tile(np.array([-1, 3, 5, 7, 1, 2, 9, 11]), (B, 1))
    a = recursive_reject(zt, zd, tokens, parent, [N] * B, mode=MODE_PATH, seed=3)
    b = recursive_reject(zt, zd, tokens, parent, [N] * B, mode=MODE_ALL_GROUPS, seed=3)
    for key in ("accepted_nodes", "n_accepted", "last_token", "final_node"):
        assert np.array_equal(a[key], b[key])
    assert np.all(np.isfinite(b["theta"][:, 1:]))
    seen = np.isfinite(a["theta"])
    assert np.allclose(a["theta"][seen], b["theta"][seen])


def test_philox_driven_walk_statistics_single_child_tree():
    # root with one child: accepted w.p. sum_x min(p,q) when the child is drawn from p;
    # on rejection the last token follows Norm[(q-p)^+]; on acceptance it follows the
    # target row of the child.
    V, B = 5, 1 << 13
    rng = np.random.default_rng(12)
    zt = rng.normal(0, 1, size=(2, V)).astype(np.float32)
    zd = rng.normal(0, 1, size=(2, V)).astype(np.float32)
    q, p = special.softmax(zt[0].astype(np.float64)), special.softmax(zd[0].astype(np.float64))
    child = rng.choice(V, size=B, p=p)
    tokens = np.stack([np.full(B, -1), child], 1)
    parent = np.tile(np.array([-1, 0]), (B, 1))
    out = recursive_reject(np.tile(zt, (B, 1, 1)), np.tile(zd, (B, 1, 1)), tokens, parent,
                           [2] * B, seed=77, step=1)
    acc = out["n_accepted"] == 1
    rate = np.minimum(p, q).sum()
    assert abs(acc.mean() - rate) < 5 * np.sqrt(rate * (1 - rate) / B)
    res = np.maximum(q - p, 0); res /= res.sum()
    rej_counts = np.bincount(out["last_token"][~acc], minlength=V)
    keep = res > 0
    assert np.all(rej_counts[~keep] == 0)
    assert stats.chisquare(rej_counts[keep], res[keep] * (~acc).sum()).pvalue > 1e-4
    acc_counts = np.bincount(out["last_token"][acc], minlength=V)
    assert stats.chisquare(acc_counts, special.softmax(zt[1].astype(np.float64)) * acc.sum()).pvalue > 1e-4
    # emitted first token (accepted child or residual draw) follows q
    first = np.where(acc, child, out["last_token"])
    assert stats.chisquare(np.bincount(first, minlength=V), q * B).pvalue > 1e-4
    # uniforms come from stream tag 1 at (seq b, node 1)
    assert out["uniforms"][5, 1] == philox.accept_uniform(77, 1, 5, 1)


def test_identical_models_accept_everything_and_sample_the_leaf():
    rng = np.random.default_rng(13)
    N, V = 4, 10
    z = rng.normal(size=(1, N, V)).astype(np.float32)
    parent = np.array([[-1, 0, 1, 2]])
    tokens = np.array([[-1, 4, 2, 7]])
    out = recursive_reject(z, z, tokens, parent, [N], seed=1)
    assert out["n_accepted"][0] == 3 and list(out["accepted_nodes"][0, :3]) == [1, 2, 3]
    assert out["final_node"][0] == 3
    g = philox.gumbel_row(1, 0, philox.TAG_LAST_GUMBEL, 0, 3, V)
    assert out["last_token"][0] == np.argmax(special.log_softmax(z[0, 3].astype(np.float64)) + g)


def test_interleaved_children_are_taken_in_stored_order():
    # RSD-S style level: children of different parents interleaved; the walk must only
    # test children of the current node, in increasing node index.
    V = 6
    zt = np.zeros((5, V), dtype=np.float32)
    zd = np.zeros((5, V), dtype=np.float32)
    zt[0, 2] = 5.0                        # target strongly prefers token 2 at the root
    parent = np.array([-1, 0, 0, 2, 1])
    tokens = np.array([-1, 1, 2, 3, 4])
    u = np.array([0.5, 0.9, 0.5, 0.0, 0.0])
    r = recursive_reject_core(zt, zd, tokens, parent, 5, u, lambda n: np.zeros(V))
    # node 1 (token 1): theta = q/p small -> rejected with u=0.9; node 2 accepted; then only
    # node 3 is a child of 2
    assert list(r["accepted_nodes"]) == [2, 3]
    assert np.isnan(r["theta"][4])
