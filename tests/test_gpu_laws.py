"""The laws the paper proves, checked on the GPU path itself by sampling (beyond token-for-token parity
with the oracle): Gumbel-Top-k draws follow sampling without replacement (Sec. 3.2.1), and the first
token a verified iteration emits follows the target distribution (Theorem 3.1), whatever the draft."""
import itertools

import numpy as np
import pytest
import torch
from scipy import special, stats

from paper_2402_14160_amd import binding, draft_tree
from tests.gpu_util import dev, say, to_np

pytestmark = pytest.mark.gpu


def _chi2_ok(obs, exp):
    big = exp >= 5
    chi2 = np.sum((obs[big] - exp[big]) ** 2 / exp[big])
    return stats.chi2.sf(chi2, int(big.sum()) - 1)


def test_gumbel_topk_rows_follow_sampling_without_replacement():
    V, k, R = 8, 2, 60000
    say(f"law of {R} Gumbel-Top-{k} draws, vocabulary {V}")
    rng = np.random.default_rng(0)
    logits = rng.normal(0, 1.5, size=V).astype(np.float32)
    p = special.softmax(logits.astype(np.float64))
    rows = torch.from_numpy(np.tile(logits, (R, 1))).to(dev())
    out = binding.gumbel_topk(rows, k, seed=77, step=3)
    toks = to_np(out["tokens"])
    assert (to_np(out["count"]) == k).all()
    keys = list(itertools.permutations(range(V), k))
    index = {key: i for i, key in enumerate(keys)}
    obs = np.zeros(len(keys))
    for a, b in toks:
        obs[index[(int(a), int(b))]] += 1
    exp = np.array([p[a] * p[b] / (1 - p[a]) for a, b in keys]) * R
    pval = _chi2_ok(obs, exp)
    say(f"  chi-square p-value {pval:.3f}")
    assert pval > 1e-4
    assert np.all(np.abs(obs - exp) <= 5 * np.sqrt(exp) + 1)


@pytest.mark.parametrize("mode", [binding.MODE_PATH, binding.MODE_ALL_GROUPS])
def test_first_emitted_token_follows_the_target_distribution(mode):
    """Every sequence has the same two rows of logits at its root (a draft that differs markedly from
    the target) and drafts three children without replacement; the token emitted first -- the accepted
    child's, or the residual sample when all three are rejected -- must be distributed as the target."""
    V, K, B = 8, 3, 20000
    say(f"law of the first emitted token over {B} sequences, mode {mode}")
    rng = np.random.default_rng(1)
    zt_row = rng.normal(0, 1.5, size=V).astype(np.float32)
    zd_row = (zt_row + rng.normal(0, 1.5, size=V)).astype(np.float32)
    q = special.softmax(zt_row.astype(np.float64))
    N = 1 + K
    zt = torch.from_numpy(rng.normal(0, 1, size=(B, N, V)).astype(np.float32))
    zd = torch.from_numpy(rng.normal(0, 1, size=(B, N, V)).astype(np.float32))
    zt[:, 0], zd[:, 0] = torch.from_numpy(zt_row), torch.from_numpy(zd_row)
    d = dev()
    zt, zd = zt.to(d), zd.to(d)
    tree = draft_tree.create_draft_tree_const(zd, [[[K]]] * B, seed=5, step=0)
    g = binding.recursive_reject(zd, zt, tree["tokens"], tree["parent"], tree["n_nodes"], mode=mode,
                                 seed=5, step=0)
    n_acc, acc_tok, last = to_np(g["n_accepted"]), to_np(g["accepted_tokens"]), to_np(g["last_token"])
    first = np.where(n_acc > 0, acc_tok[:, 0], last)
    obs = np.bincount(first, minlength=V).astype(np.float64)
    pval = _chi2_ok(obs, q * B)
    say(f"  accepted at level one: {np.mean(n_acc > 0):.3f}; chi-square p-value {pval:.3f}")
    assert pval > 1e-4
    assert np.all(np.abs(obs - q * B) <= 5 * np.sqrt(q * B) + 1)
    assert 0.2 < np.mean(n_acc > 0) < 0.999            # both branches of the verification are exercised


def test_two_sbs_levels_sample_sequences_without_replacement():
    """Theorem 3.2 on the GPU path: with a tabulated toy model (the next-token logits depend on the
    previous token only) two Stochastic Beam Search levels of width 2 return, in order, two length-2
    sequences drawn without replacement from the model's sequence distribution."""
    V, W, B = 4, 2, 40000
    say(f"law of the two sequences kept by {B} two-level beam searches, vocabulary {V}")
    rng = np.random.default_rng(2)
    root = rng.normal(0, 1.2, size=V).astype(np.float32)
    nxt = rng.normal(0, 1.2, size=(V, V)).astype(np.float32)
    p_root = special.softmax(root.astype(np.float64))
    p_next = special.softmax(nxt.astype(np.float64), axis=1)
    seqs = list(itertools.product(range(V), range(V)))
    p_seq = {s: p_root[s[0]] * p_next[s[0], s[1]] for s in seqs}
    keys = list(itertools.permutations(seqs, 2))
    exp = np.array([p_seq[a] * p_seq[b] / (1 - p_seq[a]) for a, b in keys]) * B
    d = dev()
    zeros = torch.zeros((B, 1), dtype=torch.float32, device=d)
    l0 = binding.sbs_step(torch.from_numpy(root).to(d).expand(B, 1, V).contiguous(), zeros, zeros,
                          torch.ones(B, dtype=torch.int32, device=d), W, seed=9, step=0)
    t0 = l0["tokens"].long()                                            # [B, W] first tokens of the beams
    z1 = torch.from_numpy(nxt).to(d)[t0]                                 # [B, W, V]: rows of the table
    node = torch.tensor([[1, 2]], dtype=torch.int32, device=d).expand(B, W).contiguous()
    l1 = binding.sbs_step(z1.contiguous(), l0["sum_logprob"], l0["trunc_gumbel"],
                          torch.full((B,), W, dtype=torch.int32, device=d), W, node_id=node, seed=9, step=0)
    first = torch.gather(t0, 1, l1["parent"].long())
    out = torch.stack([first, l1["tokens"].long()], dim=2).cpu().numpy()  # [B, W, 2]
    index = {key: i for i, key in enumerate(keys)}
    obs = np.zeros(len(keys))
    for pair in out:
        obs[index[((int(pair[0, 0]), int(pair[0, 1])), (int(pair[1, 0]), int(pair[1, 1])))]] += 1
    pval = _chi2_ok(obs, exp)
    say(f"  chi-square p-value {pval:.3f}")
    assert pval > 1e-4
    # the carried sum of log-probabilities is the log-probability of the kept sequence
    s_out = to_np(l1["sum_logprob"])
    want = np.log(np.array([[p_seq[(int(p[0, 0]), int(p[0, 1]))], p_seq[(int(p[1, 0]), int(p[1, 1]))]] for p in out[:200]]))
    assert np.allclose(s_out[:200], want, rtol=0, atol=1e-5)
