"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Inputs are generated on the GPU exactly as bench.py does; the oracle recomputes sampled
outputs (whole trees, whole attention heads, whole verification walks of sampled
sequences) from copies of the same inputs, and size-independent properties are checked on
everything."""
import numpy as np
import pytest
import torch

import bench
from oracle import rrs as o_rrs
from oracle import tree_attention as o_attn
from paper_2402_14160_amd import binding, draft_tree, workloads
from tests.gpu_util import NEAR_TIE, oracle_tree_const, say, to_np

pytestmark = pytest.mark.gpu


def _case(index):
    cfg = workloads.config(index)
    return cfg, bench.build_case(cfg, 0, torch, binding, draft_tree, workloads)


@pytest.mark.parametrize("index", [1, 2, 3, 4])
def test_full_size_step_matches_oracle_on_samples(index):
    cfg, case = _case(index)
    say(f"full size {cfg['name']}")
    B, N, V = cfg["B"], cfg["N"], cfg["V"]
    tree = case["tree"]
    n_nodes = to_np(tree["n_nodes"])
    parent, tokens = to_np(tree["parent"]), to_np(tree["tokens"])
    rng = np.random.default_rng(index)
    seqs = sorted(set([0, B - 1] + rng.integers(0, B, size=2).tolist()))[:3]

    # ---- trees: structure everywhere, exact tokens on sampled sequences -----------------
    assert np.all(n_nodes == cfg["N"])
    for b in range(B):
        n = int(n_nodes[b])
        assert binding.validate_tree(parent[b, :n]) == 0
        assert np.all((tokens[b, 1:n] >= 0) & (tokens[b, 1:n] < V))
        for p in set(parent[b, 1:n].tolist()):          # siblings are distinct tokens
            kids = tokens[b, 1:n][parent[b, 1:n] == p]
            assert len(set(kids.tolist())) == len(kids)
    for b in seqs:
        zd_b = to_np(case["zd"][b])
        if cfg["sampler"] == "gumbel":
            counts = workloads.tree_child_counts(cfg, 0)[b]
            ref = oracle_tree_const(zd_b, counts, b, 0, 0)
        else:
            from oracle import draft_tree as o_tree
            ref = o_tree.create_draft_tree_sbs(zd_b, cfg["width"], cfg["depth"], seq=b, seed=0, step=0)
        n = len(ref["tokens"])
        assert n == int(n_nodes[b])
        assert np.array_equal(tokens[b, :n], ref["tokens"]) and np.array_equal(parent[b, :n], ref["parent"])

    # ---- attention: sampled (sequence, KV head) groups against the fp64 oracle ------------
    case["attn"]()
    torch.cuda.synchronize()
    out = case["attn_out"]
    assert torch.isfinite(out).all()
    group = cfg["Hq"] // cfg["Hkv"]
    f = lambda t: t.to(torch.float32).cpu().numpy()
    worst = 0.0
    for b in seqs[:2]:
        for g in sorted(set([0, cfg["Hkv"] - 1, int(rng.integers(0, cfg["Hkv"]))]))[:2]:
            hs = slice(g * group, (g + 1) * group)
            ref, _ = o_attn.tree_attention(f(case["q"][b:b + 1, hs]), f(case["kp"][b:b + 1, g:g + 1]),
                                           f(case["vp"][b:b + 1, g:g + 1]), f(case["kt"][b:b + 1, g:g + 1]),
                                           f(case["vt"][b:b + 1, g:g + 1]), [cfg["P"]], [int(n_nodes[b])],
                                           parent[b:b + 1], case["scale"])
            worst = max(worst, float(np.abs(to_np(out[b, hs]) - ref[0]).max()))
    say(f"  attention max abs err on samples: {worst:.2e}")
    assert worst < 1e-2

    # ---- recursive rejection sampling: sampled sequences against the oracle ---------------
    got = binding.recursive_reject(case["zd"], case["zt"], tree["tokens"], tree["parent"], tree["n_nodes"],
                                   mode=binding.MODE_ALL_GROUPS, seed=0, step=0)
    path = binding.recursive_reject(case["zd"], case["zt"], tree["tokens"], tree["parent"], tree["n_nodes"],
                                    mode=binding.MODE_PATH, seed=0, step=0, diagnostics=False)
    for key in ("accepted_nodes", "n_accepted", "last_token", "final_node"):
        assert torch.equal(got[key], path[key]), key        # both modes decide identically
    acc, n_acc, last = to_np(got["accepted_nodes"]), to_np(got["n_accepted"]), to_np(got["last_token"])
    theta, uni = to_np(got["theta"]), to_np(got["uniforms"])
    assert np.all((last >= 0) & (last < V)) and np.all(to_np(got["flags"]) == 0)
    for b in range(B):                                      # accepted path is a root path of accepted tests
        cur = 0
        for j in acc[b, :n_acc[b]]:
            assert parent[b, j] == cur and uni[b, j] < theta[b, j]
            earlier = [c for c in range(1, j) if parent[b, c] == cur]
            assert all(uni[b, c] >= theta[b, c] for c in earlier)
            cur = j
        assert int(got["final_node"][b]) == cur
        assert np.all(acc[b, n_acc[b]:] == -1)
    near = 0
    for b in seqs:
        ref = o_rrs.recursive_reject(to_np(case["zt"][b:b + 1]), to_np(case["zd"][b:b + 1]), tokens[b:b + 1],
                                     parent[b:b + 1], n_nodes[b:b + 1], mode=o_rrs.MODE_ALL_GROUPS,
                                     seq_id=[b], seed=0, step=0)
        both = np.isfinite(ref["theta"][0])
        assert np.allclose(theta[b][both], ref["theta"][0][both], rtol=1e-5, atol=1e-6)
        assert np.array_equal(uni[b, 1:int(n_nodes[b])].astype(np.float64), ref["uniforms"][0, 1:int(n_nodes[b])])
        if ref["near_tie"][0] or ref["last_gap"][0] < NEAR_TIE:
            near += 1
            continue
        k = int(ref["n_accepted"][0])
        assert int(n_acc[b]) == k and np.array_equal(acc[b, :k], ref["accepted_nodes"][0, :k])
        assert int(last[b]) == int(ref["last_token"][0])
    say(f"  rrs near-tie samples: {near} of {len(seqs)}; mean accepted {n_acc.mean():.2f}")
    assert near <= 1
    del case
    torch.cuda.empty_cache()
