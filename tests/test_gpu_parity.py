"""GPU parity: every C-ABI call against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import baselines as o_base
from oracle import filter_kv as o_filter
from oracle import prob_filter as o_pfilter
from oracle import rrs as o_rrs
from oracle import sbs as o_sbs
from oracle import tree_attention as o_attn
from paper_2402_14160_amd import binding, draft_tree, workloads
from tests.gpu_util import (LOGP_TOL, NEAR_TIE, PSI_TOL, check_topk_against_oracle, dev, oracle_tree_const,
                            say, to_np)

pytestmark = pytest.mark.gpu


# --------------------------------------------------------------------------- lse
@pytest.mark.parametrize("R,V,inv_t", [(3, 64, 1.0), (5, 1001, 1.0), (7, 32000, 1.0 / 0.3),
                                       (4, 50272, 1.0)])
def test_log_softmax_lse(R, V, inv_t):
    say(f"lse R={R} V={V}")
    zt, _ = workloads.make_logits("zipf", 1, R, V, seed=1)
    ld = (V + 3) // 4 * 4
    buf = torch.zeros((R, ld), dtype=torch.float32)
    buf[:, :V] = zt[0]
    got = to_np(binding.log_softmax_lse(buf.to(dev())[:, :V], inv_t))
    z = zt[0].numpy().astype(np.float64) * np.float32(inv_t).astype(np.float64)
    ref = np.log(np.sum(np.exp(z - z.max(1, keepdims=True)), 1)) + z.max(1)
    assert np.allclose(got, ref, rtol=0, atol=LOGP_TOL)


# ------------------------------------------------------------------- gumbel top-k
@pytest.mark.parametrize("kind,R,V,k_max,inv_t", [
    ("normal", 3, 64, 2, 1.0),          # config 0 shape
    ("zipf", 9, 1001, 5, 1.0),          # ragged vocabulary tail
    ("zipf", 22, 32000, 3, 1.0),        # config 1 rows
    ("zipf", 12, 32000, 8, 1.0 / 0.3),  # temperature 0.3
    ("zipf", 6, 50272, 6, 1.0),         # OPT vocabulary, second kernel instance
    ("zipf", 2, 65536, 16, 1.0),        # limits
])
def test_gumbel_topk_matches_oracle(kind, R, V, k_max, inv_t):
    say(f"gumbel_topk {kind} R={R} V={V} k={k_max}")
    _, zd = workloads.make_logits(kind, 1, R, V, seed=2)
    ld = (V + 3) // 4 * 4
    buf = torch.zeros((R, ld), dtype=torch.float32)
    buf[:, :V] = zd[0]
    rng = np.random.default_rng(0)
    ks = rng.integers(0, k_max + 1, size=R).astype(np.int32)
    ks[0] = k_max
    seq = rng.integers(0, 100, size=R).astype(np.int32)
    node = rng.integers(0, 256, size=R).astype(np.int32)
    g = binding.gumbel_topk(buf.to(dev())[:, :V], k_max, k_per_row=torch.from_numpy(ks).to(dev()),
                            inv_temperature=inv_t, seq_id=torch.from_numpy(seq).to(dev()),
                            node_id=torch.from_numpy(node).to(dev()), seed=0xABCDEF0123, step=3)
    near = check_topk_against_oracle(zd[0].numpy(), g, ks, np.float32(inv_t), seq, node,
                                     0xABCDEF0123, 3, k_max)
    say(f"  near-tie rows: {near} of {R}")
    assert near <= 1
    g2 = binding.gumbel_topk(buf.to(dev())[:, :V], k_max, k_per_row=torch.from_numpy(ks).to(dev()),
                             inv_temperature=inv_t, seq_id=torch.from_numpy(seq).to(dev()),
                             node_id=torch.from_numpy(node).to(dev()), seed=0xABCDEF0123, step=3)
    for key in ("tokens", "perturbed", "logprob", "lse", "count"):
        assert torch.equal(g[key], g2[key]), key     # run-to-run determinism
    g3 = binding.gumbel_topk(buf.to(dev())[:, :V], k_max, k_per_row=torch.from_numpy(ks).to(dev()),
                             inv_temperature=inv_t, seq_id=torch.from_numpy(seq).to(dev()),
                             node_id=torch.from_numpy(node).to(dev()), seed=0xABCDEF0123, step=3,
                             want_scores=False)
    assert torch.equal(g3["tokens"], g["tokens"]) and torch.equal(g3["count"], g["count"])


def test_gumbel_topk_defaults_and_filtered_rows():
    say("gumbel_topk defaults / -inf rows")
    V, R, k = 5000, 4, 8
    _, zd = workloads.make_logits("zipf", 1, R, V, seed=3)
    z = zd[0].clone()
    z[1, 3:] = -float("inf")                 # 3 finite entries: count < k, slow selection path
    z[2, :] = -float("inf")                  # nothing to sample
    z[3, ::2] = -float("inf")
    g = binding.gumbel_topk(z.to(dev()), k, seed=9)
    near = check_topk_against_oracle(z.numpy(), g, np.full(R, k), 1.0, np.zeros(R, int),
                                     np.arange(R), 9, 0, k)
    assert near == 0
    assert to_np(g["count"]).tolist() == [8, 3, 0, 8]


def test_gumbel_topk_rejects_bad_arguments():
    z = torch.zeros((2, 64), dtype=torch.float32, device=dev())
    for kwargs in (dict(k_max=17), dict(k_max=65), dict(k_max=4, inv_temperature=0.0)):
        with pytest.raises(binding.RsdError) as e:
            binding.gumbel_topk(z, **kwargs)
        assert e.value.code == -2
    with pytest.raises(binding.RsdError):
        binding.gumbel_topk(torch.zeros((1, 70000), dtype=torch.float32, device=dev()), 2)


# -------------------------------------------------------------------------- SBS
@pytest.mark.parametrize("B,W_in,V,W,inv_t", [(1, 1, 64, 2, 1.0), (3, 6, 32000, 6, 1.0),
                                               (2, 6, 50272, 6, 1.0), (2, 12, 4000, 12, 1 / 0.3),
                                               (1, 16, 8192, 16, 1.0)])   # widest beam: 256 candidate slots
def test_sbs_step_matches_oracle(B, W_in, V, W, inv_t):
    say(f"sbs_step B={B} W_in={W_in} V={V} W={W}")
    _, zd = workloads.make_logits("zipf", B, W_in, V, seed=4)
    rng = np.random.default_rng(1)
    sigma = (-rng.exponential(3.0, size=(B, W_in))).astype(np.float32)
    gamma = (-np.sort(rng.exponential(1.0, size=(B, W_in)), axis=1)).astype(np.float32)
    n_in = rng.integers(1, W_in + 1, size=B).astype(np.int32)
    n_in[0] = W_in
    node = rng.integers(0, 200, size=(B, W_in)).astype(np.int32)
    seq = rng.integers(0, 50, size=B).astype(np.int32)
    d = dev()
    g = binding.sbs_step(zd.to(d), torch.from_numpy(sigma).to(d), torch.from_numpy(gamma).to(d),
                         torch.from_numpy(n_in).to(d), W, inv_temperature=inv_t,
                         seq_id=torch.from_numpy(seq).to(d), node_id=torch.from_numpy(node).to(d),
                         seed=77, step=2)
    ref = o_sbs.sbs_step(zd.numpy(), sigma, gamma, n_in, W, inv_temperature=np.float32(inv_t),
                         seq_id=seq, node_id=node, seed=77, step=2)
    assert np.array_equal(to_np(g["n_out"]), ref["n_out"])
    near = 0
    for b in range(B):
        n = int(ref["n_out"][b])
        if ref["min_gap"][b] < NEAR_TIE:
            near += 1
            continue
        assert np.array_equal(to_np(g["tokens"])[b, :n], ref["tokens"][b, :n])
        assert np.array_equal(to_np(g["parent"])[b, :n], ref["parent"][b, :n])
        assert np.allclose(to_np(g["sum_logprob"])[b, :n], ref["sum_logprob"][b, :n], rtol=1e-6, atol=LOGP_TOL)
        assert np.allclose(to_np(g["trunc_gumbel"])[b, :n], ref["trunc_gumbel"][b, :n], rtol=0, atol=PSI_TOL)
        assert np.all(to_np(g["tokens"])[b, n:] == -1)
        live = int(n_in[b])
        assert np.allclose(to_np(g["lse"])[b, :live], ref["lse"][b, :live], rtol=0, atol=LOGP_TOL)
    say(f"  near-tie sequences: {near} of {B}")
    assert near <= 1


def test_sbs_step_split_rows_with_sparse_and_dead_rows():
    """Few rows: each row is split over several workgroups.  One live row keeps only three finite
    entries (all in one segment, so the other segments have no candidate), another sequence has dead
    rows, and the root step (one row per sequence) takes the widest split."""
    say("sbs_step with rows split into segments, sparse and dead rows")
    d = dev()
    for B, W_in, V, W, seed in [(2, 4, 16384, 4, 5), (3, 1, 50272, 6, 6)]:
        _, zd = workloads.make_logits("zipf", B, W_in, V, seed=seed)
        zd = zd.clone()
        keep = zd[B - 1, 0, [7, 4100, 4101]].clone()
        zd[B - 1, 0, :] = -float("inf")
        zd[B - 1, 0, [7, 4100, 4101]] = keep
        rng = np.random.default_rng(seed)
        sigma = (-rng.exponential(3.0, size=(B, W_in))).astype(np.float32)
        gamma = (-np.sort(rng.exponential(1.0, size=(B, W_in)), axis=1)).astype(np.float32)
        n_in = np.full(B, W_in, dtype=np.int32)
        if W_in > 1:
            n_in[0] = 2                                                  # rows 2, 3 of sequence 0 are dead
        g = binding.sbs_step(zd.to(d), torch.from_numpy(sigma).to(d), torch.from_numpy(gamma).to(d),
                             torch.from_numpy(n_in).to(d), W, seed=31, step=1)
        ref = o_sbs.sbs_step(zd.numpy(), sigma, gamma, n_in, W, seed=31, step=1)
        assert np.array_equal(to_np(g["n_out"]), ref["n_out"])
        near = 0
        for b in range(B):
            n = int(ref["n_out"][b])
            if ref["min_gap"][b] < NEAR_TIE:
                near += 1
                continue
            assert np.array_equal(to_np(g["tokens"])[b, :n], ref["tokens"][b, :n])
            assert np.array_equal(to_np(g["parent"])[b, :n], ref["parent"][b, :n])
            assert np.allclose(to_np(g["sum_logprob"])[b, :n], ref["sum_logprob"][b, :n], rtol=1e-6, atol=LOGP_TOL)
            assert np.allclose(to_np(g["trunc_gumbel"])[b, :n], ref["trunc_gumbel"][b, :n], rtol=0, atol=PSI_TOL)
            assert np.all(to_np(g["tokens"])[b, n:] == -1)
            live = int(n_in[b])
            assert np.allclose(to_np(g["lse"])[b, :live], ref["lse"][b, :live], rtol=0, atol=LOGP_TOL)
        assert near <= 1
        if W_in == 1:
            assert int(ref["n_out"][B - 1]) == 3                          # only three finite entries


# ------------------------------------------------------------------ tree building
def test_draft_trees_match_oracle_gumbel_and_sbs():
    say("draft trees (config 0 and a small config-1-like case)")
    d = dev()
    for kind, V, branching, n_cap, seed in (("normal", 64, (2, 2), 7, 0), ("zipf", 32000, (3, 2, 2, 1), 34, 5)):
        _, zd = workloads.make_logits(kind, 2, n_cap, V, seed=seed)
        counts = [workloads.full_tree_child_counts(branching)] * 2
        g = draft_tree.create_draft_tree_const(zd.to(d), counts, seed=seed, step=1)
        for b in range(2):
            ref = oracle_tree_const(zd[b].numpy(), counts[b], b, seed, 1)
            n = len(ref["tokens"])
            assert int(g["n_nodes"][b]) == n
            assert np.array_equal(to_np(g["tokens"])[b, :n], ref["tokens"])
            assert np.array_equal(to_np(g["parent"])[b, :n], ref["parent"])
    _, zd = workloads.make_logits("zipf", 2, 37, 50272, seed=6)
    g = draft_tree.create_draft_tree_sbs(zd.to(d), 6, 6, seed=6, step=0)
    from oracle import draft_tree as o_tree
    for b in range(2):
        ref = o_tree.create_draft_tree_sbs(zd[b].numpy(), 6, 6, seq=b, seed=6, step=0)
        n = len(ref["tokens"])
        assert int(g["n_nodes"][b]) == n == 37
        assert np.array_equal(to_np(g["tokens"])[b, :n], ref["tokens"])
        assert np.array_equal(to_np(g["parent"])[b, :n], ref["parent"])


# --------------------------------------------------------------- tree attention
def _random_tree(rng, n, max_children=4):
    parent = [-1]
    frontier = [0]
    while len(parent) < n:
        nxt = []
        for p in frontier:
            for _ in range(int(rng.integers(0, max_children + 1))):
                if len(parent) < n:
                    parent.append(p); nxt.append(len(parent) - 1)
        frontier = nxt or [len(parent) - 1]
        if not nxt and len(parent) < n:
            parent.append(frontier[0]); frontier = [len(parent) - 1]
    return np.array(parent[:n], dtype=np.int32)


def _attention_case(B, Hq, Hkv, N, D, P, dtype, seed, n_nodes=None, plens=None, splits=0):
    rng = np.random.default_rng(seed)
    q, kp, vp, kt, vt = workloads.make_qkv(B, Hq, Hkv, N, D, max(P, 1), dtype, seed)
    n_nodes = np.full(B, N, dtype=np.int32) if n_nodes is None else np.asarray(n_nodes, dtype=np.int32)
    plens = np.full(B, P, dtype=np.int32) if plens is None else np.asarray(plens, dtype=np.int32)
    parent = np.stack([_random_tree(rng, N) for _ in range(B)])
    d = dev()
    scale = workloads.attention_scale(D)
    out, lse = binding.tree_attention(q.to(d), kp.to(d) if P > 0 else None, vp.to(d) if P > 0 else None,
                                      kt.to(d), vt.to(d), torch.from_numpy(plens).to(d),
                                      torch.from_numpy(n_nodes).to(d), torch.from_numpy(parent).to(d),
                                      scale, num_splits=splits, return_lse=True)
    f = lambda t: t.to(torch.float32).numpy()
    ref, ref_lse = o_attn.tree_attention(f(q), f(kp), f(vp), f(kt), f(vt), plens, n_nodes, parent, scale)
    out, lse = to_np(out), to_np(lse)
    err = 0.0
    for b in range(B):
        n = int(n_nodes[b])
        if n:
            err = max(err, np.abs(out[b, :, :n] - ref[b, :, :n]).max())
            assert np.allclose(lse[b, :, :n], ref_lse[b, :, :n], rtol=0, atol=2e-2 if dtype == "bf16" else 1e-4)
    return err


def test_tree_attention_fp32_config0():
    say("attention fp32 config 0")
    err = _attention_case(1, 1, 1, 7, 64, 32, "f32", 0)
    say(f"  max abs err {err:.2e}")
    assert err < 1e-4
    assert _attention_case(2, 4, 2, 9, 48, 70, "f32", 1, n_nodes=[9, 5], plens=[70, 3]) < 1e-4


@pytest.mark.parametrize("B,Hq,Hkv,N,D,P,splits,n_nodes,plens", [
    (1, 2, 2, 34, 128, 1024, 0, None, None),          # config-1 shape, few heads, auto split
    (2, 4, 2, 37, 128, 200, 1, None, [200, 131]),     # GQA, ragged prefix tail, one split
    (2, 4, 2, 37, 128, 200, 3, [37, 20], [200, 64]),  # forced splits, per-sequence sizes
    (1, 8, 1, 65, 128, 300, 2, None, None),           # 65 nodes: two tree tiles, 520 stacked rows
    (2, 2, 2, 130, 128, 64, 0, [130, 1], None),       # three ancestor words; single-node tree
    (1, 2, 1, 16, 64, 96, 0, None, None),             # head_dim 64
    (1, 2, 2, 20, 128, 0, 0, None, None),             # no prefix at all
    (2, 2, 2, 12, 128, 80, 0, [0, 12], [80, 0]),      # empty tree in one sequence, empty prefix in other
    (2, 8, 2, 40, 128, 200, 0, [40, 17], [200, 77]),  # wide-row variant: 160 stacked rows, ragged blocks
    (1, 16, 2, 65, 128, 257, 3, None, None),          # wide rows, forced splits, 65 nodes
    (1, 8, 1, 24, 64, 130, 0, None, None),            # wide rows with head_dim 64
    (1, 4, 1, 130, 128, 64, 1, None, None),           # wide rows, three ancestor words
    (2, 8, 1, 48, 128, 300, 0, [48, 20], [300, 150]),  # 384 rows: one 256-row block + one 128-row block
    (1, 16, 1, 40, 64, 200, 2, None, None),           # 640 rows, head_dim 64, forced splits
])
def test_tree_attention_bf16(B, Hq, Hkv, N, D, P, splits, n_nodes, plens):
    say(f"attention bf16 B={B} Hq={Hq} Hkv={Hkv} N={N} D={D} P={P} splits={splits}")
    err = _attention_case(B, Hq, Hkv, N, D, P, "bf16", 3, n_nodes=n_nodes, plens=plens, splits=splits)
    say(f"  max abs err {err:.2e}")
    assert err < 1e-2


@pytest.mark.parametrize("L,B,Hq,Hkv,N,D,P,dtype,splits", [
    (5, 1, 4, 4, 34, 128, 300, "bf16", 0),     # config-1-like: one sequence, layers fill the launch
    (3, 2, 8, 1, 65, 128, 200, "bf16", 0),     # stacked heads: 32-row kernel plus remainder rows
    (2, 2, 4, 2, 20, 64, 130, "bf16", 3),      # forced prefix splits: partial results per (layer, sequence)
    (3, 2, 2, 1, 7, 48, 40, "f32", 0),         # fp32 kernel
])
def test_tree_attention_layers_equals_per_layer_oracle(L, B, Hq, Hkv, N, D, P, dtype, splits):
    """One call over L layers that share the tree: every layer's output against the oracle called on
    that layer alone, with ragged trees / prefixes and layer tensors that are strided views."""
    say(f"attention over {L} layers B={B} Hq={Hq} Hkv={Hkv} N={N} D={D} P={P} {dtype} splits={splits}")
    rng = np.random.default_rng(L * 100 + N)
    d = dev()
    cap = P + 8                                        # prefix cache with spare rows: strided layers
    parts = [workloads.make_qkv(B, Hq, Hkv, N, D, cap, dtype, 50 + l) for l in range(L)]
    q, kp, vp, kt, vt = (torch.stack([p[i] for p in parts]) for i in range(5))
    n_nodes = rng.integers(1, N + 1, size=B).astype(np.int32); n_nodes[0] = N
    plens = rng.integers(0, P + 1, size=B).astype(np.int32); plens[0] = P
    parent = np.stack([_random_tree(rng, N) for _ in range(B)])
    scale = workloads.attention_scale(D)
    out, lse = binding.tree_attention_layers(q.to(d), kp.to(d)[:, :, :, :P], vp.to(d)[:, :, :, :P], kt.to(d),
                                             vt.to(d), torch.from_numpy(plens).to(d),
                                             torch.from_numpy(n_nodes).to(d), torch.from_numpy(parent).to(d),
                                             scale, num_splits=splits, return_lse=True)
    out, lse = to_np(out), to_np(lse)
    f = lambda t: t.to(torch.float32).numpy()
    tol, ltol = (1e-2, 2e-2) if dtype == "bf16" else (1e-4, 1e-4)
    worst = 0.0
    for l in range(L):
        ref, ref_lse = o_attn.tree_attention(f(q[l]), f(kp[l][:, :, :P]), f(vp[l][:, :, :P]), f(kt[l]), f(vt[l]),
                                             plens, n_nodes, parent, scale)
        for b in range(B):
            n = int(n_nodes[b])
            worst = max(worst, float(np.abs(out[l, b, :, :n] - ref[b, :, :n]).max()))
            assert np.allclose(lse[l, b, :, :n], ref_lse[b, :, :n], rtol=0, atol=ltol)
    say(f"  max abs err {worst:.2e}")
    assert worst < tol
    # the single-layer call on layer 1 gives the same numbers when the launch plan is the same (forced splits)
    if splits:
        one = binding.tree_attention(q[1].to(d), kp[1].to(d)[:, :, :P], vp[1].to(d)[:, :, :P], kt[1].to(d), vt[1].to(d),
                                     torch.from_numpy(plens).to(d), torch.from_numpy(n_nodes).to(d),
                                     torch.from_numpy(parent).to(d), scale, num_splits=splits)
        for b in range(B):
            n = int(n_nodes[b])
            assert np.array_equal(to_np(one)[b, :, :n], out[1, b, :, :n])


def test_tree_attention_one_key_prefix_wide_rows():
    """A one-key prefix under 272 stacked rows: few visible keys per row, so single keys dominate, and the
    fixed softmax reference of the 32-row kernel (taken from the first tile, here that one key) makes the
    dominant exponential something other than 1.  The row sum has to be the sum of the bf16-rounded
    probabilities that multiply V, or the dominant key's rounding error (2^-8 relative) reaches the output."""
    say("attention bf16, one-key prefix, 16 query heads per KV head")
    err = _attention_case(3, 48, 3, 17, 64, 1, "bf16", 617961752, n_nodes=[17, 3, 3], plens=[1, 1, 1])
    say(f"  max abs err {err:.2e}")
    assert err < 1e-2


@pytest.mark.parametrize("Hq,Hkv", [(8, 1), (2, 2)])
def test_tree_attention_rising_scores(Hq, Hkv):
    """Scores that climb far above those of the first tile (by more than 64 in log2 units).  With eight
    query heads per KV head (320 stacked rows) blocks of the 256-row kernel leave their fixed-reference
    pass and repeat with the running-maximum pass; with one (40 rows) the 16-row kernel, which raises its
    running maximum only past a slack, has to raise it again and again."""
    say(f"attention bf16, scores rising by orders of magnitude along the prefix, {Hq} q / {Hkv} kv heads")
    B, N, D, P = 2, 40, 128, 320
    rng = np.random.default_rng(11)
    q, kp, vp, kt, vt = workloads.make_qkv(B, Hq, Hkv, N, D, P, "bf16", 11)
    kp = kp.to(torch.float32)
    kp[0, :, 128:] *= 40.0           # sequence 0: later keys score ~40x larger; sequence 1 stays ordinary
    kp = kp.to(torch.bfloat16)
    n_nodes = np.full(B, N, dtype=np.int32)
    plens = np.full(B, P, dtype=np.int32)
    parent = np.stack([_random_tree(rng, N) for _ in range(B)])
    d = dev()
    scale = workloads.attention_scale(D)
    out, lse = binding.tree_attention(q.to(d), kp.to(d), vp.to(d), kt.to(d), vt.to(d),
                                      torch.from_numpy(plens).to(d), torch.from_numpy(n_nodes).to(d),
                                      torch.from_numpy(parent).to(d), scale, num_splits=1, return_lse=True)
    f = lambda t: t.to(torch.float32).numpy()
    ref, ref_lse = o_attn.tree_attention(f(q), f(kp), f(vp), f(kt), f(vt), plens, n_nodes, parent, scale)
    span = (ref_lse[0].max() - ref_lse[1].max()) / np.log(2.0)
    say(f"  lse gap between the sequences {span:.0f} (log2 units)")
    assert span > 64
    assert np.abs(to_np(out) - ref).max() < 1e-2
    assert np.allclose(to_np(lse), ref_lse, rtol=2e-3, atol=2e-2)


def test_tree_attention_strided_prefix_and_bad_arguments():
    say("attention strided prefix cache")
    d = dev()
    B, H, N, D, P, cap = 1, 2, 10, 128, 100, 160
    q, kp, vp, kt, vt = workloads.make_qkv(B, H, H, N, D, cap, "bf16", 8)
    parent = torch.tensor([[-1, 0, 0, 1, 1, 2, 3, 3, 5, 8]], dtype=torch.int32)
    args = (torch.tensor([P], dtype=torch.int32, device=d), torch.tensor([N], dtype=torch.int32, device=d),
            parent.to(d), 0.1)
    full = binding.tree_attention(q.to(d), kp.to(d), vp.to(d), kt.to(d), vt.to(d), *args)
    sliced = binding.tree_attention(q.to(d), kp.to(d)[:, :, :P], vp.to(d)[:, :, :P], kt.to(d), vt.to(d), *args)
    assert torch.equal(full, sliced)          # capacity 160, length 100: same result via strides
    with pytest.raises(binding.RsdError) as e:
        binding.tree_attention(q.to(d)[..., :96].contiguous(), None, None, kt.to(d)[..., :96].contiguous(),
                               vt.to(d)[..., :96].contiguous(), *args)
    assert e.value.code == -6
    for bad_scale in (0.0, -0.1, float("inf"), float("nan")):       # row maxima are taken before scaling
        with pytest.raises(binding.RsdError) as e:
            binding.tree_attention(q.to(d), kp.to(d), vp.to(d), kt.to(d), vt.to(d), *args[:3], bad_scale)
        assert e.value.code == -2


# ------------------------------------------------------------- probability filtering
FILTER_TOL = 1e-6   # probability mass: fp32 exponentials and sums on the GPU against the fp64 oracle


def _filter_tol(z_row, ref_row, inv_t):
    """Relative tolerance of one row's decision.  The kernel raises 2 to y = (z - max)/T * log2(e) held
    in fp32, whose spacing at the cut is |y| * 2^-23: one rounding in the scale and one in the fused
    multiply-add move an entry by up to |y| * 2^-22 * ln 2 of its probability, so neighbours closer
    than that cannot be told apart.  Never below FILTER_TOL, which covers the sums."""
    keep = np.isfinite(ref_row)
    if not keep.any():                                                      # a row with no finite logit
        return FILTER_TOL
    y_cut = (float(z_row[keep].min()) - float(z_row[keep].max())) * inv_t * np.log2(np.e)
    return max(FILTER_TOL, abs(y_cut) * 2.0 ** -22 * np.log(2.0))


def _check_filtered(got, z, ref, margin, inv_t, top_k, top_p):
    """Every row: the kept set is a top set, keeps the logits unchanged, and is a valid answer up to the
    row's tolerance (reaches the target, and would fall short without its least probable entries, which
    stay or go together when they are equally probable).  Rows that the oracle decided by a margin above
    the tolerance must match it exactly."""
    near = 0
    for r in range(z.shape[0]):
        kept = np.isfinite(got[r])
        assert np.array_equal(got[r][kept], z[r][kept])
        tol = _filter_tol(z[r], ref[r], inv_t)
        if margin[r] >= tol:
            assert np.array_equal(got[r], ref[r]), r
            continue
        near += 1
        fin = np.isfinite(z[r])
        assert kept.any() and not (kept & ~fin).any()
        assert z[r][kept].min() >= z[r][fin & ~kept].max(initial=-np.inf)         # a top set
        x = z[r].astype(np.float64) * np.float64(np.float32(inv_t))
        prob = np.where(fin, np.exp(x - x[fin].max()), 0.0)
        sizes = [int(fin.sum())]                            # candidate sizes of the set top-p acts on
        if top_k:                                                               # top-k acts first
            srt = np.sort(prob)[::-1]
            kth = srt[min(top_k, int(fin.sum())) - 1]
            in_k = prob >= kth * (1 - tol)
            assert not (kept & ~in_k).any()
            # entries within the tolerance of the k-th may or may not have been taken as tied with it
            sizes = list(range(int((prob >= kth).sum()), int(in_k.sum()) + 1))
        if top_p < 1.0:
            order = np.argsort(-prob, kind="stable")
            ok = False
            for m in sizes:                                 # top-p on the distribution over the top m
                pm = np.zeros_like(prob)
                pm[order[:m]] = prob[order[:m]]
                pm /= pm.sum()
                mass = pm[kept].sum()
                least = pm[kept].min()                      # entries as probable as it stay together
                ok |= (mass >= top_p - tol and
                       mass - pm[kept & (pm <= least * (1 + tol))].sum() < top_p + tol)
            assert ok
    return near


@pytest.mark.parametrize("kind,R,V,inv_t,top_k,top_p", [
    ("zipf", 6, 32000, 1.0, 0, 0.95),        # the instruction-following setting: nucleus 0.95 at T = 1
    ("zipf", 4, 50272, 1.0, 0, 0.95),
    ("zipf", 5, 32000, 1.0 / 0.3, 0, 0.9),   # sharper rows
    ("normal", 7, 1001, 1.0, 50, 1.0),       # top-k only, ragged tail
    ("normal", 5, 1003, 1.0, 40, 0.8),       # both filters
    ("normal", 3, 64, 1.0, 0, 0.5),
    ("zipf", 2, 65536, 1.0, 1000, 0.99),     # largest row
])
def test_filter_logits(kind, R, V, inv_t, top_k, top_p):
    say(f"filter_logits {kind} R={R} V={V} 1/T={inv_t:.2f} top_k={top_k} top_p={top_p}")
    zt, _ = workloads.make_logits(kind, 1, R, V, seed=4)
    z = zt[0].clone()
    z[0, 5:40] = -float("inf")                                    # already-filtered entries stay out
    ld = (V + 3) // 4 * 4
    buf = torch.zeros((R, ld), dtype=torch.float32)
    buf[:, :V] = z
    d_in = buf.to(dev())[:, :V]
    out, kept = binding.filter_logits(d_in, inv_t, top_k, top_p, return_kept=True)
    ref, kept_ref, margin = o_pfilter.filter_logits(z.numpy(), inv_t, top_k, top_p)
    near = _check_filtered(to_np(out), z.numpy(), ref, margin, inv_t, top_k, top_p)
    say(f"  kept per row {kept_ref.tolist()}, rows decided within the tolerance: {near}")
    assert np.array_equal(to_np(kept), np.isfinite(to_np(out)).sum(1))
    ok = margin >= np.array([_filter_tol(z.numpy()[r], ref[r], inv_t) for r in range(R)])
    assert np.array_equal(to_np(kept)[ok], kept_ref[ok])
    assert np.abs(to_np(kept) - kept_ref).max() <= 2
    # in place
    binding.filter_logits(d_in, inv_t, top_k, top_p, out=d_in)
    assert torch.equal(d_in, out)


@pytest.mark.parametrize("V,top_k,top_p", [
    (32000, 0, 0.9),
    (32000, 100, 1.0),
    (4099, 2000, 0.7),        # ragged row, both filters
    (50272, 3000, 0.95),
])
def test_filter_logits_hard_rows(V, top_k, top_p):
    """Rows that stress the threshold search: sorted values (every wave holds one value range), one
    value repeated through the row and coarsely quantised values (tie groups larger than the candidate
    buffer), a dominant peak, a handful of finite entries, none at all."""
    say(f"filter_logits hard rows V={V} top_k={top_k} top_p={top_p}")
    rng = np.random.default_rng(V + top_k)
    base = (rng.standard_normal(V) * 3).astype(np.float32)
    rows = [np.sort(base), np.sort(base)[::-1].copy(), np.full(V, 0.5, np.float32),
            np.round(base * 2) / 2, base.copy(), np.full(V, -np.inf, np.float32), base.copy(),
            np.where(np.arange(V) % 2 == 0, np.float32(1.0), np.float32(-2.0)).astype(np.float32),
            np.full(V, -np.inf, np.float32)]
    rows[4][:] = -np.inf
    rows[4][[3, V // 2, V - 1]] = [0.1, 0.2, 0.1]
    rows[6][V // 3] += 30.0
    rows[8][V - 2] = 7.0                                           # a single finite entry
    z = np.stack(rows).astype(np.float32)
    ld = (V + 3) // 4 * 4
    buf = torch.zeros((z.shape[0], ld), dtype=torch.float32)
    buf[:, :V] = torch.from_numpy(z)
    out, kept = binding.filter_logits(buf.to(dev())[:, :V], 1.0, top_k, top_p, return_kept=True)
    ref, kept_ref, margin = o_pfilter.filter_logits(z, 1.0, top_k, top_p)
    near = _check_filtered(to_np(out), z, ref, margin, 1.0, top_k, top_p)
    say(f"  kept per row {kept_ref.tolist()}, rows decided within the tolerance: {near}")
    assert np.array_equal(to_np(kept), np.isfinite(to_np(out)).sum(1))
    ok = margin >= np.array([_filter_tol(z[r], ref[r], 1.0) for r in range(z.shape[0])])
    assert np.array_equal(to_np(kept)[ok], kept_ref[ok])


@pytest.mark.parametrize("V,top_k,top_p", [
    (32000, 4000, 1.0),       # the k-th entry lies below what fp32 tells apart from zero
    (32000, 31000, 1.0),      # several such bands
    (4099, 4099, 1.0),        # everything finite is kept
    (32000, 4000, 0.999),     # with top-p those entries carry no mass and go
])
def test_filter_logits_wide_rows(V, top_k, top_p):
    """Sharp rows (1/T = 10/3 on logits spread over +-40): the relative probabilities span more than the
    fp32 exponent range, so top-k alone has to rank entries whose fp32 exponential is zero."""
    say(f"filter_logits wide rows V={V} top_k={top_k} top_p={top_p}")
    rng = np.random.default_rng(V + top_k)
    z = (rng.standard_normal((4, V)) * 10).astype(np.float32)
    z[1] = np.sort(z[1])
    z[2, ::7] = -np.inf
    z[3] = np.round(z[3])                                          # ties inside every band
    inv_t = 1.0 / 0.3
    ld = (V + 3) // 4 * 4
    buf = torch.zeros((z.shape[0], ld), dtype=torch.float32)
    buf[:, :V] = torch.from_numpy(z)
    out, kept = binding.filter_logits(buf.to(dev())[:, :V], inv_t, top_k, top_p, return_kept=True)
    ref, kept_ref, margin = o_pfilter.filter_logits(z, inv_t, top_k, top_p)
    near = _check_filtered(to_np(out), z, ref, margin, inv_t, top_k, top_p)
    say(f"  kept per row {kept_ref.tolist()}, rows decided within the tolerance: {near}")
    assert np.array_equal(to_np(kept), np.isfinite(to_np(out)).sum(1))
    ok = margin >= np.array([_filter_tol(z[r], ref[r], inv_t) for r in range(z.shape[0])])
    assert np.array_equal(to_np(kept)[ok], kept_ref[ok])


def test_filtered_logits_through_drafting_and_verification():
    """Nucleus-filtered draft and target logits (p = 0.95, T = 1) through tree drafting and recursive
    rejection sampling: the samplers and the verifier take the -inf entries as they are."""
    say("top-p 0.95 on both models, then draft tree + RRS")
    B, V, counts_shape, n_cap = 3, 32000, (3, 2, 2), 22
    zt, zd = workloads.make_logits("zipf", B, n_cap, V, seed=9)
    ft, _, mt = o_pfilter.filter_logits(zt.reshape(-1, V).numpy(), 1.0, 0, 0.95)
    fd, _, md = o_pfilter.filter_logits(zd.reshape(-1, V).numpy(), 1.0, 0, 0.95)
    d = dev()
    # the GPU filter on the same rows (its own parity is the test above); drafting and verification
    # below take the oracle-filtered rows on both sides, so that one tail entry decided within
    # FILTER_TOL cannot make the two sides work on different distributions
    got_t = to_np(binding.filter_logits(zt.to(d), top_p=0.95)).reshape(-1, V)
    _check_filtered(got_t, zt.reshape(-1, V).numpy(), ft, mt, 1.0, 0, 0.95)
    gt = torch.from_numpy(ft).reshape(B, n_cap, V).to(d)
    gd = torch.from_numpy(fd).reshape(B, n_cap, V).to(d)
    counts = [workloads.full_tree_child_counts(counts_shape)] * B
    tree = draft_tree.create_draft_tree_const(gd, counts, seed=9, step=1)
    for b in range(B):                                             # the tree itself, against the oracle's
        rt = oracle_tree_const(fd.reshape(B, n_cap, V)[b], counts[b], b, 9, 1)
        assert np.array_equal(to_np(tree["tokens"])[b, :n_cap], rt["tokens"])
        assert np.array_equal(to_np(tree["parent"])[b, :n_cap], rt["parent"])
    g = binding.recursive_reject(gd, gt, tree["tokens"], tree["parent"], tree["n_nodes"],
                                 mode=binding.MODE_ALL_GROUPS, seed=9, step=1)
    ref = o_rrs.recursive_reject(ft.reshape(B, n_cap, V), fd.reshape(B, n_cap, V), to_np(tree["tokens"]),
                                 to_np(tree["parent"]), to_np(tree["n_nodes"]), mode=o_rrs.MODE_ALL_GROUPS,
                                 seed=9, step=1)
    near = 0
    for b in range(B):
        if ref["near_tie"][b] or ref["last_gap"][b] < NEAR_TIE:
            near += 1
            continue
        k = int(ref["n_accepted"][b])
        assert int(g["n_accepted"][b]) == k
        assert np.array_equal(to_np(g["accepted_nodes"])[b, :k], ref["accepted_nodes"][b, :k])
        assert int(g["last_token"][b]) == int(ref["last_token"][b])
        assert np.isfinite(ft.reshape(B, n_cap, V)[b, int(ref["final_node"][b]), int(ref["last_token"][b])])
    assert near <= 1


# ------------------------------------------------------------------ FilterKVCache
@pytest.mark.parametrize("dtype,B,H,N,D,cap,L", [
    ("bf16", 3, 4, 12, 128, 40, 5),     # ordinary case, ragged prefix lengths and path lengths
    ("bf16", 2, 2, 9, 64, 12, 6),       # cache nearly full: rows dropped, flag raised
    ("f32", 2, 3, 7, 48, 32, 3),        # fp32 rows of 192 bytes
    ("bf16", 64, 32, 64, 128, 96, 4),   # stress-configuration head count and tree size
])
def test_filter_kv_cache(dtype, B, H, N, D, cap, L):
    say(f"filter_kv_cache {dtype} B={B} H={H} N={N} D={D} capacity={cap} depth={L}")
    rng = np.random.default_rng(5)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator().manual_seed(5)
    kc = torch.randn((B, H, cap + 8, D), generator=g).to(tdt)   # 8 spare rows: capacity < allocation
    vc = torch.randn((B, H, cap + 8, D), generator=g).to(tdt)
    kt = torch.randn((B, H, N, D), generator=g).to(tdt)
    vt = torch.randn((B, H, N, D), generator=g).to(tdt)
    plen = rng.integers(0, cap - 2, size=B).astype(np.int32)
    plen[0] = cap - 3                                            # forces an overflow when the path is long
    n_acc = rng.integers(0, L + 1, size=B).astype(np.int32)
    n_acc[0] = L
    acc = -np.ones((B, L), dtype=np.int32)
    for b in range(B):
        acc[b, :n_acc[b]] = np.sort(rng.choice(np.arange(1, N), size=n_acc[b], replace=False))
    d = dev()
    kc_d, vc_d = kc.to(d), vc.to(d)
    new_len, flags = binding.filter_kv_cache(kc_d[:, :, :cap], vc_d[:, :, :cap], kt.to(d), vt.to(d),
                                             torch.from_numpy(plen).to(d), torch.from_numpy(acc).to(d),
                                             torch.from_numpy(n_acc).to(d))
    f = lambda t: t.to(torch.float32).numpy()
    k_ref, v_ref, len_ref, flag_ref = o_filter.filter_kv_cache(f(kc[:, :, :cap]), f(vc[:, :, :cap]), f(kt), f(vt),
                                                               plen, acc, n_acc)
    assert np.array_equal(to_np(new_len), len_ref)
    assert np.array_equal(to_np(flags), flag_ref)
    assert flag_ref[0] == (1 if plen[0] + 1 + L > cap else 0)
    assert np.array_equal(f(kc_d.cpu())[:, :, :cap], k_ref)      # byte copies: exact
    assert np.array_equal(f(vc_d.cpu())[:, :, :cap], v_ref)
    assert torch.equal(kc_d.cpu()[:, :, cap:], kc[:, :, cap:])   # rows beyond the capacity untouched
    assert torch.equal(vc_d.cpu()[:, :, cap:], vc[:, :, cap:])


# ------------------------------------------------------- recursive rejection sampling
def _rrs_case(kind, B, V, counts, n_cap, seed, inv_t, mode, sbs=None):
    d = dev()
    zt, zd = workloads.make_logits(kind, B, n_cap, V, seed=seed)
    if sbs is None:
        tree = draft_tree.create_draft_tree_const(zd.to(d), counts, seed=seed, step=2, inv_temperature=inv_t)
    else:
        tree = draft_tree.create_draft_tree_sbs(zd.to(d), sbs[0], sbs[1], seed=seed, step=2, inv_temperature=inv_t)
    g = binding.recursive_reject(zd.to(d), zt.to(d), tree["tokens"], tree["parent"], tree["n_nodes"],
                                 inv_temperature=inv_t, mode=mode, seed=seed, step=2)
    ref = o_rrs.recursive_reject(zt.numpy(), zd.numpy(), to_np(tree["tokens"]), to_np(tree["parent"]),
                                 to_np(tree["n_nodes"]), inv_temperature=np.float32(inv_t), mode=mode,
                                 seed=seed, step=2)
    assert np.array_equal(to_np(g["uniforms"]).astype(np.float64)[:, 1:] *
                          (np.arange(1, n_cap)[None] < to_np(tree["n_nodes"])[:, None]),
                          ref["uniforms"][:, 1:] * (np.arange(1, n_cap)[None] < to_np(tree["n_nodes"])[:, None]))
    th_g, th_r = to_np(g["theta"]).astype(np.float64), ref["theta"]
    both = np.isfinite(th_r)
    assert np.array_equal(np.isfinite(th_g), both)
    assert np.allclose(th_g[both], th_r[both], rtol=1e-5, atol=1e-6)
    near = 0
    for b in range(B):
        if ref["near_tie"][b] or ref["last_gap"][b] < NEAR_TIE:
            near += 1
            continue
        k = int(ref["n_accepted"][b])
        assert int(g["n_accepted"][b]) == k
        assert np.array_equal(to_np(g["accepted_nodes"])[b, :k], ref["accepted_nodes"][b, :k])
        assert np.array_equal(to_np(g["accepted_tokens"])[b, :k], ref["accepted_tokens"][b, :k])
        assert np.all(to_np(g["accepted_nodes"])[b, k:] == -1)
        assert int(g["final_node"][b]) == int(ref["final_node"][b])
        assert int(g["last_token"][b]) == int(ref["last_token"][b]), (b, k)
        assert int(g["flags"][b]) == (1 if ref["flags"][b] else 0)
    return near, ref


@pytest.mark.parametrize("mode", [binding.MODE_PATH, binding.MODE_ALL_GROUPS])
@pytest.mark.parametrize("kind,B,V,branching,inv_t", [
    ("normal", 4, 64, (2, 2), 1.0),
    ("zipf", 3, 32000, (3, 2, 2, 1), 1.0),
    ("zipf", 2, 32000, (8, 4, 2), 1.0 / 0.3),
    ("zipf", 2, 50272, (4, 3), 1.0),         # resident variant with the draft row partly in LDS
    ("zipf", 2, 40004, (5, 2), 1.0),         # the same, chunks that end inside a wave
    ("zipf", 2, 65536, (3, 2), 1.0),         # largest row: the streaming variant
])
def test_recursive_reject_matches_oracle(mode, kind, B, V, branching, inv_t):
    say(f"rrs mode={mode} {kind} B={B} V={V} b={branching} invT={inv_t:.2f}")
    counts = [workloads.full_tree_child_counts(branching)] * B
    n_cap = 1 + sum(int(np.prod(branching[:l + 1])) for l in range(len(branching)))
    near, ref = _rrs_case(kind, B, V, counts, n_cap, 11, inv_t, mode)
    say(f"  near-tie sequences: {near} of {B}; accepted lengths {ref['n_accepted'].tolist()}")
    assert near <= 1


@pytest.mark.parametrize("V,inv_t,closeness", [
    (32000, 1.0 / 0.3, 0.1),     # sharp rows, drafter close to the target: residual masses down to ~1e-5
    (32000, 1.0 / 0.3, 1.0),     # sharp rows, the ordinary drafter
    (32000, 1.0, 0.02),          # flat rows and a very close drafter: many entries cancel a little
    (50272, 1.0 / 0.3, 0.1),     # the variant with most of the draft row in LDS
    (4000, 1.0 / 0.3, 0.05),     # small-vocabulary variant
])
def test_recursive_reject_small_residual_mass(V, inv_t, closeness):
    """Stages whose residual mass S_k = sum (q^(k) - p^(k))^+ is a small fraction of what went in:
    the leading digits of q - p cancel at the probable tokens, and the thresholds of the later
    siblings see that error divided by S_k.  Every sibling's threshold of every group (ALL_GROUPS)
    is compared with the oracle at the ordinary tolerance; the oracle's own chain confirms that the
    regime is reached."""
    say(f"rrs small residual mass V={V} invT={inv_t:.2f} draft-target distance x{closeness}")
    d = dev()
    B, branching = 4, (5, 3)
    n_cap = 1 + 5 + 15
    zt, zd = workloads.make_logits("zipf", B, n_cap, V, seed=31)
    zd = (zt + closeness * (zd - zt)).contiguous()
    counts = [workloads.full_tree_child_counts(branching)] * B
    tree = draft_tree.create_draft_tree_const(zd.to(d), counts, seed=31, step=4, inv_temperature=inv_t)
    g = binding.recursive_reject(zd.to(d), zt.to(d), tree["tokens"], tree["parent"], tree["n_nodes"],
                                 inv_temperature=inv_t, mode=binding.MODE_ALL_GROUPS, seed=31, step=4)
    tokens, parent, n_nodes = to_np(tree["tokens"]), to_np(tree["parent"]), to_np(tree["n_nodes"])
    ref = o_rrs.recursive_reject(zt.numpy(), zd.numpy(), tokens, parent, n_nodes,
                                 inv_temperature=np.float32(inv_t), mode=o_rrs.MODE_ALL_GROUPS, seed=31, step=4)
    # how small the residual masses get (oracle arithmetic, per stage, relative to the stage's input)
    smallest = 1.0
    for b in range(B):
        for node in range(int(n_nodes[b])):
            kids = o_rrs.children_of(parent[b], n_nodes[b], node)
            if len(kids) < 2:
                continue
            q = o_rrs.softmax_row(zt[b, node].numpy(), np.float32(inv_t))
            p = o_rrs.softmax_row(zd[b, node].numpy(), np.float32(inv_t))
            for x in tokens[b, kids[:-1]]:
                mass = np.maximum(q - p, 0.0).sum()
                smallest = min(smallest, float(mass))
                _, res, _ = o_rrs.sibling_chain(q, p, [x])
                q = res[1]
                p = p.copy(); p[x] = 0.0; p /= p.sum()
    th_g, th_r = to_np(g["theta"]).astype(np.float64), ref["theta"]
    both = np.isfinite(th_r)
    assert np.array_equal(np.isfinite(th_g), both)
    err = np.abs(th_g[both] - th_r[both]) / (1e-6 + 1e-5 * np.abs(th_r[both]))
    say(f"  smallest stage residual mass {smallest:.2e}; worst threshold error {err.max():.2f} of the tolerance")
    if closeness <= 0.1:
        assert smallest < 1e-2
    assert np.allclose(th_g[both], th_r[both], rtol=1e-5, atol=1e-6)
    near = 0
    for b in range(B):
        if ref["near_tie"][b] or ref["last_gap"][b] < NEAR_TIE:
            near += 1
            continue
        k = int(ref["n_accepted"][b])
        assert int(g["n_accepted"][b]) == k
        assert np.array_equal(to_np(g["accepted_nodes"])[b, :k], ref["accepted_nodes"][b, :k])
        assert int(g["final_node"][b]) == int(ref["final_node"][b])
        assert int(g["last_token"][b]) == int(ref["last_token"][b]), (b, k)
    assert near <= 1


def test_recursive_reject_on_sbs_tree_and_ragged_subtrees():
    say("rrs on an SBS tree (interleaved parents) and random subtrees")
    near, ref = _rrs_case("zipf", 3, 32000, None, 37, 13, 1.0, binding.MODE_ALL_GROUPS, sbs=(6, 6))
    assert near <= 1
    counts = [workloads.random_subtree_child_counts((8, 4, 2), 40, s) for s in range(3)]
    near, ref = _rrs_case("zipf", 3, 32000, counts, 40, 14, 1.0, binding.MODE_PATH)
    assert near <= 1


def test_recursive_reject_identical_models_and_single_node():
    say("rrs identical models / root only")
    d = dev()
    zt, _ = workloads.make_logits("zipf", 2, 5, 4000, seed=15)
    tokens = torch.tensor([[-1, 7, 9, 11, 13], [-1, 0, 0, 0, 0]], dtype=torch.int32, device=d)
    parent = torch.tensor([[-1, 0, 1, 2, 3], [-1, -1, -1, -1, -1]], dtype=torch.int32, device=d)
    n_nodes = torch.tensor([5, 1], dtype=torch.int32, device=d)
    g = binding.recursive_reject(zt.to(d), zt.to(d), tokens, parent, n_nodes, seed=1)
    ref = o_rrs.recursive_reject(zt.numpy(), zt.numpy(), to_np(tokens), to_np(parent), to_np(n_nodes), seed=1)
    assert to_np(g["n_accepted"]).tolist() == [4, 0] == ref["n_accepted"].tolist()
    assert to_np(g["last_token"]).tolist() == ref["last_token"].tolist()
    assert to_np(g["final_node"]).tolist() == [4, 0]


# ------------------------------------------------------------------ limits, degenerate inputs
@pytest.mark.parametrize("mode", [binding.MODE_PATH, binding.MODE_ALL_GROUPS])
def test_recursive_reject_at_the_limits(mode):
    """Sixteen siblings under one parent (the largest group), and a 256-node chain (the largest tree,
    255 levels deep)."""
    say(f"rrs limits mode={mode}")
    near, ref = _rrs_case("zipf", 2, 32000, [workloads.full_tree_child_counts((16,))] * 2, 17, 21, 1.0, mode)
    assert near <= 1
    d = dev()
    B, N, V = 2, 256, 64
    zt, zd = workloads.make_logits("normal", B, N, V, seed=22)
    rng = np.random.default_rng(22)
    tokens = torch.from_numpy(rng.integers(0, V, size=(B, N)).astype(np.int32))
    parent = torch.arange(-1, N - 1, dtype=torch.int32)[None].repeat(B, 1)
    n_nodes = torch.tensor([N, 100], dtype=torch.int32)
    # a target close to the draft, so that the walk goes deep into the chain
    zt = zd + 0.05 * (zt - zd)
    g = binding.recursive_reject(zd.to(d), zt.to(d), tokens.to(d), parent.to(d), n_nodes.to(d), mode=mode, seed=3)
    ref = o_rrs.recursive_reject(zt.numpy(), zd.numpy(), tokens.numpy(), parent.numpy(), n_nodes.numpy(),
                                 mode=mode, seed=3)
    say(f"  chain: accepted {ref['n_accepted'].tolist()}")
    skipped = 0
    for b in range(B):
        if ref["near_tie"][b] or ref["last_gap"][b] < NEAR_TIE:
            skipped += 1
            continue
        k = int(ref["n_accepted"][b])
        assert int(g["n_accepted"][b]) == k
        assert np.array_equal(to_np(g["accepted_nodes"])[b, :k], ref["accepted_nodes"][b, :k])
        assert int(g["last_token"][b]) == int(ref["last_token"][b])
    assert skipped == 0           # (fixed seeds: no close call on either chain)
    assert max(ref["n_accepted"]) >= 8


def test_recursive_reject_many_nodes_plan_in_global_memory():
    """B * N_max above 8192: the planning kernel keeps its child counts in global memory instead of LDS.
    40 sequences of up to 256 nodes (random trees of ragged size), small vocabulary, ALL_GROUPS."""
    say("rrs with B * N_max = 10240 (> 8192 nodes)")
    d = dev()
    B, N, V = 40, 256, 256
    rng = np.random.default_rng(77)
    zt, zd = workloads.make_logits("normal", B, N, V, seed=77)
    n_nodes = rng.integers(2, N + 1, size=B).astype(np.int32)
    n_nodes[0] = N
    parent = np.stack([_random_tree(rng, N, max_children=3) for _ in range(B)])
    tokens = np.zeros((B, N), dtype=np.int32)
    for b in range(B):                       # siblings carry distinct tokens (drawn without replacement)
        for node in range(N):
            kids = np.nonzero(parent[b] == node)[0]
            tokens[b, kids] = rng.choice(V, size=len(kids), replace=False)
    g = binding.recursive_reject(zd.to(d), zt.to(d), torch.from_numpy(tokens).to(d), torch.from_numpy(parent).to(d),
                                 torch.from_numpy(n_nodes).to(d), mode=binding.MODE_ALL_GROUPS, seed=5, step=1)
    ref = o_rrs.recursive_reject(zt.numpy(), zd.numpy(), tokens, parent, n_nodes, mode=o_rrs.MODE_ALL_GROUPS,
                                 seed=5, step=1)
    th_g, th_r = to_np(g["theta"]).astype(np.float64), ref["theta"]
    both = np.isfinite(th_r)
    assert np.array_equal(np.isfinite(th_g), both)       # NaN everywhere else (root, padding, unverified)
    assert np.allclose(th_g[both], th_r[both], rtol=1e-5, atol=1e-6)
    near = 0
    for b in range(B):
        if ref["near_tie"][b] or ref["last_gap"][b] < NEAR_TIE:
            near += 1
            continue
        k = int(ref["n_accepted"][b])
        assert int(g["n_accepted"][b]) == k
        assert np.array_equal(to_np(g["accepted_nodes"])[b, :k], ref["accepted_nodes"][b, :k])
        assert int(g["last_token"][b]) == int(ref["last_token"][b])
    assert near <= 2


@pytest.mark.parametrize("V,B,inv_t", [
    (4096, 120, 1.0),          # 256 threads, rows in registers
    (32000, 110, 1.0 / 0.7),   # 512 threads, rows in registers
    (50272, 100, 1.0),         # 512 threads, draft row partly in LDS
    (65536, 100, 1.0),         # streaming variant
])
def test_recursive_reject_several_groups_per_workgroup(V, B, inv_t):
    """More sibling groups than the chip has compute units, so that every persistent workgroup of
    the ALL_GROUPS pass takes several items off the work queue and the hand-over between items
    (rows of the next group requested while the current one is verified) is exercised, in every
    vocabulary-size variant.  Random ragged subtrees of the (3, 2, 2) tree: about 7 groups a sequence."""
    counts = [workloads.random_subtree_child_counts((3, 2, 2), 14, 900 + b) for b in range(B)]
    groups = sum(1 for c in counts for level in c for k in level if k > 0)
    say(f"rrs with {groups} groups at V = {V}")
    assert groups > 2 * 256
    near, _ = _rrs_case("zipf", B, V, counts, 14, 31 + V % 97, inv_t, binding.MODE_ALL_GROUPS)
    say(f"  near ties {near}")
    assert near <= max(3, B // 20)


def test_tree_attention_largest_tree():
    say("attention bf16 with 256 nodes (four ancestor words, four tree tiles)")
    err = _attention_case(1, 2, 1, 256, 128, 70, "bf16", 5, n_nodes=[256], plens=[70])
    say(f"  max abs err {err:.2e}")
    assert err < 1e-2
    err = _attention_case(2, 2, 2, 256, 64, 0, "bf16", 6, n_nodes=[256, 200], plens=[0, 0])
    assert err < 1e-2


def test_non_finite_logits_are_flagged_not_fatal():
    say("rrs with a NaN in a target row")
    d = dev()
    zt, zd = workloads.make_logits("normal", 2, 7, 64, seed=23)
    counts = [workloads.full_tree_child_counts((2, 2))] * 2
    tree = draft_tree.create_draft_tree_const(zd.to(d), counts, seed=23, step=0)
    zt[1, 0, 5] = float("nan")
    for mode in (binding.MODE_PATH, binding.MODE_ALL_GROUPS):
        g = binding.recursive_reject(zd.to(d), zt.to(d), tree["tokens"], tree["parent"], tree["n_nodes"],
                                     mode=mode, seed=23)
        torch.cuda.synchronize()
        flags = to_np(g["flags"])
        assert flags[0] == 0 and flags[1] & binding.FLAG_NONFINITE
        assert 0 <= int(g["n_accepted"][1]) <= 2 and -1 <= int(g["last_token"][1]) < 64


# ------------------------------------------------------------------ baseline verifiers (Sec. 2)
@pytest.mark.parametrize("method,gamma", [(binding.BASELINE_KSEQ, 4.0), (binding.BASELINE_KSEQ, 1.0),
                                          (binding.BASELINE_MULTIROUND, 1.0)])
@pytest.mark.parametrize("kind,R,V,K,inv_t", [("normal", 6, 64, 3, 1.0), ("zipf", 5, 32000, 4, 1.0),
                                               ("zipf", 4, 50257, 4, 1.0 / 0.3), ("zipf", 3, 1001, 8, 1.0)])
def test_baseline_verifiers_match_oracle(method, gamma, kind, R, V, K, inv_t):
    """K-SEQ and multi-round rejection sampling on i.i.d. drafts (K independent Gumbel-max draws from the
    draft row): thresholds, accepted draft and emitted token against the oracle."""
    say(f"baseline verify method={method} gamma={gamma} {kind} R={R} V={V} K={K}")
    d = dev()
    zt, zd = workloads.make_logits(kind, 1, R, V, seed=17)
    zt, zd = zt[0], zd[0]
    if method == binding.BASELINE_KSEQ and gamma > K:
        gamma = float(K)
    ld = (V + 3) // 4 * 4
    bt = torch.zeros((R, ld), dtype=torch.float32); bd = torch.zeros((R, ld), dtype=torch.float32)
    bt[:, :V], bd[:, :V] = zt, zd
    gt, gd = bt.to(d)[:, :V], bd.to(d)[:, :V]
    # K i.i.d. draws from the draft distribution: one Gumbel-max sample per (row, k), each on its own noise
    cols = []
    for k in range(K):
        node = torch.arange(R, dtype=torch.int32, device=d) + 1000 * (k + 1)
        cols.append(binding.gumbel_topk(gd, 1, inv_temperature=inv_t, node_id=node, seed=17, step=5,
                                        want_scores=False)["tokens"])
    drafts = torch.cat(cols, dim=1).contiguous()
    seq = torch.arange(R, dtype=torch.int32, device=d) % 3
    g = binding.baseline_verify(gd, gt, drafts, method, gamma=gamma, inv_temperature=inv_t, seq_id=seq, seed=17, step=5)
    ref = o_base.verify(zt.numpy(), zd.numpy(), to_np(drafts), method, gamma=gamma, inv_temperature=np.float32(inv_t),
                        seq_id=to_np(seq), seed=17, step=5)
    assert np.allclose(to_np(g["theta"]), ref["theta"], rtol=1e-5, atol=1e-6)
    near = 0
    for r in range(R):
        if ref["near_tie"][r] or ref["last_gap"][r] < NEAR_TIE:
            near += 1
            continue
        assert int(g["accepted"][r]) == int(ref["accepted"][r])
        assert int(g["token"][r]) == int(ref["token"][r]), r
        if method == binding.BASELINE_MULTIROUND or gamma >= K:
            assert int(g["flags"][r]) == (1 if ref["flags"][r] else 0)
    say(f"  accepted {ref['accepted'].tolist()}, near ties {near}")
    assert near <= 1


def test_baseline_verifiers_identical_models_and_bad_arguments():
    say("baseline verify: identical models, argument errors")
    d = dev()
    zt, _ = workloads.make_logits("zipf", 1, 3, 4000, seed=19)
    z = zt[0].to(d)
    drafts = torch.tensor([[5, 5, 9], [1, 2, 3], [7, 7, 7]], dtype=torch.int32, device=d)
    for method in (binding.BASELINE_KSEQ, binding.BASELINE_MULTIROUND):
        g = binding.baseline_verify(z, z, drafts, method, gamma=1.0, seed=2)
        # p = q: the first draft is accepted with certainty (gamma = 1)
        assert to_np(g["accepted"]).tolist() == [0, 0, 0]
        assert to_np(g["token"]).tolist() == [5, 1, 7]
        assert np.all(to_np(g["theta"])[:, 0] == 1.0)
    with pytest.raises(binding.RsdError) as e:
        binding.baseline_verify(z, z, drafts, binding.BASELINE_KSEQ, gamma=5.0)      # gamma > K
    assert e.value.code == -2
    with pytest.raises(binding.RsdError) as e:
        binding.baseline_verify(z, z, drafts, 7)
    assert e.value.code == -6
