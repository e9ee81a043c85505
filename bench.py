#!/usr/bin/env python3
"""Benchmark of the RSD draft-tree hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that
is already resident in HBM: drafting (Gumbel-Top-k per tree level, or the
Stochastic Beam Search steps), one layer of tree-masked attention, and recursive
rejection sampling.  The headline value is the metric's own definition,
tree nodes / (t_attention_one_layer + t_rrs); the figure over the whole step
(drafting included) is reported beside it as value_full_step, and ms_per_step is
the whole step.

Prints ONE JSON line.  Default workload: the largest single-GPU configuration
("cfg4_stress"); the other configurations are timed briefly and listed under
"per_config".
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch of the dominant kernel come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# scaled by the same counters over plain device copies.  The figure is not kept here: it is read
# from the committed summary of those runs (a line "traffic_bytes_per_launch: <number>"), which also
# names the kernel source it was taken on; a summary taken on another kernel source gives null.
TRAFFIC_SUMMARY = {"cfg4_stress": os.path.join(ROOT, "profiles", "cfg4_stress_attention_traffic.md")}
ATTENTION_SOURCE = os.path.join(ROOT, "paper_2402_14160_amd", "csrc", "tree_attention.hip")


def measured_traffic(name):
    """(bytes per launch, provenance) from the committed counter summary, or (None, reason)."""
    import hashlib
    import re
    path = TRAFFIC_SUMMARY.get(name)
    if not path or not os.path.exists(path):
        return None, "no counter summary committed for this workload"
    text = open(path).read()
    m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text)
    h = re.search(r"kernel_source_sha256_16:\s*([0-9a-f]{16})", text)
    if not m or not h:
        return None, "counter summary has no machine-readable figure"
    now = hashlib.sha256(open(ATTENTION_SOURCE, "rb").read()).hexdigest()[:16]
    if h.group(1) != now:
        return None, f"counter summary was taken on kernel source {h.group(1)}, this build is {now}"
    return float(m.group(1)), os.path.relpath(path, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
# plain vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second (half the
# published 157.3 TFLOP/s fp32 vector figure counts an FMA as two flops and packs two per lane)
VALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
# vector instructions the tokens-only Gumbel-Top-k kernel issues per vocabulary entry: rocprofv3
# SQ_INSTS_VALU x 64 lanes / entries over the three level launches of the stress configuration
# (profiles/cfg4_stress_gumbel_topk_counters.md, which also gives the measured busy fraction of the
# vector ALUs, SQ_ACTIVE_INST_VALU against SQ_BUSY_CYCLES: the rate the pipeline really runs at)
GUMBEL_VALU_PER_ENTRY = 31.0
N_LAYERS = {"cfg1_llama2_7b": 32, "cfg2_opt_13b_sbs": 40, "cfg3_llama2_70b_gqa": 80, "cfg4_stress": 32}
# draft size / target size of the model pairs the shapes stand for (App. C: a 115M drafter for the
# Llama 2 targets, OPT-125M for OPT-13B): the relative draft cost r of the memory-bound speed-up
DRAFT_TO_TARGET = {"cfg1_llama2_7b": 0.115 / 7.0, "cfg2_opt_13b_sbs": 0.125 / 13.0,
                   "cfg3_llama2_70b_gqa": 0.115 / 70.0, "cfg4_stress": 0.115 / 7.0}


def build_case(cfg, seed, torch, binding, draft_tree, workloads):
    """Generate inputs on the GPU, grow the trees with the HIP samplers, and return the
    resident tensors plus the three phase closures."""
    dev = torch.device("cuda:0")
    B, N, V = cfg["B"], cfg["N"], cfg["V"]
    zt, zd = workloads.make_logits(cfg["logits"], B, N, V, seed, device=dev)
    q, kp, vp, kt, vt = workloads.make_qkv(B, cfg["Hq"], cfg["Hkv"], N, cfg["D"], cfg["P"],
                                           cfg["dtype"], seed + 1, device=dev)
    plen = torch.full((B,), cfg["P"], dtype=torch.int32, device=dev)
    scale = workloads.attention_scale(cfg["D"])
    case = dict(cfg=cfg, zt=zt, zd=zd, q=q, kp=kp, vp=vp, kt=kt, vt=vt, plen=plen, scale=scale)

    if cfg["sampler"] == "gumbel":
        counts = workloads.tree_child_counts(cfg, seed)
        tree = draft_tree.create_draft_tree_const(zd, counts, seed=seed, step=0)
        # resident per-level row matrices, as a draft model would hand them over
        levels = []
        depth = max(len(c) for c in counts)
        for level in range(depth):
            rb, rn, ks = [], [], []
            for b in range(B):
                lo_hi = tree["level_off"][b]
                if level >= len(counts[b]) or level + 1 >= len(lo_hi):
                    continue
                lo, hi = lo_hi[level], lo_hi[level + 1]
                for i in range(lo, hi):
                    if counts[b][level][i - lo] > 0:
                        rb.append(b); rn.append(i); ks.append(counts[b][level][i - lo])
            if not ks:
                continue
            rows = zd[torch.tensor(rb, device=dev), torch.tensor(rn, device=dev)].contiguous()
            levels.append(dict(rows=rows, k_max=max(ks),
                               k=torch.tensor(ks, dtype=torch.int32, device=dev),
                               seq=torch.tensor(rb, dtype=torch.int32, device=dev),
                               node=torch.tensor(rn, dtype=torch.int32, device=dev)))
        case["draft_rows"] = sum(l["rows"].shape[0] for l in levels)

        def draft():
            for l in levels:
                binding.gumbel_topk(l["rows"], l["k_max"], k_per_row=l["k"], seq_id=l["seq"],
                                    node_id=l["node"], seed=seed, step=0, want_scores=False)
    else:
        W, L = cfg["width"], cfg["depth"]
        tree = draft_tree.create_draft_tree_sbs(zd, W, L, seed=seed, step=0)
        levels = []
        for level in range(L):
            w_in = 1 if level == 0 else W
            lo = 0 if level == 0 else 1 + (level - 1) * W
            rows = zd[:, lo:lo + w_in].contiguous()
            node = (lo + torch.arange(w_in, device=dev, dtype=torch.int32))[None].expand(B, w_in).contiguous()
            levels.append(dict(rows=rows, node=node,
                               sigma=torch.zeros((B, w_in), dtype=torch.float32, device=dev),
                               gamma=torch.zeros((B, w_in), dtype=torch.float32, device=dev),
                               n_in=torch.full((B,), w_in, dtype=torch.int32, device=dev)))
        case["draft_rows"] = sum(l["rows"].shape[0] * l["rows"].shape[1] for l in levels)

        def draft():
            sigma, gamma = levels[0]["sigma"], levels[0]["gamma"]
            for l in levels:
                out = binding.sbs_step(l["rows"], sigma, gamma, l["n_in"], W, node_id=l["node"],
                                       seed=seed, step=0)
                sigma, gamma = out["sum_logprob"], out["trunc_gumbel"]

    case["tree"] = tree
    attn_out = torch.empty((B, cfg["Hq"], N, cfg["D"]), dtype=torch.float32, device=dev)
    mode = binding.MODE_ALL_GROUPS

    def attn():
        binding.tree_attention(q, kp, vp, kt, vt, plen, tree["n_nodes"], tree["parent"], scale, out=attn_out)

    def rrs():
        return binding.recursive_reject(zd, zt, tree["tokens"], tree["parent"], tree["n_nodes"],
                                        mode=mode, seed=seed, step=0, diagnostics=False)

    case.update(draft=draft, attn=attn, rrs=rrs, attn_out=attn_out)
    return case


def algorithmic_figures(case):
    """Bytes / flops that one step has to move / do at the least."""
    cfg, tree = case["cfg"], case["tree"]
    B, V, D, P = cfg["B"], cfg["V"], cfg["D"], cfg["P"]
    esz = 2 if cfg["dtype"] == "bf16" else 4
    n_nodes = tree["n_nodes"].cpu().tolist()
    parent = tree["parent"].cpu()
    attn_bytes = attn_flops = 0
    groups = 0
    for b in range(B):
        n = n_nodes[b]
        attn_bytes += 2 * (P + n) * cfg["Hkv"] * D * esz + cfg["Hq"] * n * D * (esz + 4)
        attn_flops += 4 * n * (P + n) * D * cfg["Hq"]
        groups += len(set(parent[b, 1:n].tolist()))
    # every sibling group reads its draft row and its target row once; the last token reads
    # one more row pair per sequence
    rrs_bytes = (groups + B) * 2 * V * 4
    draft_bytes = case["draft_rows"] * V * 4
    return dict(attn_bytes=attn_bytes, attn_flops=attn_flops, rrs_bytes=rrs_bytes,
                draft_bytes=draft_bytes, nodes=sum(n_nodes), groups=groups)


def time_case(case, steps, warmup, torch):
    ev = lambda: torch.cuda.Event(enable_timing=True)
    for _ in range(warmup):
        case["draft"](); case["attn"](); case["rrs"]()
    torch.cuda.synchronize()
    marks = [[ev() for _ in range(4)] for _ in range(steps)]
    t0 = time.perf_counter()
    for s in range(steps):
        marks[s][0].record()
        case["draft"]()
        marks[s][1].record()
        case["attn"]()
        marks[s][2].record()
        case["rrs"]()
        marks[s][3].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    phase = [sum(m[i].elapsed_time(m[i + 1]) for m in marks) / steps for i in range(3)]
    return dict(ms_per_step=wall * 1000.0 / steps, draft_ms=phase[0], attn_ms=phase[1], rrs_ms=phase[2])


def graph_step_ms(case, torch, steps=20):
    """The same step captured once into a HIP graph and replayed: what the GPU needs for it without the
    host's per-call launch work (the difference matters for the small, latency-bound configurations)."""
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        case["draft"](); case["attn"](); case["rrs"]()
    for _ in range(2):
        graph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    del graph
    return e0.elapsed_time(e1) / steps


def report(case, t):
    fig = algorithmic_figures(case)
    cfg = case["cfg"]
    attn_s, rrs_s, draft_s = t["attn_ms"] / 1e3, t["rrs_ms"] / 1e3, t["draft_ms"] / 1e3
    intensity = fig["attn_flops"] / fig["attn_bytes"]
    ridge = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    out = dict(
        workload=cfg["name"], nodes=fig["nodes"], ms_per_step=round(t["ms_per_step"], 4),
        nodes_per_s_full_step=fig["nodes"] / (t["ms_per_step"] / 1e3),
        nodes_per_s_attn_rrs=fig["nodes"] / (attn_s + rrs_s),
        draft_ms=round(t["draft_ms"], 4), attn_ms=round(t["attn_ms"], 4), rrs_ms=round(t["rrs_ms"], 4),
        attn_GBps=fig["attn_bytes"] / attn_s / 1e9, attn_TFLOPs=fig["attn_flops"] / attn_s / 1e12,
        attn_frac_hbm=fig["attn_bytes"] / attn_s / 1e9 / HBM_PEAK_GBS,
        attn_frac_mfma=fig["attn_flops"] / attn_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        attn_bound="mfma" if intensity > ridge else "hbm",
        rrs_GBps=fig["rrs_bytes"] / rrs_s / 1e9, rrs_frac_hbm=fig["rrs_bytes"] / rrs_s / 1e9 / HBM_PEAK_GBS,
        draft_alu_frac=(fig["draft_bytes"] / 4 * GUMBEL_VALU_PER_ENTRY / draft_s / VALU_PEAK_LANE_OPS
                        if draft_s > 0 and cfg["sampler"] == "gumbel" else None),
        draft_GBps=fig["draft_bytes"] / draft_s / 1e9 if draft_s > 0 else None,
        draft_frac_hbm=fig["draft_bytes"] / draft_s / 1e9 / HBM_PEAK_GBS if draft_s > 0 else None,
    )
    return out, fig


def model_step(rep, fig, layers):
    """Tree nodes per second of a whole-model verification step: all layers' tree attention (measured
    in one multi-layer call; scaled from the measured layers when the model's K/V does not fit the
    memory budget of the benchmark) plus one recursive rejection sampling call."""
    if not layers:
        return {}
    scale = layers["layers_of_model"] / layers["layers"]
    t = layers["layers_ms"] * scale / 1e3 + rep["rrs_ms"] / 1e3
    return dict(model_step_nodes_per_s=fig["nodes"] / t,
                model_step_layers_measured=layers["layers"], model_step_layers_of_model=layers["layers_of_model"])


def cpu_baseline(case, fig, torch, budget_s=12.0):
    """The oracle, as it stands, on a bounded sample of the same workload: whole sequences
    (drafting of their non-leaf rows, tree attention of a few KV heads scaled to all heads,
    recursive rejection sampling over all groups) until about `budget_s` seconds of CPU work."""
    import numpy as np

    from oracle import gumbel_topk as o_topk
    from oracle import rrs as o_rrs
    from oracle import sbs as o_sbs
    from oracle import tree_attention as o_attn
    cfg, tree = case["cfg"], case["tree"]
    B = cfg["B"]
    heads = min(16, cfg["Hkv"])
    group = cfg["Hq"] // cfg["Hkv"]
    f = lambda t: t.to(torch.float32).cpu().numpy()
    nodes, scaled, spent, used = 0, 0.0, 0.0, 0
    for b in range(B):
        n = int(tree["n_nodes"][b])
        q = f(case["q"][b:b + 1, :heads * group]); kp = f(case["kp"][b:b + 1, :heads]); vp = f(case["vp"][b:b + 1, :heads])
        kt = f(case["kt"][b:b + 1, :heads]); vt = f(case["vt"][b:b + 1, :heads])
        parent = tree["parent"][b:b + 1].cpu().numpy(); tokens = tree["tokens"][b:b + 1].cpu().numpy()
        zt = case["zt"][b:b + 1].cpu().numpy(); zd = case["zd"][b:b + 1].cpu().numpy()
        t0 = time.perf_counter()
        o_attn.tree_attention(q, kp, vp, kt, vt, [cfg["P"]], [n], parent, case["scale"])
        t_attn = time.perf_counter() - t0
        t0 = time.perf_counter()
        o_rrs.recursive_reject(zt, zd, tokens, parent, [n], mode=o_rrs.MODE_ALL_GROUPS, seq_id=[b], seed=0, step=0)
        nonleaf = sorted(set(parent[0, 1:n].tolist()))
        if cfg["sampler"] == "gumbel":
            o_topk.gumbel_topk(zd[0, nonleaf], 2, seq_id=np.full(len(nonleaf), b), node_id=np.array(nonleaf), seed=0)
        else:
            for lo in range(0, len(nonleaf), cfg["width"]):
                rows = nonleaf[lo:lo + cfg["width"]]
                o_sbs.sbs_step(zd[:, rows], np.zeros((1, len(rows))), np.zeros((1, len(rows))), [len(rows)],
                               cfg["width"], seed=0)
        t_rest = time.perf_counter() - t0
        nodes += n
        used += 1
        spent += t_attn + t_rest
        scaled += t_attn * cfg["Hkv"] / heads + t_rest
        if spent >= budget_s:
            break
    try:
        import threadpoolctl
        threads = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    return dict(value=nodes / scaled, unit="tree nodes/s", cores=threads, kind="oracle",
                sample=(f"{used} of {B} sequences: drafting of their non-leaf rows, tree attention of {heads} of "
                        f"{cfg['Hkv']} KV heads (time scaled to all heads), recursive rejection sampling over all "
                        f"groups; {spent:.1f} s of CPU work"),
                seconds_per_sequence=scaled / used)


def calibrate_copy(torch, gib=1, repeats=10):
    """Plain device-to-device copies of known size: the reference that the FETCH_SIZE / WRITE_SIZE
    counters of a profiler run are scaled by."""
    dev = torch.device("cuda:0")
    n = gib << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(repeats):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps(dict(calibration="device copy", bytes_read=n, bytes_written=n, repeats=repeats)))


def vocab_pass(case, torch, binding, steps=10):
    """The plain log-softmax normaliser over every target row: the pure HBM-bound vocabulary pass."""
    zt = case["zt"]
    B, N, V = zt.shape
    rows = zt.view(B * N, V)
    for _ in range(2):
        binding.log_softmax_lse(rows)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        binding.log_softmax_lse(rows)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    gbs = rows.numel() * 4 / ms / 1e6
    return dict(lse_ms=round(ms, 4), lse_GBps=gbs, lse_frac_hbm=gbs / HBM_PEAK_GBS)


def layers_pass(case, torch, binding, workloads, steps=5, mem_budget=48 << 30):
    """Tree attention of ALL layers of the model the shape stands for in one call
    (rsd_tree_attention_layers: the layers share the tree, its mask and the launch plan), on
    distinct K/V buffers per layer, so nothing is served from the on-package cache.  Also times the
    single-layer call rotated over those buffers (the cold figure of the one-layer call)."""
    cfg, tree = case["cfg"], case["tree"]
    if cfg["name"] not in N_LAYERS or cfg["dtype"] != "bf16":
        return {}
    dev = case["q"].device
    B, Hq, Hkv, N, D, P = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["N"], cfg["D"], cfg["P"]
    per_layer = 2 * B * Hkv * (P + N) * D * 2
    want = N_LAYERS[cfg["name"]]
    L = max(1, min(want, mem_budget // per_layer))
    q = torch.empty((L, B, Hq, N, D), dtype=torch.bfloat16, device=dev)
    kp = torch.empty((L, B, Hkv, P, D), dtype=torch.bfloat16, device=dev)
    vp = torch.empty_like(kp)
    kt = torch.empty((L, B, Hkv, N, D), dtype=torch.bfloat16, device=dev)
    vt = torch.empty_like(kt)
    for l in range(L):
        ql, kpl, vpl, ktl, vtl = workloads.make_qkv(B, Hq, Hkv, N, D, P, "bf16", 1000 + l, device=dev)
        q[l], kp[l], vp[l], kt[l], vt[l] = ql, kpl, vpl, ktl, vtl
        del ql, kpl, vpl, ktl, vtl
    out = torch.empty((L, B, Hq, N, D), dtype=torch.float32, device=dev)
    nn, par, plen, scale = tree["n_nodes"], tree["parent"], case["plen"], case["scale"]
    run = lambda: binding.tree_attention_layers(q, kp, vp, kt, vt, plen, nn, par, scale, out=out)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    run()
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    # one-layer call on a different layer's buffers every time (cold) ...
    one = lambda l: binding.tree_attention(q[l], kp[l], vp[l], kt[l], vt[l], plen, nn, par, scale, out=out[l])
    one(0)
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    reps = max(L, 8)
    e0.record()
    for i in range(reps):
        one(i % L)
    e1.record()
    torch.cuda.synchronize()
    cold_ms = e0.elapsed_time(e1) / reps
    fig = algorithmic_figures(case)
    res = dict(layers=L, layers_of_model=want, layers_ms=round(ms, 4), ms_per_layer=round(ms / L, 5),
               layers_GBps=fig["attn_bytes"] * L / ms / 1e6, layers_TFLOPs=fig["attn_flops"] * L / ms / 1e9,
               layers_frac_hbm=fig["attn_bytes"] * L / ms / 1e6 / HBM_PEAK_GBS,
               layers_frac_mfma=fig["attn_flops"] * L / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
               one_layer_cold_ms=round(cold_ms, 4),
               one_layer_cold_GBps=fig["attn_bytes"] / cold_ms / 1e6,
               one_layer_cold_TFLOPs=fig["attn_flops"] / cold_ms / 1e9)
    del q, kp, vp, kt, vt, out
    torch.cuda.empty_cache()
    return res


def rrs_path_pass(case, torch, binding, steps=20):
    """The same verification in path mode (only the sibling groups along the accepted path, as the
    paper's level-by-level loop does): identical decisions, less work; reported beside the timed
    all-groups call."""
    tree = case["tree"]
    run = lambda: binding.recursive_reject(case["zd"], case["zt"], tree["tokens"], tree["parent"], tree["n_nodes"],
                                           mode=binding.MODE_PATH, seed=0, step=0, diagnostics=False)
    for _ in range(2):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    return dict(rrs_path_mode_ms=round(e0.elapsed_time(e1) / steps, 4))


def filter_kv_pass(case, torch, binding, steps=20):
    """FilterKVCache (the step after the verification) on the step's own accepted paths, into a small
    cache of the same head layout: a latency-bound gather, timed on its own and not part of `value`."""
    cfg = case["cfg"]
    B, Hkv, D = cfg["B"], cfg["Hkv"], cfg["D"]
    res = case["rrs"]()
    kt, vt = case["kt"], case["vt"]
    cap = 8 + res["accepted_nodes"].shape[1] + 1
    kc = torch.zeros((B, Hkv, cap, D), dtype=kt.dtype, device=kt.device)
    vc = torch.zeros_like(kc)
    plen = torch.full((B,), 8, dtype=torch.int32, device=kt.device)
    run = lambda: binding.filter_kv_cache(kc, vc, kt, vt, plen, res["accepted_nodes"], res["n_accepted"])
    for _ in range(2):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    rows = int(res["n_accepted"].sum().item()) + B
    # tokens decoded per iteration (accepted draft tokens + the sampled last token), the paper's block
    # efficiency, here on synthetic logits whose draft/target gap is a recipe, not a trained pair
    block_eff = rows / B
    out = dict(filter_kv_ms=round(e0.elapsed_time(e1) / steps, 4), filter_kv_rows=rows * Hkv,
               block_efficiency_synthetic=round(block_eff, 3))
    if cfg["name"] in DRAFT_TO_TARGET:
        # memory-bound speed-up (App. C, performance metrics): block efficiency / (depth * r + 1)
        depth = cfg["depth"] if cfg["sampler"] == "sbs" else len(cfg["branching"])
        out["mbsu_synthetic"] = round(block_eff / (depth * DRAFT_TO_TARGET[cfg["name"]] + 1.0), 3)
    return out


def acceptance_pass(case, torch, binding, trials=8):
    """Acceptance of one level of K drafts at the root of every sequence, method against method on the
    same synthetic logit rows (the comparison of the paper's toy example and first experiment, here on
    a recipe instead of a trained model pair): recursive rejection sampling on K drafts drawn without
    replacement, against K-SEQ (gamma = K) and multi-round rejection sampling on K i.i.d. drafts.  K is
    the workload's own first-level branching, plus a sweep over the number of drafts."""
    cfg = case["cfg"]
    K_own = cfg["branching"][0] if cfg["sampler"] == "gumbel" else cfg["width"]
    zt, zd = case["zt"][:, 0].contiguous(), case["zd"][:, 0].contiguous()
    B, V = zt.shape
    dev = zt.device
    seq = torch.arange(B, dtype=torch.int32, device=dev)

    def rates(K):
        rows3 = lambda t: torch.stack([t] + [t] * K, dim=1).contiguous()      # [B, K + 1, V]: only row 0 is read
        zt3, zd3 = rows3(zt), rows3(zd)
        parent = torch.tensor([[-1] + [0] * K] * B, dtype=torch.int32, device=dev)
        n_nodes = torch.full((B,), K + 1, dtype=torch.int32, device=dev)
        hits = dict(rrs=0, kseq=0, multiround=0)
        for t in range(trials):
            top = binding.gumbel_topk(zd, K, seq_id=seq, seed=99, step=t, want_scores=False)["tokens"]
            tokens = torch.cat([torch.full((B, 1), -1, dtype=torch.int32, device=dev), top], dim=1).contiguous()
            r = binding.recursive_reject(zd3, zt3, tokens, parent, n_nodes, mode=binding.MODE_PATH, seed=99, step=t,
                                         diagnostics=False)
            hits["rrs"] += int((r["n_accepted"] > 0).sum().item())
            iid = torch.cat([binding.gumbel_topk(zd, 1, seq_id=seq, node_id=seq * 0 + 1000 + k, seed=99, step=t,
                                                 want_scores=False)["tokens"] for k in range(K)], dim=1).contiguous()
            for name, method, gamma in (("kseq", binding.BASELINE_KSEQ, float(K)),
                                        ("multiround", binding.BASELINE_MULTIROUND, 1.0)):
                g = binding.baseline_verify(zd, zt, iid, method, gamma=gamma, seq_id=seq, seed=99, step=t)
                hits[name] += int((g["accepted"] >= 0).sum().item())
        n = B * trials
        return dict(K=K, trials=n, rrs_without_replacement=round(hits["rrs"] / n, 4),
                    kseq_gamma_K=round(hits["kseq"] / n, 4), multiround=round(hits["multiround"] / n, 4))

    own = rates(K_own)
    own["by_number_of_drafts"] = [own if K == K_own else rates(K) for K in (1, 2, 4, 8, 16) if K <= V]
    own["by_number_of_drafts"] = [{k: v for k, v in r.items() if k != "by_number_of_drafts"}
                                  for r in own["by_number_of_drafts"]]
    return dict(level_acceptance_synthetic=own)


def filter_logits_pass(case, torch, binding, steps=5):
    """Nucleus filtering (top-p 0.95, the paper's instruction-following setting) of every target row:
    a preprocessing pass of that setting, timed on its own and not part of `value`."""
    zt = case["zt"]
    B, N, V = zt.shape
    rows = zt.view(B * N, V)
    out = torch.empty_like(rows)
    for _ in range(2):
        binding.filter_logits(rows, top_p=0.95, out=out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        binding.filter_logits(rows, top_p=0.95, out=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    del out
    return dict(top_p_filter_ms=round(ms, 4), top_p_filter_GBps=rows.numel() * 8 / ms / 1e6)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg4_stress", help="primary workload (name or index)")
    ap.add_argument("--no-others", action="store_true", help="skip the brief runs of the other configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run plain device copies of known size (profiler counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (no collectives are part of the hot path); "
                 "run with --gpus 1")

    import torch

    from paper_2402_14160_amd import binding, draft_tree, workloads
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    binding.lib()   # fails loudly if the HIP library is missing
    if args.calibrate_copy:
        calibrate_copy(torch)
        return

    key = int(args.config) if args.config.isdigit() else args.config
    cfg = workloads.config(key)
    case = build_case(cfg, args.seed, torch, binding, draft_tree, workloads)
    torch.cuda.synchronize()
    t = time_case(case, args.steps, args.warmup, torch)
    rep, fig = report(case, t)
    vocab = vocab_pass(case, torch, binding)
    vocab["graph_ms_per_step"] = round(graph_step_ms(case, torch), 4)
    vocab.update(rrs_path_pass(case, torch, binding))
    vocab.update(filter_kv_pass(case, torch, binding))
    vocab.update(filter_logits_pass(case, torch, binding))
    vocab.update(acceptance_pass(case, torch, binding))
    layers = layers_pass(case, torch, binding, workloads)
    vocab.update(layers)
    vocab.update(model_step(rep, fig, layers))

    # roofline of the dominant kernel: the tree-attention launch
    bound = rep["attn_bound"]
    traffic, traffic_source = measured_traffic(cfg["name"])
    if bound == "hbm":
        roof = dict(bound="hbm", achieved=rep["attn_GBps"], peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=rep["attn_frac_hbm"], traffic=traffic, traffic_source=traffic_source,
                    kernel="tree_attn_bf16_kernel", algorithmic_bytes=fig["attn_bytes"])
    else:
        roof = dict(bound="mfma", achieved=rep["attn_TFLOPs"], peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=rep["attn_frac_mfma"], traffic=traffic, traffic_source=traffic_source,
                    kernel="tree_attn_bf16_w32_kernel", algorithmic_flops=fig["attn_flops"])

    per_config = {}
    if not args.no_others:
        for other in workloads.CONFIGS:
            if other["name"] == cfg["name"]:
                continue
            del case
            torch.cuda.empty_cache()
            case = build_case(dict(other), args.seed, torch, binding, draft_tree, workloads)
            tt = time_case(case, max(5, args.steps), args.warmup, torch)
            per_config[other["name"]], ofig = report(case, tt)
            per_config[other["name"]]["graph_ms_per_step"] = round(graph_step_ms(case, torch), 4)
            olayers = layers_pass(case, torch, binding, workloads)
            per_config[other["name"]].update(olayers)
            per_config[other["name"]].update(model_step(per_config[other["name"]], ofig, olayers))
        del case
        torch.cuda.empty_cache()
        case = build_case(cfg, args.seed, torch, binding, draft_tree, workloads)

    cpu = None if args.no_cpu else cpu_baseline(case, fig, torch)

    line = dict(
        metric="draft-tree nodes verified/sec (attn+RRS) at 1 GPU; % HBM and % MFMA peak",
        value=rep["nodes_per_s_attn_rrs"], unit="tree nodes/s", n_gpus=1, steps=args.steps,
        warmup=args.warmup, ms_per_step=rep["ms_per_step"], higher_is_better=True, scaling="weak",
        vs_baseline=None, dtype="bf16" if cfg["dtype"] == "bf16" else "f32", data="synthetic",
        config=dict(workload=cfg["name"], batch=cfg["B"], vocab=cfg["V"], nodes_per_seq=cfg["N"],
                    q_heads=cfg["Hq"], kv_heads=cfg["Hkv"], head_dim=cfg["D"], kv_prefix=cfg["P"],
                    sampler=cfg["sampler"], rrs_mode="all_groups"),
        value_definition="tree nodes / (one layer of tree attention + recursive rejection sampling), both timed "
                         "inside the whole step",
        value_full_step=rep["nodes_per_s_full_step"],
        phases=dict(draft_ms=rep["draft_ms"], attn_ms=rep["attn_ms"], rrs_ms=rep["rrs_ms"],
                    attn_GBps=rep["attn_GBps"], attn_TFLOPs=rep["attn_TFLOPs"],
                    rrs_GBps=rep["rrs_GBps"],
                    rrs_frac_hbm=rep["rrs_frac_hbm"],
                    draft_GBps=rep["draft_GBps"], draft_alu_frac=rep["draft_alu_frac"], **vocab),
        roofline=roof, cpu_baseline=cpu, per_config=per_config,
    )
    print(json.dumps(line))


if __name__ == "__main__":
    main()
