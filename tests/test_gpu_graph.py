"""One decode iteration's calls captured into a HIP graph and replayed: the library enqueues kernels only
(no allocation, no memset, no synchronisation), so a captured step must give, on every replay, what the
same calls give eagerly on the inputs then in the buffers."""
import pytest
import torch

from paper_2402_14160_amd import binding, workloads
from tests.gpu_util import dev, say, to_np

pytestmark = pytest.mark.gpu


def _step(bufs):
    """Draft one level, attend, verify, update the cache -- on static buffers."""
    top = binding.gumbel_topk(bufs["zd"][:, 0].contiguous(), 3, seed=4, step=1)
    out = binding.tree_attention(bufs["q"], bufs["kc"][:, :, :bufs["P"]], bufs["vc"][:, :, :bufs["P"]],
                                 bufs["kt"], bufs["vt"], bufs["plen"], bufs["n_nodes"], bufs["parent"], 0.09)
    rrs = binding.recursive_reject(bufs["zd"], bufs["zt"], bufs["tokens"], bufs["parent"], bufs["n_nodes"],
                                   mode=binding.MODE_ALL_GROUPS, seed=4, step=1)
    kc, vc = bufs["kc"].clone(), bufs["vc"].clone()
    new_len, _ = binding.filter_kv_cache(kc, vc, bufs["kt"], bufs["vt"], bufs["plen"],
                                         rrs["accepted_nodes"], rrs["n_accepted"])
    return dict(tokens=top["tokens"], attn=out, n_acc=rrs["n_accepted"], last=rrs["last_token"],
                acc=rrs["accepted_nodes"], new_len=new_len, kc=kc)


def test_captured_step_replays_like_eager():
    say("one iteration captured in a HIP graph, three replays on changing inputs")
    d = dev()
    B, N, V, H, D, P, cap = 4, 10, 32000, 4, 128, 192, 256
    parent = torch.tensor([[-1, 0, 0, 0, 1, 1, 2, 2, 3, 3]] * B, dtype=torch.int32, device=d)
    bufs = dict(P=P, parent=parent, n_nodes=torch.full((B,), N, dtype=torch.int32, device=d),
                plen=torch.full((B,), P, dtype=torch.int32, device=d))

    def fill(seed):
        zt, zd = workloads.make_logits("zipf", B, N, V, seed=seed)
        q, kp, vp, kt, vt = workloads.make_qkv(B, H, H, N, D, cap, "bf16", seed)
        g = torch.Generator().manual_seed(seed)
        tokens = torch.stack([torch.randperm(V, generator=g)[:N] for _ in range(B)]).to(torch.int32)
        vals = dict(zt=zt, zd=zd, q=q, kc=kp, vc=vp, kt=kt, vt=vt, tokens=tokens)
        for k, v in vals.items():
            if k in bufs:
                bufs[k].copy_(v.to(d))
            else:
                bufs[k] = v.to(d).contiguous()

    fill(0)
    for _ in range(2):                      # warm-up: one-time kernel attributes are set outside capture
        _step(bufs)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = _step(bufs)
    for seed in (1, 2, 3):
        fill(seed)                          # eager copies into the static input buffers
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = {k: v.clone() for k, v in captured.items()}
        want = _step(bufs)                  # the same calls, eagerly, on the same inputs
        torch.cuda.synchronize()
        for k in want:
            assert torch.equal(got[k], want[k]), (seed, k)
        say(f"  replay with seed {seed}: accepted {to_np(want['n_acc']).tolist()}")
