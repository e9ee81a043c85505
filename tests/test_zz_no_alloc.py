"""rsd_sbs_step_static: the Stochastic Beam Search step for callers that cannot allocate.  Called
through the C ABI with every input and output tensor made beforehand, it must give what
rsd_sbs_step gives (same kernels: bit-identical), on two calls in a row that share the library's
scratch array, the second one smaller than the first, and it must refuse a request that does not
fit the array."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import sbs as o_sbs
from paper_2402_14160_amd import binding, workloads
from tests.gpu_util import LOGP_TOL, dev, say, to_np

pytestmark = pytest.mark.gpu

KEYS = ("tokens", "parent", "sum_logprob", "trunc_gumbel", "n_out", "lse")


def _inputs(B, W_in, V, seed):
    d = dev()
    _, zd = workloads.make_logits("zipf", B, W_in, V, seed=seed)
    rng = np.random.default_rng(seed)
    sigma = (-rng.exponential(3.0, size=(B, W_in))).astype(np.float32)
    gamma = (-np.sort(rng.exponential(1.0, size=(B, W_in)), axis=1)).astype(np.float32)
    n_in = rng.integers(1, W_in + 1, size=B).astype(np.int32)
    n_in[0] = W_in
    host = dict(zd=zd.numpy(), sigma=sigma, gamma=gamma, n_in=n_in)
    return host, (zd.to(d), torch.from_numpy(sigma).to(d), torch.from_numpy(gamma).to(d),
                  torch.from_numpy(n_in).to(d))


def _outputs(B, W_in, W):
    d = dev()
    return dict(tokens=torch.full((B, W), -7, dtype=torch.int32, device=d),
                parent=torch.full((B, W), -7, dtype=torch.int32, device=d),
                sum_logprob=torch.zeros((B, W), dtype=torch.float32, device=d),
                trunc_gumbel=torch.zeros((B, W), dtype=torch.float32, device=d),
                n_out=torch.full((B,), -7, dtype=torch.int32, device=d),
                lse=torch.zeros((B, W_in), dtype=torch.float32, device=d))


def test_sbs_step_static_matches_workspace_variant_twice():
    say("sbs_step_static: two calls in a row on the shared scratch array, the second one smaller")
    # first call: rows split into segments (few rows, large vocabulary); second: fewer, shorter rows
    for B, W_in, V, W, seed in [(8, 6, 50272, 6, 41), (2, 3, 4000, 4, 42)]:
        host, args = _inputs(B, W_in, V, seed)
        outs = _outputs(B, W_in, W)
        torch.cuda.synchronize()
        events = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]
        before = events()
        got = binding.sbs_step(*args, W, seed=seed, step=3, out=outs, static_scratch=True)
        assert events() == before                                # no allocation went through torch
        want = binding.sbs_step(*args, W, seed=seed, step=3)
        torch.cuda.synchronize()
        for k in KEYS:
            assert torch.equal(got[k], want[k]), (B, W_in, V, k)
        # and both against the oracle (token / parent lists and the normalisers)
        ref = o_sbs.sbs_step(host["zd"], host["sigma"], host["gamma"], host["n_in"], W, seed=seed, step=3)
        assert np.array_equal(to_np(got["n_out"]), ref["n_out"])
        for b in range(B):
            n, live = int(ref["n_out"][b]), int(host["n_in"][b])
            if ref["min_gap"][b] < 1e-5:
                continue
            assert np.array_equal(to_np(got["tokens"])[b, :n], ref["tokens"][b, :n])
            assert np.array_equal(to_np(got["parent"])[b, :n], ref["parent"][b, :n])
            assert np.allclose(to_np(got["lse"])[b, :live], ref["lse"][b, :live], rtol=0, atol=LOGP_TOL)


def test_sbs_step_static_rejects_what_does_not_fit():
    lib = binding.lib()
    fake = ctypes.c_void_p(4096)          # never dereferenced: the size check comes first
    B, W_in, V, W = 4096, 16, 1024, 16    # 65536 rows of 16 candidates: far beyond the array
    assert lib.rsd_sbs_step_workspace_bytes(B, W_in, V, W) > 524288
    rc = lib.rsd_sbs_step_static(fake, fake, fake, fake, None, None, B, W_in, V, W, 1.0, 0, 0,
                                 fake, fake, fake, fake, fake, None, None)
    assert rc == -7
    assert b"scratch" in lib.rsd_status_string(rc)
    assert lib.rsd_sbs_step_static(None, fake, fake, fake, None, None, 1, 1, 64, 1, 1.0, 0, 0,
                                   fake, fake, fake, fake, fake, None, None) == -1
