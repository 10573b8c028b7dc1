"""moe_expert_counts_static, the entry point for callers that cannot allocate or pass a workspace: its output
against moe_expert_counts (and the oracle's counts) bit for bit, on two calls in a row of which the second is
the smaller one (the built-in array still holds the first call's histograms), then a larger one again."""
import numpy as np
import pytest
import torch

import gpu_util as G
from paper_2411_10003_amd import binding, workload as wl

pytestmark = pytest.mark.gpu


def _counts_both_ways(cfg, seed):
    rng = np.random.default_rng(seed)
    p = rng.dirichlet(np.full(cfg.E, 0.3))                                   # skewed routing, some experts near empty
    idx = rng.choice(cfg.E, size=(cfg.T, cfg.k), p=p).astype(np.int32)
    hd = G.make_handle(cfg)
    d_idx = G.dev(idx)
    with_ws = torch.full((cfg.E,), -1, dtype=torch.int32, device=G.DEV)
    static = torch.full((cfg.E,), -2, dtype=torch.int32, device=G.DEV)
    hd.expert_counts(d_idx, with_ws)
    print(f"[no-alloc] T={cfg.T} k={cfg.k} E={cfg.E}: moe_expert_counts_static", flush=True)
    hd.expert_counts_static(d_idx, static)
    torch.cuda.synchronize()
    assert torch.equal(static, with_ws)
    assert np.array_equal(G.host(static), G.orc.counts(idx, cfg.E))
    assert int(G.host(static).sum()) == cfg.A


def test_static_counts_match_on_consecutive_calls():
    big = wl.scaled(wl.CONFIGS[3], T=20000, d=64, h=64)                      # 157 chunks x 16 experts, ragged last chunk
    small = wl.scaled(wl.CONFIGS[4], T=700, d=64, h=64)                      # 3 chunks x 64 experts: other strides, fewer words
    _counts_both_ways(big, 1)
    _counts_both_ways(small, 2)
    _counts_both_ways(wl.scaled(wl.CONFIGS[1], T=5000, d=64, h=64, E=100, k=3, P=10, n_replicas=1), 3)


def test_static_counts_reject_inputs_beyond_the_array():
    cfg = wl.scaled(wl.CONFIGS[4], T=300000, d=64, h=64, E=1024, k=1, P=16, n_replicas=0)  # 1172 chunks x 1024 experts > 2^20 words
    hd = G.make_handle(cfg)
    idx = torch.zeros(cfg.T, cfg.k, dtype=torch.int32, device=G.DEV)
    counts = torch.zeros(cfg.E, dtype=torch.int32, device=G.DEV)
    with pytest.raises(binding.MoeError) as ei:
        hd.expert_counts_static(idx, counts)
    assert ei.value.status == -8
