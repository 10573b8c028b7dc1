"""The gate checked against the mathematics alone (Section 2.1 of the paper defines only the linear map and the
top-k choice), with no reference to any summation order: the device logits against a float64 product within a
bound that depends on the operands only, and the device's top-k against the float64 top-k for every token whose
float64 margin is wide enough to be decided in fp32.  The bit-for-bit comparison with the oracle's fixed order is
a separate test; this one would still hold if that order were wrong on both sides."""
import numpy as np
import pytest
import torch

import gpu_util as G
from paper_2411_10003_amd import binding, workload as wl

pytestmark = pytest.mark.gpu

CASES = [
    wl.CONFIGS[0],                                                          # fp32 tokens, tiny, complete
    wl.scaled(wl.CONFIGS[1], T=2048, h=64),                                 # d = 1024, E = 16, k = 2
    wl.scaled(wl.CONFIGS[2], T=2048, h=64),                                 # d = 2048, E = 32
    wl.scaled(wl.CONFIGS[3], h=64),                                         # the gate of the largest workload, full size
    wl.scaled(wl.CONFIGS[4], h=64),                                         # E = 64, k = 1, full size
    wl.scaled(wl.CONFIGS[1], T=1000, d=320, h=64, E=100, k=3, P=10, n_replicas=1),   # passes of 64 experts, tails
    wl.scaled(wl.CONFIGS[0], T=333, d=100, E=8, k=2, P=4),                  # fp32 tokens, column tail
]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: f"{c.dtype}-T{c.T}-d{c.d}-E{c.E}-k{c.k}")
def test_gate_against_float64(cfg):
    inp = wl.make_inputs(cfg, 0, with_weights=False)
    X, Wg, bg = inp["X"], inp["Wg"], inp["bg"]
    hd = G.make_handle(cfg)
    b = binding.LayerBuffers(hd, False)
    hd.gate_topk(G.dev(X, cfg.dtype), G.dev(Wg), G.dev(bg), b.logits, b.idx, b.w)
    torch.cuda.synchronize()
    got, idx, w = G.host(b.logits).astype(np.float64), G.host(b.idx), G.host(b.w).astype(np.float64)

    X64, W64, b64 = X.astype(np.float64), Wg.astype(np.float64), bg.astype(np.float64)
    L = X64 @ W64 + b64                                                     # library routine, float64
    bound = 1e-5 * (np.linalg.norm(X64, axis=1)[:, None] * np.linalg.norm(W64, axis=0)[None, :] + np.abs(b64)[None, :])
    excess = np.abs(got - L) / bound
    assert excess.max() <= 1.0, f"logit off by {excess.max():.2f} times the bound at {np.unravel_index(excess.argmax(), L.shape)}"

    # float64 top-k, ties to the lowest index; a token is decided when every gap down to rank k+1 is wide
    k, E = cfg.k, cfg.E
    order = np.lexsort((np.broadcast_to(np.arange(E), L.shape), -L), axis=1)
    v = np.take_along_axis(L, order, axis=1)
    thr = 1e-5 * np.abs(L).max(axis=1)
    gaps = v[:, :k] - v[:, 1:k + 1] if k < E else v[:, :k - 1] - v[:, 1:k]
    decided = (gaps > thr[:, None]).all(axis=1)
    n_out = int((~decided).sum())
    print(f"[{cfg.dtype} T={cfg.T} d={cfg.d} E={E} k={k}] largest logit error {excess.max():.3f} of the bound; "
          f"{n_out} of {cfg.T} tokens closer than 1e-5 max|logit| to a tie (compared for validity only)", flush=True)
    assert n_out <= max(2, cfg.T // 200)
    assert np.array_equal(idx[decided], order[decided, :k].astype(np.int32))
    # the others: every chosen expert is within the margin of the k-th float64 value, and no expert is chosen twice
    chosen = np.take_along_axis(L, idx.astype(np.int64), axis=1)
    assert (chosen >= (v[:, k - 1] - thr)[:, None]).all()
    assert all(len(set(row)) == k for row in idx[~decided].tolist())

    # gate weights from the float64 logits (softmax over all experts, renormalised over the chosen when asked)
    p = np.exp(L - L.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    ws = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if cfg.renorm:
        ws = ws / ws.sum(axis=1, keepdims=True)
    assert np.allclose(w, ws, rtol=2e-4, atol=1e-7)
