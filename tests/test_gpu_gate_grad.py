"""GPU parity of the gate-parameter gradients and of the complete input gradient against the oracle."""
import numpy as np
import pytest
import torch

import gpu_util as G
from paper_2411_10003_amd import binding, workload as wl

pytestmark = pytest.mark.gpu


def _case(index, **kw):
    cfg = wl.scaled(wl.CONFIGS[index], **kw) if kw else wl.CONFIGS[index]
    return cfg, G.Case(cfg)


def _check(cfg, case, seed=0):
    rng = np.random.default_rng(seed)
    T, d, E, k, A = cfg.T, cfg.d, cfg.E, cfg.k, cfg.A
    tol = G.TOL[cfg.dtype]
    hd = G.make_handle(cfg)
    # logit gradients as moe_gate_bwd produces them (fp32); both sides get the same values
    dl = rng.standard_normal((T, E)).astype(np.float32)
    if cfg.renorm:                                            # only the selected experts carry a gradient
        mask = np.zeros((T, E), bool)
        np.put_along_axis(mask, case.route["idx"].astype(np.int64), True, axis=1)
        dl[~mask] = 0.0
    d_dl = G.dev(dl)
    dWg = torch.full((d, E), 7.0, dtype=torch.float32, device=G.DEV)
    dbg = torch.full((E,), 7.0, dtype=torch.float32, device=G.DEV)
    hd.gate_bwd_params(case.dX, d_dl, dWg, dbg)
    want_W, want_b = G.orc.gate_bwd_params(case.inp["X"], dl)
    G.assert_rows_close(G.host(dWg), want_W, 1e-5, "dWg")      # fp32 sums in every dtype
    G.assert_rows_close(G.host(dbg), want_b, 1e-5, "dbg")
    dWg2 = torch.zeros_like(dWg); dbg2 = torch.zeros_like(dbg)
    hd.gate_bwd_params(case.dX, d_dl, dWg2, dbg2)              # fixed summation order: same bits
    assert torch.equal(dWg, dWg2) and torch.equal(dbg, dbg2)

    dXp = rng.standard_normal((A, d)).astype(np.float32)
    if cfg.dtype == "bf16":
        wl.round_to_bf16(dXp)
    pos = case.lay["pos"]
    dX = torch.zeros(T, d, dtype=hd.elt, device=G.DEV)
    hd.input_grad(G.dev(dXp, cfg.dtype), G.dev(pos), d_dl, case.dWg, dX)
    want = G.orc.input_grad(dXp, pos, dl, case.inp["Wg"], k)
    G.assert_rows_close(G.host(dX), want, tol, "dX")
    # without a logit gradient it is the backward of the send: the same bits as moe_dispatch_bwd
    dX0 = torch.zeros_like(dX); dX1 = torch.zeros_like(dX)
    hd.input_grad(G.dev(dXp, cfg.dtype), G.dev(pos), torch.zeros_like(d_dl), case.dWg, dX0)
    hd.dispatch_bwd(G.dev(dXp, cfg.dtype), G.dev(pos), dX1)
    assert torch.equal(dX0, dX1)
    # the gate path alone, made large enough (x64, exact in fp32) to stand clear of the rounding of the sum
    big = (dl * np.float32(64.0)).astype(np.float32)
    hd.input_grad(G.dev(dXp, cfg.dtype), G.dev(pos), G.dev(big), case.dWg, dX0)
    gate_only = big.astype(np.float64) @ case.inp["Wg"].astype(np.float64).T
    assert G.rel_l2(G.host(dX0).astype(np.float64) - G.orc.dispatch_bwd(dXp, pos, k), gate_only) <= 0.05


@pytest.mark.parametrize("index,kw", [
    (0, {}),                                                   # fp32, E = 8, k = 1
    (1, dict(T=1001, d=512, h=128)),                           # bf16, E = 16, ragged token count
    (2, dict(T=777, d=192, h=128)),                            # E = 32, a strip that is not full
    (3, dict(T=2048, d=1024, h=128)),                          # E = 16, k = 2
    (4, dict(T=600, d=576, h=128)),                            # E = 64, k = 1, softmax weights (dense gradient)
    (1, dict(T=300, d=1024, h=64, E=128, k=2, P=8, n_replicas=1)),     # two passes of 64 experts, renormalised top-2
    (4, dict(T=530, d=320, h=64, E=100, k=1, P=10, n_replicas=1)),     # a second pass that is partly empty, dense gradient
    (0, dict(T=200, d=100, E=72, k=2, P=4, renorm=1)),                 # fp32 tokens, column tail, 72 experts
])
def test_gate_gradients_small(index, kw):
    cfg, case = _case(index, **kw)
    _check(cfg, case, seed=index)


@pytest.mark.timeout(600)
def test_gate_gradients_full_config3():
    """At the full size of the benchmark configuration (T = 32768, d = 4096): complete comparison."""
    cfg = wl.scaled(wl.CONFIGS[3], h=64)                       # the expert width plays no part here
    case = G.Case(cfg)
    _check(cfg, case, seed=33)


def test_argument_errors():
    cfg = wl.scaled(wl.CONFIGS[1], T=256, d=128, h=128)
    hd = G.make_handle(cfg)
    z = torch.zeros(4, device=G.DEV)
    with pytest.raises((binding.MoeError, ValueError)):
        hd.gate_bwd_params(None, z, z, z)
    with pytest.raises((binding.MoeError, ValueError)):
        hd.input_grad(z, None, z, z, z)
