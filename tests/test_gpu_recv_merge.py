"""Receive side (Eq. 2 of the paper: a device computes its own inputs of the experts it hosts and those the
first all-to-all delivers for the experts it owns).  The expert computation runs once over the send buffer and
once over a receive buffer laid out by moe_recv_layout; the weight gradients of the second pass are added to
those of the first.  Received rows are synthetic; the oracle evaluates each row with the weights of its expert
and sums the two weight gradients."""
import numpy as np
import pytest
import torch

import gpu_util as G
from paper_2411_10003_amd import binding, workload as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("index,kw,recv", [
    (3, dict(T=768, d=256, h=384), [300, 0, 513, 7]),           # SwiGLU, G = 4: ragged, an empty group, a tail
    (2, dict(T=640, d=128, h=256), [0, 257, 0, 31, 0, 0, 90, 5]),   # GELU, G = 8
])
def test_expert_computation_over_send_and_receive_buffers(index, kw, recv):
    cfg = wl.scaled(wl.CONFIGS[index], **kw)
    case = G.Case(cfg)
    inp, lay = case.inp, case.lay
    d, h, k, Gn, dt = cfg.d, cfg.h, cfg.k, case.G, cfg.dtype
    tol = G.TOL[dt]
    recv = np.array(recv[:cfg.G_max], dtype=np.int64)
    recv[Gn:] = 0                                              # nothing arrives for slots that host no expert
    offs = np.concatenate([[0], np.cumsum(recv)]).astype(np.int32)          # [G_max + 1], constant after the hosted groups
    R = int(offs[-1])
    rng = np.random.default_rng(900 + index)
    Xr = rng.standard_normal((R, d)).astype(np.float32)
    dYr = rng.standard_normal((R, d)).astype(np.float32)
    wl.round_to_bf16(Xr); wl.round_to_bf16(dYr)
    hosted_e = wl.hosted_experts(case.expert_dest, cfg.self_dest)
    idx_r = np.repeat(hosted_e[:len(recv)][:Gn] if Gn else hosted_e, recv[:Gn]).astype(np.int32)   # expert of every received row

    # ---- device: local pass, then the receive pass with the same weights, gradients accumulated
    hd = G.make_handle(cfg)
    b = binding.LayerBuffers(hd, True)
    idx, cnt = G.dev(case.route["idx"]), G.dev(case.route["counts"])
    hd.dispatch(case.ddest, case.dX, idx, cnt, b.layout, b.Xp)
    b.Yp.copy_(G.dev(inp["Yp_fill"], dt))
    hd.expert_ffn_fwd(b.Xp, b.layout, case.dW1, case.dW2, case.dW3, b.Yp, b.Z, b.U)
    dYp = rng.standard_normal((cfg.A, d)).astype(np.float32)
    wl.round_to_bf16(dYp)
    b.dXp.copy_(G.dev(inp["dXp_fill"], dt))
    hd.expert_ffn_bwd(G.dev(dYp, dt), b.Xp, b.Z, b.U, b.layout, case.dW1, case.dW2, case.dW3, b.dXp, b.dW1, b.dW2, b.dW3)

    hr = binding.Handle(T=max(R, 1), d=d, h=h, E=cfg.E, k=1, P=cfg.P, self_dest=cfg.self_dest, G=cfg.G_max, dtype=dt,
                        act=cfg.act, renorm=0, device=G.DEV)
    lay_r = hr.new_layout()
    hr.recv_layout(b.layout, G.dev(offs), lay_r)
    el = hd.elt
    dXr = G.dev(Xr, dt) if R else torch.zeros(1, d, dtype=el, device=G.DEV)
    Yr = torch.full((max(R, 1), d), 3.0, dtype=el, device=G.DEV)
    Zr = torch.zeros(max(R, 1), h, dtype=el, device=G.DEV)
    Ur = torch.zeros(max(R, 1), h, dtype=el, device=G.DEV) if cfg.act == "swiglu" else None
    hr.expert_ffn_fwd(dXr, lay_r, case.dW1, case.dW2, case.dW3, Yr, Zr, Ur)
    dXr_out = torch.full((max(R, 1), d), 5.0, dtype=el, device=G.DEV)
    ddYr = G.dev(dYr, dt) if R else torch.zeros(1, d, dtype=el, device=G.DEV)
    hr.expert_ffn_bwd_acc(ddYr, dXr, Zr, Ur, lay_r, case.dW1, case.dW2, case.dW3, dXr_out, b.dW1, b.dW2, b.dW3)
    torch.cuda.synchronize()
    assert hd.read_status() == 0
    assert np.array_equal(G.host(lay_r.slot_offsets)[int(lay["dest_slots"][cfg.self_dest]):][:Gn + 1], offs[:Gn + 1])

    # ---- oracle: received rows are one-expert assignments (k = 1) of a second batch
    goe = case.goe
    a_r = np.arange(R, dtype=np.int32)
    if R:
        Yr_o = G.orc.ffn_fwd(Xr, idx_r, goe, inp["W1"], inp["W2"], inp.get("W3"), 1, cfg.act, a_r)
        assert G.rel_l2(G.host(Yr)[:R], Yr_o) <= tol
        dXr_o = G.orc.ffn_bwd_rows(Xr, idx_r, goe, inp["W1"], inp["W2"], inp.get("W3"), 1, cfg.act, a_r, dYr.astype(np.float64))
        assert G.rel_l2(G.host(dXr_out)[:R], dXr_o) <= tol
    # local rows are untouched by the receive pass
    hosted = case.hosted
    assert G.rel_l2(G.host(b.Yp)[lay["pos"][hosted]], case.oracle_ffn(hosted)) <= tol
    # weight gradients: the sum over both buffers
    loc = G.orc.ffn_bwd_weights(inp["X"], case.idx_flat, goe, inp["W1"], inp["W2"], inp.get("W3"), k, cfg.act, dYp[lay["pos"]], cfg.G_max)
    rec = G.orc.ffn_bwd_weights(Xr, idx_r, goe, inp["W1"], inp["W2"], inp.get("W3"), 1, cfg.act, dYr, cfg.G_max) if R else (0, 0, 0)
    assert G.rel_l2(G.host(b.dW1)[:Gn], (loc[0] + rec[0])[:Gn]) <= tol
    assert G.rel_l2(G.host(b.dW2)[:Gn], (loc[1] + rec[1])[:Gn]) <= tol
    if cfg.act == "swiglu":
        assert G.rel_l2(G.host(b.dW3)[:Gn], (loc[2] + rec[2])[:Gn]) <= tol
    # the receive pass must matter: against the local gradients alone the difference is large
    if R:
        assert G.rel_l2(G.host(b.dW1)[:Gn], loc[0][:Gn]) > 10 * tol
