"""GPU parity, call by call and end to end, at sizes the oracle finishes in seconds: every output
of the HIP path is compared element by element with the oracle on the same seeded inputs.
Integer results (indices, counts, offsets, permutations) and copies must match bit for bit, the
gate logits too (fixed summation order); floating results within rel-L2 1e-5 (fp32) / 1e-2 (bf16)."""
import numpy as np
import pytest
import torch

from paper_2411_10003_amd import workload as wl

pytestmark = pytest.mark.gpu

@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


@pytest.fixture(scope="module")
def orc():
    from oracle import moe_oracle
    moe_oracle.build()
    return moe_oracle


def _cfg(ci, **kw):
    return wl.scaled(wl.CONFIGS[ci], **kw)


# shapes chosen to span several tiles and ragged tails: T not a multiple of the 64 tokens of a block, d with
# one, two and many 64-column chunks (fewer than, as many as and several times the chunks requested ahead),
# E below, at and above a multiple of 16, E above 64 (several expert passes), k up to 3
GATE_CASES = [
    _cfg(0),                                                  # the tiny fp32 configuration, complete
    _cfg(0, T=333, d=100, E=8, k=1, P=4),                     # fp32, column tail (d % 64 != 0)
    _cfg(0, T=200, d=1024, E=16, k=2, P=4),                   # fp32 tokens, whole chunks
    _cfg(1, T=1000, d=320, h=64),
    _cfg(1, T=1001, d=512, h=64),                             # exactly the chunks requested ahead, ragged last block
    _cfg(1, T=130, d=64, h=64),                               # one chunk
    _cfg(1, T=130, d=128, h=64),                              # two chunks
    _cfg(1, T=640, d=4096, h=64),                             # the long rows of the largest configuration
    _cfg(2, T=777, d=256, h=64, E=32, k=2),
    _cfg(2, T=640, d=2048, h=64, E=32, k=2),
    _cfg(4, T=515, d=192, h=64, E=64, k=1, P=16),
    _cfg(4, T=640, d=2048, h=64, E=64, k=1, P=16),
    _cfg(1, T=300, d=128, h=64, E=100, k=3, P=10, n_replicas=1),
    _cfg(1, T=300, d=1024, h=64, E=128, k=2, P=8, n_replicas=1),   # two passes of 64 experts, whole chunks
    _cfg(1, T=65, d=64, h=64, E=5, k=2, P=5, n_replicas=1),
    _cfg(1, T=130, d=256, h=64, E=48, k=2, P=8, n_replicas=1),     # bf16, E a multiple of 16 the ring kernel does not take
    _cfg(1, T=130, d=192, h=64, E=80, k=2, P=8, n_replicas=1),     # two passes, the second one partly empty
    _cfg(0, T=130, d=128, E=16, k=2, P=4),                         # fp32 tokens, two whole chunks
    _cfg(1, T=100, d=8192, h=64),                                  # rows longer than any workload's
]


@pytest.mark.parametrize("cfg", GATE_CASES, ids=lambda c: f"{c.dtype}-T{c.T}-d{c.d}-E{c.E}-k{c.k}")
def test_gate_topk_and_counts(G, cfg):
    case = G.Case(cfg)
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, False)
    G.gpu_route(hd, case, b)
    torch.cuda.synchronize()
    r = case.route
    assert np.array_equal(G.host(b.logits).view(np.uint32), r["logits"].view(np.uint32))     # bit for bit
    assert np.array_equal(G.host(b.idx), r["idx"])
    assert np.allclose(G.host(b.w), r["w"], rtol=1e-5, atol=1e-7)
    assert np.array_equal(G.host(b.counts), r["counts"])
    assert int(G.host(b.counts).sum()) == cfg.T * cfg.k


def test_gate_exact_ties_go_to_lowest_index(G):
    cfg = _cfg(1, T=130, d=128, h=64, E=16, k=2)
    case = G.Case(cfg)
    Wg = np.repeat(case.inp["Wg"][:, :1], cfg.E, axis=1).copy()       # all columns equal: every logit ties
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, False)
    hd.gate_topk(case.dX, G.dev(Wg), G.dev(np.zeros(cfg.E, np.float32)), b.logits, b.idx, b.w)
    torch.cuda.synchronize()
    assert np.array_equal(G.host(b.idx), np.broadcast_to(np.array([0, 1], np.int32), (cfg.T, 2)))
    assert np.allclose(G.host(b.w), 0.5, rtol=1e-6)


@pytest.mark.parametrize("cfg", [_cfg(1, T=200, d=256, h=64), _cfg(0, T=200, d=100, E=8, k=2, P=4)],
                         ids=lambda c: f"{c.dtype}-d{c.d}-E{c.E}")
def test_gate_with_infinities_and_nans(G, orc, cfg):
    """Non-finite inputs take the IEEE route on both sides: an infinite token value or bias gives an infinite
    or NaN logit, NaN ranks as -inf in the selection, and the other tokens are untouched."""
    case = G.Case(cfg)
    X, Wg, bg = case.inp["X"].copy(), case.inp["Wg"].copy(), case.inp["bg"].copy()
    X[3, 5] = np.inf                      # logits of token 3: +-inf by the sign of Wg[5, e]
    X[7, 0] = np.nan                      # all logits of token 7 are NaN
    X[11, 17] = -np.inf
    X[11, 18] = np.inf                    # inf - inf somewhere along the chains of token 11
    bg[2] = -np.inf                       # expert 2 is never chosen by a finite token
    ref = orc.route(X, Wg, bg, cfg.k, cfg.renorm)
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, False)
    hd.gate_topk(G.dev(X, cfg.dtype), G.dev(Wg), G.dev(bg), b.logits, b.idx, b.w)
    torch.cuda.synchronize()
    got = G.host(b.logits)
    both_nan = np.isnan(got) & np.isnan(ref["logits"])
    assert np.array_equal(np.isnan(got), np.isnan(ref["logits"]))
    assert np.array_equal(got.view(np.uint32)[~both_nan], ref["logits"].view(np.uint32)[~both_nan])
    assert np.isnan(got[7]).all() and np.isinf(got[3]).any() and (got[:, 2][~np.isnan(got[:, 2])] == -np.inf).all()
    assert np.array_equal(G.host(b.idx), ref["idx"])
    finite = np.isfinite(ref["w"]).all(axis=1)
    assert finite.sum() >= cfg.T - 3
    assert np.allclose(G.host(b.w)[finite], ref["w"][finite], rtol=1e-5, atol=1e-7)
    assert not (G.host(b.idx)[finite] == 2).any()


PLANS = ["planner", "all_owner", "all_self", "round_robin", "self_last"]


@pytest.mark.parametrize("plan", PLANS)
@pytest.mark.parametrize("ci", [0, 1, 4])
def test_dispatch_layout_and_copy(G, orc, ci, plan):
    cfg = _cfg(ci, T=1500 if ci else 512, d=128 if ci else 64, h=64)
    E, P = cfg.E, cfg.P
    if plan == "self_last":
        cfg = wl.scaled(cfg, self_dest=P - 1)
    case0 = G.Case(cfg)
    dest = {
        "planner": case0.expert_dest,
        "all_owner": np.array([wl.owner_of(e, E, P) for e in range(E)], np.int32),
        "all_self": np.full(E, cfg.self_dest, np.int32),
        "round_robin": (np.arange(E) % P).astype(np.int32),
        "self_last": np.array([wl.owner_of(e, E, P) for e in range(E)], np.int32),
    }[plan]
    case = G.Case(cfg, expert_dest=dest)
    hd = G.make_handle(cfg, G=E)
    b = G.binding.LayerBuffers(hd, False)
    idx = G.dev(case.route["idx"])
    cnt = G.dev(case.route["counts"])
    hd.dispatch(case.ddest, case.dX, idx, cnt, b.layout, b.Xp)
    assert hd.read_status() == 0
    G.assert_layout_equal(b, case.lay)
    Xp = G.host(b.Xp)
    assert np.array_equal(Xp, orc.dispatch(case.inp["X"], case.lay["perm"], cfg.k))
    # determinism: a second run gives the same bits
    b2 = G.binding.LayerBuffers(hd, False)
    hd.dispatch(case.ddest, case.dX, idx, cnt, b2.layout, b2.Xp)
    torch.cuda.synchronize()
    assert torch.equal(b.layout.perm, b2.layout.perm) and torch.equal(b.Xp, b2.Xp)


def test_dispatch_with_empty_experts_and_one_giant_group(G, orc):
    cfg = _cfg(1, T=900, d=64, h=64, E=16, k=2)
    case = G.Case(cfg)
    # reroute by hand: expert 3 takes every first choice, expert 7 every second one
    idx = np.empty((cfg.T, 2), np.int32)
    idx[:, 0], idx[:, 1] = 3, 7
    cnt = orc.counts(idx, cfg.E)
    dest = wl.make_plan(cfg, cnt)
    lay = orc.place(idx, cnt, dest, cfg.P)
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, False)
    hd.expert_counts(G.dev(idx), b.counts)
    hd.dispatch(G.dev(dest), case.dX, G.dev(idx), b.counts, b.layout, b.Xp)
    torch.cuda.synchronize()
    assert np.array_equal(G.host(b.counts), cnt)
    G.assert_layout_equal(b, lay)
    assert np.array_equal(G.host(b.Xp), orc.dispatch(case.inp["X"], lay["perm"], cfg.k))


def test_dispatch_depends_on_its_arguments_only(G, orc):
    """moe_dispatch keeps nothing from earlier calls: rewriting idx in place after moe_expert_counts, or another
    handle counting into the same workspace in between, must not change its result.  moe_dispatch_after_counts is
    the explicit form for the unbroken sequence counts -> dispatch and gives the same bits."""
    cfg = _cfg(1, T=1500, d=128, h=64)
    case = G.Case(cfg)
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, False)
    idx1 = case.route["idx"]
    rng = np.random.default_rng(5)
    idx2 = np.stack([rng.permutation(cfg.E)[:cfg.k] for _ in range(cfg.T)]).astype(np.int32)   # another routing
    cnt2 = orc.counts(idx2, cfg.E)
    lay2 = orc.place(idx2, cnt2, case.expert_dest, cfg.P)
    # (a) idx rewritten in place between the two calls
    d_idx = G.dev(idx1)
    hd.expert_counts(d_idx, b.counts)
    d_idx.copy_(G.dev(idx2))
    hd.dispatch(case.ddest, case.dX, d_idx, G.dev(cnt2), b.layout, b.Xp)
    torch.cuda.synchronize()
    G.assert_layout_equal(b, lay2)
    assert np.array_equal(G.host(b.Xp), orc.dispatch(case.inp["X"], lay2["perm"], cfg.k))
    # (b) a second handle used the same workspace in between
    hd_other = G.make_handle(cfg)
    hd_other.ws = hd.ws
    d_idx1, d_idx2 = G.dev(idx1), G.dev(idx2)
    hd.expert_counts(d_idx1, b.counts)
    hd_other.expert_counts(d_idx2, torch.empty_like(b.counts))
    hd.dispatch(case.ddest, case.dX, d_idx1, b.counts, b.layout, b.Xp)
    torch.cuda.synchronize()
    G.assert_layout_equal(b, case.lay)
    # (c) the explicit reuse after an unbroken counts call
    b3 = G.binding.LayerBuffers(hd, False)
    hd.expert_counts(d_idx1, b3.counts)
    hd.dispatch_after_counts(case.ddest, case.dX, d_idx1, b3.counts, b3.layout, b3.Xp)
    torch.cuda.synchronize()
    G.assert_layout_equal(b3, case.lay)
    assert torch.equal(b3.Xp, b.Xp) and np.array_equal(G.host(b3.Xp), orc.dispatch(case.inp["X"], case.lay["perm"], cfg.k))


def test_plan_errors_are_reported(G):
    cfg = _cfg(1, T=128, d=64, h=64)
    case = G.Case(cfg)
    hd = G.make_handle(cfg, G=2)                     # capacity below the 4 hosted experts of the plan
    b = G.binding.LayerBuffers(hd, False)
    idx, cnt = G.dev(case.route["idx"]), G.dev(case.route["counts"])
    hd.dispatch(case.ddest, case.dX, idx, cnt, b.layout, b.Xp)
    assert hd.read_status() == -3
    bad = case.expert_dest.copy()
    bad[5] = cfg.P + 3
    hd2 = G.make_handle(cfg)
    hd2.dispatch(G.dev(bad), case.dX, idx, cnt, b.layout, b.Xp)
    assert hd2.read_status() == -3
    hd2.dispatch(case.ddest, case.dX, idx, cnt, b.layout, b.Xp)
    assert hd2.read_status() == 0


FFN_CASES = [
    _cfg(0),                                                              # fp32 GELU, complete
    _cfg(0, T=300, d=36, h=50, act="swiglu", backward=True),              # fp32 SwiGLU, odd sizes
    _cfg(1, T=1100, d=128, h=320, backward=True),                         # bf16 GELU, ragged tiles
    _cfg(3, T=900, d=192, h=256, backward=True),                          # bf16 SwiGLU
    _cfg(4, T=2000, d=128, h=128, backward=True),                         # 64 experts, k = 1, tiny groups
    # contractions of 128 slices and more: the few tiles there are get split along the contraction (two to four
    # parts, over both segments of the SwiGLU input gradient) and are finished by the second launch
    _cfg(3, T=500, d=128, h=4096, backward=True),
    _cfg(1, T=600, d=4096, h=128, backward=True),
    # the shortest contractions there are: two slices (one pair) per segment, so the loop's first and last slice are
    # all of it, and the SwiGLU input gradient changes segment after its first pair
    _cfg(3, T=700, d=64, h=64, backward=True),
    _cfg(1, T=700, d=64, h=192, backward=True),
]


def _ffn_io(G, case, hd, b):
    """Run dispatch -> FFN forward on the device with oracle routing as the input."""
    idx, cnt = G.dev(case.route["idx"]), G.dev(case.route["counts"])
    hd.dispatch(case.ddest, case.dX, idx, cnt, b.layout, b.Xp)
    b.Yp.copy_(G.dev(case.inp["Yp_fill"], case.cfg.dtype))
    hd.expert_ffn_fwd(b.Xp, b.layout, case.dW1, case.dW2, case.dW3, b.Yp, b.Z, b.U)
    torch.cuda.synchronize()


@pytest.mark.parametrize("cfg", FFN_CASES, ids=lambda c: f"{c.dtype}-{c.act}-T{c.T}-d{c.d}-h{c.h}-E{c.E}")
def test_ffn_forward_and_combine(G, orc, cfg):
    tol = G.TOL[cfg.dtype]
    case = G.Case(cfg)
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, cfg.backward)
    _ffn_io(G, case, hd, b)
    pos, hosted = case.lay["pos"], case.hosted
    Y, Z, U, Act = case.oracle_ffn(hosted, True)
    rows = pos[hosted]
    Yp_gpu = G.host(b.Yp)
    G.assert_rows_close(Yp_gpu[rows], Y, tol, "Yp_gpu[rows]")
    G.assert_rows_close(G.host(b.Z)[rows], Z, tol, "b.Z[rows]")
    if cfg.act == "swiglu":
        G.assert_rows_close(G.host(b.U)[rows], U, tol, "b.U[rows]")
    # rows of other destinations are untouched
    remote = np.setdiff1d(np.arange(cfg.A), rows)
    assert np.array_equal(Yp_gpu[remote], case.inp["Yp_fill"][remote])
    # combine on inputs both sides share: the oracle's Yp rounded to the storage type
    Yp_in = case.oracle_Yp_full().astype(np.float32)
    if cfg.dtype == "bf16":
        wl.round_to_bf16(Yp_in)
    w32 = case.route["w"].astype(np.float32)
    hd.combine(G.dev(Yp_in, cfg.dtype), G.dev(pos), G.dev(w32), b.out)
    torch.cuda.synchronize()
    want = orc.combine(Yp_in, pos, w32, cfg.k)
    G.assert_rows_close(G.host(b.out), want, tol, "b.out")
    # end to end (device routing and device FFN output) against the oracle chain
    G.gpu_route(hd, case, b)
    hd.dispatch(case.ddest, case.dX, b.idx, b.counts, b.layout, b.Xp)
    hd.expert_ffn_fwd(b.Xp, b.layout, case.dW1, case.dW2, case.dW3, b.Yp, b.Z, b.U)
    hd.combine(b.Yp, b.layout.pos, b.w, b.out)
    torch.cuda.synchronize()
    want = orc.combine(case.oracle_Yp_full(), pos, case.route["w"], cfg.k)
    G.assert_rows_close(G.host(b.out), want, tol, "b.out")
    # forward only: without Z and U the output holds the same bits and the two buffers are not written
    Yp_kept = b.Yp.clone()
    b.Yp.fill_(3.0); b.Z.fill_(5.0)
    if b.U is not None:
        b.U.fill_(5.0)
    hd.expert_ffn_fwd(b.Xp, b.layout, case.dW1, case.dW2, case.dW3, b.Yp, None, None)
    torch.cuda.synchronize()
    assert torch.equal(b.Yp[torch.as_tensor(rows, device=b.Yp.device).long()], Yp_kept[torch.as_tensor(rows, device=b.Yp.device).long()])
    assert bool((b.Z == 5.0).all()) and (b.U is None or bool((b.U == 5.0).all()))
    if cfg.act == "swiglu":                                    # kept together or not at all
        with pytest.raises(G.binding.MoeError):
            hd.expert_ffn_fwd(b.Xp, b.layout, case.dW1, case.dW2, case.dW3, b.Yp, b.Z, None)


def test_identity_experts_return_x_times_weight_sum(G):
    cfg = _cfg(1, T=700, d=128, h=64)
    case = G.Case(cfg)
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, False)
    G.gpu_route(hd, case, b)
    hd.dispatch(case.ddest, case.dX, b.idx, b.counts, b.layout, b.Xp)
    hd.combine(b.Xp, b.layout.pos, b.w, b.out)                   # Yp := Xp on all rows
    torch.cuda.synchronize()
    want = case.inp["X"].astype(np.float64) * case.route["w"].sum(axis=1, keepdims=True)
    G.assert_rows_close(G.host(b.out), want, 4e-3, "b.out")   # one bf16 rounding of the output


@pytest.mark.parametrize("cfg", [c for c in FFN_CASES if c.backward],
                         ids=lambda c: f"{c.dtype}-{c.act}-T{c.T}-d{c.d}-h{c.h}-E{c.E}")
def test_backward_calls(G, orc, cfg):
    tol = G.TOL[cfg.dtype]
    dt = cfg.dtype
    case = G.Case(cfg)
    inp, lay, r = case.inp, case.lay, case.route
    pos, hosted = lay["pos"], case.hosted
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, True)
    _ffn_io(G, case, hd, b)                                       # fills Xp, Z, U on the device

    # --- combine_bwd on shared inputs
    Yp_in = case.oracle_Yp_full().astype(np.float32)
    if dt == "bf16":
        wl.round_to_bf16(Yp_in)
    w32 = r["w"].astype(np.float32)
    hd.combine_bwd(G.dev(inp["dOut"], dt), G.dev(Yp_in, dt), G.dev(pos), G.dev(w32), b.dYp, b.dw)
    torch.cuda.synchronize()
    dYp_o, dw_o = orc.combine_bwd(inp["dOut"], Yp_in, pos, w32, cfg.k)
    G.assert_rows_close(G.host(b.dYp), dYp_o, tol, "b.dYp")
    G.assert_rows_close(G.host(b.dw), dw_o, tol, "b.dw", floor=1.0)

    # --- expert_ffn_bwd on shared inputs: dYp = oracle's, rounded to the storage type
    dYp_in = dYp_o.astype(np.float32)
    if dt == "bf16":
        wl.round_to_bf16(dYp_in)
    b.dXp.copy_(G.dev(inp["dXp_fill"], dt))
    hd.expert_ffn_bwd(G.dev(dYp_in, dt), b.Xp, b.Z, b.U, b.layout, case.dW1, case.dW2, case.dW3,
                      b.dXp, b.dW1, b.dW2, b.dW3)
    torch.cuda.synchronize()
    dXh = orc.ffn_bwd_rows(inp["X"], case.idx_flat, case.goe, inp["W1"], inp["W2"], inp.get("W3"), cfg.k, cfg.act,
                           hosted, dYp_in[pos[hosted]].astype(np.float64))
    dXp_gpu = G.host(b.dXp)
    G.assert_rows_close(dXp_gpu[pos[hosted]], dXh, tol, "dXp_gpu[pos[hosted]]")
    remote = np.setdiff1d(np.arange(cfg.A), pos[hosted])
    assert np.array_equal(dXp_gpu[remote], inp["dXp_fill"][remote])
    dYa = dYp_in[pos]                                            # by assignment
    dW1o, dW2o, dW3o = orc.ffn_bwd_weights(inp["X"], case.idx_flat, case.goe, inp["W1"], inp["W2"], inp.get("W3"),
                                           cfg.k, cfg.act, dYa, cfg.G_max)
    Gn = case.G
    G.assert_rows_close(G.host(b.dW1)[:Gn], dW1o[:Gn], tol, "b.dW1[:Gn]")
    G.assert_rows_close(G.host(b.dW2)[:Gn], dW2o[:Gn], tol, "b.dW2[:Gn]")
    if cfg.act == "swiglu":
        G.assert_rows_close(G.host(b.dW3)[:Gn], dW3o[:Gn], tol, "b.dW3[:Gn]")
    for g in range(cfg.G_max):                                   # empty or unused groups are written as zeros
        o, e = case.group_rows(g) if g < Gn else (0, 0)
        if e == o:
            assert not G.host(b.dW1)[g].any() and not G.host(b.dW2)[g].any()

    # --- the activation of the forward pass read from the workspace instead of being recomputed (moe_set_act_saved):
    # the forward call puts it back there; what does not depend on it keeps its bits, dW2 stays within tolerance
    if dt == "bf16":
        plain = [t.clone() if t is not None else None for t in (b.dW1, b.dW2, b.dW3, b.dXp)]
        hd.expert_ffn_fwd(b.Xp, b.layout, case.dW1, case.dW2, case.dW3, b.Yp, b.Z, b.U)
        hd.set_act_saved(True)
        b.dW2.fill_(float("nan"))
        hd.expert_ffn_bwd(G.dev(dYp_in, dt), b.Xp, b.Z, b.U, b.layout, case.dW1, case.dW2, case.dW3,
                          b.dXp, b.dW1, b.dW2, b.dW3)
        hd.set_act_saved(False)
        torch.cuda.synchronize()
        assert torch.equal(b.dW1, plain[0]) and torch.equal(b.dXp, plain[3])
        if cfg.act == "swiglu":
            assert torch.equal(b.dW3, plain[2])
        G.assert_rows_close(G.host(b.dW2)[:Gn], dW2o[:Gn], tol, "dW2 from the saved activation")
        for g in range(cfg.G_max):
            o, e = case.group_rows(g) if g < Gn else (0, 0)
            if e == o:
                assert not G.host(b.dW2)[g].any()
        # back to the recomputed form for what follows
        hd.expert_ffn_bwd(G.dev(dYp_in, dt), b.Xp, b.Z, b.U, b.layout, case.dW1, case.dW2, case.dW3,
                          b.dXp, b.dW1, b.dW2, b.dW3)
        torch.cuda.synchronize()
        assert torch.equal(b.dW2, plain[1])

    # --- accumulate form: a second contribution is added to what the buffers hold.  Doubling is exact in
    # fp32, so running the same backward again on top must give exactly twice the first result; seeding the
    # buffers with another value checks against the oracle's sum.
    first = [t.clone() if t is not None else None for t in (b.dW1, b.dW2, b.dW3)]
    dXp_first = b.dXp.clone()
    hd.expert_ffn_bwd_acc(G.dev(dYp_in, dt), b.Xp, b.Z, b.U, b.layout, case.dW1, case.dW2, case.dW3,
                          b.dXp, b.dW1, b.dW2, b.dW3)
    torch.cuda.synchronize()
    assert torch.equal(b.dW1, first[0] * 2) and torch.equal(b.dW2, first[1] * 2)
    if cfg.act == "swiglu":
        assert torch.equal(b.dW3, first[2] * 2)
    assert torch.equal(b.dXp, dXp_first)                          # the row gradient is overwritten as before
    b.dW1.fill_(0.5); b.dW2.fill_(-0.25)
    if b.dW3 is not None:
        b.dW3.fill_(2.0)
    hd.expert_ffn_bwd_acc(G.dev(dYp_in, dt), b.Xp, b.Z, b.U, b.layout, case.dW1, case.dW2, case.dW3,
                          b.dXp, b.dW1, b.dW2, b.dW3)
    torch.cuda.synchronize()
    G.assert_rows_close(G.host(b.dW1)[:Gn] - 0.5, dW1o[:Gn], tol, "b.dW1[:Gn] - 0.5")
    G.assert_rows_close(G.host(b.dW2)[:Gn] + 0.25, dW2o[:Gn], tol, "b.dW2[:Gn]  0.25")
    for g in range(cfg.G_max):                                   # an empty or unused group adds zero
        o, e = case.group_rows(g) if g < Gn else (0, 0)
        if e == o:
            assert (G.host(b.dW1)[g] == 0.5).all() and (G.host(b.dW2)[g] == -0.25).all()

    # --- dispatch_bwd and gate_bwd on shared inputs
    dXp_in = inp["dXp_fill"].copy()
    hd.dispatch_bwd(G.dev(dXp_in, dt), G.dev(pos), b.dX)
    dw32 = dw_o.astype(np.float32)
    hd.gate_bwd(G.dev(dw32), G.dev(r["logits"]), G.dev(r["idx"]), b.dlogits)
    torch.cuda.synchronize()
    G.assert_rows_close(G.host(b.dX), orc.dispatch_bwd(dXp_in, pos, cfg.k), tol, "b.dX")
    # a token's logit gradient is a difference of nearly equal terms where its two gate weights or their gradients
    # are close: measured against the typical row, not against what is left after the cancellation
    G.assert_rows_close(G.host(b.dlogits), orc.gate_bwd(dw32, r["logits"], r["idx"], cfg.renorm), 1e-5, "b.dlogits", floor=1.0)


@pytest.mark.parametrize("cfg", [c for c in FFN_CASES if c.backward][:3],
                         ids=lambda c: f"{c.dtype}-{c.act}-T{c.T}")
def test_layer_forward_backward_end_to_end(G, orc, cfg):
    """The device chain on its own intermediates against the oracle chain in double."""
    tol = G.TOL[cfg.dtype]
    dt = cfg.dtype
    case = G.Case(cfg)
    inp, lay, r = case.inp, case.lay, case.route
    pos, hosted = lay["pos"], case.hosted
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, True)
    b.Yp.copy_(G.dev(inp["Yp_fill"], dt))
    b.dXp.copy_(G.dev(inp["dXp_fill"], dt))
    G.binding.layer_forward(hd, b, case.dX, case.dWg, case.dbg, case.ddest, case.dW1, case.dW2, case.dW3)
    G.binding.layer_backward(hd, b, G.dev(inp["dOut"], dt), case.dW1, case.dW2, case.dW3)
    torch.cuda.synchronize()
    Yp_o = case.oracle_Yp_full()
    dYp_o, dw_o = orc.combine_bwd(inp["dOut"], Yp_o, pos, r["w"], cfg.k)
    dXp_o = inp["dXp_fill"].astype(np.float64)
    dXp_o[pos[hosted]] = orc.ffn_bwd_rows(inp["X"], case.idx_flat, case.goe, inp["W1"], inp["W2"], inp.get("W3"),
                                          cfg.k, cfg.act, hosted, dYp_o[pos[hosted]])
    dW1o, dW2o, dW3o = orc.ffn_bwd_weights(inp["X"], case.idx_flat, case.goe, inp["W1"], inp["W2"], inp.get("W3"),
                                           cfg.k, cfg.act, dYp_o[pos].astype(np.float32), cfg.G_max)
    Gn = case.G
    G.assert_rows_close(G.host(b.out), orc.combine(Yp_o, pos, r["w"], cfg.k), tol, "b.out")
    G.assert_rows_close(G.host(b.dw), dw_o, tol, "b.dw", floor=1.0)
    G.assert_rows_close(G.host(b.dX), orc.dispatch_bwd(dXp_o, pos, cfg.k), tol, "b.dX")
    G.assert_rows_close(G.host(b.dW1)[:Gn], dW1o[:Gn], tol, "b.dW1[:Gn]")
    G.assert_rows_close(G.host(b.dW2)[:Gn], dW2o[:Gn], tol, "b.dW2[:Gn]")
    if cfg.act == "swiglu":
        G.assert_rows_close(G.host(b.dW3)[:Gn], dW3o[:Gn], tol, "b.dW3[:Gn]")
    # d_gate, the plain relative L2 error over the whole tensor (observed about 2e-3)
    dl_o = orc.gate_bwd(dw_o, r["logits"], r["idx"], cfg.renorm)
    dl_err = float(np.linalg.norm(G.host(b.dlogits) - dl_o))
    print(f"[{cfg.dtype}-{cfg.act}-T{cfg.T}] end-to-end dlogits: plain rel-L2 {dl_err / np.linalg.norm(dl_o):.3e}, "
          f"against max(|dw|, |dlogits|) {dl_err / max(np.linalg.norm(dw_o), np.linalg.norm(dl_o)):.3e}", flush=True)
    assert dl_err <= tol * np.linalg.norm(dl_o)                # the plain relative L2 error


def test_argument_errors_do_not_launch(G):
    cfg = _cfg(1, T=128, d=64, h=64)
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, False)
    with pytest.raises(G.binding.MoeError) as ei:
        hd._check(hd.lib.moe_combine(hd._h, None, b.layout.pos.data_ptr(), b.w.data_ptr(), b.out.data_ptr(), None), "moe_combine")
    assert ei.value.status == -1
    with pytest.raises(G.binding.MoeError) as ei:                      # misaligned workspace
        hd._check(hd.lib.moe_expert_counts(hd._h, b.idx.data_ptr(), b.counts.data_ptr(), hd.ws.data_ptr() + 4, None),
                  "moe_expert_counts")
    assert ei.value.status == -4
    with pytest.raises(G.binding.MoeError):
        G.binding.Handle(T=128, d=100, h=64, E=8, k=2, P=4, self_dest=0, G=2, dtype="bf16", act="gelu", renorm=1)
