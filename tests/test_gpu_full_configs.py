"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (the same calls on the same buffers).  Routing, counts, layout, permutation and the
send buffer are compared completely and bit for bit; FFN outputs, layer outputs and gradients on
sampled rows, tokens and hidden units that the oracle computes one by one, each compared row by
row: a row in every 256-row tile of every hosted group (hence in every tile band, every ragged
last tile and every tile of the contraction-split last round), group boundaries, random picks,
and a hidden unit in every 256-wide block of the weight gradients."""
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


def _check_pass(G, orc, case, hd, b, n_random=16, seed=0, label=""):
    cfg = case.cfg
    tol = G.TOL[cfg.dtype]
    dt = cfg.dtype
    inp, lay, r = case.inp, case.lay, case.route
    pos, k = lay["pos"], cfg.k
    rep = []
    print(f"[{label}] running the device pass", flush=True)
    b.Yp.copy_(G.dev(inp["Yp_fill"], dt))
    G.binding.layer_forward(hd, b, case.dX, case.dWg, case.dbg, case.ddest, case.dW1, case.dW2, case.dW3)
    if cfg.backward:
        b.dXp.copy_(G.dev(inp["dXp_fill"], dt))
        G.binding.layer_backward(hd, b, G.dev(inp["dOut"], dt), case.dW1, case.dW2, case.dW3)
    torch.cuda.synchronize()
    assert hd.read_status() == 0

    # ---- complete, bit for bit
    assert np.array_equal(G.host(b.logits).view(np.uint32), r["logits"].view(np.uint32))
    assert np.array_equal(G.host(b.idx), r["idx"])
    assert np.array_equal(G.host(b.counts), r["counts"]) and int(r["counts"].sum()) == cfg.A
    assert np.allclose(G.host(b.w), r["w"], rtol=1e-5, atol=1e-7)
    G.assert_layout_equal(b, lay)
    assert np.array_equal(G.host(b.Xp), orc.dispatch(inp["X"], lay["perm"], k))

    # ---- which tiles there are: one sampled row in every 256-row tile of every hosted group, so that every tile
    # band, every ragged last tile and every tile of the contraction-split last round holds a compared row (a row
    # is compared over all its columns, hence over every column tile)
    groups = [case.group_rows(g) for g in range(case.G)]
    row_tiles = G.ffn_row_tiles(groups)
    n_blocks = torch.cuda.get_device_properties(0).multi_processor_count // 8 * 8
    swiglu = cfg.act == "swiglu"
    launches = {"fwd1": (-(-cfg.h // (128 if swiglu else 256)), cfg.d // 32), "fwd2": (-(-cfg.d // 256), cfg.h // 32),
                "bwd1": (-(-cfg.h // 256), cfg.d // 32), "bwd2": (-(-cfg.d // 256), (2 if swiglu else 1) * cfg.h // 32)}
    split = {n: G.ffn_split_tiles(len(row_tiles), ct, ks, n_blocks, G.FFN_BAND[n]) for n, (ct, ks) in launches.items()}
    for n, tiles in split.items():                               # every split tile lies in a sampled row tile
        assert all(0 <= rt < len(row_tiles) for rt, _ in tiles), n
    a_s = case.sample_assignments(n_random, seed, every_tile=True)
    sampled_rows = np.sort(pos[a_s])
    for ti, (g, r0, r1) in enumerate(row_tiles):
        i = np.searchsorted(sampled_rows, r0)
        assert i < sampled_rows.size and sampled_rows[i] < r1, f"row tile {ti} of group {g} holds no sampled row"
    print(f"[{label}] {len(row_tiles)} row tiles in {-(-len(row_tiles) // 8)} bands, all sampled ({a_s.size} rows); "
          f"tiles of the split last round: " + ", ".join(f"{n} {len(t)}" for n, t in split.items()), flush=True)

    # ---- sampled assignments: forward FFN
    if a_s.size:
        Y, Z, U, Act = case.oracle_ffn(a_s, True)
        rows = torch.from_numpy(pos[a_s].astype(np.int64)).to(G.DEV)
        G.assert_rows_close(G.host(b.Yp[rows]), Y, tol, "Yp", report=rep)
        G.assert_rows_close(G.host(b.Z[rows]), Z, tol, "Z", report=rep)
        if swiglu:
            G.assert_rows_close(G.host(b.U[rows]), U, tol, "U", report=rep)

    # ---- sampled tokens: layer output (all k assignments of each token)
    rng = np.random.default_rng(seed + 1)
    t_s = np.unique(np.concatenate([a_s[:: max(1, a_s.size // 32)] // k, rng.integers(0, cfg.T, 8)]))[:40].astype(np.int32)
    a_t = (t_s[:, None] * k + np.arange(k)[None, :]).reshape(-1).astype(np.int32)
    host_mask = case.goe[case.idx_flat[a_t]] >= 0
    Yt = inp["Yp_fill"][pos[a_t]].astype(np.float64)             # rows of other destinations: the seeded fill
    if host_mask.any():
        Yt[host_mask] = case.oracle_ffn(a_t[host_mask])
    pos_c = np.arange(a_t.size, dtype=np.int32)                  # compact layout: row i holds assignment a_t[i]
    w_c = r["w"][t_s]
    out_o = orc.combine(Yt, pos_c, w_c, k)
    t_dev = torch.from_numpy(t_s.astype(np.int64)).to(G.DEV)
    G.assert_rows_close(G.host(b.out[t_dev]), out_o, tol, "out", report=rep)
    if not cfg.backward:
        print(f"[{label}] worst row / pooled: " + "; ".join(f"{n} {w:.2e} / {p_:.2e}" for n, w, p_ in rep), flush=True)
        return

    # ---- backward on the sampled tokens
    dOut_t = inp["dOut"][t_s]
    dYt, dw_o = orc.combine_bwd(dOut_t, Yt, pos_c, w_c, k)
    rows_t = torch.from_numpy(pos[a_t].astype(np.int64)).to(G.DEV)
    G.assert_rows_close(G.host(b.dYp[rows_t]), dYt, tol, "dYp", report=rep)
    G.assert_rows_close(G.host(b.dw[t_dev]), dw_o, tol, "dw", floor=1.0, report=rep)
    dXt = inp["dXp_fill"][pos[a_t]].astype(np.float64)
    if host_mask.any():
        dXt[host_mask] = orc.ffn_bwd_rows(inp["X"], case.idx_flat, case.goe, inp["W1"], inp["W2"], inp.get("W3"),
                                          k, cfg.act, a_t[host_mask], dYt[host_mask])
    G.assert_rows_close(G.host(b.dX[t_dev]), orc.dispatch_bwd(dXt, pos_c, k), tol, "dX", report=rep)
    dl_o = orc.gate_bwd(dw_o, r["logits"][t_s], r["idx"][t_s], cfg.renorm)
    dl_err = float(np.linalg.norm(G.host(b.dlogits[t_dev]) - dl_o))
    print(f"[{label}] end-to-end dlogits on {t_s.size} tokens: plain rel-L2 {dl_err / max(np.linalg.norm(dl_o), 1e-300):.3e}, "
          f"against max(|dw|, |dlogits|) {dl_err / max(np.linalg.norm(dw_o), np.linalg.norm(dl_o)):.3e}", flush=True)
    assert dl_err <= tol * np.linalg.norm(dl_o)                # the plain relative L2 error

    # ---- backward on the row of every tile: the gradient rows the return all-to-all delivers do not depend on Yp
    # (zeros stand in for it; the gate-weight gradient of this call is not used), the input gradient does the rest
    if a_s.size:
        t_a = (a_s // k).astype(np.int32)
        a_all = (t_a[:, None] * k + np.arange(k)[None, :]).reshape(-1)
        dY_all, _ = orc.combine_bwd(inp["dOut"][t_a], np.zeros((a_all.size, cfg.d)), np.arange(a_all.size, dtype=np.int32),
                                    r["w"][t_a], k)
        dY_s = dY_all[np.arange(a_s.size) * k + (a_s % k)]
        G.assert_rows_close(G.host(b.dYp[rows]), dY_s, tol, "dYp (every tile)", report=rep)
        dX_s = orc.ffn_bwd_rows(inp["X"], case.idx_flat, case.goe, inp["W1"], inp["W2"], inp.get("W3"), k, cfg.act, a_s, dY_s)
        G.assert_rows_close(G.host(b.dXp[rows]), dX_s, tol, "dXp (every tile)", report=rep)

    # ---- weight gradients: one hidden unit in every 256-wide block of h (every column tile of dW1 / dW3 and
    # every row tile of dW2; a unit is compared over all d, hence over every tile of the other axis), contracted
    # over every row of the group
    print(f"[{label}] weight-gradient samples", flush=True)
    dYa = (r["w"].reshape(-1, 1) * np.repeat(inp["dOut"], k, axis=0)).astype(np.float32)   # w[a] * dOut[t(a)]
    dW1, dW2 = b.dW1, b.dW2
    for g in range(cfg.G_max):
        o, e = case.group_rows(g) if g < case.G else (0, 0)
        if e == o:                                              # empty or unused group: written as zeros
            assert not bool(dW1[g].any()) and not bool(dW2[g].any())
            if swiglu:
                assert not bool(b.dW3[g].any())
            continue
        js = np.array(sorted(set([0, cfg.h - 1] + [int(rng.integers(j0, min(j0 + 256, cfg.h))) for j0 in range(0, cfg.h, 256)])),
                      dtype=np.int32)
        r2, c1, c3 = orc.ffn_bwd_hidden_many(inp["X"], case.idx_flat, case.goe, inp["W1"], inp["W2"], inp.get("W3"),
                                             k, cfg.act, dYa, g, js)
        jd = torch.from_numpy(js.astype(np.int64)).to(G.DEV)
        # a hidden unit's gradient in a group of a handful of rows is a sum of that many terms, each carrying an
        # error proportional to the typical size of dZ, not to its own: where the terms all happen to be small the
        # vector is measured against half the typical norm of the group's units instead of its own
        G.assert_rows_close(G.host(dW2[g][jd, :]), r2, tol, f"dW2[{g}]", floor=0.5, report=rep)
        G.assert_rows_close(G.host(dW1[g][:, jd].t()), c1, tol, f"dW1[{g}]", floor=0.5, report=rep)
        if swiglu:
            G.assert_rows_close(G.host(b.dW3[g][:, jd].t()), c3, tol, f"dW3[{g}]", floor=0.5, report=rep)
    worst = {}
    for n, w, p_ in rep:
        key = n.split("[")[0]
        worst[key] = max(worst.get(key, (0.0, 0.0)), (w, p_))
    print(f"[{label}] worst row / pooled: " + "; ".join(f"{n} {w:.2e} / {p_:.2e}" for n, (w, p_) in worst.items()), flush=True)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("ci", [1, 2, 3])
def test_full_config(G, orc, ci):
    cfg = wl.CONFIGS[ci]
    print(f"[cfg{ci}] drawing inputs and routing on the CPU", flush=True)
    case = G.Case(cfg)
    assert case.G == cfg.G_max
    share = np.sort(case.route["counts"])[::-1] / cfg.A
    print(f"[cfg{ci}] top-3 share {share[:3].sum():.3f}, bottom-3 {share[-3:].sum():.4f}, hosted rows "
          f"{[case.group_rows(g)[1] - case.group_rows(g)[0] for g in range(case.G)]}", flush=True)
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, cfg.backward)
    _check_pass(G, orc, case, hd, b, label=f"cfg{ci}")


@pytest.mark.timeout(600)
@pytest.mark.parametrize("T,h,parts", [(10240, 6272, 3), (8192, 8256, 4)])
def test_last_round_split_in_three_and_four_parts(G, orc, T, h, parts):
    """Shapes whose last round of fwd2 and bwd2 is cut along the contraction into three and four parts, with part
    boundaries that would fall on odd slices (196 and 258 slices) if the kernel did not move them to even ones."""
    cfg = wl.scaled(wl.CONFIGS[2], T=T, d=256, h=h)
    case = G.Case(cfg)
    row_tiles = G.ffn_row_tiles([case.group_rows(g) for g in range(case.G)])
    n_blocks = torch.cuda.get_device_properties(0).multi_processor_count // 8 * 8
    k_slices = h // 32
    assert min(4, n_blocks // len(row_tiles), k_slices // 64) == parts
    assert any((i * k_slices // parts) % 2 == 1 for i in range(1, parts))
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, cfg.backward)
    _check_pass(G, orc, case, hd, b, label=f"split{parts}")


@pytest.mark.timeout(900)
def test_drift_sweep(G, orc):
    """Ten iterations of the skew/drift workload: alpha cycles through {0, 0.8, 1.5}, the rank
    permutation is re-drawn every third iteration, and the plan of iteration i comes from the input
    distribution of iteration i-1 (the locality the planner relies on), so replicas go stale."""
    cfg = wl.CONFIGS[4]
    hd = G.make_handle(cfg)
    b = G.binding.LayerBuffers(hd, True)
    prev_counts = None
    weights = None
    saw_empty = saw_giant = False
    for it in range(cfg.iterations):
        print(f"[cfg4] iteration {it}: alpha {wl.alpha_for(cfg, it)}", flush=True)
        case = G.Case.__new__(G.Case)
        inp = wl.make_inputs(cfg, it, with_weights=(weights is None))
        if weights is None:
            weights = {n: inp[n] for n in ("W1", "W2")}
            dW = {n: G.dev(weights[n], cfg.dtype) for n in weights}
        inp.update(weights)
        r = orc.route(inp["X"], inp["Wg"], inp["bg"], cfg.k, cfg.renorm)
        dest = wl.make_plan(cfg, r["counts"] if prev_counts is None else prev_counts, threshold=True)
        prev_counts = r["counts"]
        case.cfg, case.inp, case.route, case.expert_dest = cfg, inp, r, dest
        case.lay = orc.place(r["idx"], r["counts"], dest, cfg.P)
        case.goe = wl.group_of_expert(dest, cfg.self_dest)
        case.G = int((dest == cfg.self_dest).sum())
        case.idx_flat = r["idx"].reshape(-1)
        case.hosted = orc.hosted_assignments(case.idx_flat, case.goe)
        case.dX, case.dWg, case.dbg = G.dev(inp["X"], cfg.dtype), G.dev(inp["Wg"]), G.dev(inp["bg"])
        case.dW1, case.dW2, case.dW3, case.ddest = dW["W1"], dW["W2"], None, G.dev(dest)
        rows = [case.group_rows(g)[1] - case.group_rows(g)[0] for g in range(case.G)]
        saw_empty |= any(x == 0 for x in rows)
        saw_giant |= any(x > cfg.T // 4 for x in rows)
        print(f"[cfg4] hosted experts {wl.hosted_experts(dest).tolist()} rows {rows}", flush=True)
        _check_pass(G, orc, case, hd, b, n_random=8, seed=it, label=f"cfg4 it{it}")
    assert saw_empty and saw_giant, "the sweep must contain an empty hosted group and one above 25 % of T"
