"""Pins of the oracle's expert-computation half: forward FFN against numpy float64 matmul
MLPs and closed forms, combine against identity experts and plan invariance, every gradient
against central finite differences and adjointness."""
import numpy as np
import pytest
from scipy.special import erf

from paper_2411_10003_amd import workload as wl


def _tiny(ci, **kw):
    base = dict(T=24, d=8, h=16)
    base.update(kw)
    return wl.scaled(wl.CONFIGS[ci], **base)


def _routed(orc, cfg, iteration=0, threshold=False):
    inp = wl.make_inputs(cfg, iteration)
    r = orc.route(inp["X"], inp["Wg"], inp["bg"], cfg.k, cfg.renorm)
    dest = wl.make_plan(cfg, r["counts"], threshold=threshold)
    lay = orc.place(r["idx"], r["counts"], dest, cfg.P)
    goe = wl.group_of_expert(dest, cfg.self_dest)
    return inp, r, dest, lay, goe


def _gelu64(z):
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def _silu64(z):
    return z / (1.0 + np.exp(-z))


@pytest.mark.parametrize("ci", [0, 1, 3])
def test_ffn_fwd_vs_numpy_mlp_per_group(orc, ci):
    cfg = _tiny(ci, T=96, d=24, h=40)
    inp, r, dest, lay, goe = _routed(orc, cfg)
    idx = r["idx"].reshape(-1)
    hosted = orc.hosted_assignments(idx, goe)
    assert hosted.size > 0
    Y, Z, U, Act = orc.ffn_fwd(inp["X"], idx, goe, inp["W1"], inp["W2"], inp.get("W3"), cfg.k, cfg.act, hosted, True)
    X64 = inp["X"].astype(np.float64)
    for g, e in enumerate(wl.hosted_experts(dest)):
        sel = np.nonzero(idx[hosted] == e)[0]
        x = X64[hosted[sel] // cfg.k]
        z = x @ inp["W1"][g].astype(np.float64)
        if cfg.act == "swiglu":
            u = x @ inp["W3"][g].astype(np.float64)
            a = _silu64(z) * u
            assert np.allclose(U[sel], u, rtol=1e-12, atol=1e-13)
        else:
            a = _gelu64(z)
        y = a @ inp["W2"][g].astype(np.float64)
        assert np.allclose(Z[sel], z, rtol=1e-12, atol=1e-13)
        assert np.allclose(Act[sel], a, rtol=1e-12, atol=1e-13)
        assert np.allclose(Y[sel], y, rtol=1e-11, atol=1e-12)


def test_ffn_single_group_is_a_dense_mlp_and_remote_rejected(orc):
    rng = np.random.default_rng(3)
    T, d, h = 10, 6, 9
    X = rng.standard_normal((T, d)).astype(np.float32)
    W1 = rng.standard_normal((1, d, h)).astype(np.float32)
    W2 = rng.standard_normal((1, h, d)).astype(np.float32)
    idx = np.zeros(T, np.int32)
    Y = orc.ffn_fwd(X, idx, np.array([0], np.int32), W1, W2, None, 1, "gelu", np.arange(T))
    ref = _gelu64(X.astype(np.float64) @ W1[0].astype(np.float64)) @ W2[0].astype(np.float64)
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-13)
    with pytest.raises(ValueError):
        orc.ffn_fwd(X, idx, np.array([-1], np.int32), W1, W2, None, 1, "gelu", np.arange(T))


def test_activation_special_values(orc):
    # one input, d = 1, h = 3: z = x * W1 picks the pre-activations directly; W2 = 1 sums them
    X = np.array([[1.0]], np.float32)
    W2 = np.ones((1, 3, 1), np.float32)
    idx = np.zeros(1, np.int32)
    goe = np.array([0], np.int32)
    W1 = np.array([[[0.0, 30.0, -30.0]]], np.float32)
    Y, Z, U, Act = orc.ffn_fwd(X, idx, goe, W1, W2, None, 1, "gelu", [0], True)
    assert Act[0, 0] == 0.0 and Act[0, 1] == 30.0 and abs(Act[0, 2]) < 1e-100   # gelu(0)=0, gelu(x)->x, gelu(-x)->0
    W1 = np.array([[[0.5, 1.0, -2.0]]], np.float32)
    Y, Z, U, Act = orc.ffn_fwd(X, idx, goe, W1, W2, None, 1, "gelu", [0], True)
    # Phi(0.5), Phi(1), Phi(-2) from standard normal tables
    phi = np.array([0.6914624612740131, 0.8413447460685429, 0.022750131948179195])
    assert np.allclose(Act[0], np.array([0.5, 1.0, -2.0]) * phi, rtol=1e-13)
    # SwiGLU with the gate branch u == 1 is a plain silu MLP; silu(0) = 0, silu(ln 3) = 0.75 ln 3
    W1 = np.array([[[0.0, np.log(3.0), 1.0]]], np.float32)
    W3 = np.ones((1, 1, 3), np.float32)
    Y, Z, U, Act = orc.ffn_fwd(X, idx, goe, W1, W2, W3, 1, "swiglu", [0], True)
    z = W1[0, 0].astype(np.float64)
    assert np.all(U[0] == 1.0) and Act[0, 0] == 0.0
    assert np.allclose(Act[0], z / (1 + np.exp(-z)), rtol=1e-14)
    assert np.isclose(Act[0, 1], 0.75 * z[1], rtol=1e-12)
    W3 = np.full((1, 1, 3), 2.0, np.float32)
    Y2 = orc.ffn_fwd(X, idx, goe, W1, W2, W3, 1, "swiglu", [0])
    assert np.allclose(Y2, 2.0 * Y, rtol=1e-14)                                   # linear in the u branch


@pytest.mark.parametrize("ci", [0, 1])
def test_combine_identity_experts_and_plan_invariance(orc, ci):
    cfg = _tiny(ci, T=200, d=16)
    inp, r, dest, lay, goe = _routed(orc, cfg)
    X64 = inp["X"].astype(np.float64)
    Yp = orc.dispatch(inp["X"], lay["perm"], cfg.k).astype(np.float64)            # identity experts everywhere
    out = orc.combine(Yp, lay["pos"], r["w"], cfg.k)
    assert np.allclose(out, X64 * r["w"].sum(axis=1, keepdims=True), rtol=1e-13, atol=1e-14)
    if cfg.renorm:
        assert np.allclose(out, X64, rtol=1e-13, atol=1e-14)
    # values do not depend on the placement: a different plan gives the same output
    rng = np.random.default_rng(5)
    Ya = rng.standard_normal((cfg.A, cfg.d))                                      # per-assignment expert outputs
    outs = []
    for plan in (dest, np.array([wl.owner_of(e, cfg.E, cfg.P) for e in range(cfg.E)], np.int32),
                 np.zeros(cfg.E, np.int32), (np.arange(cfg.E) % cfg.P).astype(np.int32)):
        l2 = orc.place(r["idx"], r["counts"], plan, cfg.P)
        Yp2 = np.empty_like(Ya)
        Yp2[l2["pos"]] = Ya
        outs.append(orc.combine(Yp2, l2["pos"], r["w"], cfg.k))
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])
    ref = (Ya.reshape(cfg.T, cfg.k, cfg.d) * r["w"][:, :, None]).sum(axis=1)
    assert np.allclose(outs[0], ref, rtol=1e-13, atol=1e-14)
    # a token subset gives the same rows
    sub = np.array([3, 0, 17], np.int32)
    assert np.array_equal(orc.combine(Yp, lay["pos"], r["w"], cfg.k, sub), out[sub])


def test_adjointness_of_dispatch_and_combine(orc):
    cfg = _tiny(1, T=64, d=8)
    inp, r, dest, lay, goe = _routed(orc, cfg)
    rng = np.random.default_rng(6)
    R = rng.standard_normal((cfg.A, cfg.d))
    Xp = orc.dispatch(inp["X"], lay["perm"], cfg.k).astype(np.float64)
    lhs = float((Xp * R).sum())
    rhs = float((inp["X"].astype(np.float64) * orc.dispatch_bwd(R, lay["pos"], cfg.k)).sum())
    assert np.isclose(lhs, rhs, rtol=1e-12)
    Y = rng.standard_normal((cfg.A, cfg.d))
    G = rng.standard_normal((cfg.T, cfg.d)).astype(np.float32)
    dYp, dw = orc.combine_bwd(G, Y, lay["pos"], r["w"], cfg.k)
    lhs = float((orc.combine(Y, lay["pos"], r["w"], cfg.k) * G).sum())
    assert np.isclose(lhs, float((Y * dYp).sum()), rtol=1e-12)
    assert np.isclose(lhs, float((r["w"] * dw).sum()), rtol=1e-12)               # combine is bilinear in (w, Y)


# ---- finite differences ------------------------------------------------------------------
EPS = 2.0 ** -11


def _grid(a):
    """Snap to multiples of 2^-8 so that +-EPS perturbations are exact in fp32."""
    return (np.round(np.asarray(a, np.float64) * 256.0) / 256.0).astype(np.float32)


def _layer_loss(orc, X, idx, goe, W1, W2, W3, k, act, pos, w, G, Yfill):
    """sum(out * G) with out = combine(place(ffn(x))) ; routing (idx, w) held fixed."""
    hosted = orc.hosted_assignments(idx, goe)
    Y = orc.ffn_fwd(X, idx, goe, W1, W2, W3, k, act, hosted)
    Yp = Yfill.copy()
    Yp[pos[hosted]] = Y
    return float((orc.combine(Yp, pos, w, k) * G).sum()), Yp


@pytest.mark.parametrize("ci", [1, 3, 4])
def test_backward_vs_finite_differences(orc, ci):
    cfg = _tiny(ci, T=8, d=6, h=10, backward=True)
    inp, r, dest, lay, goe = _routed(orc, cfg)
    k, act = cfg.k, cfg.act
    idx = r["idx"].reshape(-1)
    X, W1, W2 = _grid(inp["X"]), _grid(inp["W1"] * 2), _grid(inp["W2"] * 2)
    W3 = _grid(inp["W3"] * 2) if act == "swiglu" else None
    G = inp["dOut"]
    w, pos = r["w"], lay["pos"]
    Yfill = inp["Yp_fill"].astype(np.float64)
    hosted = orc.hosted_assignments(idx, goe)
    assert 0 < hosted.size < cfg.A
    L0, Yp = _layer_loss(orc, X, idx, goe, W1, W2, W3, k, act, pos, w, G, Yfill)

    # analytic chain
    dYp, dw = orc.combine_bwd(G, Yp, pos, w, k)
    dXh = orc.ffn_bwd_rows(X, idx, goe, W1, W2, W3, k, act, hosted, dYp[pos[hosted]])
    dXp = np.zeros((cfg.A, cfg.d))                     # remote rows contribute nothing in this check
    dXp[pos[hosted]] = dXh
    dX = orc.dispatch_bwd(dXp, pos, k)
    dYa = dYp[pos].astype(np.float32)                  # by assignment; exact enough: compared at 1e-5
    Gn = int(goe.max()) + 1
    dW1, dW2, dW3 = orc.ffn_bwd_weights(X, idx, goe, W1, W2, W3, k, act, dYa, Gn)
    # the threaded form over a list of hidden units is the same call per unit: same bits, any order of units
    js = np.arange(cfg.h, dtype=np.int32)[::-1].copy()
    for g in range(Gn):
        r2, c1, c3 = orc.ffn_bwd_hidden_many(X, idx, goe, W1, W2, W3, k, act, dYa, g, js)
        assert np.array_equal(r2, dW2[g][js]) and np.array_equal(c1, dW1[g][:, js].T)
        assert c3 is None if W3 is None else np.array_equal(c3, dW3[g][:, js].T)

    def fd(arr, index, fn):
        old = arr[index]
        arr[index] = old + np.float32(EPS)
        lp = fn()
        arr[index] = old - np.float32(EPS)
        lm = fn()
        arr[index] = old
        return (lp - lm) / (2 * EPS)

    loss = lambda: _layer_loss(orc, X, idx, goe, W1, W2, W3, k, act, pos, w, G, Yfill)[0]
    rng = np.random.default_rng(9)
    scale = max(1.0, float(np.abs(dX).max()))
    for _ in range(12):
        i = (rng.integers(cfg.T), rng.integers(cfg.d))
        assert abs(fd(X, i, loss) - dX[i]) <= 2e-5 * scale, ("dX", i)
    used = sorted(set(int(goe[e]) for e in idx[hosted]))
    for name, Wm, dWm in (("dW1", W1, dW1), ("dW2", W2, dW2)) + ((("dW3", W3, dW3),) if W3 is not None else ()):
        sc = max(1.0, float(np.abs(dWm).max()))
        for _ in range(12):
            g = used[rng.integers(len(used))]
            i = (g, rng.integers(Wm.shape[1]), rng.integers(Wm.shape[2]))
            assert abs(fd(Wm, i, loss) - dWm[i]) <= 2e-5 * sc, (name, i)
        for g in range(Gn):
            if g not in used:
                assert not dWm[g].any()                # an empty group's gradient is exactly zero
    # dw: the loss is linear in w, so a difference is exact
    for a in range(cfg.A):
        t, j = divmod(a, k)
        w2 = w.copy()
        w2[t, j] += 0.5
        lp = _layer_loss(orc, X, idx, goe, W1, W2, W3, k, act, pos, w2, G, Yfill)[0]
        assert np.isclose((lp - L0) / 0.5, dw[t, j], rtol=1e-9, atol=1e-9)


@pytest.mark.parametrize("k,renorm,E", [(1, 0, 8), (2, 1, 8), (2, 0, 5), (3, 1, 6)])
def test_gate_bwd_vs_finite_differences(orc, k, renorm, E):
    rng = np.random.default_rng(20 + k + renorm)
    T = 6
    logits = _grid(rng.standard_normal((T, E)) * 1.5)
    idx, w, p = orc.topk(logits, k, renorm)
    dw = rng.standard_normal((T, k))
    dl = orc.gate_bwd(dw, logits, idx, renorm)
    assert np.allclose(dl.sum(axis=1), 0.0, atol=1e-14)           # softmax Jacobian has zero row sums
    if renorm:
        mask = np.ones((T, E), bool)
        np.put_along_axis(mask, idx.astype(np.int64), False, axis=1)
        assert not dl[mask].any()

    def wsel(lg):
        """Gate weights with the selection held fixed, straight from the definition."""
        pe = np.exp(lg.astype(np.float64) - lg.max(axis=1, keepdims=True))
        pe /= pe.sum(axis=1, keepdims=True)
        ws = np.take_along_axis(pe, idx.astype(np.int64), axis=1)
        return ws / ws.sum(axis=1, keepdims=True) if renorm else ws

    assert np.allclose(wsel(logits), w, rtol=1e-13)
    eps = 2.0 ** -10
    for t in range(T):
        for e in range(E):
            lp, lm = logits.copy(), logits.copy()
            lp[t, e] += np.float32(eps)
            lm[t, e] -= np.float32(eps)
            num = ((wsel(lp) - wsel(lm)) * dw).sum() / (2 * eps)
            assert abs(num - dl[t, e]) <= 1e-5 * max(1.0, np.abs(dl).max()), (t, e)


def test_gate_linear_backward_vs_matmul_and_finite_differences(orc):
    """The gate is linear in Wg, b and X (Section 2.1), so its backward is two matrix products: checked
    against numpy's, and against central differences of <logits, dlogits> with exactly representable steps."""
    rng = np.random.default_rng(77)
    T, d, E, k = 9, 12, 5, 2
    X = _grid(rng.standard_normal((T, d)))
    Wg = _grid(rng.standard_normal((d, E)) * 0.5)
    bg = _grid(rng.standard_normal(E))
    dl = rng.standard_normal((T, E))
    dWg, dbg = orc.gate_bwd_params(X, dl)
    assert np.allclose(dWg, X.astype(np.float64).T @ dl, rtol=1e-13, atol=1e-13)
    assert np.allclose(dbg, dl.sum(axis=0), rtol=1e-13, atol=1e-13)
    assert dWg.shape == (d, E) and not np.allclose(dWg, (X.astype(np.float64).T @ dl).T.reshape(d, E))   # not the transpose

    def inner(Xv, Wv, bv):                                   # <logits, dlogits> in double from the definition
        return float(((Xv.astype(np.float64) @ Wv.astype(np.float64) + bv.astype(np.float64)) * dl).sum())

    eps = np.float32(2.0 ** -6)
    for (c, e) in [(0, 0), (3, 4), (11, 2)]:
        Wp, Wm = Wg.copy(), Wg.copy()
        Wp[c, e] += eps; Wm[c, e] -= eps
        assert abs((inner(X, Wp, bg) - inner(X, Wm, bg)) / (2 * float(eps)) - dWg[c, e]) < 1e-9
    for e in range(E):
        bp, bm = bg.copy(), bg.copy()
        bp[e] += eps; bm[e] -= eps
        assert abs((inner(X, Wg, bp) - inner(X, Wg, bm)) / (2 * float(eps)) - dbg[e]) < 1e-9

    # input gradient = expert path (sum of the k returned rows) + gate path dlogits Wg^T
    A = T * k
    pos = rng.permutation(A).astype(np.int32)
    dXp = rng.standard_normal((A, d))
    dX = orc.input_grad(dXp, pos, dl, Wg, k)
    assert np.allclose(dX, orc.dispatch_bwd(dXp, pos, k) + dl @ Wg.astype(np.float64).T, rtol=1e-13, atol=1e-13)
    for (t, c) in [(0, 0), (4, 7), (8, 11)]:
        Xp_, Xm_ = X.copy(), X.copy()
        Xp_[t, c] += eps; Xm_[t, c] -= eps
        gate_path = (inner(Xp_, Wg, bg) - inner(Xm_, Wg, bg)) / (2 * float(eps))
        expert_path = sum(dXp[pos[t * k + j], c] for j in range(k))
        assert abs(gate_path + expert_path - dX[t, c]) < 1e-9
    # with dlogits = 0 the gate path vanishes and the result is the plain backward of the send
    assert np.array_equal(orc.input_grad(dXp, pos, np.zeros((T, E)), Wg, k), orc.dispatch_bwd(dXp, pos, k))
