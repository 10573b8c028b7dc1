"""Pins of the oracle's routing half (gate logits, top-k, weights, counts, layout, positions,
dispatch) against things that are not the oracle: exact rational arithmetic, brute force,
closed forms, numpy library routines and the totals of the paper's Fig. 6 example."""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2411_10003_amd import workload as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---- exact fp32 arithmetic on rationals (independent of C's fmaf) ------------------------
def _round_f32(q: Fraction) -> Fraction:
    """Round a rational to the nearest fp32 value, ties to even (no overflow handling)."""
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    e = 0
    # find e with 2^23 <= a / 2^e < 2^24, clamped at the subnormal exponent
    while a / Fraction(2) ** e >= 2 ** 24:
        e += 1
    while a / Fraction(2) ** e < 2 ** 23 and e > -149:
        e -= 1
    m = a / Fraction(2) ** e
    fl = m.numerator // m.denominator
    rem = m - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return sign * fl * Fraction(2) ** e


def _column_order(d):
    """(block, column) in the order of the reading: blocks of 32 columns; position n of a block is
    its column 8 * (n % 4) + n // 4; columns at or past d are skipped."""
    return [(blk, 32 * blk + 8 * (n % 4) + n // 4) for blk in range((d + 31) // 32) for n in range(32)
            if 32 * blk + 8 * (n % 4) + n // 4 < d]


def _logit_exact_order(x, wcol, b):
    """The fixed summation order, written with rationals: two partial sums fed by alternating
    blocks of 32 columns, one fused multiply-add per column, (s0 + s1) + bias."""
    s = [Fraction(0), Fraction(0)]
    for blk, c in _column_order(len(x)):
        s[blk % 2] = _round_f32(Fraction(float(x[c])) * Fraction(float(wcol[c])) + s[blk % 2])
    return _round_f32(_round_f32(s[0] + s[1]) + Fraction(float(b)))


def test_column_order_is_a_permutation_with_the_stated_head():
    order = [c for _, c in _column_order(100)]
    assert sorted(order) == list(range(100))
    assert order[:9] == [0, 8, 16, 24, 1, 9, 17, 25, 2]
    assert order[32:36] == [32, 40, 48, 56]
    assert order[-4:] == [96, 97, 98, 99]          # the last block keeps only columns below d


@pytest.mark.parametrize("d", [24, 64, 100, 192, 257])
def test_logits_bitwise_vs_rational_fma(orc, d):
    rng = np.random.default_rng(d)
    T, E = 3, 4
    X = rng.standard_normal((T, d)).astype(np.float32)
    Wg = (rng.standard_normal((d, E)) / np.sqrt(d)).astype(np.float32)
    bg = rng.standard_normal(E).astype(np.float32)
    got = orc.gate_logits(X, Wg, bg)
    for t in range(T):
        for e in range(E):
            want = _logit_exact_order(X[t], Wg[:, e], bg[e])
            assert Fraction(float(got[t, e])) == want, (t, e)


def test_logits_close_to_fp64_and_layout_of_Wg(orc):
    rng = np.random.default_rng(7)
    T, d, E = 33, 320, 6          # E != d, so a transposed Wg cannot pass
    X = rng.standard_normal((T, d)).astype(np.float32)
    Wg = rng.standard_normal((d, E)).astype(np.float32)
    bg = rng.standard_normal(E).astype(np.float32)
    got = orc.gate_logits(X, Wg, bg).astype(np.float64)
    ref = X.astype(np.float64) @ Wg.astype(np.float64) + bg.astype(np.float64)
    bound = 1e-5 * (np.linalg.norm(X, axis=1)[:, None] * np.linalg.norm(Wg, axis=0)[None, :] + np.abs(bg))
    assert np.all(np.abs(got - ref) <= bound)


def test_logits_zero_gate_matrix_returns_bias_exactly(orc):
    rng = np.random.default_rng(8)
    X = rng.standard_normal((5, 130)).astype(np.float32)
    bg = rng.standard_normal(9).astype(np.float32)
    got = orc.gate_logits(X, np.zeros((130, 9), np.float32), bg)
    assert np.array_equal(got, np.broadcast_to(bg, (5, 9)))


# ---- top-k ------------------------------------------------------------------------------
def _brute_topk(row, k):
    v = [(-np.inf if np.isnan(x) else float(x)) for x in row]
    order = sorted(range(len(v)), key=lambda e: (-v[e], e))
    return order[:k]


@pytest.mark.parametrize("k", [1, 2, 3])
def test_topk_vs_bruteforce_sort_with_ties(orc, k):
    rng = np.random.default_rng(11 + k)
    T, E = 400, 7
    logits = rng.integers(-2, 3, size=(T, E)).astype(np.float32)   # many exact ties
    logits[5, :] = 0.0
    logits[6, 2] = -0.0
    logits[7, 3] = np.nan
    logits[8, :] = np.nan
    idx, w, p = orc.topk(logits, k, 0)
    for t in range(T):
        assert list(idx[t]) == _brute_topk(logits[t], k), t


def test_topk_zero_gate_picks_lowest_ranks(orc):
    cfg = wl.scaled(wl.CONFIGS[1], T=64, d=64)
    inp = wl.make_inputs(cfg, with_weights=False)
    r = orc.route(inp["X"], np.zeros_like(inp["Wg"]), inp["bg"], cfg.k, cfg.renorm)
    best = np.argsort(inp["rank"], kind="stable")[: cfg.k]       # rank 1 has the largest bias
    assert np.array_equal(r["idx"], np.broadcast_to(best.astype(np.int32), (cfg.T, cfg.k)))
    expect = np.zeros(cfg.E, np.int32)
    expect[best] = cfg.T
    assert np.array_equal(r["counts"], expect)


def test_topk_duplicate_columns_tie_to_lowest_index(orc):
    rng = np.random.default_rng(12)
    T, d, E = 50, 128, 6
    X = rng.standard_normal((T, d)).astype(np.float32)
    col = rng.standard_normal(d).astype(np.float32)
    Wg = np.repeat(col[:, None], E, axis=1)
    r = orc.route(X, Wg, np.zeros(E, np.float32), 2, 1)
    assert np.array_equal(r["idx"], np.broadcast_to(np.array([0, 1], np.int32), (T, 2)))


def test_topk_k_equals_E_is_a_permutation(orc):
    rng = np.random.default_rng(13)
    logits = rng.standard_normal((100, 2)).astype(np.float32)
    idx, w, p = orc.topk(logits, 2, 1)
    assert np.array_equal(np.sort(idx, axis=1), np.broadcast_to(np.array([0, 1], np.int32), (100, 2)))
    assert np.array_equal(idx[:, 0], (logits[:, 1] > logits[:, 0]).astype(np.int32))


# ---- gate weights -----------------------------------------------------------------------
def test_weights_closed_forms(orc):
    rng = np.random.default_rng(14)
    logits = rng.standard_normal((200, 2)).astype(np.float32) * 3
    idx, w, p = orc.topk(logits, 1, 0)
    diff = np.abs(logits[:, 0].astype(np.float64) - logits[:, 1].astype(np.float64))
    assert np.allclose(w[:, 0], 1.0 / (1.0 + np.exp(-diff)), rtol=1e-14)        # E = 2: a sigmoid
    logits = rng.standard_normal((200, 9)).astype(np.float32) * 2
    idx, w, p = orc.topk(logits, 1, 0)
    ref = np.exp(logits.astype(np.float64))
    ref /= ref.sum(axis=1, keepdims=True)
    assert np.allclose(p, ref, rtol=1e-13)
    assert np.allclose(w[:, 0], ref.max(axis=1), rtol=1e-13)
    assert np.all(w > 1.0 / 9) and np.all(w <= 1.0)
    idx, w, p = orc.topk(logits, 2, 1)
    assert np.allclose(w.sum(axis=1), 1.0, rtol=1e-14)
    l2 = np.take_along_axis(logits.astype(np.float64), idx.astype(np.int64), axis=1)
    sm = np.exp(l2 - l2.max(axis=1, keepdims=True))
    sm /= sm.sum(axis=1, keepdims=True)
    assert np.allclose(w, sm, rtol=1e-13)                                       # softmax of the two selected
    assert np.all(w[:, 0] >= w[:, 1])                                           # best first


# ---- counts / layout / positions / dispatch ---------------------------------------------
@pytest.mark.parametrize("ci", [0, 1, 4])
def test_counts_layout_positions_vs_numpy(orc, ci):
    cfg = wl.scaled(wl.CONFIGS[ci], T=777, d=64)
    inp = wl.make_inputs(cfg, iteration=2, with_weights=False)
    r = orc.route(inp["X"], inp["Wg"], inp["bg"], cfg.k, cfg.renorm)
    idx = r["idx"].reshape(-1)
    cnt = r["counts"]
    assert np.array_equal(cnt, np.bincount(idx, minlength=cfg.E))
    assert int(cnt.sum()) == cfg.T * cfg.k
    dest = wl.make_plan(cfg, cnt)
    lay = orc.place(r["idx"], cnt, dest, cfg.P)
    so, do, ds, soe = lay["slot_offsets"], lay["dest_offsets"], lay["dest_slots"], lay["slot_of_expert"]
    A = cfg.A
    # offsets
    assert so[0] == 0 and so[-1] == A and np.all(np.diff(so) >= 0)
    assert do[0] == 0 and do[-1] == A and ds[0] == 0 and ds[-1] == cfg.E
    for p in range(cfg.P):
        assert do[p] == so[ds[p]]
        assert do[p + 1] - do[p] == int(cnt[dest == p].sum())
        assert ds[p + 1] - ds[p] == int((dest == p).sum())
    # slot order is (destination, expert)
    order = sorted(range(cfg.E), key=lambda e: (int(dest[e]), e))
    assert [int(soe[e]) for e in order] == list(range(cfg.E))
    # permutation: bijection, inverse, purity, stability, library stable sort
    pos, perm = lay["pos"], lay["perm"]
    assert np.array_equal(np.sort(perm), np.arange(A))
    assert np.array_equal(perm[pos], np.arange(A))
    key = soe[idx]
    assert np.array_equal(perm, np.argsort(key, kind="stable"))
    for e in range(cfg.E):
        s = soe[e]
        rows = perm[so[s]:so[s + 1]]
        assert np.all(idx[rows] == e)
        assert np.all(np.diff(rows) > 0)
    # dispatch
    Xp = orc.dispatch(inp["X"], perm, cfg.k)
    assert np.array_equal(Xp, inp["X"][perm // cfg.k])


def test_layout_rejects_bad_destination(orc):
    with pytest.raises(ValueError):
        orc.layout(np.array([1, 2], np.int32), np.array([0, 5], np.int32), 2)


def _read_golden():
    vals = {}
    with open(os.path.join(GOLDEN, "fig6_placement_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *rest = line.split()
            vals[key] = [int(x) for x in rest]
    return vals


def test_fig6_example_counts_and_replica_purity(orc):
    g = _read_golden()
    E, P = g["experts"][0], g["devices"][0]
    # nine inputs whose best expert is fixed by a one-hot feature; identity gate
    experts = [0, 1, 0, 2, 0, 0, 1, 0, 2]
    X = np.zeros((9, 64), np.float32)
    for t, e in enumerate(experts):
        X[t, e] = 4.0
        X[t, 3:] = np.float32(0.01 * t)
    Wg = np.zeros((64, E), np.float32)
    Wg[:E, :E] = np.eye(E, dtype=np.float32)
    r = orc.route(X, Wg, np.zeros(E, np.float32), 1, 0)
    assert list(r["counts"]) == g["counts"]
    for key, me in (("expert_dest_dev1", 1), ("expert_dest_dev0", 0)):
        dest = np.array(g[key], np.int32)
        lay = orc.place(r["idx"], r["counts"], dest, P)
        do = lay["dest_offsets"]
        # rows kept on this device = inputs of the experts placed on it; the rest go to the owner
        assert do[me + 1] - do[me] == sum(c for c, p in zip(g["counts"], g[key]) if p == me)
        for e in range(E):
            s = lay["slot_of_expert"][e]
            rows = lay["perm"][lay["slot_offsets"][s]:lay["slot_offsets"][s + 1]]
            assert [experts[a] for a in rows] == [e] * g["counts"][e]
            assert np.all(rows >= 0)
            assert do[dest[e]] <= lay["slot_offsets"][s] <= do[dest[e] + 1]


def test_skew_generator_matches_fig3_band():
    """Fig. 3: at 16 experts the three heaviest hold > 50 % of the inputs, the three lightest < 5 %.
    The generator's bias alone (softmax of -alpha ln rank, alpha = 1.2) sits inside that band."""
    rank = np.arange(1, 17, dtype=np.float64)
    share = rank ** -1.2
    share /= share.sum()
    assert share[:3].sum() > 0.5 and share[-3:].sum() < 0.05


def test_make_plan_replicates_heaviest_not_owned():
    cfg = wl.CONFIGS[1]
    cnt = np.arange(16)[::-1].copy()         # expert 0 heaviest; 0,1 owned by destination 0
    dest = wl.make_plan(cfg, cnt)
    assert list(wl.hosted_experts(dest)) == [0, 1, 2, 3]
    cnt[[2, 9]] = 100
    dest = wl.make_plan(cfg, cnt)
    assert list(wl.hosted_experts(dest)) == [0, 1, 2, 9]
    assert dest[5] == 2 and dest[15] == 7
    cfg4 = wl.CONFIGS[4]
    flat = np.full(64, 256)
    assert list(wl.hosted_experts(wl.make_plan(cfg4, flat, threshold=True))) == [0, 1, 2, 3]
