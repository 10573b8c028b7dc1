"""Pins of the planner oracle (performance model Eqs. 1-6 and 8, balance test Eq. 7, Algorithm 1).

The expected numbers of the worked examples were derived by hand from the paper's rules (the trace is
written out in the docstrings), never produced by the code under test.  The property tests restate the
rules of the search as checks on its trace, using the placement's definition for the loads.
"""
import itertools

import numpy as np
import pytest

from oracle import planner_oracle as po

GATING4 = np.array([[6, 1, 1, 0],
                    [5, 2, 0, 1],
                    [4, 0, 3, 1],
                    [1, 1, 0, 6]], dtype=np.int64)


def model(**kw):
    base = dict(size_input=1.0, size_params=2.0, size_grads=2.0, B=1.0, t=1.0, alpha=0.2)
    base.update(kw)
    return po.PlannerModel(**base)


def test_equations_on_hand_numbers():
    """Eqs. 1-6 on numbers small enough to check in the head (D = 4)."""
    m = model(size_input=2.0, B=4.0, t=8.0, size_params=16.0, size_grads=8.0)
    R, H = [10, 2, 1, 2], [16, 4, 4, 8]
    assert po.t_a2a(R, m) == 10 * 2.0 / 4.0                          # Eq. 1: the slowest receiver
    assert po.t_fec(H, m) == 16 / 8.0                                # Eq. 2: the most loaded device
    assert po.t_trans(3, 1, 4, m) == 3 * (4 - 1) * 16.0 / (4 * 4.0)  # Eq. 4
    assert po.t_agg(3, 1, 4, m) == 3 * (4 - 1) * 8.0 / (4 * 4.0)     # Eq. 5
    # Eq. 6: four all-to-alls, forward + backward (= 2 x forward) expert computation, Trans, Agg
    assert po.layer_time(R, H, 3, 1, m) == 4 * 5.0 + 3 * 2.0 + 9.0 + 4.5
    assert po.layer_time(R, H, 0, 0, m) == 26.0


def test_equation_8_hides_trans_and_agg_behind_computation():
    m = model(size_input=2.0, B=4.0, t=8.0, size_params=16.0, size_grads=8.0, overlap=True, T_FNEC=1.0, T_BNEC=0.25)
    R, H = [10, 2, 1, 2], [16, 4, 4, 8]
    # T_Trans = 9 against T_FEC + T_FNEC = 2 + 1: 6 remain; T_Agg = 4.5 against T_BEC + T_BNEC = 4 + 0.25: 0.25 remain
    assert po.layer_time(R, H, 3, 1, m) == 26.0 + 6.0 + 0.25
    # fully hidden
    assert po.layer_time(R, H, 1, 3, m) == 26.0


def test_balance_condition_eq9():
    m = model(alpha=0.5)
    # I = 32 inputs, E = 4: threshold 4; the difference must be strictly below it
    assert po.balanced([9, 7, 8, 8], 32, 4, m)
    assert not po.balanced([10, 6, 8, 8], 32, 4, m)
    assert not po.balanced([16, 4, 4, 8], 32, 4, m)


def test_loads_follow_the_placement_definition():
    """Section 4.1: without replicas every input of expert e is computed by e's owner."""
    hosts = po.placement(4, 4, [], [])
    H, R = po.loads(GATING4, hosts)
    assert H.tolist() == [16, 4, 4, 8] and R.tolist() == [10, 2, 1, 2]
    # expert 0 also on devices 1 and 2: their 5 and 4 inputs stay at home
    hosts = po.placement(4, 4, [0], [[3]])
    H, R = po.loads(GATING4, hosts)
    assert H.tolist() == [7, 9, 8, 8] and R.tolist() == [1, 2, 1, 2]


def test_greedy_search_hand_trace_eq7():
    """Algorithm 1 by hand, n = 1, alpha = 0.2 (threshold 1.6), unit costs, parameters of 2 bytes.

    start   H = [16,4,4,8], R = [10,2,1,2], T' = 4*10 + 3*16 = 88
    iter 1  heaviest device 0 -> expert 0; other devices hold 5,4,1 of it: skip device 3.
            H = [7,9,8,8], R = [1,2,1,2]; Trans = Agg = 1*3*2/4 = 1.5; T' = 8 + 27 + 3 = 38 < 88: keep, cnt = 1
    iter 2  9-7 = 2 >= 1.6; heaviest device 1 -> expert 1; others hold 1,0,1: skip device 2.
            H = [8,7,8,9], R = [1,0,1,2]; T' = 8 + 27 + 6 = 41: no
    iter 3  heaviest device 3 -> expert 3; others hold 0,1,1: skip device 0.
            H = [8,8,9,7], R = [1,0,1,0]; T' = 4 + 27 + 9 = 40: no
    iter 4  heaviest device 2 -> expert 2; others hold 1,0,0: skip device 1 (tie to the lower index).
            H = [9,8,8,7], R = [1,0,0,0]; T' = 4 + 27 + 12 = 43: no
    iter 5  heaviest device 0 has been used: stop.  Output: the first selection only.
    """
    r = po.greedy_search(GATING4, 1, model())
    assert r["L"] == [0, 1, 3, 2]
    assert r["n_bottoms"] == [[3], [2], [0], [1]]
    assert [float(s["T"]) for s in r["trace"]] == [38.0, 41.0, 40.0, 43.0]
    assert [s["H"].tolist() for s in r["trace"]] == [[7, 9, 8, 8], [8, 7, 8, 9], [8, 8, 9, 7], [9, 8, 8, 7]]
    assert [s["R"].tolist() for s in r["trace"]] == [[1, 2, 1, 2], [1, 0, 1, 2], [1, 0, 1, 0], [1, 0, 0, 0]]
    assert r["cnt"] == 1 and r["T_base"] == 88.0 and r["T_output"] == 38.0
    assert r["H"].tolist() == [7, 9, 8, 8] and r["R"].tolist() == [1, 2, 1, 2]
    assert r["expert_dest"].tolist() == [[0, 1, 2, 3], [1, 1, 2, 3], [2, 1, 2, 3], [0, 1, 2, 3]]


def test_greedy_search_hand_trace_eq8():
    """Same search with Eq. 8 and T_FNEC = T_BNEC = 1: Trans and Agg (at most 6) hide behind T_FEC = 9,
    so T' = 4 T_A2A + 27: 35, 35, 31, 31.  The strict comparison keeps s = 1, then takes s = 3."""
    r = po.greedy_search(GATING4, 1, model(overlap=True, T_FNEC=1.0, T_BNEC=1.0))
    assert r["L"] == [0, 1, 3, 2]
    assert [float(s["T"]) for s in r["trace"]] == [35.0, 35.0, 31.0, 31.0]
    assert r["cnt"] == 3 and r["T_output"] == 31.0
    assert r["H"].tolist() == [8, 8, 9, 7] and r["R"].tolist() == [1, 0, 1, 0]


def test_eq8_placement_matrix():
    r = po.greedy_search(GATING4, 1, model(overlap=True, T_FNEC=1.0, T_BNEC=1.0))
    # selected: expert 0 (not on 3), expert 1 (not on 2), expert 3 (not on 0)
    hosts = r["hosts"].astype(int).tolist()
    assert hosts == [[1, 1, 0, 0],
                     [1, 1, 0, 1],
                     [1, 0, 1, 1],
                     [0, 1, 0, 1]]
    assert r["expert_dest"].tolist() == [[0, 0, 2, 3],
                                         [1, 1, 2, 1],
                                         [2, 1, 2, 2],
                                         [0, 3, 2, 3]]


def test_balanced_input_needs_no_placement():
    g = np.full((4, 8), 5, dtype=np.int64)
    r = po.greedy_search(g, 1, model(alpha=1.0))
    assert r["L"] == [] and r["cnt"] == 0 and r["T_output"] == r["T_base"]
    assert (r["expert_dest"] == np.array([e // 2 for e in range(8)])[None, :]).all()


def test_replicating_to_nobody_never_pays():
    """n = D-1 leaves one extra device per selected expert; with expensive parameters T' only grows."""
    r = po.greedy_search(GATING4, 3, model(size_params=1e6, size_grads=1e6))
    assert r["cnt"] == 0 and r["T_output"] == r["T_base"] == 88.0


def _check_trace(g, n, m):
    """The rules of Algorithm 1, restated as properties of the trace."""
    D, E = g.shape
    r = po.greedy_search(g, n, m)
    total = int(g.sum())
    per_expert = g.sum(axis=0)
    L, NB = r["L"], r["n_bottoms"]
    assert len(set(L)) == len(L)
    times = [r["T_base"]]
    for s in range(len(L) + 1):
        hosts = po.placement(D, E, L[:s], NB[:s])
        H, R = po.loads(g, hosts)
        assert int(H.sum()) == total and (R <= H).all() and (R >= 0).all()
        if s < len(L):
            assert not po.balanced(H, total, E, m)                      # the search went on
            i = int(np.argmax(H))
            e = L[s]
            assert po.owner_of(e, E, D) == i                            # from the heaviest device
            rest = [x for x in range(E) if po.owner_of(x, E, D) == i and x not in L[:s]]
            assert per_expert[e] == max(per_expert[x] for x in rest)    # its heaviest unselected expert
            assert e == min(x for x in rest if per_expert[x] == per_expert[e])
            assert len(NB[s]) == n and i not in NB[s]
            skipped = sorted(int(g[j, e]) for j in NB[s])
            others = sorted(int(g[j, e]) for j in range(D) if j != i)
            assert skipped == others[:n]                                # the n smallest holders are skipped
            times.append(po.layer_time(*po.loads(g, po.placement(D, E, L[:s + 1], NB[:s + 1]))[::-1], s + 1, n, m))
        else:                                                           # why it stopped
            i = int(np.argmax(H))
            exhausted = all(x in L for x in range(E) if po.owner_of(x, E, D) == i)
            assert po.balanced(H, total, E, m) or exhausted
    best = min(range(len(times)), key=lambda s: (times[s], s))          # first strict improvement wins ties
    assert r["cnt"] == best and r["T_output"] == times[best] <= r["T_base"]
    return r


@pytest.mark.parametrize("seed", range(12))
def test_search_rules_on_random_inputs(seed):
    rng = np.random.default_rng(1000 + seed)
    D = int(rng.choice([2, 3, 4, 8]))
    E = D * int(rng.choice([1, 2, 4]))
    p = rng.dirichlet(np.full(E, 0.3))
    g = rng.multinomial(int(rng.integers(50, 2000)), p, size=D).astype(np.int64)
    n = int(rng.integers(0, D))
    m = model(size_input=float(rng.choice([1.0, 4096.0])), size_params=float(rng.choice([2.0, 5e4, 1e6])),
              size_grads=float(rng.choice([2.0, 5e4])), B=float(rng.choice([1.0, 1e3])), t=float(rng.choice([1.0, 10.0])),
              alpha=float(rng.choice([0.1, 0.5, 1.0])), overlap=bool(seed % 2), T_FNEC=0.5, T_BNEC=1.0)
    _check_trace(g, n, m)


def test_tiny_exhaustive_never_worse_than_no_placement_and_best_prefix():
    """All 3x3 count matrices with entries in {0,1,3}: the result is the best prefix of the greedy order."""
    m = model(size_params=1.0, size_grads=1.0, alpha=0.3)
    vals = (0, 1, 3)
    for cells in itertools.product(vals, repeat=9):
        g = np.array(cells, dtype=np.int64).reshape(3, 3)
        if g.sum() == 0:
            continue
        _check_trace(g, 1, m)


def test_fixed_policies_and_balance_degree():
    """The ablation's top-r policies put the r heaviest experts everywhere (Section 6.4)."""
    hosts = po.top_policy(GATING4, 2)                     # experts 0 (16 inputs) and 3 (8 inputs)
    assert hosts.astype(int).tolist() == [[1, 0, 0, 1], [1, 1, 0, 1], [1, 0, 1, 1], [1, 0, 0, 1]]
    H, R = po.loads(GATING4, hosts)
    # inputs of experts 0 and 3 stay at home; device 1 still receives 1 + 1 inputs of expert 1, device 2 one of expert 2
    assert H.tolist() == [6, 10, 9, 7] and R.tolist() == [0, 2, 1, 0]
    assert po.balance_degree([16, 4, 4, 8]) == pytest.approx(np.sqrt(24.0))
    assert po.balance_degree(H) == pytest.approx(np.sqrt(2.5))
