"""CPU oracle of the planner -- TEST INFRASTRUCTURE, NOT PRODUCT.

Plain Python/NumPy statement of the paper's performance model (Section 4.2, Eqs. 1-6; Section 5.3,
Eq. 8) and of its greedy search (Section 4.3, Algorithm 1, balance test of Eq. 7).  Only tests, the
smoke check and the benchmark's CPU-baseline leg import this module; it imports nothing from the GPU
package.  Slow on purpose: after every selection the per-device loads are recomputed from the
definition of a lightweight placement (Section 4.1), never updated in place.

Notation follows the paper: D devices, E experts, `gating[i][e]` = inputs on device i routed to
expert e, H[i] = inputs computed on device i, R[i] = inputs device i receives from other devices,
s = number of selected experts, n = devices a selected expert is not transferred to.

Readings where Algorithm 1 is silent or garbled (each is also listed in the design notes):
  * H and R are computed before the first evaluation of T'; `Used` starts empty.
  * The paper has one expert per device and appends the device index to the expert list.  With
    E/D experts per device (contiguous blocks, Section 2.1) the heaviest device contributes its
    unselected expert with the most inputs (ties: lowest id); the search stops when the heaviest
    device has no unselected expert left, which is the paper's `i in Used` when E = D.
  * The loop runs while the load is NOT balanced.
  * BottomK looks at the devices other than the owner (the owner always holds the parameters) and
    takes the n smallest counts, ties to the lower device index.
  * arg max over devices: ties to the lower index.
  * "3 T_FEC" = T_FEC + T_BEC with T_BEC = 2 T_FEC (Eqs. 2-3); in Eq. 8, T_BEC = 2 T_FEC.
  * All times are IEEE doubles evaluated in the association order written in `layer_time`; the
    comparison `T_changed < T_output` is strict.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Sequence

import numpy as np


@dataclass(frozen=True)
class PlannerModel:
    """Constants of the performance model (Table 2 of the paper), SI units."""
    size_input: float          # bytes of one input
    size_params: float         # bytes of one expert's parameters
    size_grads: float          # bytes of one expert's gradients
    B: float                   # average communication bandwidth, bytes/s
    t: float                   # computation throughput, inputs/s
    T_FNEC: float = 0.0        # forward time of the non-MoE layer (Eq. 8 only)
    T_BNEC: float = 0.0        # backward time of the non-MoE layer (Eq. 8 only)
    overlap: bool = False      # False: Eq. 6, True: Eq. 8
    alpha: float = 1.0         # coefficient of the balance test (Eq. 7)


def owner_of(e: int, E: int, D: int) -> int:
    """Expert parallelism gives every device E/D consecutive experts (Section 2.1)."""
    return e // (E // D)


def loads(gating: np.ndarray, hosts: np.ndarray) -> (np.ndarray, np.ndarray):
    """H and R of a lightweight placement, from its definition (Section 4.1): device j computes its
    own inputs of expert e if it holds e's parameters, otherwise it sends them to e's owner."""
    D, E = gating.shape
    H = np.zeros(D, dtype=np.int64)
    R = np.zeros(D, dtype=np.int64)
    for j in range(D):
        for e in range(E):
            c = int(gating[j, e])
            o = owner_of(e, E, D)
            if hosts[j, e]:
                H[j] += c
            else:
                H[o] += c
                R[o] += c
    return H, R


def t_a2a(R: Sequence[int], m: PlannerModel) -> float:
    """Eq. 1."""
    return (float(max(int(r) for r in R)) * m.size_input) / m.B


def t_fec(H: Sequence[int], m: PlannerModel) -> float:
    """Eq. 2 (Eq. 3 is twice this)."""
    return float(max(int(h) for h in H)) / m.t


def t_trans(s: int, n: int, D: int, m: PlannerModel) -> float:
    """Eq. 4."""
    return (float(s) * float(D - n) * m.size_params) / (float(D) * m.B)


def t_agg(s: int, n: int, D: int, m: PlannerModel) -> float:
    """Eq. 5."""
    return (float(s) * float(D - n) * m.size_grads) / (float(D) * m.B)


def layer_time(R: Sequence[int], H: Sequence[int], s: int, n: int, m: PlannerModel) -> float:
    """T'(R, H, s, n): Eq. 6, or Eq. 8 when the scheduler hides Trans and Agg behind computation."""
    D = len(H)
    a2a = t_a2a(R, m)
    fec = t_fec(H, m)
    base = 4.0 * a2a + 3.0 * fec
    tr = t_trans(s, n, D, m)
    ag = t_agg(s, n, D, m)
    if not m.overlap:
        return (base + tr) + ag
    bec = 2.0 * fec
    ptr = max(0.0, (tr - fec) - m.T_FNEC)
    pag = max(0.0, (ag - bec) - m.T_BNEC)
    return (base + ptr) + pag


def balanced(H: Sequence[int], total_inputs: int, E: int, m: PlannerModel) -> bool:
    """Eq. 7: max(H) - min(H) < alpha * I / E."""
    return float(int(max(H)) - int(min(H))) < (m.alpha * float(total_inputs)) / float(E)


def bottom_k(gating: np.ndarray, e: int, n: int) -> List[int]:
    """The n devices, owner excluded, with the fewest inputs of expert e (ties: lower index)."""
    D, E = gating.shape
    o = owner_of(e, E, D)
    cand = [j for j in range(D) if j != o]
    cand.sort(key=lambda j: (int(gating[j, e]), j))
    return sorted(cand[:n])


def placement(D: int, E: int, L: Sequence[int], n_bottoms: Sequence[Sequence[int]]) -> np.ndarray:
    """Get_PoE: hosts[j][e] for the selected experts L and the devices they skip."""
    hosts = np.zeros((D, E), dtype=bool)
    for e in range(E):
        hosts[owner_of(e, E, D), e] = True
    for e, nb in zip(L, n_bottoms):
        for j in range(D):
            if j not in nb:
                hosts[j, e] = True
    return hosts


def next_selection(gating: np.ndarray, H: np.ndarray, chosen: Sequence[int], n: int):
    """One step of the search (Section 4.3): the device with the largest load (ties: lowest index) gives up its
    heaviest expert that has not been selected yet (ties: lowest id), and the n devices that hold the fewest of
    that expert's inputs do not receive it.  None when that device has no expert left to give."""
    D, E = gating.shape
    heaviest = int(np.argmax(H))
    totals = gating.sum(axis=0)
    left = [e for e in range(E) if owner_of(e, E, D) == heaviest and e not in chosen]
    if not left:
        return None
    e_sel = min(left, key=lambda e: (-int(totals[e]), e))
    return heaviest, e_sel, bottom_k(gating, e_sel, n)


def greedy_search(gating: np.ndarray, n: int, m: PlannerModel) -> Dict[str, object]:
    """The greedy search of Section 4.3 (Algorithm 1), stated as: grow a chain of placements, each adding one
    selection to the one before, until the load is balanced or the heaviest device has nothing left; evaluate
    every placement of the chain with the performance model from its own definition; return the first placement
    of the chain whose time is the smallest (a later one has to be strictly faster to be preferred)."""
    gating = np.asarray(gating, dtype=np.int64)
    D, E = gating.shape
    assert E % D == 0 and 0 <= n <= D - 1
    total = int(gating.sum())

    chain = [([], [])]                                     # (selected experts, devices each of them skips)
    donors = []
    while True:
        experts, skipped = chain[-1]
        H, _ = loads(gating, placement(D, E, experts, skipped))
        if balanced(H, total, E, m):
            break
        step = next_selection(gating, H, experts, n)
        if step is None:
            break
        device, e_sel, nb = step
        donors.append(device)
        chain.append((experts + [e_sel], skipped + [nb]))

    evaluated = []
    for experts, skipped in chain:
        H, R = loads(gating, placement(D, E, experts, skipped))
        s = len(experts)
        evaluated.append((layer_time(R, H, s, n if s else 0, m), H, R))
    times = [t for t, _, _ in evaluated]
    cnt = min(range(len(chain)), key=lambda i: (times[i], i))          # first of the smallest times
    L, n_bottoms = chain[-1]
    trace = [dict(device=donors[i - 1], expert=L[i - 1], n_bottom=n_bottoms[i - 1], H=evaluated[i][1].copy(),
                  R=evaluated[i][2].copy(), T=times[i]) for i in range(1, len(chain))]

    hosts = placement(D, E, L[:cnt], n_bottoms[:cnt])
    expert_dest = np.empty((D, E), dtype=np.int32)
    for j in range(D):
        for e in range(E):
            expert_dest[j, e] = j if hosts[j, e] else owner_of(e, E, D)
    return dict(L=L, n_bottoms=n_bottoms, cnt=cnt, hosts=hosts, expert_dest=expert_dest,
                H=evaluated[cnt][1], R=evaluated[cnt][2], T_base=times[0], T_output=times[cnt], trace=trace)


def top_policy(gating: np.ndarray, r: int) -> np.ndarray:
    """The ablation's fixed policies (Section 6.4): the r experts with the most inputs go to all devices."""
    gating = np.asarray(gating, dtype=np.int64)
    D, E = gating.shape
    per_expert = gating.sum(axis=0)
    order = sorted(range(E), key=lambda e: (-int(per_expert[e]), e))[:r]
    return placement(D, E, order, [[] for _ in order])


def balance_degree(H: Sequence[int]) -> float:
    """Standard deviation of the load (Section 6.4, balance capability)."""
    return float(np.std(np.asarray(H, dtype=np.float64)))
