"""Seeded synthetic workloads for one GPU's share of an expert-parallel MoE layer.

This module only *draws inputs* (tokens, gate parameters, expert weights, upstream
gradients, the rows a return all-to-all would have delivered) and builds the
placement input (`expert_dest`).  It holds none of the layer's arithmetic: no gate,
no routing, no FFN.  Both the CPU oracle's tests and the GPU tests draw from here so
that the two sides see the same bits.

The shapes stand in for the paper's workloads (Section 6.1: 16384 / 32768 tokens per
iteration, one expert per device, k in {1, 2}) and its imbalance profile (Fig. 3: at
16 experts the three heaviest hold more than half of the inputs, the three lightest
under 5 %).  The skew is produced by a per-expert gate bias b_e = -alpha * ln(rank_e)
with rank a seeded permutation of 1..E; the unit-variance noise of X @ Wg spreads it.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np

BASE_SEED = 20241110


@dataclass(frozen=True)
class MoEConfig:
    name: str
    index: int
    T: int            # tokens held by this GPU
    d: int            # model width
    h: int            # expert hidden width
    E: int            # experts in the layer
    k: int            # experts per token
    P: int            # virtual destinations (devices of the expert-parallel group)
    dtype: str        # "f32" | "bf16": storage type of activations and expert weights
    act: str          # "gelu" | "swiglu"
    renorm: int       # 1: the k gate weights are renormalised to sum to one
    alpha: float      # skew of the gate bias
    n_replicas: int   # heavy experts replicated onto this GPU by the plan (upper bound for cfg 4)
    backward: bool
    self_dest: int = 0
    iterations: int = 1

    @property
    def A(self) -> int:
        return self.T * self.k

    @property
    def experts_per_dest(self) -> int:
        return self.E // self.P

    @property
    def n_owned(self) -> int:
        return self.experts_per_dest

    @property
    def G_max(self) -> int:
        return self.n_owned + self.n_replicas

    @property
    def n_mats(self) -> int:
        return 3 if self.act == "swiglu" else 2


CONFIGS: List[MoEConfig] = [
    MoEConfig("cfg0_tiny_f32_fwd", 0, T=512, d=64, h=256, E=8, k=1, P=4, dtype="f32", act="gelu",
              renorm=0, alpha=1.2, n_replicas=0, backward=False),
    MoEConfig("cfg1_bf16_fwd", 1, T=8192, d=1024, h=4096, E=16, k=2, P=8, dtype="bf16", act="gelu",
              renorm=1, alpha=1.0, n_replicas=2, backward=False),
    MoEConfig("cfg2_bf16_fwd_bwd", 2, T=16384, d=2048, h=8192, E=32, k=2, P=8, dtype="bf16", act="gelu",
              renorm=1, alpha=1.2, n_replicas=4, backward=True),
    MoEConfig("cfg3_bf16_swiglu_fwd_bwd", 3, T=32768, d=4096, h=14336, E=16, k=2, P=8, dtype="bf16",
              act="swiglu", renorm=1, alpha=1.5, n_replicas=2, backward=True),
    MoEConfig("cfg4_bf16_drift_sweep", 4, T=16384, d=2048, h=8192, E=64, k=1, P=16, dtype="bf16", act="gelu",
              renorm=0, alpha=0.0, n_replicas=4, backward=True, iterations=10),
]

CFG4_ALPHAS = (0.0, 0.8, 1.5)


def scaled(cfg: MoEConfig, **kw) -> MoEConfig:
    """A copy of `cfg` with some fields replaced (smaller shapes for fast tests)."""
    return dataclasses.replace(cfg, **kw)


def seed_for(cfg_index: int, iteration: int = 0) -> int:
    return BASE_SEED + 1000 * cfg_index + iteration


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round an fp32 array to the nearest bf16 value (ties to even), in place; stays fp32."""
    assert a.dtype == np.float32
    u = a.reshape(-1).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    u += lsb + np.uint32(0x7FFF)
    u &= np.uint32(0xFFFF0000)
    return a


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """The upper 16 bits of fp32 values that are already bf16-representable."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value is not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def _normal(rng: np.random.Generator, shape, std: float, dtype: str) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if dtype == "bf16":
        round_to_bf16(a)
    return a


def owner_of(e: int, E: int, P: int) -> int:
    """Expert parallelism divides the experts evenly, in contiguous blocks (Section 2.1)."""
    return e // (E // P)


def draw_rank(cfg: MoEConfig, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.permutation(cfg.E).astype(np.int64) + 1


def alpha_for(cfg: MoEConfig, iteration: int) -> float:
    if cfg.index == 4:
        return CFG4_ALPHAS[iteration % 3]
    return cfg.alpha


def make_inputs(cfg: MoEConfig, iteration: int = 0, *, with_weights: bool = True,
                base_seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Draw every input of one layer pass.  Draw order: rank, X, Wg, W1, W2, (W3), dOut,
    Yp fill, dXp fill.  All arrays are fp32; under dtype "bf16" the values of X, the
    expert weights, dOut and the fills are bf16-representable (rounded once, here).

    For the drift sweep (cfg 4) the rank permutation comes from the seed of iteration
    3*(i//3) (it is re-drawn every third iteration), the gate matrix and expert weights
    from the seed of iteration 0 (parameters drift slowly), the rest from iteration i.
    """
    ci = cfg.index
    s_iter = (base_seed if base_seed is not None else seed_for(ci, 0)) + iteration
    s_base = s_iter - iteration
    s_rank = s_base + 3 * (iteration // 3)
    alpha = alpha_for(cfg, iteration)

    out: Dict[str, np.ndarray] = {}
    rank = draw_rank(cfg, s_rank)
    out["rank"] = rank
    out["bg"] = (-alpha * np.log(rank.astype(np.float64))).astype(np.float32)

    rng_x = np.random.default_rng([s_iter, 1])
    out["X"] = _normal(rng_x, (cfg.T, cfg.d), 1.0, cfg.dtype)

    rng_p = np.random.default_rng([s_base, 2])
    out["Wg"] = _normal(rng_p, (cfg.d, cfg.E), cfg.d ** -0.5, "f32")
    if with_weights:
        G = cfg.G_max
        out["W1"] = _normal(rng_p, (G, cfg.d, cfg.h), cfg.d ** -0.5, cfg.dtype)
        out["W2"] = _normal(rng_p, (G, cfg.h, cfg.d), cfg.h ** -0.5, cfg.dtype)
        if cfg.act == "swiglu":
            out["W3"] = _normal(rng_p, (G, cfg.d, cfg.h), cfg.d ** -0.5, cfg.dtype)

    rng_g = np.random.default_rng([s_iter, 3])
    if cfg.backward:
        out["dOut"] = _normal(rng_g, (cfg.T, cfg.d), 1.0, cfg.dtype)
    out["Yp_fill"] = _normal(rng_g, (cfg.A, cfg.d), 1.0, cfg.dtype)
    if cfg.backward:
        out["dXp_fill"] = _normal(rng_g, (cfg.A, cfg.d), 1.0, cfg.dtype)
    return out


def make_plan(cfg: MoEConfig, counts: Sequence[int], *, threshold: bool = False) -> np.ndarray:
    """Stand-in for the planner's output: `expert_dest[e]`, the destination that computes this
    GPU's tokens of expert e.  Owned experts and the replicated heavy ones stay here; every
    other expert goes to its owner (lightweight expert placement, Section 4.1).

    Replicas are the `n_replicas` experts with the most inputs among those this GPU does not
    own (ties to the lower id).  With `threshold` an expert is only replicated when its load
    exceeds twice the mean, a one-expert form of the balance test (Eq. 7 with alpha = 1).
    """
    counts = np.asarray(counts, dtype=np.int64)
    E, P, me = cfg.E, cfg.P, cfg.self_dest
    dest = np.array([owner_of(e, E, P) for e in range(E)], dtype=np.int32)
    cand = [e for e in range(E) if dest[e] != me]
    cand.sort(key=lambda e: (-int(counts[e]), e))
    mean = float(counts.sum()) / E
    for e in cand[: cfg.n_replicas]:
        if threshold and not counts[e] > 2.0 * mean:
            continue
        dest[e] = me
    return dest


def hosted_experts(expert_dest: np.ndarray, self_dest: int = 0) -> np.ndarray:
    """Expert ids computed on this GPU, ascending: the order of the weight groups."""
    return np.nonzero(np.asarray(expert_dest) == self_dest)[0].astype(np.int32)


def group_of_expert(expert_dest: np.ndarray, self_dest: int = 0) -> np.ndarray:
    g = np.full(len(expert_dest), -1, dtype=np.int32)
    g[hosted_experts(expert_dest, self_dest)] = np.arange(int((np.asarray(expert_dest) == self_dest).sum()), dtype=np.int32)
    return g


def balance_degree(counts: Sequence[int]) -> float:
    """Standard deviation of the input distribution (Section 6.3, balance capability)."""
    return float(np.std(np.asarray(counts, dtype=np.float64)))


def make_gating(cfg: MoEConfig, counts_self: Sequence[int], iteration: int = 0, base_seed: Optional[int] = None) -> np.ndarray:
    """The P x E matrix of routing counts the planner consumes (Algorithm 1's `gating`): row
    `self_dest` is this GPU's realised histogram, every other row is a multinomial draw of the same
    number of assignments from the realised shares (devices see the same skewed distribution,
    Section 3).  Only random numbers are drawn here."""
    counts_self = np.asarray(counts_self, dtype=np.int64)
    seed = (seed_for(cfg.index, iteration) if base_seed is None else base_seed) + 500
    rng = np.random.default_rng(seed)
    A = int(counts_self.sum())
    p = counts_self.astype(np.float64) / max(A, 1)
    g = np.empty((cfg.P, cfg.E), dtype=np.int32)
    for j in range(cfg.P):
        g[j] = counts_self if j == cfg.self_dest else rng.multinomial(A, p)
    return g


def planner_constants(cfg: MoEConfig) -> dict:
    """Constants of the planner's performance model for one configuration (Table 2 of the paper):
    bytes per input / per expert from the shapes, an xGMI-class link bandwidth and an expert
    throughput of the order this library reaches.  Inputs of the harness, not measurements."""
    elt = 4 if cfg.dtype == "f32" else 2
    flops_per_input = 2.0 * cfg.n_mats * cfg.d * cfg.h
    return dict(size_input=float(cfg.d * elt), size_params=float(cfg.n_mats * cfg.d * cfg.h * elt),
                size_grads=float(cfg.n_mats * cfg.d * cfg.h * 4), B=150e9, t=1.0e15 / flops_per_input,
                T_FNEC=0.0, T_BNEC=0.0)

