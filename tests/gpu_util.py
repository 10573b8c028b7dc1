"""Helpers of the GPU parity tests: upload seeded inputs, run the HIP path through the C ABI
binding, and compute the oracle's answers for the same inputs (complete for small cases, on
sampled rows / hidden units for the full-size configurations)."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from oracle import moe_oracle as orc
from paper_2411_10003_amd import binding
from paper_2411_10003_amd import workload as wl

DEV = "cuda:0"
TOL = {"f32": 1e-5, "bf16": 1e-2}


def dev(a: Optional[np.ndarray], dtype: str = "f32"):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype == torch.float32 and dtype == "bf16":
        return t.to(torch.bfloat16).to(DEV)        # exact: the values are bf16-representable
    return t.to(DEV)


def host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()


def rel_l2(got, want) -> float:
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    den = float(np.linalg.norm(want))
    num = float(np.linalg.norm(got - want))
    return num / den if den > 0 else num


def make_handle(cfg: wl.MoEConfig, G: Optional[int] = None) -> binding.Handle:
    return binding.Handle(T=cfg.T, d=cfg.d, h=cfg.h, E=cfg.E, k=cfg.k, P=cfg.P, self_dest=cfg.self_dest,
                          G=G if G is not None else cfg.G_max, dtype=cfg.dtype, act=cfg.act, renorm=cfg.renorm,
                          device=DEV)


class Case:
    """Inputs of one layer pass on both sides plus the oracle's routing and layout (always complete)."""

    def __init__(self, cfg: wl.MoEConfig, iteration: int = 0, plan_counts=None, expert_dest=None,
                 threshold: bool = False, base_seed=None):
        self.cfg = cfg
        self.inp = wl.make_inputs(cfg, iteration, base_seed=base_seed)
        i = self.inp
        self.route = orc.route(i["X"], i["Wg"], i["bg"], cfg.k, cfg.renorm)
        if expert_dest is None:
            basis = self.route["counts"] if plan_counts is None else plan_counts
            expert_dest = wl.make_plan(cfg, basis, threshold=threshold)
        self.expert_dest = np.asarray(expert_dest, np.int32)
        self.lay = orc.place(self.route["idx"], self.route["counts"], self.expert_dest, cfg.P)
        self.goe = wl.group_of_expert(self.expert_dest, cfg.self_dest)
        self.G = int((self.expert_dest == cfg.self_dest).sum())
        self.idx_flat = self.route["idx"].reshape(-1)
        self.hosted = orc.hosted_assignments(self.idx_flat, self.goe)
        # device copies
        dt = cfg.dtype
        self.dX = dev(i["X"], dt)
        self.dWg = dev(i["Wg"])
        self.dbg = dev(i["bg"])
        self.dW1 = dev(i["W1"], dt)
        self.dW2 = dev(i["W2"], dt)
        self.dW3 = dev(i.get("W3"), dt)
        self.ddest = dev(self.expert_dest)

    # ---- oracle pieces --------------------------------------------------------------------
    def group_rows(self, g: int):
        """(first row, end row) of hosted group g in the send layout."""
        s = int(self.lay["dest_slots"][self.cfg.self_dest]) + g
        return int(self.lay["slot_offsets"][s]), int(self.lay["slot_offsets"][s + 1])

    def oracle_ffn(self, a_list, want_hidden=False):
        i, c = self.inp, self.cfg
        return orc.ffn_fwd(i["X"], self.idx_flat, self.goe, i["W1"], i["W2"], i.get("W3"), c.k, c.act, a_list, want_hidden)

    def oracle_Yp_full(self) -> np.ndarray:
        """Send-layout outputs: oracle FFN on hosted rows, the seeded fill on the others (float64)."""
        Yp = self.inp["Yp_fill"].astype(np.float64)
        if self.hosted.size:
            Yp[self.lay["pos"][self.hosted]] = self.oracle_ffn(self.hosted)
        return Yp

    def sample_assignments(self, n_random: int, seed: int = 0) -> np.ndarray:
        """Hosted assignments at group and tile boundaries plus random ones."""
        rng = np.random.default_rng(seed)
        rows = []
        for g in range(self.G):
            o, e = self.group_rows(g)
            for r in (o, o + 1, o + 255, o + 256, o + 257, e - 2, e - 1):
                if o <= r < e:
                    rows.append(r)
        perm = self.lay["perm"]
        a = [int(perm[r]) for r in rows]
        if self.hosted.size:
            a += [int(x) for x in rng.choice(self.hosted, size=min(n_random, self.hosted.size), replace=False)]
        return np.array(sorted(set(a)), np.int32)


def gpu_route(hd: binding.Handle, case: Case, b: binding.LayerBuffers):
    hd.gate_topk(case.dX, case.dWg, case.dbg, b.logits, b.idx, b.w)
    hd.expert_counts(b.idx, b.counts)


def assert_layout_equal(b: binding.LayerBuffers, lay: Dict[str, np.ndarray]):
    L = b.layout
    for name in ("slot_of_expert", "slot_offsets", "dest_offsets", "dest_slots", "pos", "perm"):
        got = host(getattr(L, name))
        assert np.array_equal(got, lay[name]), name
