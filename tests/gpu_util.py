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


def rows_close(got, want, tol: float, floor: float = 0.02, elt: float = 8.0):
    """Row-by-row comparison of two arrays whose last axis is a row.  Returns (worst row error, its row,
    worst element error in units of the row's rms, pooled rel-L2).  A row's error is ||got - want|| over
    max(||want||, floor * typical row norm): the relative L2 error of that row, with rows far below the
    typical norm measured against a floor so that an all-but-zero row does not divide by nothing."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    n = want.shape[-1] if want.ndim else 1
    g2, w2 = got.reshape(-1, n), want.reshape(-1, n)
    if w2.shape[0] == 0:
        return 0.0, -1, 0.0, 0.0
    rn = np.linalg.norm(w2, axis=1)
    typical = float(np.sqrt(np.mean(rn * rn)))
    den = np.maximum(rn, floor * typical)
    diff = g2 - w2
    if typical == 0.0:
        worst = float(np.abs(diff).max())
        return worst, int(np.argmax(np.abs(diff).max(axis=1))), worst, worst
    err = np.linalg.norm(diff, axis=1) / den
    r = int(np.argmax(err))
    elt_err = float((np.abs(diff).max(axis=1) / (den / np.sqrt(n))).max())
    return float(err[r]), r, elt_err, rel_l2(g2, w2)


def assert_rows_close(got, want, tol: float, what: str = "", floor: float = 0.02, elt: float = 8.0, report=None):
    """Every row within `tol` in relative L2, and every element within elt * tol of its row's rms: an error
    confined to one row, one tile or a few elements fails even where the norm over the whole tensor would
    hide it.  `report` (a list) collects (what, worst row error, pooled error) for printing."""
    worst, r, elt_err, pooled = rows_close(got, want, tol, floor, elt)
    if report is not None:
        report.append((what, worst, pooled))
    assert worst <= tol, f"{what}: row {r} off by {worst:.3e} (pooled {pooled:.3e}, tolerance {tol:g})"
    assert elt_err <= elt * tol, f"{what}: an element off by {elt_err:.3e} of its row's rms (allowed {elt * tol:g})"
    return worst


# ---- which tiles the grouped matrix kernel works on (the test picks its samples from this; it mirrors the
# kernel's tile walk: 256-row tiles from each group's first row, bands of 8 row tiles walked column by column,
# and the tiles left after the last full round of the chip, which are split along the contraction)
FFN_BM, FFN_SPLIT_UNITS = 256, 320
FFN_BAND = {"fwd1": 16, "fwd2": 8, "bwd1": 8, "bwd2": 8}     # row tiles per band of each contraction's tile walk


def ffn_row_tiles(group_rows):
    """[(group, first row, end row)] of every 256-row tile, in the kernel's order."""
    tiles = []
    for g, (o, e) in enumerate(group_rows):
        for r0 in range(o, e, FFN_BM):
            tiles.append((g, r0, min(r0 + FFN_BM, e)))
    return tiles


def ffn_split_tiles(total_rt: int, col_tiles: int, k_slices: int, n_blocks: int, band: int = 8):
    """(row tile, column tile) of the tiles the last, contraction-split round covers; empty if there is none."""
    n_act = total_rt * col_tiles
    n_full = (n_act // n_blocks) * n_blocks
    rem = n_act - n_full
    if rem == 0 or k_slices < 128:
        return []
    S = min(4, n_blocks // rem, max(1, k_slices // 64))
    if S <= 1 or rem * S > FFN_SPLIT_UNITS:
        return []
    out = []
    for t in range(n_full, n_act):
        b = t // (band * col_tiles)
        in_band = t - b * band * col_tiles
        band_rows = min(band, total_rt - b * band)
        out.append((b * band + in_band % band_rows, in_band // band_rows))
    return out


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

    def sample_assignments(self, n_random: int, seed: int = 0, every_tile: bool = False) -> np.ndarray:
        """Hosted assignments at group and tile boundaries plus random ones; with `every_tile` also one row,
        at a random place, in every 256-row tile of every hosted group (the last, ragged tile included)."""
        rng = np.random.default_rng(seed)
        rows = []
        for g in range(self.G):
            o, e = self.group_rows(g)
            for r in (o, o + 1, o + 255, o + 256, o + 257, e - 2, e - 1):
                if o <= r < e:
                    rows.append(r)
        if every_tile:
            for _, r0, r1 in ffn_row_tiles([self.group_rows(g) for g in range(self.G)]):
                rows.append(int(rng.integers(r0, r1)))
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
