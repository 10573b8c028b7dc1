#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic tokens already resident in HBM:
gate+top-k, expert counts, placement-aware dispatch, grouped expert FFN, combine, and for the
configurations with a backward pass combine_bwd, FFN backward, dispatch_bwd and gate_bwd.
Prints one JSON line: tokens/s, the roofline of the grouped FFN kernel (bf16 MFMA) measured with
events on the launch stream, per-call times with their HBM fractions, and the CPU oracle timed on
a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "MoE-layer tokens/sec/GPU (gate+dispatch+grouped FFN+combine); FFN MFMA util"
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3        # fp32 vector
PEAK_HBM_GBS = 8000.0          # HBM3E
# HBM-side bytes of all grouped_gemm_kernel launches of one step come from rocprofv3 FETCH_SIZE / WRITE_SIZE scaled by
# a plain copy of known size; counters cannot be read from inside this run, so the figure is parsed from the committed
# summary of those two runs, which states the workload (flops per step) it was measured on.
TRAFFIC_PROFILES = {3: os.path.join(ROOT, "profiles", "grouped_gemm_cfg3_pmc_traffic.txt")}


def measured_traffic(cfg_index: int, flops_per_step: float):
    """Bytes per step from the counter summary of this configuration, or None if there is none.  The summary names
    the flops per step of the run it was taken from: a summary of another workload is an error, not a number."""
    import re
    path = TRAFFIC_PROFILES.get(cfg_index)
    if path is None or not os.path.exists(path):
        return None
    text = open(path).read()
    m = re.search(r"traffic per step = ([0-9.eE+]+) bytes.*algorithmic flops per step ([0-9.eE+]+)", text)
    if not m:
        raise SystemExit(f"bench.py: {path} has no 'traffic per step' line")
    traffic, flops = float(m.group(1)), float(m.group(2))
    if abs(flops - flops_per_step) > 2e-3 * flops_per_step:
        raise SystemExit(f"bench.py: {path} was measured on {flops:.4e} flops per step, this run does {flops_per_step:.4e}")
    return traffic


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class PowerSampler:
    """Package power from the driver's hwmon files while the timed steps run (host side, a few reads per step).
    The grouped GEMM runs at the package power cap, so its clock, and with it the attainable MFMA rate, is set by
    energy per flop; the reading goes into the result beside the nominal-peak fraction."""

    def __init__(self):
        import glob
        self.inp = (glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input")
                    or glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average") or [None])[0]
        cap = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap")
        self.cap_w = None
        try:
            if cap:
                self.cap_w = int(open(cap[0]).read()) / 1e6
        except (OSError, ValueError):
            pass
        self.samples = []
        self._stop = False
        self._thread = None

    def _run(self):
        while not self._stop:
            try:
                self.samples.append(int(open(self.inp).read()) / 1e6)
            except (OSError, ValueError):
                return
            time.sleep(0.01)

    def __enter__(self):
        if self.inp:
            import threading
            self._thread = threading.Thread(target=self._run, daemon=True)
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        if self._thread:
            self._thread.join()

    def result(self):
        if not self.samples:
            return None
        return {"mean_w": round(float(np.mean(self.samples)), 1), "max_w": round(float(np.max(self.samples)), 1),
                "cap_w": self.cap_w, "samples": len(self.samples)}


def cpu_baseline(cfg, inp, n_tokens: int, n_hidden: int):
    """The oracle as it stands, timed on a bounded sample of the same workload, in two legs.
    Rows: the whole layer pass (every call of a step except the weight gradients) on the first n_tokens tokens;
    its time scales with the tokens.  Weight gradients: the contraction over ALL hosted rows of the workload for
    n_hidden hidden units of every hosted group; its time scales with the hidden units.  The plan comes from the
    oracle's own routing of the full batch."""
    from oracle import moe_oracle as orc
    from paper_2411_10003_amd import workload as wl
    orc.build()
    k, act, T = cfg.k, cfg.act, cfg.T
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    r_full = orc.route(inp["X"], inp["Wg"], inp["bg"], k, cfg.renorm)       # untimed: where the plan comes from
    expert_dest = wl.make_plan(cfg, r_full["counts"], threshold=(cfg.index == 4))
    goe = wl.group_of_expert(expert_dest, cfg.self_dest)
    X = inp["X"][:n_tokens]
    t0 = time.perf_counter()
    r = orc.route(X, inp["Wg"], inp["bg"], k, cfg.renorm)
    lay = orc.place(r["idx"], r["counts"], expert_dest, cfg.P)
    idx = r["idx"].reshape(-1)
    hosted = orc.hosted_assignments(idx, goe)
    orc.dispatch(X, lay["perm"], k)
    Y = orc.ffn_fwd(X, idx, goe, inp["W1"], inp["W2"], inp.get("W3"), k, act, hosted)
    Yp = inp["Yp_fill"][: n_tokens * k].astype(np.float64)
    Yp[lay["pos"][hosted]] = Y
    orc.combine(Yp, lay["pos"], r["w"], k)
    if cfg.backward:
        dOut = inp["dOut"][:n_tokens]
        dYp, dw = orc.combine_bwd(dOut, Yp, lay["pos"], r["w"], k)
        dXh = orc.ffn_bwd_rows(X, idx, goe, inp["W1"], inp["W2"], inp.get("W3"), k, act, hosted, dYp[lay["pos"][hosted]])
        dXp = inp["dXp_fill"][: n_tokens * k].astype(np.float64)
        dXp[lay["pos"][hosted]] = dXh
        orc.dispatch_bwd(dXp, lay["pos"], k)
        orc.gate_bwd(dw, r["logits"], r["idx"], cfg.renorm)
    t_rows = time.perf_counter() - t0
    rows_scaled = t_rows * (T / n_tokens)
    if not cfg.backward:
        return {"value": T / rows_scaled, "unit": "tokens/s", "cores": threads, "kind": "oracle",
                "sample": f"whole forward pass on the first {n_tokens} of {T} tokens in {t_rows:.1f} s ({threads} threads), "
                          f"scaled to {rows_scaled:.1f} s for the batch"}
    # weight gradients over every hosted row of the batch (dYp = w * dOut does not depend on the expert outputs)
    idx_full = r_full["idx"].reshape(-1)
    dYa = (r_full["w"].reshape(-1, 1) * np.repeat(inp["dOut"], k, axis=0)).astype(np.float32)
    G = int((np.asarray(expert_dest) == cfg.self_dest).sum())
    M = int((goe[idx_full] >= 0).sum())
    rng = np.random.default_rng(0)
    js = np.sort(rng.choice(cfg.h, size=n_hidden, replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    for g in range(G):
        orc.ffn_bwd_hidden_many(inp["X"], idx_full, goe, inp["W1"], inp["W2"], inp.get("W3"), k, act, dYa, g, js)
    t_w = time.perf_counter() - t0
    w_scaled = t_w * (cfg.h / n_hidden)
    total = rows_scaled + w_scaled
    return {
        "value": T / total, "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": (f"scaled: rows (every call but the weight gradients) on the first {n_tokens} of {T} tokens in {t_rows:.1f} s "
                   f"({threads} threads over rows) x {T / n_tokens:.0f} = {rows_scaled:.0f} s; weight gradients over all {M} hosted "
                   f"rows on {n_hidden} of {cfg.h} hidden units per group in {t_w:.1f} s ({min(threads, n_hidden)} threads over "
                   f"hidden units) x {cfg.h / n_hidden:.0f} = {w_scaled:.0f} s"),
    }


def ffn_group_bounds(cfg, group_rows, backward: bool):
    """Per hosted group, the time the expert computation needs at the published peaks: bound_g =
    max(flops_g / MFMA peak, bytes_g / HBM peak).  A group of few rows is bound by reading its weights (and, in
    the backward pass, writing its fp32 weight gradients), a large one by the matrix cores.  Bytes: every operand
    and result of the group's contractions once (weights, saved pre-activations, activations, gradients)."""
    es = 2 if cfg.dtype == "bf16" else 4
    d, h, nm = cfg.d, cfg.h, cfg.n_mats
    peak = (PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS) * 1e12
    out = []
    for m in group_rows:
        if m == 0:                       # nothing is read for an empty or unused group; its gradients are written as zeros
            t_b = (nm * d * h * 4 if backward else 0) / (PEAK_HBM_GBS * 1e9)
            out.append({"rows": 0, "bound_us": round(t_b * 1e6, 1), "bound": "hbm"})
            continue
        flops = 2.0 * m * d * h * nm * (3 if backward else 1)
        w_bytes = nm * d * h * es
        # forward: Xp in, Z (and U) and the activation out, the activation in again, Yp out
        nbytes = w_bytes + m * (d * es + nm * h * es + h * es + d * es)
        if backward:
            # dYp in twice, Z (and U) in, dZ (and dU) out and in twice, the activation and Xp in, dXp out, the weights
            # again, the fp32 weight gradients out (written as zeros even for an empty group)
            nbytes += w_bytes + nm * d * h * 4 + m * (2 * d * es + (nm - 1) * h * es + 3 * (nm - 1) * h * es + h * es + d * es + d * es)
        t_f, t_b = flops / peak, nbytes / (PEAK_HBM_GBS * 1e9)
        out.append({"rows": int(m), "bound_us": round(max(t_f, t_b) * 1e6, 1), "bound": "mfma" if t_f >= t_b else "hbm"})
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="index into BASELINE.json configs (default: the roofline target)")
    ap.add_argument("--iteration", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-tokens", type=int, default=0)
    ap.add_argument("--step-only", action="store_true",
                    help="skip the calls timed beside the step (planner, gate gradients, parameter transfer, receive-side pass): "
                         "for profiler runs, so that per-kernel averages cover the step's launches only")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known size) to scale rocprofv3 FETCH_SIZE/WRITE_SIZE readings")
    ap.add_argument("--no-calib", action="store_true",
                    help="skip the two calibration kernels (streaming copy, register-only bf16 MFMA loop) that give the measured peaks")
    ap.add_argument("--recompute-act", action="store_true",
                    help="backward recomputes the activation from the saved pre-activations instead of reading the forward "
                         "pass's copy in the workspace (for callers that share one workspace between layers)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build is one GPU's share of the layer; it has no multi-GPU path (use --gpus 1)")

    import torch
    from paper_2411_10003_amd import binding
    from paper_2411_10003_amd import workload as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: needs a GPU")
    binding.load()
    cfg = wl.CONFIGS[args.config]
    dev = "cuda:0"
    dt = cfg.dtype

    t0 = time.perf_counter()
    inp = wl.make_inputs(cfg, args.iteration)
    log(f"[bench] {cfg.name}: inputs drawn in {time.perf_counter() - t0:.1f} s")

    def up(a, dtype="f32"):
        t = torch.from_numpy(a)
        return (t.to(torch.bfloat16) if dtype == "bf16" else t).to(dev)

    X, Wg, bg = up(inp["X"], dt), up(inp["Wg"]), up(inp["bg"])
    W1, W2 = up(inp["W1"], dt), up(inp["W2"], dt)
    W3 = up(inp["W3"], dt) if cfg.act == "swiglu" else None
    dOut = up(inp["dOut"], dt) if cfg.backward else None

    hd = binding.Handle(T=cfg.T, d=cfg.d, h=cfg.h, E=cfg.E, k=cfg.k, P=cfg.P, self_dest=cfg.self_dest,
                        G=cfg.G_max, dtype=dt, act=cfg.act, renorm=cfg.renorm, device=dev)
    # this layer keeps its workspace from its forward to its backward pass, so the activation the forward pass
    # left there is read by the backward pass instead of being recomputed (moe_set_act_saved)
    act_saved = cfg.backward and dt == "bf16" and not args.recompute_act
    hd.set_act_saved(act_saved)
    b = binding.LayerBuffers(hd, cfg.backward)
    b.Yp.copy_(up(inp["Yp_fill"], dt))
    if cfg.backward:
        b.dXp.copy_(up(inp["dXp_fill"], dt))

    # the plan is an input of the step: built once from this batch's input distribution
    hd.gate_topk(X, Wg, bg, b.logits, b.idx, b.w)
    hd.expert_counts(b.idx, b.counts)
    counts = b.counts.cpu().numpy()
    expert_dest_np = wl.make_plan(cfg, counts, threshold=(cfg.index == 4))
    expert_dest = torch.from_numpy(expert_dest_np).to(dev)

    calls = ["gate_topk", "expert_counts", "dispatch", "expert_ffn_fwd", "combine"]
    if cfg.backward:
        calls += ["combine_bwd", "expert_ffn_bwd", "dispatch_bwd", "gate_bwd"]

    def step(ev=None):
        def mark(i):
            if ev is not None:
                ev[i].record()
        mark(0)
        hd.gate_topk(X, Wg, bg, b.logits, b.idx, b.w); mark(1)
        hd.expert_counts(b.idx, b.counts); mark(2)
        # counts -> dispatch on the same idx and workspace with nothing in between: the histograms are not rebuilt
        hd.dispatch_after_counts(expert_dest, X, b.idx, b.counts, b.layout, b.Xp); mark(3)
        # a forward-only workload does not keep the pre-activations (nothing reads them)
        hd.expert_ffn_fwd(b.Xp, b.layout, W1, W2, W3, b.Yp, b.Z if cfg.backward else None, b.U if cfg.backward else None); mark(4)
        hd.combine(b.Yp, b.layout.pos, b.w, b.out); mark(5)
        if cfg.backward:
            hd.combine_bwd(dOut, b.Yp, b.layout.pos, b.w, b.dYp, b.dw); mark(6)
            hd.expert_ffn_bwd(b.dYp, b.Xp, b.Z, b.U, b.layout, W1, W2, W3, b.dXp, b.dW1, b.dW2, b.dW3); mark(7)
            hd.dispatch_bwd(b.dXp, b.layout.pos, b.dX); mark(8)
            hd.gate_bwd(b.dw, b.logits, b.idx, b.dlogits); mark(9)

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                                   # one elementwise copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    assert hd.read_status() == 0, "plan rejected"
    do = b.layout.dest_offsets.cpu().numpy()
    M = int(do[cfg.self_dest + 1] - do[cfg.self_dest])
    so = b.layout.slot_offsets.cpu().numpy()
    ds = b.layout.dest_slots.cpu().numpy()
    group_rows = [int(so[s + 1] - so[s]) for s in range(ds[cfg.self_dest], ds[cfg.self_dest + 1])]
    share = np.sort(counts)[::-1] / counts.sum()
    log(f"[bench] counts per expert {counts.tolist()}  balance degree (std) {wl.balance_degree(counts):.1f}")
    log(f"[bench] top-3 experts hold {share[:3].sum():.1%}, bottom-3 {share[-3:].sum():.1%}; "
        f"hosted rows M={M} of A={cfg.A}; rows per hosted group {group_rows}")

    n_ev = len(calls) + 1
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    power = PowerSampler()
    t0 = time.perf_counter()
    with power:
        for s in range(args.steps):
            step(events[s])
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    call_all = {c: np.array([events[s][i].elapsed_time(events[s][i + 1]) for s in range(args.steps)])
                for i, c in enumerate(calls)}
    call_ms = {c: float(np.mean(v)) for c, v in call_all.items()}
    step_all = np.array([events[s][0].elapsed_time(events[s][n_ev - 1]) for s in range(args.steps)])
    ffn_all = call_all["expert_ffn_fwd"] + call_all.get("expert_ffn_bwd", 0.0)

    # algorithmic work
    es = 2 if dt == "bf16" else 4
    T, d, h, A, E, k = cfg.T, cfg.d, cfg.h, cfg.A, cfg.E, cfg.k
    fwd_flops = 2.0 * M * d * h * cfg.n_mats
    ffn_flops = fwd_flops * (3 if cfg.backward else 1)
    ffn_ms = call_ms["expert_ffn_fwd"] + call_ms.get("expert_ffn_bwd", 0.0)
    peak = PEAK_BF16_TFLOPS if dt == "bf16" else PEAK_F32_TFLOPS
    achieved = ffn_flops / (ffn_ms * 1e-3) / 1e12
    hbm_bytes = {
        "gate_topk": T * d * es + T * E * 4 + 8 * T * k,
        "dispatch": (1 + k) * T * d * es,
        "combine": (1 + k) * T * d * es,
        "combine_bwd": (T * d + 2 * A * d) * es,
        "dispatch_bwd": (1 + k) * T * d * es,
    }
    per_call = {}
    for c in calls:
        e = {"ms": round(call_ms[c], 4), "median_ms": round(float(np.median(call_all[c])), 4),
             "min_ms": round(float(call_all[c].min()), 4)}
        if c in hbm_bytes:
            gbs = hbm_bytes[c] / (call_ms[c] * 1e-3) / 1e9
            e.update({"GB/s": round(gbs, 1), "hbm_frac": round(gbs / PEAK_HBM_GBS, 4)})
        if c == "gate_topk":
            # co-bound: the tokens stream from HBM while 2 E flops per element run on the fp32 matrix instruction
            # (157.3 TFLOP/s); at E = 64 the arithmetic takes longer than the stream at their peaks
            gflop = 2.0 * T * d * E
            t_hbm, t_mat = hbm_bytes[c] / (PEAK_HBM_GBS * 1e9), gflop / (PEAK_F32_TFLOPS * 1e12)
            e.update({"TFLOP/s": round(gflop / (call_ms[c] * 1e-3) / 1e12, 2),
                      "matrix_frac": round(gflop / (call_ms[c] * 1e-3) / 1e12 / PEAK_F32_TFLOPS, 4),
                      "bound": "fp32 matrix rate" if t_mat > t_hbm else "hbm",
                      "us_at_peak": {"hbm": round(t_hbm * 1e6, 1), "fp32_matrix": round(t_mat * 1e6, 1)}})
        if c == "expert_ffn_fwd":
            e.update({"TFLOP/s": round(fwd_flops / (call_ms[c] * 1e-3) / 1e12, 1)})
        if c == "expert_ffn_bwd":
            e.update({"TFLOP/s": round(2 * fwd_flops / (call_ms[c] * 1e-3) / 1e12, 1)})
        per_call[c] = e

    # ---- the gate on its own, back to back: in a step it starts while the memory-side cache still holds the dirty
    # lines of the calls before it (268 MB of dX from moe_dispatch_bwd at config 3), whose write-back shares the HBM
    # with the gate's reads and is billed to the gate's time; back to back there is none
    if not args.step_only:
        ge = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        hd.gate_topk(X, Wg, bg, b.logits, b.idx, b.w)
        torch.cuda.synchronize()
        ge[0].record()
        for _ in range(20):
            hd.gate_topk(X, Wg, bg, b.logits, b.idx, b.w)
        ge[1].record()
        torch.cuda.synchronize()
        g_ms = ge[0].elapsed_time(ge[1]) / 20
        per_call["gate_topk"]["back_to_back_ms"] = round(g_ms, 4)
        per_call["gate_topk"]["hbm_frac_back_to_back"] = round(hbm_bytes["gate_topk"] / (g_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)

    # ---- measured peaks of this GPU today: a plain streaming copy and a register-only bf16 MFMA loop
    measured_peak = None
    if not args.no_calib:
        nb = 1 << 30
        src = torch.empty(nb, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        sink = torch.empty(cus * 512, dtype=torch.float32, device=dev)
        iters = 40000
        binding.calib_copy(src, dst)
        mfma_flops = binding.calib_mfma(sink, iters)
        torch.cuda.synchronize()
        reps = 5
        ce = [torch.cuda.Event(enable_timing=True) for _ in range(2 * reps + 1)]
        ce[0].record()
        for i in range(reps):
            binding.calib_copy(src, dst); ce[i + 1].record()
        with PowerSampler() as cal_power:
            for i in range(reps):
                binding.calib_mfma(sink, iters); ce[reps + i + 1].record()
            torch.cuda.synchronize()
        t_copy = np.array([ce[i].elapsed_time(ce[i + 1]) for i in range(reps)])
        t_mfma = np.array([ce[reps + i].elapsed_time(ce[reps + i + 1]) for i in range(reps)])
        measured_peak = {
            "copy_GB/s": round(2.0 * nb / (float(np.median(t_copy)) * 1e-3) / 1e9, 1),
            "copy_what": "1 GiB read + 1 GiB written by a plain 16-byte-per-lane kernel, median of 5",
            "mfma_TFLOP/s": round(mfma_flops / (float(np.median(t_mfma)) * 1e-3) / 1e12, 1),
            "mfma_what": f"{cus} blocks x 8 waves x {iters} x 8 v_mfma_f32_32x32x16_bf16 on register operands, median of 5",
            "mfma_package_power": cal_power.result(),
        }
        del src, dst, sink
        log(f"[bench] measured peaks: copy {measured_peak['copy_GB/s']} GB/s, bf16 MFMA {measured_peak['mfma_TFLOP/s']} TFLOP/s")
        if dt == "bf16":
            for c in per_call:
                if "GB/s" in per_call[c]:
                    per_call[c]["frac_of_measured_copy"] = round(per_call[c]["GB/s"] / measured_peak["copy_GB/s"], 4)

    if not args.step_only:
        # the planner (Algorithm 1) on the P x E count matrix of this batch: not one of the timed calls of a step
        # (the paper runs it under the all-to-all of the previous iteration), reported beside them
        gating_np = wl.make_gating(cfg, counts, args.iteration)
        gating = torch.from_numpy(gating_np).to(dev)
        pc = wl.planner_constants(cfg)
        pbuf = binding.PlanBuffers(cfg.P, cfg.E, dev)
        plan_args = dict(n=1, overlap=False, alpha=1.0, **pc)
        binding.plan(gating, pbuf, **plan_args)
        torch.cuda.synchronize()
        pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        pe[0].record()
        for _ in range(20):
            binding.plan(gating, pbuf, **plan_args)
        pe[1].record()
        torch.cuda.synchronize()
        info = pbuf.info.cpu().numpy()
        ptimes = pbuf.times.cpu().numpy()
        per_call["plan"] = {"ms": round(pe[0].elapsed_time(pe[1]) / 20, 4), "in_step": False, "selected": int(info[1]),
                            "kept": int(info[0]), "model_T_before_s": float(ptimes[0]), "model_T_after_s": float(ptimes[1]),
                            "gating": f"{cfg.P}x{cfg.E} counts, n=1, Eq. 6"}
        if not args.no_cpu_baseline:
            from oracle import planner_oracle as po
            t0 = time.perf_counter()
            ref = po.greedy_search(gating_np.astype(np.int64), 1, po.PlannerModel(alpha=1.0, overlap=False, **pc))
            per_call["plan"]["oracle_ms"] = round((time.perf_counter() - t0) * 1e3, 3)
            assert ref["cnt"] == int(info[0]) and ref["T_output"] == float(ptimes[1]), "planner disagrees with its oracle"
            # the ablation's fixed policies (Section 6.4) through the same performance model, and the balance degree
            # (standard deviation of the per-device load, Section 6.3) without a placement and under each policy
            m_ = po.PlannerModel(alpha=1.0, overlap=False, **pc)
            g64 = gating_np.astype(np.int64)
            H0, R0 = po.loads(g64, po.placement(cfg.P, cfg.E, [], []))
            comp = {"none": {"model_T_s": float(ptimes[0]), "RB": round(po.balance_degree(H0), 1)},
                    "greedy (device)": {"model_T_s": float(ptimes[1]), "RB": round(po.balance_degree(pbuf.H.cpu().numpy()), 1)}}
            for r_top in (2, 3):
                Ht, Rt = po.loads(g64, po.top_policy(g64, r_top))
                comp[f"top{r_top}"] = {"model_T_s": po.layer_time(Rt, Ht, r_top, 0, m_), "RB": round(po.balance_degree(Ht), 1)}
            per_call["plan"]["policies"] = comp

        # the rest of the gate's backward (parameter gradients, gate path of the input gradient): beside the step
        if cfg.backward and E <= 64:
            dWg = torch.empty(d, E, dtype=torch.float32, device=dev)
            dbg = torch.empty(E, dtype=torch.float32, device=dev)
            extra = {
                "gate_bwd_params": (lambda: hd.gate_bwd_params(X, b.dlogits, dWg, dbg), T * d * es + T * E * 4),
                "input_grad": (lambda: hd.input_grad(b.dXp, b.layout.pos, b.dlogits, Wg, b.dX), (1 + k) * T * d * es + T * E * 4),
            }
            for name, (fn, nbytes) in extra.items():
                fn()
                torch.cuda.synchronize()
                ee = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                ee[0].record()
                for _ in range(10):
                    fn()
                ee[1].record()
                torch.cuda.synchronize()
                ms = ee[0].elapsed_time(ee[1]) / 10
                per_call[name] = {"ms": round(ms, 4), "in_step": False, "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                                  "hbm_frac": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}

        # Trans on one GPU: gather the hosted experts' parameters from a pool of all experts into the group slots
        # (worst case: every slot changes; a slot that already holds its expert is skipped)
        if dt == "bf16":
            n_t = cfg.n_mats
            pools = [torch.empty(E, d * h, dtype=torch.bfloat16, device=dev) for _ in range(n_t)]
            slots = [torch.empty(cfg.G_max, d * h, dtype=torch.bfloat16, device=dev) for _ in range(n_t)]
            slot_expert = torch.full((cfg.G_max,), -1, dtype=torch.int32, device=dev)
            pool_ver = torch.zeros(E, dtype=torch.int32, device=dev)
            slot_ver = torch.full((cfg.G_max,), -1, dtype=torch.int32, device=dev)
            hd.trans(expert_dest, slot_expert, pools, slots, pool_ver, slot_ver)
            torch.cuda.synchronize()
            te = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            slot_expert.fill_(-1)
            te[0].record(); hd.trans(expert_dest, slot_expert, pools, slots, pool_ver, slot_ver); te[1].record()
            hd.trans(expert_dest, slot_expert, pools, slots, pool_ver, slot_ver); te[2].record()   # nothing to move the second time
            torch.cuda.synchronize()
            moved = 2.0 * len(group_rows) * n_t * d * h * es
            ms_all, ms_none = te[0].elapsed_time(te[1]), te[1].elapsed_time(te[2])
            per_call["trans"] = {"ms": round(ms_all, 4), "in_step": False, "GB/s": round(moved / (ms_all * 1e-3) / 1e9, 1),
                                 "hbm_frac": round(moved / (ms_all * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                 "ms_when_nothing_moves": round(ms_none, 4)}
            del pools, slots

        # Receive side (Eq. 2): the rows that the other devices would send for the experts hosted here, the stand-in plan
        # applied to every row of the gating matrix; synthetic rows, expert computation forward, then backward with the
        # weight gradients added to those of the local pass
        if dt == "bf16" and cfg.backward:
            me = cfg.self_dest
            hosted_e = wl.hosted_experts(expert_dest_np, me)
            recv = np.zeros(cfg.G_max + 1, dtype=np.int64)
            for j in range(cfg.P):
                if j != me:
                    dest_j = wl.make_plan(wl.scaled(cfg, self_dest=j), gating_np[j], threshold=(cfg.index == 4))
                    for g, e in enumerate(hosted_e):
                        recv[g + 1] += int(gating_np[j, e]) if dest_j[e] == me else 0
            offs = np.cumsum(recv).astype(np.int32)
            Rn = int(offs[-1])
            if Rn > 0:
                hr = binding.Handle(T=Rn, d=d, h=h, E=E, k=1, P=cfg.P, self_dest=me, G=cfg.G_max, dtype=dt, act=cfg.act,
                                    renorm=0, device=dev)
                lay_r = hr.new_layout()
                d_offs = torch.from_numpy(offs).to(dev)
                Xr = torch.randn(Rn, d, dtype=torch.bfloat16, device=dev)
                dYr = torch.randn(Rn, d, dtype=torch.bfloat16, device=dev)
                Yr, dXr = torch.empty_like(Xr), torch.empty_like(Xr)
                Zr = torch.empty(Rn, h, dtype=torch.bfloat16, device=dev)
                Ur = torch.empty_like(Zr) if cfg.act == "swiglu" else None

                def recv_pass():
                    hr.recv_layout(b.layout, d_offs, lay_r)
                    hr.expert_ffn_fwd(Xr, lay_r, W1, W2, W3, Yr, Zr, Ur)
                    hr.expert_ffn_bwd_acc(dYr, Xr, Zr, Ur, lay_r, W1, W2, W3, dXr, b.dW1, b.dW2, b.dW3)
                recv_pass()
                torch.cuda.synchronize()
                re_ = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                re_[0].record()
                for _ in range(3):
                    recv_pass()
                re_[1].record()
                torch.cuda.synchronize()
                ms = re_[0].elapsed_time(re_[1]) / 3
                fl = 3 * 2.0 * Rn * d * h * cfg.n_mats
                per_call["recv_pass"] = {"ms": round(ms, 4), "in_step": False, "received_rows": Rn,
                                         "rows_per_group": np.diff(offs)[:len(hosted_e)].tolist(),
                                         "TFLOP/s": round(fl / (ms * 1e-3) / 1e12, 1),
                                         "mfma_frac": round(fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
                del Xr, dYr, Yr, dXr, Zr, Ur

    result = {
        "metric": METRIC, "value": T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dt, "data": "synthetic",
        "config": {"workload": f"configs[{cfg.index}] {cfg.name}: T={T} d={d} h={h} {cfg.act} E={E} k={k} P={cfg.P} "
                               f"hosted groups={len(group_rows)} alpha={wl.alpha_for(cfg, args.iteration)}",
                   "pass": "fwd+bwd" if cfg.backward else "fwd", "hosted_rows_M": M, "assignments_A": A},
        "roofline": {"bound": "mfma" if dt == "bf16" else "alu", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": measured_traffic(cfg.index, ffn_flops) if dt == "bf16" else None,
                     "kernel": "grouped_gemm_kernel (all launches of expert_ffn_fwd/bwd in a step)",
                     "flops_per_step": ffn_flops, "ms_per_step": ffn_ms,
                     "median_ms_per_step": float(np.median(ffn_all)), "min_ms_per_step": float(ffn_all.min()),
                     "frac_at_min": ffn_flops / (float(ffn_all.min()) * 1e-3) / 1e12 / peak,
                     "package_power": power.result()},
        "step_ms": {"mean": float(step_all.mean()), "median": float(np.median(step_all)), "min": float(step_all.min()),
                    "what": "first to last event of a step on the launch stream"},
        "per_call": per_call,
    }
    result["config"]["act_saved"] = bool(act_saved)
    result["config"]["pre_activations_kept"] = bool(cfg.backward)
    if measured_peak is not None:
        result["roofline"]["measured_peak"] = measured_peak
        if dt == "bf16":
            result["roofline"]["frac_of_measured"] = achieved / measured_peak["mfma_TFLOP/s"]
    gb = ffn_group_bounds(cfg, group_rows + [0] * (cfg.G_max - len(group_rows)), cfg.backward)
    bound_ms = sum(x["bound_us"] for x in gb) / 1e3
    result["roofline"]["per_group"] = {"groups": gb, "sum_of_bounds_ms": round(bound_ms, 4),
                                       "frac_of_bound": round(bound_ms / ffn_ms, 4) if ffn_ms > 0 else None,
                                       "what": "bound_g = max(flops_g / MFMA peak, bytes_g / HBM peak) at the published peaks"}
    if not args.no_cpu_baseline:
        n_tok = args.cpu_tokens or {0: 512, 1: 1024, 2: 256, 3: 512, 4: 256}[cfg.index]
        n_hid = {0: cfg.h, 1: 64, 2: 32, 3: 64, 4: 32}[cfg.index]
        t0 = time.perf_counter()
        result["cpu_baseline"] = cpu_baseline(cfg, inp, min(n_tok, T), min(n_hid, h))
        log(f"[bench] cpu baseline took {time.perf_counter() - t0:.1f} s")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
