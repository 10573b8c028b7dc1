"""Thin ctypes binding of libmoehot.so: the same entry points as include/moehot.h, taking torch
tensors.  Argument marshalling only -- every step of the layer runs in the HIP kernels of the
library.  PyTorch is used for device memory and streams.  There is no CPU or eager fallback: if
the library has not been built, `load()` raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoehot.so")

MOE_F32, MOE_BF16 = 0, 1
MOE_ACT_GELU, MOE_ACT_SWIGLU = 0, 1
DTYPES = {"f32": MOE_F32, "bf16": MOE_BF16}
ACTS = {"gelu": MOE_ACT_GELU, "swiglu": MOE_ACT_SWIGLU}
TORCH_DTYPE = {MOE_F32: torch.float32, MOE_BF16: torch.bfloat16}

EXPORTS = [
    "moe_create", "moe_destroy", "moe_workspace_bytes", "moe_status_string", "moe_last_hip_error",
    "moe_read_status", "moe_gate_topk", "moe_expert_counts", "moe_dispatch", "moe_expert_ffn_fwd",
    "moe_combine", "moe_combine_bwd", "moe_expert_ffn_bwd", "moe_dispatch_bwd", "moe_gate_bwd",
    "moe_plan", "moe_gate_bwd_params", "moe_input_grad", "moe_expert_ffn_bwd_acc", "moe_trans", "moe_recv_layout",
    "moe_dispatch_after_counts", "moe_set_act_saved", "moe_expert_counts_static", "moe_agg", "moe_calib_copy", "moe_calib_mfma",
    "moe_calib_round_bf16",
]


class MoeError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: status {status} ({detail})")


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("T", "d", "h", "E", "k", "P", "self", "G", "dtype", "act", "renorm")]


class _Layout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("slot_of_expert", "slot_offsets", "dest_offsets", "dest_slots", "pos", "perm")]


class _Planner(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("D", "E", "n", "overlap")] + \
               [(n, ctypes.c_double) for n in ("alpha", "size_input", "size_params", "size_grads", "B", "t", "T_FNEC", "T_BNEC")]


class _PlanOut(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("expert_dest", "selected", "skipped", "H", "R", "times", "info")]


_lib = None


def load() -> ctypes.CDLL:
    """Load the HIP library.  Raises if it is missing: nothing else can compute the layer."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2411_10003_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        vp, ip = ctypes.c_void_p, ctypes.c_int
        lib.moe_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(_Shape)]
        lib.moe_destroy.argtypes = [vp]
        lib.moe_workspace_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
        lib.moe_status_string.argtypes = [ip]
        lib.moe_status_string.restype = ctypes.c_char_p
        lib.moe_read_status.argtypes = [vp, vp, vp, ctypes.POINTER(ip)]
        lib.moe_gate_topk.argtypes = [vp] * 8
        lib.moe_expert_counts.argtypes = [vp] * 5
        lib.moe_dispatch.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(_Layout), vp, vp, vp]
        lib.moe_dispatch_after_counts.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(_Layout), vp, vp, vp]
        lib.moe_set_act_saved.argtypes = [vp, ip]
        lib.moe_expert_counts_static.argtypes = [vp] * 4
        lib.moe_expert_ffn_fwd.argtypes = [vp, vp, ctypes.POINTER(_Layout)] + [vp] * 8
        lib.moe_combine.argtypes = [vp] * 6
        lib.moe_combine_bwd.argtypes = [vp] * 8
        lib.moe_expert_ffn_bwd.argtypes = [vp] * 5 + [ctypes.POINTER(_Layout)] + [vp] * 9
        lib.moe_expert_ffn_bwd_acc.argtypes = [vp] * 5 + [ctypes.POINTER(_Layout)] + [vp] * 9
        lib.moe_dispatch_bwd.argtypes = [vp] * 5
        lib.moe_gate_bwd.argtypes = [vp] * 6
        lib.moe_gate_bwd_params.argtypes = [vp] * 7
        lib.moe_input_grad.argtypes = [vp] * 7
        lib.moe_trans.argtypes = [vp, vp, vp, vp, vp, ip, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(ctypes.c_size_t), vp]
        lib.moe_agg.argtypes = [vp, vp, ip, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(ctypes.c_size_t), vp]
        lib.moe_calib_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.moe_calib_mfma.argtypes = [vp, ctypes.c_size_t, ip, ctypes.POINTER(ip), ctypes.POINTER(ip), vp]
        lib.moe_calib_round_bf16.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.moe_recv_layout.argtypes = [vp, ctypes.POINTER(_Layout), vp, ctypes.POINTER(_Layout), vp]
        lib.moe_plan.argtypes = [ctypes.POINTER(_Planner), vp, ctypes.POINTER(_PlanOut), vp]
        _lib = lib
    return _lib


def _ptr(t: Optional[torch.Tensor], dtype: torch.dtype, numel: int, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name}: need a contiguous device tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if t.numel() < numel:
        raise ValueError(f"{name}: {t.numel()} elements, need {numel}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class PlanBuffers:
    """Device arrays moe_plan writes (see moe_plan_out_t)."""

    def __init__(self, D: int, E: int, device="cuda:0"):
        self.D, self.E = D, E
        self.expert_dest = torch.zeros(D, E, dtype=torch.int32, device=device)
        self.selected = torch.zeros(E, dtype=torch.int32, device=device)
        self.skipped = torch.zeros(E, dtype=torch.int64, device=device)      # bit masks, read as unsigned
        self.H = torch.zeros(D, dtype=torch.int64, device=device)
        self.R = torch.zeros(D, dtype=torch.int64, device=device)
        self.times = torch.zeros(2 + E, dtype=torch.float64, device=device)
        self.info = torch.zeros(2, dtype=torch.int32, device=device)
        self.c = _PlanOut(*(t.data_ptr() for t in (self.expert_dest, self.selected, self.skipped, self.H, self.R,
                                                   self.times, self.info)))


def plan(gating: torch.Tensor, out: PlanBuffers, *, n: int, overlap: bool, alpha: float, size_input: float,
         size_params: float, size_grads: float, B: float, t: float, T_FNEC: float = 0.0, T_BNEC: float = 0.0) -> None:
    """moe_plan: greedy search for a lightweight expert placement on the device (argument marshalling only)."""
    lib = load()
    D, E = out.D, out.E
    g = _ptr(gating, torch.int32, D * E, "gating")
    cfg = _Planner(D, E, int(n), int(bool(overlap)), float(alpha), float(size_input), float(size_params),
                   float(size_grads), float(B), float(t), float(T_FNEC), float(T_BNEC))
    rc = lib.moe_plan(ctypes.byref(cfg), g, ctypes.byref(out.c), _stream())
    if rc != 0:
        raise MoeError(rc, "moe_plan", lib.moe_status_string(rc).decode())


def calib_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    """moe_calib_copy: a plain streaming copy of src into dst (uint8 tensors of the same size)."""
    lib = load()
    n = src.numel() * src.element_size()
    rc = lib.moe_calib_copy(_ptr(src, src.dtype, src.numel(), "src"), _ptr(dst, src.dtype, src.numel(), "dst"), n, _stream())
    if rc != 0:
        raise MoeError(rc, "moe_calib_copy", lib.moe_status_string(rc).decode())


def calib_mfma(out: torch.Tensor, iters: int) -> float:
    """moe_calib_mfma: enqueue the register-only bf16 MFMA loop; returns the flops it performs."""
    lib = load()
    blocks, threads = ctypes.c_int(0), ctypes.c_int(0)
    rc = lib.moe_calib_mfma(_ptr(out, torch.float32, 1, "out"), out.numel(), int(iters), ctypes.byref(blocks),
                            ctypes.byref(threads), _stream())
    if rc != 0:
        raise MoeError(rc, "moe_calib_mfma", lib.moe_status_string(rc).decode())
    return float(blocks.value) * (threads.value // 64) * iters * 8 * 32768.0


def calib_round_bf16(x: torch.Tensor, out: torch.Tensor) -> None:
    """moe_calib_round_bf16: out[i] (int16 bit patterns) = the library's fp32 -> bf16 rounding of x[i]."""
    lib = load()
    rc = lib.moe_calib_round_bf16(_ptr(x, torch.float32, 1, "x"), _ptr(out, torch.int16, x.numel(), "out"), x.numel(), _stream())
    if rc != 0:
        raise MoeError(rc, "moe_calib_round_bf16", lib.moe_status_string(rc).decode())


class Layout:
    """Device arrays of the send layout (see moe_layout_t)."""

    def __init__(self, E: int, P: int, A: int, device):
        i32 = dict(dtype=torch.int32, device=device)
        self.slot_of_expert = torch.zeros(E, **i32)
        self.slot_offsets = torch.zeros(E + 1, **i32)
        self.dest_offsets = torch.zeros(P + 1, **i32)
        self.dest_slots = torch.zeros(P + 1, **i32)
        self.pos = torch.zeros(A, **i32)
        self.perm = torch.zeros(A, **i32)
        self.c = _Layout(*(t.data_ptr() for t in (self.slot_of_expert, self.slot_offsets, self.dest_offsets,
                                                  self.dest_slots, self.pos, self.perm)))


class Handle:
    """A moe_handle_t plus its workspace.  Methods carry the names of the C entry points."""

    def __init__(self, *, T: int, d: int, h: int, E: int, k: int, P: int, self_dest: int, G: int,
                 dtype: str, act: str, renorm: int, device="cuda:0", alloc_workspace: bool = True):
        self.lib = load()
        self.shape = _Shape(T, d, h, E, k, P, self_dest, G, DTYPES[dtype], ACTS[act], renorm)
        self.T, self.d, self.h, self.E, self.k, self.P, self.G = T, d, h, E, k, P, G
        self.A = T * k
        self.swiglu = act == "swiglu"
        self.elt = TORCH_DTYPE[DTYPES[dtype]]
        self.device = torch.device(device)
        self._h = ctypes.c_void_p()
        self._check(self.lib.moe_create(ctypes.byref(self._h), ctypes.byref(self.shape)), "moe_create")
        n = ctypes.c_size_t()
        self._check(self.lib.moe_workspace_bytes(self._h, ctypes.byref(n)), "moe_workspace_bytes")
        self.workspace_bytes = n.value
        self.ws = torch.empty(n.value, dtype=torch.uint8, device=self.device) if alloc_workspace else None

    def close(self):
        if self._h:
            self.lib.moe_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int, where: str):
        if rc != 0:
            detail = self.lib.moe_status_string(rc).decode()
            if rc == -7:
                detail += f", hipError {self.lib.moe_last_hip_error()}"
            raise MoeError(rc, where, detail)

    def _ws(self) -> int:
        if self.ws is None:
            raise ValueError("no workspace attached")
        return self.ws.data_ptr()

    def new_layout(self) -> Layout:
        return Layout(self.E, self.P, self.A, self.device)

    # ---- the entry points ---------------------------------------------------------------
    def read_status(self) -> int:
        v = ctypes.c_int(0)
        self._check(self.lib.moe_read_status(self._h, self._ws(), _stream(), ctypes.byref(v)), "moe_read_status")
        return v.value

    def gate_topk(self, X, Wg, bg, logits, idx, w):
        f32, i32 = torch.float32, torch.int32
        self._check(self.lib.moe_gate_topk(
            self._h, _ptr(X, self.elt, self.T * self.d, "X"), _ptr(Wg, f32, self.d * self.E, "Wg"),
            _ptr(bg, f32, self.E, "bg"), _ptr(logits, f32, self.T * self.E, "logits"),
            _ptr(idx, i32, self.A, "idx"), _ptr(w, f32, self.A, "w"), _stream()), "moe_gate_topk")

    def expert_counts(self, idx, counts):
        i32 = torch.int32
        self._check(self.lib.moe_expert_counts(self._h, _ptr(idx, i32, self.A, "idx"), _ptr(counts, i32, self.E, "counts"),
                                               self._ws(), _stream()), "moe_expert_counts")

    def expert_counts_static(self, idx, counts):
        i32 = torch.int32
        self._check(self.lib.moe_expert_counts_static(self._h, _ptr(idx, i32, self.A, "idx"), _ptr(counts, i32, self.E, "counts"),
                                                      _stream()), "moe_expert_counts_static")

    def dispatch(self, expert_dest, X, idx, counts, layout: Layout, Xp, after_counts: bool = False):
        i32 = torch.int32
        fn = self.lib.moe_dispatch_after_counts if after_counts else self.lib.moe_dispatch
        self._check(fn(
            self._h, _ptr(expert_dest, i32, self.E, "expert_dest"), _ptr(X, self.elt, self.T * self.d, "X"),
            _ptr(idx, i32, self.A, "idx"), _ptr(counts, i32, self.E, "counts"), ctypes.byref(layout.c),
            _ptr(Xp, self.elt, self.A * self.d, "Xp"), self._ws(), _stream()),
            "moe_dispatch_after_counts" if after_counts else "moe_dispatch")

    def dispatch_after_counts(self, expert_dest, X, idx, counts, layout: Layout, Xp):
        self.dispatch(expert_dest, X, idx, counts, layout, Xp, after_counts=True)

    def set_act_saved(self, saved: bool):
        self._check(self.lib.moe_set_act_saved(self._h, int(bool(saved))), "moe_set_act_saved")

    def expert_ffn_fwd(self, Xp, layout: Layout, W1, W2, W3, Yp, Z, U):
        e, dh = self.elt, self.G * self.d * self.h
        self._check(self.lib.moe_expert_ffn_fwd(
            self._h, _ptr(Xp, e, self.A * self.d, "Xp"), ctypes.byref(layout.c), _ptr(W1, e, dh, "W1"), _ptr(W2, e, dh, "W2"),
            _ptr(W3, e, dh, "W3"), _ptr(Yp, e, self.A * self.d, "Yp"), _ptr(Z, e, self.A * self.h, "Z"),
            _ptr(U, e, self.A * self.h, "U"), self._ws(), _stream()), "moe_expert_ffn_fwd")

    def combine(self, Yp, pos, w, out):
        self._check(self.lib.moe_combine(
            self._h, _ptr(Yp, self.elt, self.A * self.d, "Yp"), _ptr(pos, torch.int32, self.A, "pos"),
            _ptr(w, torch.float32, self.A, "w"), _ptr(out, self.elt, self.T * self.d, "out"), _stream()), "moe_combine")

    def combine_bwd(self, dOut, Yp, pos, w, dYp, dw):
        e = self.elt
        self._check(self.lib.moe_combine_bwd(
            self._h, _ptr(dOut, e, self.T * self.d, "dOut"), _ptr(Yp, e, self.A * self.d, "Yp"),
            _ptr(pos, torch.int32, self.A, "pos"), _ptr(w, torch.float32, self.A, "w"),
            _ptr(dYp, e, self.A * self.d, "dYp"), _ptr(dw, torch.float32, self.A, "dw"), _stream()), "moe_combine_bwd")

    def expert_ffn_bwd(self, dYp, Xp, Z, U, layout: Layout, W1, W2, W3, dXp, dW1, dW2, dW3, accumulate: bool = False):
        e, f32, dh = self.elt, torch.float32, self.G * self.d * self.h
        fn = self.lib.moe_expert_ffn_bwd_acc if accumulate else self.lib.moe_expert_ffn_bwd
        self._check(fn(
            self._h, _ptr(dYp, e, self.A * self.d, "dYp"), _ptr(Xp, e, self.A * self.d, "Xp"),
            _ptr(Z, e, self.A * self.h, "Z"), _ptr(U, e, self.A * self.h, "U"), ctypes.byref(layout.c),
            _ptr(W1, e, dh, "W1"), _ptr(W2, e, dh, "W2"), _ptr(W3, e, dh, "W3"),
            _ptr(dXp, e, self.A * self.d, "dXp"), _ptr(dW1, f32, dh, "dW1"), _ptr(dW2, f32, dh, "dW2"),
            _ptr(dW3, f32, dh, "dW3"), self._ws(), _stream()), "moe_expert_ffn_bwd_acc" if accumulate else "moe_expert_ffn_bwd")

    def expert_ffn_bwd_acc(self, *args):
        self.expert_ffn_bwd(*args, accumulate=True)

    def dispatch_bwd(self, dXp, pos, dX):
        self._check(self.lib.moe_dispatch_bwd(
            self._h, _ptr(dXp, self.elt, self.A * self.d, "dXp"), _ptr(pos, torch.int32, self.A, "pos"),
            _ptr(dX, self.elt, self.T * self.d, "dX"), _stream()), "moe_dispatch_bwd")

    def gate_bwd(self, dw, logits, idx, dlogits):
        f32 = torch.float32
        self._check(self.lib.moe_gate_bwd(
            self._h, _ptr(dw, f32, self.A, "dw"), _ptr(logits, f32, self.T * self.E, "logits"),
            _ptr(idx, torch.int32, self.A, "idx"), _ptr(dlogits, f32, self.T * self.E, "dlogits"), _stream()), "moe_gate_bwd")

    def trans(self, expert_dest, slot_expert, pools, groups, pool_version=None, slot_version=None):
        """moe_trans: gather the hosted experts' tensors from the pools into the group slots."""
        n = len(pools)
        per = [p.numel() // self.E * p.element_size() for p in pools]
        for p, g, b in zip(pools, groups, per):
            if not (p.is_cuda and g.is_cuda and p.is_contiguous() and g.is_contiguous()):
                raise ValueError("trans: need contiguous device tensors")
            if p.numel() % self.E or g.numel() * g.element_size() < self.G * b or p.dtype != g.dtype:
                raise ValueError("trans: pool / group sizes do not match")
        pa = (ctypes.c_void_p * n)(*(p.data_ptr() for p in pools))
        ga = (ctypes.c_void_p * n)(*(g.data_ptr() for g in groups))
        ba = (ctypes.c_size_t * n)(*per)
        self._check(self.lib.moe_trans(
            self._h, _ptr(expert_dest, torch.int32, self.E, "expert_dest"), _ptr(pool_version, torch.int32, self.E, "pool_version"),
            _ptr(slot_expert, torch.int32, self.G, "slot_expert"), _ptr(slot_version, torch.int32, self.G, "slot_version"),
            n, pa, ga, ba, _stream()), "moe_trans")

    def agg(self, expert_dest, group_grads, pool_grads):
        """moe_agg: add the hosted groups' weight gradients to the per-expert gradient pools."""
        n = len(group_grads)
        per = [p.numel() // self.E for p in pool_grads]
        for p, g, b in zip(pool_grads, group_grads, per):
            if not (p.is_cuda and g.is_cuda and p.is_contiguous() and g.is_contiguous()):
                raise ValueError("agg: need contiguous device tensors")
            if p.dtype != torch.float32 or g.dtype != torch.float32 or p.numel() % self.E or g.numel() < self.G * b:
                raise ValueError("agg: pool / group sizes or dtypes do not match")
        ga = (ctypes.c_void_p * n)(*(g.data_ptr() for g in group_grads))
        pa = (ctypes.c_void_p * n)(*(p.data_ptr() for p in pool_grads))
        ba = (ctypes.c_size_t * n)(*per)
        self._check(self.lib.moe_agg(self._h, _ptr(expert_dest, torch.int32, self.E, "expert_dest"), n, ga, pa, ba, _stream()),
                    "moe_agg")

    def recv_layout(self, local: Layout, recv_offsets, out: Layout):
        self._check(self.lib.moe_recv_layout(
            self._h, ctypes.byref(local.c), _ptr(recv_offsets, torch.int32, self.G + 1, "recv_offsets"),
            ctypes.byref(out.c), _stream()), "moe_recv_layout")

    def gate_bwd_params(self, X, dlogits, dWg, dbg):
        f32 = torch.float32
        self._check(self.lib.moe_gate_bwd_params(
            self._h, _ptr(X, self.elt, self.T * self.d, "X"), _ptr(dlogits, f32, self.T * self.E, "dlogits"),
            _ptr(dWg, f32, self.d * self.E, "dWg"), _ptr(dbg, f32, self.E, "dbg"), self._ws(), _stream()),
            "moe_gate_bwd_params")

    def input_grad(self, dXp, pos, dlogits, Wg, dX):
        f32 = torch.float32
        self._check(self.lib.moe_input_grad(
            self._h, _ptr(dXp, self.elt, self.A * self.d, "dXp"), _ptr(pos, torch.int32, self.A, "pos"),
            _ptr(dlogits, f32, self.T * self.E, "dlogits"), _ptr(Wg, f32, self.d * self.E, "Wg"),
            _ptr(dX, self.elt, self.T * self.d, "dX"), _stream()), "moe_input_grad")


class LayerBuffers:
    """Every device buffer of one layer pass, allocated once (nothing is allocated per step)."""

    def __init__(self, hd: Handle, backward: bool):
        dev, e = hd.device, hd.elt
        f32 = dict(dtype=torch.float32, device=dev)
        i32 = dict(dtype=torch.int32, device=dev)
        T, d, h, E, A, G = hd.T, hd.d, hd.h, hd.E, hd.A, hd.G
        self.logits = torch.empty(T, E, **f32)
        self.idx = torch.empty(T, hd.k, **i32)
        self.w = torch.empty(T, hd.k, **f32)
        self.counts = torch.empty(E, **i32)
        self.layout = hd.new_layout()
        self.Xp = torch.empty(A, d, dtype=e, device=dev)
        self.Yp = torch.empty(A, d, dtype=e, device=dev)
        self.Z = torch.empty(A, h, dtype=e, device=dev)
        self.U = torch.empty(A, h, dtype=e, device=dev) if hd.swiglu else None
        self.out = torch.empty(T, d, dtype=e, device=dev)
        if backward:
            self.dYp = torch.empty(A, d, dtype=e, device=dev)
            self.dw = torch.empty(T, hd.k, **f32)
            self.dXp = torch.empty(A, d, dtype=e, device=dev)
            self.dW1 = torch.empty(G, d, h, **f32)
            self.dW2 = torch.empty(G, h, d, **f32)
            self.dW3 = torch.empty(G, d, h, **f32) if hd.swiglu else None
            self.dX = torch.empty(T, d, dtype=e, device=dev)
            self.dlogits = torch.empty(T, E, **f32)


def layer_forward(hd: Handle, b: LayerBuffers, X, Wg, bg, expert_dest, W1, W2, W3):
    """The forward calls in order; rows of other destinations in b.Yp are left as the caller set them."""
    hd.gate_topk(X, Wg, bg, b.logits, b.idx, b.w)
    hd.expert_counts(b.idx, b.counts)
    hd.dispatch_after_counts(expert_dest, X, b.idx, b.counts, b.layout, b.Xp)   # same idx, same workspace, nothing in between
    hd.expert_ffn_fwd(b.Xp, b.layout, W1, W2, W3, b.Yp, b.Z, b.U)
    hd.combine(b.Yp, b.layout.pos, b.w, b.out)


def layer_backward(hd: Handle, b: LayerBuffers, dOut, W1, W2, W3):
    """The backward calls in order; rows of other destinations in b.dXp are left as the caller set them."""
    hd.combine_bwd(dOut, b.Yp, b.layout.pos, b.w, b.dYp, b.dw)
    hd.expert_ffn_bwd(b.dYp, b.Xp, b.Z, b.U, b.layout, W1, W2, W3, b.dXp, b.dW1, b.dW2, b.dW3)
    hd.dispatch_bwd(b.dXp, b.layout.pos, b.dX)
    hd.gate_bwd(b.dw, b.logits, b.idx, b.dlogits)
