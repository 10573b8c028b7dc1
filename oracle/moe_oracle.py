"""ctypes front end of the CPU oracle (moe_oracle.c) -- TEST INFRASTRUCTURE, NOT PRODUCT.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this module.  It
marshals numpy arrays into the C functions and strings them together in the order the
layer runs; every piece of arithmetic lives in the C file.  It imports nothing from the
GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")

ACT = {"gelu": 0, "swiglu": 1}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Contraction and fast-math stay off: the gate order is exact."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-mavx2", "-mfma",
               "-ffp-contract=off", "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def gate_logits(X, Wg, bg) -> np.ndarray:
    X, Wg, bg = _f32(X), _f32(Wg), _f32(bg)
    T, d = X.shape
    E = Wg.shape[1]
    assert Wg.shape[0] == d and bg.shape == (E,)
    out = np.empty((T, E), dtype=np.float32)
    lib().orc_gate_logits(_p(X), _p(Wg), _p(bg), T, d, E, _p(out))
    return out


def topk(logits, k: int, renorm: int):
    logits = _f32(logits)
    T, E = logits.shape
    assert 1 <= k <= E
    idx = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float64)
    probs = np.empty((T, E), dtype=np.float64)
    lib().orc_topk(_p(logits), T, E, k, int(renorm), _p(idx), _p(w), _p(probs))
    return idx, w, probs


def counts(idx, E: int) -> np.ndarray:
    idx = _i32(idx).reshape(-1)
    assert idx.size == 0 or (idx.min() >= 0 and idx.max() < E)
    out = np.empty(E, dtype=np.int32)
    lib().orc_counts(_p(idx), idx.size, E, _p(out))
    return out


def layout(cnt, expert_dest, P: int):
    cnt, expert_dest = _i32(cnt), _i32(expert_dest)
    E = cnt.size
    slot_of_expert = np.empty(E, dtype=np.int32)
    slot_offsets = np.empty(E + 1, dtype=np.int32)
    dest_offsets = np.empty(P + 1, dtype=np.int32)
    dest_slots = np.empty(P + 1, dtype=np.int32)
    rc = lib().orc_layout(_p(cnt), _p(expert_dest), E, P, _p(slot_of_expert), _p(slot_offsets),
                          _p(dest_offsets), _p(dest_slots))
    if rc != 0:
        raise ValueError("expert_dest out of range")
    return slot_of_expert, slot_offsets, dest_offsets, dest_slots


def positions(idx, slot_of_expert, slot_offsets):
    idx = _i32(idx).reshape(-1)
    A, E = idx.size, len(slot_of_expert)
    pos = np.empty(A, dtype=np.int32)
    perm = np.empty(A, dtype=np.int32)
    lib().orc_positions(_p(idx), A, E, _p(_i32(slot_of_expert)), _p(_i32(slot_offsets)), _p(pos), _p(perm))
    return pos, perm


def dispatch(X, perm, k: int) -> np.ndarray:
    X, perm = _f32(X), _i32(perm)
    A, d = perm.size, X.shape[1]
    Xp = np.empty((A, d), dtype=np.float32)
    lib().orc_dispatch(_p(X), _p(perm), A, d, k, _p(Xp))
    return Xp


def ffn_fwd(X, idx, group_of_expert, W1, W2, W3, k: int, act: str, a_list, want_hidden: bool = False):
    """Expert FFN of the listed assignments.  Returns Y[n,d] (and Z, U, Act [n,h] if asked)."""
    X, idx, goe, a_list = _f32(X), _i32(idx).reshape(-1), _i32(group_of_expert), _i32(a_list)
    W1, W2 = _f32(W1), _f32(W2)
    W3 = _f32(W3) if act == "swiglu" else None
    d, h, n = X.shape[1], W1.shape[2], a_list.size
    assert W1.shape[1] == d and W2.shape[1:] == (h, d)
    Y = np.empty((n, d), dtype=np.float64)
    Z = np.empty((n, h), dtype=np.float64) if want_hidden else None
    U = np.empty((n, h), dtype=np.float64) if (want_hidden and W3 is not None) else None
    Act = np.empty((n, h), dtype=np.float64) if want_hidden else None
    rc = lib().orc_ffn_fwd(_p(X), _p(idx), _p(goe), _p(W1), _p(W2), _p(W3), d, h, k, ACT[act],
                           _p(a_list), n, _p(Y), _p(Z), _p(U), _p(Act))
    if rc != 0:
        raise ValueError("assignment of an expert that is not hosted")
    if want_hidden:
        return Y, Z, U, Act
    return Y


def combine(Yp, pos, w, k: int, t_list=None) -> np.ndarray:
    Yp, pos, w = _f64(Yp), _i32(pos), _f64(w)
    d = Yp.shape[1]
    T = pos.size // k
    t_list = np.arange(T, dtype=np.int32) if t_list is None else _i32(t_list)
    out = np.empty((t_list.size, d), dtype=np.float64)
    lib().orc_combine(_p(Yp), _p(pos), _p(w), d, k, _p(t_list), t_list.size, _p(out))
    return out


def combine_bwd(dOut, Yp, pos, w, k: int):
    dOut, Yp, pos, w = _f32(dOut), _f64(Yp), _i32(pos), _f64(w)
    T, d = dOut.shape
    dYp = np.empty((T * k, d), dtype=np.float64)
    dw = np.empty((T, k), dtype=np.float64)
    lib().orc_combine_bwd(_p(dOut), _p(Yp), _p(pos), _p(w), T, d, k, _p(dYp), _p(dw))
    return dYp, dw


def ffn_bwd_rows(X, idx, group_of_expert, W1, W2, W3, k: int, act: str, a_list, dY) -> np.ndarray:
    X, idx, goe, a_list = _f32(X), _i32(idx).reshape(-1), _i32(group_of_expert), _i32(a_list)
    W1, W2 = _f32(W1), _f32(W2)
    W3 = _f32(W3) if act == "swiglu" else None
    dY = _f64(dY)
    d, h, n = X.shape[1], W1.shape[2], a_list.size
    assert dY.shape == (n, d)
    dX = np.empty((n, d), dtype=np.float64)
    rc = lib().orc_ffn_bwd_rows(_p(X), _p(idx), _p(goe), _p(W1), _p(W2), _p(W3), d, h, k, ACT[act],
                                _p(a_list), n, _p(dY), _p(dX))
    if rc != 0:
        raise ValueError("assignment of an expert that is not hosted")
    return dX


def ffn_bwd_hidden(X, idx, group_of_expert, W1, W2, W3, k: int, act: str, dYa, g: int, j: int):
    """(dW2[g][j,:], dW1[g][:,j], dW3[g][:,j] or None) for one hidden unit of one group."""
    X, idx, goe = _f32(X), _i32(idx).reshape(-1), _i32(group_of_expert)
    W1, W2 = _f32(W1), _f32(W2)
    W3 = _f32(W3) if act == "swiglu" else None
    dYa = _f32(dYa)
    d, h, A = X.shape[1], W1.shape[2], idx.size
    assert dYa.shape == (A, d) and 0 <= j < h and 0 <= g < W1.shape[0]
    r2 = np.empty(d, dtype=np.float64)
    c1 = np.empty(d, dtype=np.float64)
    c3 = np.empty(d, dtype=np.float64) if W3 is not None else None
    lib().orc_ffn_bwd_hidden(_p(X), _p(idx), _p(goe), _p(W1), _p(W2), _p(W3), d, h, k, A, ACT[act],
                             _p(dYa), int(g), int(j), _p(r2), _p(c1), _p(c3))
    return r2, c1, c3


def ffn_bwd_hidden_many(X, idx, group_of_expert, W1, W2, W3, k: int, act: str, dYa, g: int, js):
    """ffn_bwd_hidden for several hidden units of one group (one per thread): rows of (dW2[g][js,:],
    dW1[g][:,js].T, dW3[g][:,js].T or None)."""
    X, idx, goe = _f32(X), _i32(idx).reshape(-1), _i32(group_of_expert)
    W1, W2 = _f32(W1), _f32(W2)
    W3 = _f32(W3) if act == "swiglu" else None
    dYa, js = _f32(dYa), _i32(js).reshape(-1)
    d, h, A = X.shape[1], W1.shape[2], idx.size
    assert dYa.shape == (A, d) and 0 <= g < W1.shape[0] and (js.size == 0 or (js.min() >= 0 and js.max() < h))
    r2 = np.empty((js.size, d), dtype=np.float64)
    c1 = np.empty((js.size, d), dtype=np.float64)
    c3 = np.empty((js.size, d), dtype=np.float64) if W3 is not None else None
    lib().orc_ffn_bwd_hidden_many(_p(X), _p(idx), _p(goe), _p(W1), _p(W2), _p(W3), d, h, k, A, ACT[act],
                                  _p(dYa), int(g), _p(js), int(js.size), _p(r2), _p(c1), _p(c3))
    return r2, c1, c3


def ffn_bwd_weights(X, idx, group_of_expert, W1, W2, W3, k: int, act: str, dYa, G: int):
    """Full weight gradients (small cases): loops ffn_bwd_hidden over every group and hidden unit."""
    d, h = X.shape[1], W1.shape[2]
    dW1 = np.zeros((G, d, h))
    dW2 = np.zeros((G, h, d))
    dW3 = np.zeros((G, d, h)) if act == "swiglu" else None
    for g in range(G):
        for j in range(h):
            r2, c1, c3 = ffn_bwd_hidden(X, idx, group_of_expert, W1, W2, W3, k, act, dYa, g, j)
            dW2[g, j, :] = r2
            dW1[g, :, j] = c1
            if dW3 is not None:
                dW3[g, :, j] = c3
    return dW1, dW2, dW3


def dispatch_bwd(dXp, pos, k: int) -> np.ndarray:
    dXp, pos = _f64(dXp), _i32(pos)
    d = dXp.shape[1]
    T = pos.size // k
    dX = np.empty((T, d), dtype=np.float64)
    lib().orc_dispatch_bwd(_p(dXp), _p(pos), T, d, k, _p(dX))
    return dX


def gate_bwd(dw, logits, idx, renorm: int) -> np.ndarray:
    dw, logits, idx = _f64(dw), _f32(logits), _i32(idx)
    T, E = logits.shape
    k = idx.shape[1]
    out = np.empty((T, E), dtype=np.float64)
    lib().orc_gate_bwd(_p(dw), _p(logits), _p(idx), T, E, k, int(renorm), _p(out))
    return out


def gate_bwd_params(X, dlogits):
    """dWg[d,E], dbg[E] of the gate's linear map."""
    X, dlogits = _f32(X), _f64(dlogits)
    T, d = X.shape
    E = dlogits.shape[1]
    dWg = np.empty((d, E), dtype=np.float64)
    dbg = np.empty(E, dtype=np.float64)
    lib().orc_gate_bwd_params(_p(X), _p(dlogits), T, d, E, _p(dWg), _p(dbg))
    return dWg, dbg


def input_grad(dXp, pos, dlogits, Wg, k: int) -> np.ndarray:
    """Expert-path plus gate-path gradient of the layer input."""
    dXp, pos, dlogits, Wg = _f64(dXp), _i32(pos), _f64(dlogits), _f32(Wg)
    d, E = Wg.shape
    T = pos.size // k
    dX = np.empty((T, d), dtype=np.float64)
    lib().orc_input_grad(_p(dXp), _p(pos), _p(dlogits), _p(Wg), T, d, E, k, _p(dX))
    return dX


# ------------------------------------------------------------------------------------------
# The layer in call order (routing part is cheap and always complete; the FFN part is
# evaluated for the assignments asked for).

def route(X, Wg, bg, k: int, renorm: int) -> Dict[str, np.ndarray]:
    logits = gate_logits(X, Wg, bg)
    idx, w, probs = topk(logits, k, renorm)
    E = Wg.shape[1]
    return {"logits": logits, "idx": idx, "w": w, "probs": probs, "counts": counts(idx, E)}


def place(idx, cnt, expert_dest, P: int) -> Dict[str, np.ndarray]:
    slot_of_expert, slot_offsets, dest_offsets, dest_slots = layout(cnt, expert_dest, P)
    pos, perm = positions(idx, slot_of_expert, slot_offsets)
    return {"slot_of_expert": slot_of_expert, "slot_offsets": slot_offsets, "dest_offsets": dest_offsets,
            "dest_slots": dest_slots, "pos": pos, "perm": perm}


def hosted_assignments(idx, group_of_expert) -> np.ndarray:
    """Assignment ids (ascending) whose expert is computed on this device."""
    goe = _i32(group_of_expert)
    return np.nonzero(goe[_i32(idx).reshape(-1)] >= 0)[0].astype(np.int32)
