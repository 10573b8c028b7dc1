"""Expert computation (Section 4.2, Eq. 2-3) on a row space whose hidden activations exceed 2^31 elements
and whose largest group exceeds 2^32 bytes per hidden matrix: element offsets must be 64-bit and the
32-bit offsets of the buffer loads of the weight-gradient contraction must be re-based on the way.
Sampled rows and hidden units against the oracle; the rows sit at the start, around the 2^31-element
and 2^32-byte marks, at the group boundary and at the end."""
import numpy as np
import pytest
import torch

import gpu_util as G
from paper_2411_10003_amd import binding, workload as wl

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(600)
def test_rows_beyond_32_bit_offsets():
    d, h, act, dt = 64, 14336, "swiglu", "bf16"
    rows = [160000, 3840]
    A = sum(rows)
    assert A * h > 2 ** 31 and rows[0] * h * 2 > 2 ** 32
    tol = G.TOL[dt]
    rng = np.random.default_rng(4242)

    def draw(*shape, scale=1.0):
        a = (rng.standard_normal(shape) * scale).astype(np.float32)
        wl.round_to_bf16(a)
        return a
    X, dY = draw(A, d), draw(A, d)
    W1, W3, W2 = draw(2, d, h, scale=d ** -0.5), draw(2, d, h, scale=d ** -0.5), draw(2, h, d, scale=h ** -0.5)
    idx = np.repeat(np.arange(2, dtype=np.int32), rows)          # expert of every row; k = 1, rows in group order
    goe = np.arange(2, dtype=np.int32)

    hd = binding.Handle(T=A, d=d, h=h, E=2, k=1, P=1, self_dest=0, G=2, dtype=dt, act=act, renorm=0, device=G.DEV)
    L = hd.new_layout()
    L.slot_offsets.copy_(torch.tensor([0, rows[0], A], dtype=torch.int32))
    L.dest_slots.copy_(torch.tensor([0, 2], dtype=torch.int32))
    bf = dict(dtype=torch.bfloat16, device=G.DEV)
    dXp_in, ddY = G.dev(X, dt), G.dev(dY, dt)
    dW = [G.dev(w, dt) for w in (W1, W2, W3)]
    Yp, Z, U = torch.zeros(A, d, **bf), torch.empty(A, h, **bf), torch.empty(A, h, **bf)
    dXp = torch.zeros(A, d, **bf)
    g1 = torch.empty(2, d, h, dtype=torch.float32, device=G.DEV)
    g3 = torch.empty_like(g1)
    g2 = torch.empty(2, h, d, dtype=torch.float32, device=G.DEV)
    print("[large rows] device pass", flush=True)
    hd.expert_ffn_fwd(dXp_in, L, dW[0], dW[1], dW[2], Yp, Z, U)
    hd.expert_ffn_bwd(ddY, dXp_in, Z, U, L, dW[0], dW[1], dW[2], dXp, g1, g2, g3)
    torch.cuda.synchronize()

    m31 = 2 ** 31 // h                                           # first row whose elements lie past 2^31
    m32 = 2 ** 32 // (2 * h)                                     # first row past 2^32 bytes
    sample = sorted(set([0, 1, 255, 256, m31 - 1, m31, m31 + 1, m32 - 1, m32, m32 + 1, rows[0] - 1, rows[0], rows[0] + 1, A - 1]
                        + [int(x) for x in rng.integers(0, A, 12)]))
    a_s = np.array(sample, dtype=np.int32)
    print("[large rows] sampled rows", flush=True)
    Yo, Zo, Uo, _ = G.orc.ffn_fwd(X, idx, goe, W1, W2, W3, 1, act, a_s, True)
    r = torch.from_numpy(a_s.astype(np.int64)).to(G.DEV)
    assert G.rel_l2(G.host(Yp[r]), Yo) <= tol
    assert G.rel_l2(G.host(Z[r]), Zo) <= tol
    assert G.rel_l2(G.host(U[r]), Uo) <= tol
    dXo = G.orc.ffn_bwd_rows(X, idx, goe, W1, W2, W3, 1, act, a_s, dY[a_s].astype(np.float64))
    assert G.rel_l2(G.host(dXp[r]), dXo) <= tol
    print("[large rows] sampled hidden units", flush=True)
    for g in range(2):
        for j in (0, 4097, h - 1):
            r2, c1, c3 = G.orc.ffn_bwd_hidden(X, idx, goe, W1, W2, W3, 1, act, dY, g, j)
            assert G.rel_l2(G.host(g2[g, j, :]), r2) <= tol, (g, j)
            assert G.rel_l2(G.host(g1[g, :, j]), c1) <= tol, (g, j)
            assert G.rel_l2(G.host(g3[g, :, j]), c3) <= tol, (g, j)
