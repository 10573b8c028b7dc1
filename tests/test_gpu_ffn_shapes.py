"""A sweep of seeded shapes through the grouped FFN, forward and backward, against the oracle: contraction lengths from
one pair of slices to a few hundred, hidden and model widths that are odd multiples of 64, token counts that leave
ragged and empty groups, both activations, k = 1 and 2.  The checks are those of test_gpu_parity.py (row by row)."""
import numpy as np
import pytest

from paper_2411_10003_amd import workload as wl
import test_gpu_parity as P

pytestmark = pytest.mark.gpu

G = P.G          # module-scoped fixtures of the parity tests
orc = P.orc


def _shapes():
    rng = np.random.default_rng(20241128)
    out = []
    for i in range(14):
        d = int(rng.choice([64, 128, 192, 320, 448, 576, 1024]))
        h = int(rng.choice([64, 128, 192, 320, 704, 1088, 2048]))
        T = int(rng.integers(150, 1800))
        E, P_ = [(8, 4), (16, 8), (32, 8), (16, 4)][int(rng.integers(0, 4))]
        k = int(rng.integers(1, 3))
        act = "swiglu" if rng.integers(0, 2) else "gelu"
        base = 3 if act == "swiglu" else 1
        out.append(wl.scaled(wl.CONFIGS[base], T=T, d=d, h=h, E=E, k=k, P=P_, act=act, backward=True,
                             n_replicas=int(rng.integers(0, 3)), alpha=float(rng.choice([0.0, 1.0, 1.6]))))
    return out


SHAPES = _shapes()


@pytest.mark.parametrize("cfg", SHAPES, ids=lambda c: f"{c.act}-T{c.T}-d{c.d}-h{c.h}-E{c.E}-k{c.k}-r{c.n_replicas}")
def test_forward(G, orc, cfg):
    P.test_ffn_forward_and_combine(G, orc, cfg)


@pytest.mark.parametrize("cfg", SHAPES, ids=lambda c: f"{c.act}-T{c.T}-d{c.d}-h{c.h}-E{c.E}-k{c.k}-r{c.n_replicas}")
def test_backward(G, orc, cfg):
    P.test_backward_calls(G, orc, cfg)
