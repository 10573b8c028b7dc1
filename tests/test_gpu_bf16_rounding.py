"""The fp32 -> bf16 rounding behind every bf16 output of the library (one hardware conversion per pair of values):
round to nearest, ties to even, NaN stays NaN, checked bit for bit against the definition written out on integers."""
import numpy as np
import pytest
import torch

import gpu_util as G
from paper_2411_10003_amd import binding

pytestmark = pytest.mark.gpu


def _rne(bits: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even of fp32 bit patterns to their upper 16 bits (inputs that are not NaN)."""
    b = bits.astype(np.uint64)
    return (((b + 0x7FFF + ((b >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)


def test_rounding_is_nearest_even_and_keeps_nan():
    rng = np.random.default_rng(7)
    special = np.array([0x00000000, 0x80000000, 0x00000001, 0x00007FFF, 0x00008000, 0x00008001, 0x00018000, 0x00017FFF,
                        0x3F800000, 0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001, 0x7F7FFFFF, 0x7F7F8000, 0x7F7F7FFF,
                        0x7F800000, 0xFF800000, 0x007FFFFF, 0x00800000, 0x807F8000, 0xBF808000, 0xBF818000], dtype=np.uint32)
    # every tie (lower half exactly 0x8000) next to an even and an odd kept bit, at random exponents
    hi = rng.integers(0, 0x7F80, 4096, dtype=np.uint32)
    ties = ((hi << 16) | 0x8000).astype(np.uint32)
    rnd = rng.integers(0, 2 ** 32, 1 << 20, dtype=np.uint64).astype(np.uint32)
    bits = np.concatenate([special, ties, ties | 0x80000000, rnd])
    x = torch.from_numpy(bits.view(np.float32).copy()).to(G.DEV)
    out = torch.zeros(bits.size, dtype=torch.int16, device=G.DEV)
    binding.calib_round_bf16(x, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16)
    nan = (bits & 0x7FFFFFFF) > 0x7F800000
    assert np.array_equal(got[~nan], _rne(bits[~nan]))
    assert ((got[nan] & 0x7FFF) > 0x7F80).all()                   # NaN in, NaN out
    assert nan.sum() > 1000 and (~nan).sum() > 1000000
    # a tie goes to the even neighbour, both ways
    assert got[8] == 0x3F80 and got[9] == 0x3F80 and got[10] == 0x3F82 and got[21] == 0xBF80 and got[22] == 0xBF82
    # the largest finite values round to infinity, as the definition says
    assert got[13] == 0x7F80 and got[14] == 0x7F80 and got[15] == 0x7F7F
