"""The blockwise recipe (paper Sec. 3.2-3.3) reproduces the token walk for any
chunk size, forward and backward -- the paper's claim that local inversions
give the same result.  Checks the reading of the block formulas (product
order, which masks are strict, missing "I -" in the chunk product) that the
GPU kernels implement, before any GPU is involved."""
import numpy as np
import pytest

import blockwise_model as bm
from paper_2505_16381_amd import synth_inputs as si


def _head(L, d, seed):
    x = si.make_inputs(1, 1, L, d, "bf16", seed, 0.0, with_do=True)
    x = {n: a[0, 0].astype(np.float64) for n, a in x.items()}
    x["beta"][3 % L] = 0.0
    x["beta"][5 % L] = 1.0
    x["beta"][7 % L] = 2.0
    return x


@pytest.mark.parametrize("C", [1, 2, 16, 64])
@pytest.mark.parametrize("L", [64, 150])
def test_forward_blockwise_equals_walk(oracle, C, L):
    d = 8
    x = _head(L, d, 21)
    o_ref, lse_ref = oracle.fwd(*(x[n][None, None] for n in ("q", "k", "v", "w", "beta")), 0.4)
    o, lse = bm.forward_blockwise(x["q"], x["k"], x["v"], x["w"], x["beta"], C, 0.4)
    np.testing.assert_allclose(o, o_ref[0, 0], atol=1e-11)
    np.testing.assert_allclose(lse, lse_ref[0, 0], atol=1e-11)


@pytest.mark.parametrize("C", [4, 64])
def test_backward_blockwise_equals_walk_adjoint(oracle, C):
    L, d = 150, 8
    x = _head(L, d, 22)
    ref = oracle.bwd(*(x[n][None, None] for n in ("q", "k", "v", "w", "beta", "dO")), 0.4)
    got = bm.backward_blockwise(x["q"], x["k"], x["v"], x["w"], x["beta"], x["dO"], C, 0.4)
    for name, r, g in zip(("dq", "dk", "dv", "dw", "dbeta"), ref, got):
        assert np.abs(r[0, 0] - g).max() < 1e-10 * max(1.0, np.abs(r).max()), name


def test_chunk_product_and_boundary_rows():
    """P = I - dP is the product of the chunk's H in descending order; row t of Qb
    is q_t carried to the chunk's left edge, row s of Kb is k_s carried to its right edge."""
    C, d = 16, 6
    x = _head(C, d, 23)
    pre = bm.chunk_prep(x["q"], x["k"], x["w"], x["beta"])
    Hs = [np.eye(d) - x["beta"][t] * np.outer(x["w"][t], x["w"][t]) for t in range(C)]
    seq = np.eye(d)
    for t in range(C):
        seq = Hs[t] @ seq                       # H_{C-1} ... H_0
    np.testing.assert_allclose(np.eye(d) - pre["dP"], seq, atol=1e-12)
    for t in range(C):
        u = x["q"][t].copy()
        for s in range(t, -1, -1):
            u = Hs[s] @ u                       # H_0 ... H_t q_t
        np.testing.assert_allclose(pre["Qb"][t], u, atol=1e-12)
        z = x["k"][t].copy()
        for s in range(t + 1, C):
            z = Hs[s] @ z                       # H_{C-1} ... H_{t+1} k_t
        np.testing.assert_allclose(pre["Kb"][t], z, atol=1e-12)
