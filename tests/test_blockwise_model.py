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


@pytest.mark.parametrize("with_gates", [False, True])
@pytest.mark.parametrize("lengths", [[48, 48, 48], [64, 32, 20], [16, 96, 1]])
def test_sequence_split_into_segments_reproduces_the_walk(oracle, lengths, with_gates):
    """The sequence-parallel scheme of Sec. 3.5 as the kernels read it, in fp64 on the CPU: every segment runs the
    block recipe on its own tokens only (chunks of 16, super-blocks of 2 chunks here); a query's state is carried to
    its segment's left edge; a hop attends ALL keys of an earlier segment -- keys carried to their super-block's
    right edge, one product per super-block, the first one's included -- and partial softmaxes are merged through
    their running maximum and sum.  With forget gates every segment counts its gate sums from its own start and a
    hop adds the totals of the segments passed.  The result equals the token walk over the whole sequence."""
    C, SB, d, scale = 16, 2, 8, 0.4
    L = sum(lengths)
    x = _head(L, d, 31 + L)
    logf = None
    if with_gates:
        logf = -np.log1p(np.exp(-np.random.default_rng(L).normal(1.0, 1.0, L)))
    args = [x[n][None, None] for n in ("q", "k", "v", "w", "beta")]
    o_ref, lse_ref = oracle.fwd(*args, scale, logf=None if logf is None else logf[None, None])
    starts = np.concatenate([[0], np.cumsum(lengths)])

    def prep_segment(a, b):
        n = b - a
        nc = -(-n // C)
        pad = lambda t: bm._pad(t[a:b], nc * C)
        q, k, v, w, beta = (pad(x[m]) for m in ("q", "k", "v", "w", "beta"))
        pre = [bm.chunk_prep(q[c * C:(c + 1) * C], k[c * C:(c + 1) * C], w[c * C:(c + 1) * C], beta[c * C:(c + 1) * C]) for c in range(nc)]
        # second level: keys carried to their super-block's right edge, super-block products
        kb2, p2 = [None] * nc, []
        for J in range(-(-nc // SB)):
            R = np.eye(d)
            for c in range(min((J + 1) * SB, nc) - 1, J * SB - 1, -1):
                kb2[c] = pre[c]["Kb"] @ R.T
                R = R @ (np.eye(d) - pre[c]["dP"])
            p2.append(R)
        cum = np.cumsum(bm._pad(logf[a:b], nc * C)) if logf is not None else np.zeros(nc * C)
        return dict(n=n, nc=nc, pre=pre, kb2=kb2, p2=p2, v=v, cum=cum)

    seg = [prep_segment(int(starts[r]), int(starts[r + 1])) for r in range(len(lengths))]
    o = np.zeros((L, d))
    lse = np.zeros(L)
    for r, s in enumerate(seg):
        nc = s["nc"]
        for c in range(nc):
            rows = slice(c * C, (c + 1) * C)
            # own segment: diagonal block, then the chunks to the left one by one; the product of chunk 0 too
            X = s["pre"][c]["Qb"].copy()
            S = [np.where(np.tril(np.ones((C, C))) > 0, scale * s["pre"][c]["Sd"] - s["cum"][None, rows], -np.inf)]
            V = [s["v"][rows]]
            for j in range(c - 1, -1, -1):
                S.append(scale * X @ s["pre"][j]["Kb"].T - s["cum"][None, j * C:(j + 1) * C])
                V.append(s["v"][j * C:(j + 1) * C])
                X = X - X @ s["pre"][j]["dP"]
            passed = 0.0
            for t in range(r - 1, -1, -1):             # hops, nearest earlier segment first
                e = seg[t]
                assert e["n"] == e["nc"] * C            # an earlier segment is a whole number of chunks
                total = e["cum"][-1]
                for j in range(e["nc"] - 1, -1, -1):
                    S.append(scale * X @ e["kb2"][j].T + (passed + total - e["cum"][None, j * C:(j + 1) * C]))
                    V.append(e["v"][j * C:(j + 1) * C])
                    if j % SB == 0:
                        X = X @ e["p2"][j // SB]
                passed += total
            S = np.concatenate(S, axis=1)
            V = np.concatenate(V, axis=0)
            m = S.max(axis=1, keepdims=True)
            P = np.exp(S - m)
            l = P.sum(axis=1, keepdims=True)
            g0 = int(starts[r]) + c * C
            nrow = min(C, s["n"] - c * C)
            o[g0:g0 + nrow] = (P @ V / l)[:nrow]
            lse[g0:g0 + nrow] = (m + np.log(l) + s["cum"][rows, None])[:nrow, 0]
    np.testing.assert_allclose(o, o_ref[0, 0], atol=1e-10)
    np.testing.assert_allclose(lse, lse_ref[0, 0], atol=1e-10)
