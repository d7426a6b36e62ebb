"""NumPy fp64 model of the paper's BLOCKWISE recipe (Sec. 3.2-3.3) -- test helper.

It is neither the oracle (which is the token walk in oracle/) nor the GPU code:
it exists so that the reading of the blockwise formulas that the kernels
implement -- chunk UT transform, boundary-adjusted queries/keys, chunk
products, right-to-left scan, and the hand-derived chunk-level backward -- can
be checked against the oracle on the CPU at several chunk sizes.

Row-vector convention, one head at a time, chunk c = tokens [cC,(c+1)C):

    G  = W W^T                     A = I + strictLower(diag(beta) G)
    N  = A^{-1} diag(beta)         (the paper's T^{-1} of the chunk)
    U  = N W                       dP = W^T U    (chunk product P = I - dP)
    F  = tril(Q W^T)               Y  = N strictLower(W K^T)
    Qb = Q - F U                   Kb = K - Y^T W
    Sd = tril(Q K^T - F Y)         (diagonal block, unscaled)
    scan: X = Qb_c; for j = c-1..0: S_cj = X Kb_j^T ; X <- X - X dP_j
"""
import numpy as np


def chunk_prep(Q, K, W, beta):
    C = Q.shape[0]
    G = W @ W.T
    A = np.eye(C) + np.tril(beta[:, None] * G, -1)
    Ainv = np.linalg.inv(A)
    N = Ainv * beta[None, :]
    U = N @ W
    dP = W.T @ U
    F = np.tril(Q @ W.T)
    Gk = np.tril(W @ K.T, -1)
    Y = N @ Gk
    Qb = Q - F @ U
    Kb = K - Y.T @ W
    Sd = np.tril(Q @ K.T - F @ Y)
    return dict(G=G, Ainv=Ainv, N=N, U=U, dP=dP, F=F, Gk=Gk, Y=Y, Qb=Qb, Kb=Kb, Sd=Sd)


def _pad(x, Lp):
    pad = [(0, Lp - x.shape[0])] + [(0, 0)] * (x.ndim - 1)
    return np.pad(x, pad)


def logits_blockwise(q, k, w, beta, C, scale):
    """Dense lower-triangular scaled logits [L,L] of one head via the block recipe."""
    L, d = q.shape
    nc = -(-L // C)
    Lp = nc * C
    q, k, w, beta = (_pad(x, Lp) for x in (q, k, w, beta))   # padding: beta = 0 => H = I
    pre = [chunk_prep(q[c * C:(c + 1) * C], k[c * C:(c + 1) * C], w[c * C:(c + 1) * C],
                      beta[c * C:(c + 1) * C]) for c in range(nc)]
    S = np.zeros((Lp, Lp))
    for c in range(nc):
        S[c * C:(c + 1) * C, c * C:(c + 1) * C] = pre[c]["Sd"]
        X = pre[c]["Qb"].copy()
        for j in range(c - 1, -1, -1):
            S[c * C:(c + 1) * C, j * C:(j + 1) * C] = X @ pre[j]["Kb"].T
            X = X - X @ pre[j]["dP"]
    return scale * S[:L, :L], pre


def forward_blockwise(q, k, v, w, beta, C, scale):
    L = q.shape[0]
    S, _ = logits_blockwise(q, k, w, beta, C, scale)
    mask = np.tril(np.ones((L, L), dtype=bool))
    S = np.where(mask, S, -np.inf)
    m = S.max(-1, keepdims=True)
    e = np.exp(S - m)
    z = e.sum(-1, keepdims=True)
    return (e / z) @ v, (m + np.log(z))[:, 0]


def chunk_prep_backward(Q, K, W, beta, pre, dQb, dKb, ddP, dSd):
    """Adjoint of chunk_prep: gradients w.r.t. Q, K, W, beta of the chunk, given
    gradients of its outputs Qb, Kb, dP and Sd (dSd is used on its lower triangle)."""
    N, U, F, Gk, Y, G, Ainv = (pre[n] for n in ("N", "U", "F", "Gk", "Y", "G", "Ainv"))
    dSd = np.tril(dSd)
    dQ = dQb + dSd @ K
    dK = dKb + dSd.T @ Q
    dF = -dSd @ Y.T - dQb @ U.T
    dY = -F.T @ dSd - W @ dKb.T
    dU = -F.T @ dQb + W @ ddP
    dW = -Y @ dKb + U @ ddP.T
    dF = np.tril(dF)
    dQ += dF @ W
    dW += dF.T @ Q
    dN = dY @ Gk.T + dU @ W.T
    dGk = np.tril(N.T @ dY, -1)
    dW += dGk @ K + N.T @ dU
    dK += dGk.T @ W
    R = Ainv.T @ dN                      # A^{-T} dN
    dbeta = np.diag(R).copy()            # from N = A^{-1} diag(beta)
    M = np.tril(-R @ N.T, -1)            # dA restricted to the strict lower triangle
    dbeta += (M * G).sum(-1)             # from A = I + strictLower(diag(beta) G)
    dG = beta[:, None] * M
    dW += (dG + dG.T) @ W
    return dQ, dK, dW, dbeta


def backward_blockwise(q, k, v, w, beta, dO, C, scale):
    """dq, dk, dv, dw, dbeta of sum(dO*o) via the block recipe (one head)."""
    L, d = q.shape
    nc = -(-L // C)
    Lp = nc * C
    S, pre = logits_blockwise(q, k, w, beta, C, scale)
    mask = np.tril(np.ones((L, L), dtype=bool))
    Sm = np.where(mask, S, -np.inf)
    m = Sm.max(-1, keepdims=True)
    e = np.exp(Sm - m)
    P = e / e.sum(-1, keepdims=True)
    o = P @ v
    delta = (dO * o).sum(-1, keepdims=True)
    dS = scale * P * (dO @ v.T - delta)          # gradient w.r.t. the UNSCALED block logits
    dv = P.T @ dO
    dSp = np.zeros((Lp, Lp)); dSp[:L, :L] = dS
    qp, kp, wp, bp = (_pad(x, Lp) for x in (q, k, w, beta))
    dQb = np.zeros((Lp, d)); dKb = np.zeros((Lp, d)); ddP = np.zeros((nc, d, d))
    sl = lambda c: slice(c * C, (c + 1) * C)
    for c in range(nc):
        Xs = {}
        X = pre[c]["Qb"].copy()
        for j in range(c - 1, -1, -1):
            Xs[j] = X
            X = X - X @ pre[j]["dP"]
        dXn = np.zeros((C, d))
        for j in range(c):                        # adjoint runs left to right
            dSj = dSp[sl(c), sl(j)]
            ddP[j] -= Xs[j].T @ dXn
            dKb[sl(j)] += dSj.T @ Xs[j]
            dXn = dSj @ pre[j]["Kb"] + dXn - dXn @ pre[j]["dP"].T
        dQb[sl(c)] = dXn
    dq = np.zeros((Lp, d)); dk = np.zeros((Lp, d)); dw = np.zeros((Lp, d)); db = np.zeros(Lp)
    for c in range(nc):
        a, b_, c_, e_ = chunk_prep_backward(qp[sl(c)], kp[sl(c)], wp[sl(c)], bp[sl(c)], pre[c],
                                            dQb[sl(c)], dKb[sl(c)], ddP[c], dSp[sl(c), sl(c)])
        dq[sl(c)], dk[sl(c)], dw[sl(c)], db[sl(c)] = a, b_, c_, e_
    return dq[:L], dk[:L], dv, dw[:L], db[:L]
