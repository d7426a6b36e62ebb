"""Pins of the PaTH-FoX part of the oracle (CPU): the paper's "Extension: PaTH-FoX" formula,
A_ij proportional to (prod_{s=j+1..i} f_s) exp(PaTH logit)."""
import numpy as np
import torch

from oracle import path_oracle
from paper_2505_16381_amd import synth_inputs as si


def _x(L=23, d=6, seed=31, B=1, H=2):
    x = si.make_inputs(B, H, L, d, "fp32", seed, 0.0, with_do=True)
    rng = np.random.default_rng(seed + 1)
    x["logf"] = np.log(1.0 / (1.0 + np.exp(-rng.normal(1.0, 1.0, size=(B, H, L)))))     # log sigmoid
    return x


def test_no_gates_and_unit_gates_are_plain_path():
    x = _x()
    a = path_oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], 0.4)
    b = path_oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], 0.4, logf=np.zeros_like(x["logf"]))
    assert all(np.array_equal(u, v) for u, v in zip(a, b))


def test_beta_zero_is_fox_attention_written_out():
    # H = I: plain softmax attention with the additive bias c_i - c_j, c = cumsum(log f), from textbook formulas
    x = _x(L=17, d=5, seed=8)
    scale = 0.37
    o, lse = path_oracle.fwd(x["q"], x["k"], x["v"], x["w"], np.zeros_like(x["beta"]), scale, logf=x["logf"])
    q, k, v = (x[n].astype(np.float64) for n in "qkv")
    c = np.cumsum(x["logf"], axis=-1)
    z = scale * np.einsum("bhid,bhjd->bhij", q, k) + c[..., :, None] - c[..., None, :]
    z = np.where(np.tril(np.ones((17, 17), bool)), z, -np.inf)
    lse_ref = np.log(np.exp(z).sum(-1))
    o_ref = np.einsum("bhij,bhjd->bhid", np.exp(z - lse_ref[..., None]), v)
    assert np.abs(o - o_ref).max() <= 1e-12 and np.abs(lse - lse_ref).max() <= 1e-12


def test_weights_are_path_weights_times_the_gate_products():
    # the formula itself: unnormalised weight = prod f * exp(PaTH logit); normalise and compare
    x = _x(L=11, d=4, seed=2, H=1)
    scale = 0.5
    S = path_oracle.logits(x["q"][0, 0], x["k"][0, 0], x["w"][0, 0], x["beta"][0, 0], scale)
    f = np.exp(x["logf"][0, 0])
    o, lse = path_oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale, logf=x["logf"])
    for i in range(11):
        wgt = np.array([np.prod(f[j + 1:i + 1]) * np.exp(S[i, j]) for j in range(i + 1)])
        o_ref = (wgt[:, None] * x["v"][0, 0, :i + 1].astype(np.float64)).sum(0) / wgt.sum()
        assert np.abs(o[0, 0, i] - o_ref).max() <= 1e-12
        assert abs(lse[0, 0, i] - np.log(wgt.sum())) <= 1e-12


def _dense_loss(q, k, v, w, beta, logf, dO, scale):
    """Dense torch model (fp64) from explicit d x d transition matrices; autograd gives the gradients."""
    L, d = q.shape
    eye = torch.eye(d, dtype=torch.float64)
    Hs = [eye - beta[t] * torch.outer(w[t], w[t]) for t in range(L)]
    c = torch.cumsum(logf, 0)
    rows = []
    for i in range(L):
        u = q[i]
        zs = []
        for j in range(i, -1, -1):
            zs.append(scale * torch.dot(u, k[j]) + c[i] - c[j])
            u = Hs[j] @ u
        z = torch.stack(zs[::-1])
        p = torch.softmax(z, 0)
        rows.append(p @ v[:i + 1])
    o = torch.stack(rows)
    return (o * dO).sum()


def test_backward_matches_autograd_of_a_dense_model_including_dlogf():
    x = _x(L=14, d=5, seed=77, H=1)
    scale = 0.45
    t = {n: torch.tensor(x[n][0, 0].astype(np.float64), requires_grad=(n != "dO")) for n in ("q", "k", "v", "w", "beta", "logf", "dO")}
    loss = _dense_loss(t["q"], t["k"], t["v"], t["w"], t["beta"], t["logf"], t["dO"], scale)
    loss.backward()
    got = path_oracle.bwd(x["q"], x["k"], x["v"], x["w"], x["beta"], x["dO"], scale, logf=x["logf"])
    for name, g in zip(("q", "k", "v", "w", "beta", "logf"), got):
        ref = t[name].grad.numpy()
        assert np.abs(g[0, 0] - ref).max() <= 1e-10 * max(1.0, np.abs(ref).max()), name
    assert got[5][0, 0, 0] == 0.0        # the first gate is on no path


def test_dlogf_by_central_differences():
    x = _x(L=12, d=4, seed=5, H=1)
    scale = 0.6
    got = path_oracle.bwd(x["q"], x["k"], x["v"], x["w"], x["beta"], x["dO"], scale, logf=x["logf"])[5]
    h = 1e-6
    for s in (1, 5, 11):
        lp, lm = x["logf"].copy(), x["logf"].copy()
        lp[0, 0, s] += h
        lm[0, 0, s] -= h
        op = path_oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale, logf=lp)[0]
        om = path_oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale, logf=lm)[0]
        fd = ((op - om) * x["dO"]).sum() / (2 * h)
        assert abs(fd - got[0, 0, s]) <= 1e-6 * max(1.0, abs(fd))
