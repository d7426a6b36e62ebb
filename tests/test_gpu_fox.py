"""GPU parity of PaTH-FoX (forget-gate bias on the logits) against the oracle (run with -m gpu).
Bars as for plain PaTH: o 1e-4 / lse 1e-3 (fp32 I/O), o 2e-2 / lse 1e-3 (bf16 I/O); gradients
2e-2 relative to the tensor's maximum (bf16), 1e-4 (fp32)."""
import numpy as np
import pytest

from paper_2505_16381_amd import synth_inputs as si

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2505_16381_amd as pa
    assert torch.cuda.is_available()
    pa.load_library()
    return torch, pa


def _inputs(B, H, L, d, dtype, seed, gate_mean=2.0):
    x = si.make_inputs(B, H, L, d, dtype, seed, 0.0, with_do=True)
    rng = np.random.default_rng(seed + 7)
    z = rng.normal(gate_mean, 1.0, size=(B, H, L)).astype(np.float32)
    logf = (-np.log1p(np.exp(-z))).astype(np.float32)                  # log sigmoid(z)
    x["logf"] = si.round_to_bf16(logf) if dtype == "bf16" else logf
    return x


def _dev(gpu, x, dtype):
    torch, _ = gpu
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    return {n: torch.from_numpy(a).to("cuda").to(td).contiguous() for n, a in x.items()}


@pytest.mark.parametrize("dtype,L,d", [("fp32", 64, 64), ("fp32", 300, 128), ("fp32", 1100, 64), ("bf16", 200, 64),
                                       ("bf16", 1030, 128), ("bf16", 2048, 64)])
def test_fox_forward_matches_the_oracle(gpu, oracle, dtype, L, d):
    torch, pa = gpu
    x = _inputs(1, 2, L, d, dtype, 1200 + L + d)
    dv = _dev(gpu, x, dtype)
    scale = d ** -0.5
    o, lse = pa.path_attn_fox_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], dv["logf"], scale=scale)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale, logf=x["logf"])
    eo = np.abs(o.float().cpu().numpy() - o_ref).max()
    el = np.abs(lse.cpu().numpy() - lse_ref).max()
    print(f"[fox fwd {dtype} L={L} d={d}] max|do|={eo:.2e} max|dlse|={el:.2e}", flush=True)
    assert eo <= (1e-4 if dtype == "fp32" else 2e-2) and el <= 1e-3


def test_unit_gates_reproduce_plain_path(gpu):
    """log f = 0 everywhere: the gated kernel subtracts a zero gate sum from the base-2 logit in a step of its
    own (two roundings in the exponent where the plain kernel's fused multiply-add has one), so o may differ from
    plain PaTH's by a rounding step of the bf16 result (2^-6 for |o| in [2,4)) and lse by a few fp32 steps --
    not bit for bit, and not more."""
    torch, pa = gpu
    x = _inputs(1, 2, 500, 64, "bf16", 1300)
    dv = _dev(gpu, x, "bf16")
    zero = torch.zeros_like(dv["logf"])
    o1, l1 = pa.path_attn_fox_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], zero, scale=0.125)
    o0, l0 = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=0.125)
    assert float((o1.float() - o0.float()).abs().max()) <= 2.0 ** -6 and float((l1 - l0).abs().max()) <= 1e-5


NAMES = ("dq", "dk", "dv", "dw", "dbeta", "dlogf")


@pytest.mark.parametrize("dtype,L,d", [("fp32", 64, 64), ("fp32", 200, 128), ("fp32", 1100, 64), ("bf16", 300, 64),
                                       ("bf16", 1030, 128), ("fp32", 2200, 64), ("bf16", 3100, 128)])
def test_fox_backward_matches_the_oracle(gpu, oracle, dtype, L, d):
    torch, pa = gpu
    x = _inputs(1, 2, L, d, dtype, 1400 + L + d)
    dv = _dev(gpu, x, dtype)
    scale = d ** -0.5
    o, lse = pa.path_attn_fox_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], dv["logf"], scale=scale)
    got = pa.path_attn_fox_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], dv["logf"], o, lse, dv["dO"], scale=scale)
    torch.cuda.synchronize()
    ref = oracle.bwd(x["q"], x["k"], x["v"], x["w"], x["beta"], x["dO"], scale, logf=x["logf"])
    msg, worst = [], 0.0
    for n, g, r in zip(NAMES, got, ref):
        g = g.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(g).all(), n
        e = np.abs(g - r).max() / max(np.abs(r).max(), 1e-2)
        msg.append(f"{n}={e:.2e}")
        worst = max(worst, e)
    print(f"[fox bwd {dtype} L={L} d={d}] rel err " + " ".join(msg), flush=True)
    assert worst <= (1e-4 if dtype == "fp32" else 2e-2), msg
    assert float(got[5][:, :, 0].abs().max()) == 0.0


def test_fox_headline_shape_sampled_head(gpu, oracle):
    """PaTH-FoX at the shape bench.py times (B=4, H=16, L=8192, d=128, bf16; eight super-blocks, every
    key-side and scan kernel in its FoX instantiation at full grid size): the whole batch runs on the
    GPU, one head is checked against the oracle, forward and backward."""
    torch, pa = gpu
    B, H, L, d = 4, 16, 8192, 128
    x = _inputs(B, H, L, d, "bf16", 1500)
    dv = _dev(gpu, x, "bf16")
    scale = d ** -0.5
    o, lse = pa.path_attn_fox_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], dv["logf"], scale=scale)
    got = pa.path_attn_fox_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], dv["logf"], o, lse, dv["dO"], scale=scale)
    torch.cuda.synchronize()
    head = 29
    sel = lambda a: np.ascontiguousarray(a.reshape((B * H,) + a.shape[2:])[head][None, None])
    xs = {n: sel(a) for n, a in x.items()}
    o_ref, lse_ref = oracle.fwd(xs["q"], xs["k"], xs["v"], xs["w"], xs["beta"], scale, logf=xs["logf"])
    eo = np.abs(sel(o.float().cpu().numpy()) - o_ref).max()
    el = np.abs(sel(lse.cpu().numpy()) - lse_ref).max()
    print(f"[fox headline fwd] max|do|={eo:.2e} max|dlse|={el:.2e}", flush=True)
    assert eo <= 2e-2 and el <= 1e-3
    ref = oracle.bwd(xs["q"], xs["k"], xs["v"], xs["w"], xs["beta"], xs["dO"], scale, logf=xs["logf"])
    msg, worst = [], 0.0
    for n, g, r in zip(NAMES, got, ref):
        g = sel(g.float().cpu().numpy()).astype(np.float64)
        assert np.isfinite(g).all(), n
        e = np.abs(g - r).max() / max(np.abs(r).max(), 1e-2)
        msg.append(f"{n}={e:.2e}")
        worst = max(worst, e)
    print("[fox headline bwd] rel err " + " ".join(msg), flush=True)
    assert worst <= 2e-2, msg
