"""GPU parity of the backward path against the oracle's adjoint walk (run with -m gpu).

Bar (the benchmark states none for gradients): per tensor,
max|g - g_oracle| / max(max|g_oracle|, 1e-2) <= 1e-4 (fp32 I/O) or 2e-2 (bf16 I/O).
"""
import numpy as np
import pytest

from paper_2505_16381_amd import synth_inputs as si

pytestmark = pytest.mark.gpu
TOL = {"fp32": 1e-4, "bf16": 2e-2}
NAMES = ("dq", "dk", "dv", "dw", "dbeta")


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2505_16381_amd as pa
    assert torch.cuda.is_available()
    pa.load_library()
    return torch, pa


def _run_bwd(gpu, x, dtype, scale):
    torch, pa = gpu
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    dv = {n: torch.from_numpy(a).to("cuda").to(td).contiguous() for n, a in x.items()}
    o, lse = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
    grads = pa.path_attn_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], scale=scale)
    torch.cuda.synchronize()
    return [g.float().cpu().numpy().astype(np.float64) for g in grads]


def _check(gpu, oracle, x, dtype, scale, heads=None, tag=""):
    got = _run_bwd(gpu, x, dtype, scale)
    if heads is not None:
        B, H = x["q"].shape[:2]
        sel = lambda a: np.stack([a.reshape((B * H,) + a.shape[2:])[h] for h in heads])[None]
        xs = {n: sel(a) for n, a in x.items()}
        got = [sel(g) for g in got]
    else:
        xs = x
    ref = oracle.bwd(xs["q"], xs["k"], xs["v"], xs["w"], xs["beta"], xs["dO"], scale)
    msg = []
    worst = 0.0
    for n, g, r in zip(NAMES, got, ref):
        assert np.isfinite(g).all(), n
        e = np.abs(g - r).max() / max(np.abs(r).max(), 1e-2)   # floor: exact-zero gradients (L = 1)
        msg.append(f"{n}={e:.2e}")
        worst = max(worst, e)
    print(f"[{tag}] dtype={dtype} rel err " + " ".join(msg), flush=True)
    assert worst <= TOL[dtype], (tag, msg)


@pytest.mark.parametrize("L,d", [(64, 64), (130, 64), (200, 128), (1, 64), (65, 128)])
def test_bwd_fp32_small(gpu, oracle, L, d):
    x = si.make_inputs(1, 2, L, d, "fp32", 500 + L + d, 0.0, with_do=True)
    _check(gpu, oracle, x, "fp32", d ** -0.5, tag=f"bwd fp32 L={L} d={d}")


@pytest.mark.parametrize("L,d", [(64, 64), (300, 64), (512, 128), (77, 128)])
def test_bwd_bf16_small(gpu, oracle, L, d):
    x = si.make_inputs(2, 2, L, d, "bf16", 600 + L + d, 0.0, with_do=True)
    _check(gpu, oracle, x, "bf16", d ** -0.5, tag=f"bwd bf16 L={L} d={d}")


@pytest.mark.parametrize("dtype,L,d", [("fp32", 1100, 64), ("bf16", 1100, 128), ("fp32", 1024, 128), ("bf16", 580, 64),
                                       ("fp32", 2200, 64), ("bf16", 3100, 128)])
def test_bwd_several_superblocks(gpu, oracle, dtype, L, d):
    """Long enough that the second blocking level (super-blocks of 16 chunks = 1024 tokens, far key
    blocks with their own products) and its adjoint carry pairs; from two super-blocks (no far
    product applied yet) to four, ragged and exact lengths."""
    x = si.make_inputs(1, 2, L, d, dtype, 650 + L + d, 0.0, with_do=True)
    _check(gpu, oracle, x, dtype, d ** -0.5, tag=f"bwd superblocks L={L} d={d}")


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_bwd_special_betas(gpu, oracle, dtype):
    x = si.make_inputs(1, 2, 200, 64, dtype, 700, 0.0, with_do=True)
    x["beta"][..., 0::3] = 0.0
    x["beta"][..., 1::3] = 1.0
    x["beta"][..., 2::3] = 2.0
    _check(gpu, oracle, x, dtype, 0.125, tag="bwd special betas")


@pytest.mark.parametrize("dtype,scale", [("fp32", 1.0), ("fp32", 0.03), ("bf16", 1.0), ("bf16", 0.3)])
def test_bwd_other_scales(gpu, oracle, dtype, scale):
    """`scale` is a free argument (the paper's logits are unscaled, scale = 1): the kernels fold it into the
    exponent and into the finished sums, so values far from d^-1/2 are worth a case of their own.  With
    scale = 1 the inputs are shrunk so that the logits stay in the range the other tests cover."""
    L, d = 1100, 64
    x = si.make_inputs(1, 2, L, d, dtype, 760 + int(100 * scale), 0.0, with_do=True)
    if scale == 1.0:
        x["q"] = (x["q"] * 0.35).astype(x["q"].dtype)
        if dtype == "bf16":
            x["q"] = si.round_to_bf16(x["q"])
    _check(gpu, oracle, x, dtype, scale, tag=f"bwd scale={scale}")


@pytest.mark.parametrize("L,d", [(1100, 128), (300, 64)])
def test_bwd_bf16_large_magnitude_inputs(gpu, oracle, L, d):
    """q and k at 64 times, dO at 1024 times their usual size (bf16 I/O: the transported operands and the state
    gradients travel as fp16, range 65504; see the header's range rule), `scale` reduced by 64^2: the logits are
    the usual ones, the carried operands are 64 times and the state gradients 16 times larger than in the other
    cases (powers of two: the inputs stay exact bf16 values)."""
    x = si.make_inputs(1, 2, L, d, "bf16", 830 + L + d, 0.0, with_do=True)
    for n, f in (("q", 64), ("k", 64), ("dO", 1024)):
        x[n] = (x[n] * f).astype(np.float32)
    _check(gpu, oracle, x, "bf16", d ** -0.5 / 4096, tag=f"bwd bf16 x64 inputs L={L} d={d}")


def test_bwd_gradient_identities_on_gpu(gpu):
    """w.dw = 2 beta dbeta and dw_0 = dbeta_0 = 0 hold for the GPU gradients too (fp32)."""
    x = si.make_inputs(1, 2, 192, 64, "fp32", 800, 0.0, with_do=True)
    dq, dk, dv, dw, db = _run_bwd(gpu, x, "fp32", 0.125)
    lhs = (x["w"].astype(np.float64) * dw).sum(-1)
    rhs = 2 * x["beta"].astype(np.float64) * db
    assert np.abs(lhs - rhs).max() <= 1e-4 * max(1.0, np.abs(rhs).max())
    assert np.abs(dw[:, :, 0]).max() <= 1e-6 and np.abs(db[:, :, 0]).max() <= 1e-6
    assert np.abs(dv.sum(2) - x["dO"].astype(np.float64).sum(2)).max() <= 1e-3


def test_config3_backward_full_shape_sampled_heads(gpu, oracle):
    """Full benchmark shape on the GPU; the oracle (not row-separable) on a sample of heads: both ends and
    every residue of the head index modulo 8 (the kernels number their workgroups per XCD, head = 8 * slot +
    xcd) twice over."""
    x, c = si.make_config(3)
    heads = [0, 1, 10, 19, 28, 37, 46, 55, 64, 73, 82, 91, 100, 109, 118, 127]
    assert sorted(h % 8 for h in heads) == sorted(list(range(8)) * 2)
    _check(gpu, oracle, x, "bf16", c["d"] ** -0.5, heads=heads, tag="cfg3")


def test_headline_shape_backward_sampled_head(gpu, oracle):
    """The shape and launch configuration bench.py times (B=4, H=16, L=8192, d=128, bf16):
    the whole batch runs on the GPU, five heads (first, last, three residues modulo 8 in between) are checked
    against the oracle."""
    x, c = si.make_config(2, with_do=True)
    _check(gpu, oracle, x, "bf16", c["d"] ** -0.5, heads=[0, 13, 41, 50, 63], tag="headline shape")


def test_bwd_long_context_with_beta_near_two(gpu, oracle):
    """Sixteen super-blocks (16384 tokens, d = 128) with beta drawn as in the long-context configuration (near 2, some
    exactly 2.0 after rounding): the far chains of the second level and their adjoint over many blocks."""
    x = si.make_inputs(1, 1, 16384, 128, "bf16", 5555, 2.0, with_do=True)
    _check(gpu, oracle, x, "bf16", 128 ** -0.5, tag="bwd long context, beta near 2")
