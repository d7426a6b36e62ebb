"""The memory-bounded backward (run with -m gpu): path_attn_bwd in a workspace that holds only some of the heads
passes over the heads in groups -- same kernels, same arithmetic -- and must give bit-identical gradients to the
full-workspace call (which the other files hold against the oracle), also with a ragged last group, on both
layouts, with gates, and at the headline shape inside 4 GB."""
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


def _dev(torch, x, dtype):
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    return {n: torch.from_numpy(a).to("cuda").to(td).contiguous() for n, a in x.items()}


@pytest.mark.parametrize("dtype,B,H,L,d,heads", [("bf16", 1, 5, 1100, 128, 2), ("bf16", 2, 3, 300, 64, 1), ("fp32", 1, 5, 1100, 64, 3),
                                                 ("fp32", 3, 2, 200, 128, 4)])
def test_grouped_backward_is_bit_identical(gpu, oracle, dtype, B, H, L, d, heads):
    torch, pa = gpu
    x = si.make_inputs(B, H, L, d, dtype, 3100 + L + d + heads, 0.0, with_do=True)
    dv = _dev(torch, x, dtype)
    dt = pa.PATH_F32 if dtype == "fp32" else pa.PATH_BF16
    scale = d ** -0.5
    o, lse = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
    full = pa.path_attn_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], scale=scale)
    nbytes = pa.path_attn_bwd_workspace_bytes_for_heads(B, H, L, d, dt, heads)
    assert 0 < nbytes < pa.path_attn_workspace_bytes(B, H, L, d, dt, True)
    assert pa.path_attn_bwd_heads_per_pass(B, H, L, d, dt, nbytes) == heads
    assert pa.path_attn_bwd_heads_per_pass(B, H, L, d, dt, nbytes - 1) == heads - 1
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    part = pa.path_attn_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], scale=scale, workspace=ws)
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(zip(full, part)):
        assert torch.equal(a, b), i
    # and against the oracle directly, once
    ref = oracle.bwd(x["q"], x["k"], x["v"], x["w"], x["beta"], x["dO"], scale)
    tol = 1e-4 if dtype == "fp32" else 2e-2
    for g, r in zip(part, ref):
        assert np.abs(g.float().cpu().numpy() - r).max() / max(np.abs(r).max(), 1e-2) <= tol
    # less than one head's worth is refused before anything is launched
    small = torch.empty(pa.path_attn_bwd_workspace_bytes_for_heads(B, H, L, d, dt, 1) - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(pa.PathAttnError) as e:
        pa.path_attn_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], scale=scale, workspace=small)
    assert e.value.code == 5


def test_grouped_backward_on_the_other_layout_and_with_gates(gpu):
    torch, pa = gpu
    B, H, L, d = 2, 3, 700, 64
    x = si.make_inputs(B, H, L, d, "bf16", 3300, 0.0, with_do=True)
    rng = np.random.default_rng(3)
    x["logf"] = si.round_to_bf16((-np.log1p(np.exp(-rng.normal(2.0, 1.0, size=(B, H, L)))).astype(np.float32)))
    dv = _dev(torch, x, "bf16")
    t = {n: (a.permute(0, 2, 1, 3).contiguous() if a.dim() == 4 else a.permute(0, 2, 1).contiguous()) for n, a in dv.items()}   # [B,L,H,d]
    scale = d ** -0.5
    o, lse = pa.path_attn_fwd_layout(t["q"], t["k"], t["v"], t["w"], t["beta"], pa.PATH_LAYOUT_BLHD, log_f=t["logf"], scale=scale)
    full = pa.path_attn_bwd_layout(t["q"], t["k"], t["v"], t["w"], t["beta"], o, lse, t["dO"], pa.PATH_LAYOUT_BLHD, log_f=t["logf"], scale=scale)
    ws = torch.empty(pa.path_attn_bwd_workspace_bytes_for_heads(B, H, L, d, pa.PATH_BF16, 4), dtype=torch.uint8, device="cuda")
    part = pa.path_attn_bwd_layout(t["q"], t["k"], t["v"], t["w"], t["beta"], o, lse, t["dO"], pa.PATH_LAYOUT_BLHD, log_f=t["logf"],
                                   scale=scale, workspace=ws)
    torch.cuda.synchronize()
    assert len(full) == 6
    for i, (a, b) in enumerate(zip(full[:5], part[:5])):
        assert torch.equal(a, b), i
    # dlog_f: its column and row sums are shared-memory float adds in no fixed order (see the header), so two runs
    # agree only up to the rounding of those sums -- one step of the bf16 result
    a, b = full[5].float(), part[5].float()
    assert float((a - b).abs().max()) <= 2.0 ** -7 * float(a.abs().max())


def test_headline_backward_inside_four_gigabytes(gpu, oracle):
    """B=4, H=16, L=8192, d=128 (bf16): the full workspace is 12.8 GB; with 16 heads per pass the backward runs in
    under 4 GB.  Two heads (one from the first group, one from the last) against the oracle."""
    torch, pa = gpu
    x, c = si.make_config(2, with_do=True)
    B, H, L, d = c["B"], c["H"], c["L"], c["d"]
    dv = _dev(torch, x, "bf16")
    scale = d ** -0.5
    nbytes = pa.path_attn_bwd_workspace_bytes_for_heads(B, H, L, d, pa.PATH_BF16, 16)
    print(f"[bounded backward] workspace for 16 heads per pass: {nbytes / 2**30:.2f} GiB (all 64: "
          f"{pa.path_attn_workspace_bytes(B, H, L, d, pa.PATH_BF16, True) / 2**30:.2f} GiB)", flush=True)
    assert nbytes <= 4 * 10 ** 9
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    o, lse = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
    got = pa.path_attn_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], scale=scale, workspace=ws)
    torch.cuda.synchronize()
    heads = [5, 58]
    sel = lambda a: np.stack([a.reshape((B * H,) + a.shape[2:])[h] for h in heads])[None]
    xs = {n: sel(a) for n, a in x.items()}
    ref = oracle.bwd(xs["q"], xs["k"], xs["v"], xs["w"], xs["beta"], xs["dO"], scale)
    for n, g, r in zip(("dq", "dk", "dv", "dw", "dbeta"), got, ref):
        g = sel(g.float().cpu().numpy())
        e = np.abs(g - r).max() / max(np.abs(r).max(), 1e-2)
        print(f"[bounded backward headline] {n} rel err {e:.2e}", flush=True)
        assert e <= 2e-2, n
