"""GPU tests of the training pair (path_attn_train_fwd / path_attn_train_bwd: forward and backward that
share one workspace, the chunk transform runs once): parity against the oracle, to the bars of the
calls they stand in for, and bit-equality with those calls (run with -m gpu)."""
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


def _inputs(B, H, L, d, dtype, seed, fox):
    x = si.make_inputs(B, H, L, d, dtype, seed, 0.0, with_do=True)
    if fox:
        rng = np.random.default_rng(seed + 7)
        z = rng.normal(2.0, 1.0, size=(B, H, L)).astype(np.float32)
        logf = (-np.log1p(np.exp(-z))).astype(np.float32)
        x["logf"] = si.round_to_bf16(logf) if dtype == "bf16" else logf
    return x


def _dev(torch, x, dtype):
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    return {n: torch.from_numpy(a).to("cuda").to(td).contiguous() for n, a in x.items()}


@pytest.mark.parametrize("dtype,L,d,fox", [("fp32", 200, 64, False), ("fp32", 1100, 128, True), ("bf16", 300, 128, False),
                                           ("bf16", 2200, 64, False), ("bf16", 1030, 128, True)])
def test_training_pair_matches_the_oracle_and_the_separate_calls(gpu, oracle, dtype, L, d, fox):
    torch, pa = gpu
    B, H = 1, 2
    x = _inputs(B, H, L, d, dtype, 2100 + L + d, fox)
    dv = _dev(torch, x, dtype)
    scale = d ** -0.5
    dt = pa.PATH_F32 if dtype == "fp32" else pa.PATH_BF16
    ws = torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, dt, True), dtype=torch.uint8, device="cuda")
    logf = dv.get("logf")
    o, lse = pa.path_attn_train_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], ws, log_f=logf, scale=scale)
    got = pa.path_attn_train_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], ws, log_f=logf, scale=scale)
    torch.cuda.synchronize()

    # the separate calls, each in a workspace of its own
    if fox:
        o2, lse2 = pa.path_attn_fox_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], logf, scale=scale)
        got2 = pa.path_attn_fox_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], logf, o2, lse2, dv["dO"], scale=scale)
    else:
        o2, lse2 = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
        got2 = pa.path_attn_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o2, lse2, dv["dO"], scale=scale)
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(lse, lse2)
    for i, (a, b) in enumerate(zip(got, got2)):
        if i < 5:
            assert torch.equal(a, b), i
        else:   # dlog_f sums LDS adds whose order is not fixed: equal up to the rounding of the output type
            assert float((a.float() - b.float()).abs().max()) <= (1e-5 if dtype == "fp32" else 1e-2) * max(float(b.float().abs().max()), 1e-2)

    o_ref, lse_ref = oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale, **({"logf": x["logf"]} if fox else {}))
    eo = np.abs(o.float().cpu().numpy().astype(np.float64) - o_ref).max()
    el = np.abs(lse.cpu().numpy().astype(np.float64) - lse_ref).max()
    assert eo <= (1e-4 if dtype == "fp32" else 2e-2) and el <= 1e-3, (eo, el)
    ref = oracle.bwd(x["q"], x["k"], x["v"], x["w"], x["beta"], x["dO"], scale, **({"logf": x["logf"]} if fox else {}))
    worst = 0.0
    for g, r in zip(got, ref):
        g = g.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(g).all()
        worst = max(worst, np.abs(g - r).max() / max(np.abs(r).max(), 1e-2))
    print(f"[train pair {dtype} L={L} d={d} fox={fox}] o {eo:.2e} lse {el:.2e} grads {worst:.2e}", flush=True)
    assert worst <= (1e-4 if dtype == "fp32" else 2e-2)


def test_training_pair_at_the_headline_shape_equals_the_separate_calls(gpu):
    """The shape and launch configuration bench.py times (B=4, H=16, L=8192, d=128, bf16, the pair): o, lse and all
    gradients are bit-equal to those of path_attn_fwd / path_attn_bwd, which tests/test_gpu_fwd.py and
    tests/test_gpu_bwd.py hold against the oracle at this shape."""
    torch, pa = gpu
    x, c = si.make_config(2, with_do=True)
    dv = _dev(torch, x, "bf16")
    B, H, L, d = c["B"], c["H"], c["L"], c["d"]
    scale = d ** -0.5
    ws = torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, pa.PATH_BF16, True), dtype=torch.uint8, device="cuda")
    for rep in range(2):       # twice in the same workspace: nothing of the first step may leak into the second
        o, lse = pa.path_attn_train_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], ws, scale=scale)
        got = pa.path_attn_train_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], ws, scale=scale)
    torch.cuda.synchronize()
    o2, lse2 = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
    got2 = pa.path_attn_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o2, lse2, dv["dO"], scale=scale)
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(lse, lse2)
    for i, (a, b) in enumerate(zip(got, got2)):
        assert torch.isfinite(a.float()).all(), i
        assert torch.equal(a, b), i


def test_training_pair_rejects_a_forward_sized_workspace(gpu):
    torch, pa = gpu
    B, H, L, d = 1, 1, 128, 64
    x = _dev(torch, _inputs(B, H, L, d, "fp32", 5, False), "fp32")
    small = torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, pa.PATH_F32, False), dtype=torch.uint8, device="cuda")
    with pytest.raises(pa.PathAttnError):
        pa.path_attn_train_fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], small)


@pytest.mark.parametrize("dtype,L,d", [("bf16", 2200, 128), ("fp32", 1100, 64)])
def test_backward_in_stages_equals_the_whole_call(gpu, dtype, L, d):
    """path_attn_train_bwd_stages, one stage after the other in the order of the stage bits, is exactly
    path_attn_train_bwd (bench.py times the stages this way); an unknown bit is refused."""
    torch, pa = gpu
    B, H = 1, 3
    x = _inputs(B, H, L, d, dtype, 2300 + L + d, False)
    dv = _dev(torch, x, dtype)
    scale = d ** -0.5
    dt = pa.PATH_F32 if dtype == "fp32" else pa.PATH_BF16
    ws = torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, dt, True), dtype=torch.uint8, device="cuda")
    o, lse = pa.path_attn_train_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], ws, scale=scale)
    whole = pa.path_attn_train_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], ws, scale=scale)
    torch.cuda.synchronize()
    o, lse = pa.path_attn_train_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], ws, scale=scale)
    outs = [torch.full_like(dv["q"], 7.0) for _ in range(4)] + [torch.full_like(dv["beta"], 7.0)]
    for bit in (pa.PATH_BWD_STAGE_SCAN, pa.PATH_BWD_STAGE_KEYS_NEAR, pa.PATH_BWD_STAGE_KEYS_FAR, pa.PATH_BWD_STAGE_DDP, pa.PATH_BWD_STAGE_CHUNK):
        pa.path_attn_train_bwd_stages(bit, dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], outs, ws, scale=scale)
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(zip(whole, outs)):
        assert torch.equal(a, b), i
    with pytest.raises(pa.PathAttnError) as e:
        pa.path_attn_train_bwd_stages(64, dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], outs, ws, scale=scale)
    assert e.value.code == 4


def test_mfma_probe_runs_and_reports_its_work(gpu):
    torch, pa = gpu
    sink = torch.zeros(1024 * 4 * 64, dtype=torch.float32, device="cuda")
    for wps in (1, 2, 4):
        flops = pa.path_probe_mfma(sink, wps, 50)
        assert flops == 256.0 * 4 * wps * 50 * 16 * 2 * 32 * 32 * 16
        assert pa.path_probe_mfma(sink, wps, 50, random_operands=True) == flops
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink).all())
    with pytest.raises(pa.PathAttnError):
        pa.path_probe_mfma(sink, 3, 50)
