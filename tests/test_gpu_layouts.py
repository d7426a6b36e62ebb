"""GPU tests of the layout-taking and variable-length entry points (run with -m gpu).

[B,L,H,d] tensors and packed sequences are read and written in place through their strides; every
sum is taken in the same order as for [B,H,L,d], so the results must be BIT-EQUAL to those of the
[B,H,L,d] entry points on the transposed / unpacked data (PaTH-FoX's dlog_f excepted: it sums LDS
adds whose order is not fixed).  One case of each is also held against the oracle, to the usual bars
(o 1e-4 / 2e-2, lse 1e-3, gradients 1e-4 / 2e-2 of the tensor's maximum)."""
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


def _to_blhd(t):        # [B,H,L,(d)] -> [B,L,H,(d)], contiguous
    return (t.permute(0, 2, 1, 3) if t.dim() == 4 else t.permute(0, 2, 1)).contiguous()


def _close_dlogf(a, b, dtype):
    return float((a.float() - b.float()).abs().max()) <= (1e-5 if dtype == "fp32" else 1e-2) * max(float(b.float().abs().max()), 1e-2)


@pytest.mark.parametrize("dtype,L,d,fox", [("fp32", 200, 64, False), ("fp32", 1100, 128, True), ("bf16", 300, 128, False),
                                           ("bf16", 1030, 64, True), ("bf16", 2200, 128, False)])
def test_blhd_layout_is_bit_equal_to_bhld(gpu, dtype, L, d, fox):
    torch, pa = gpu
    B, H = 2, 3
    dv = _dev(torch, _inputs(B, H, L, d, dtype, 3100 + L + d, fox), dtype)
    scale = d ** -0.5
    logf = dv.get("logf")
    # reference: the [B,H,L,d] entry points
    if fox:
        o, lse = pa.path_attn_fox_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], logf, scale=scale)
        g = pa.path_attn_fox_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], logf, o, lse, dv["dO"], scale=scale)
    else:
        o, lse = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
        g = pa.path_attn_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], scale=scale)
    # the same data as [B,L,H,d]
    t = {n: _to_blhd(a) for n, a in dv.items()}
    o2, lse2 = pa.path_attn_fwd_layout(t["q"], t["k"], t["v"], t["w"], t["beta"], pa.PATH_LAYOUT_BLHD, log_f=t.get("logf"), scale=scale)
    g2 = pa.path_attn_bwd_layout(t["q"], t["k"], t["v"], t["w"], t["beta"], o2, lse2, t["dO"], pa.PATH_LAYOUT_BLHD,
                                 log_f=t.get("logf"), scale=scale)
    torch.cuda.synchronize()
    assert torch.equal(o2, _to_blhd(o)) and torch.equal(lse2, _to_blhd(lse))
    for i, (a, b) in enumerate(zip(g2, g)):
        if i < 5:
            assert torch.equal(a, _to_blhd(b)), i
        else:
            assert _close_dlogf(a, _to_blhd(b), dtype)
    # ... and the BHLD layout through the same entry points
    o3, lse3 = pa.path_attn_fwd_layout(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], pa.PATH_LAYOUT_BHLD, log_f=logf, scale=scale)
    assert torch.equal(o3, o) and torch.equal(lse3, lse)


@pytest.mark.parametrize("dtype,d,fox", [("fp32", 64, False), ("bf16", 128, False), ("bf16", 64, True)])
def test_packed_sequences_equal_the_sequences_run_one_by_one(gpu, oracle, dtype, d, fox):
    torch, pa = gpu
    H = 2
    lens = [200, 64, 1030, 1]
    cu = np.concatenate([[0], np.cumsum(lens)]).tolist()
    scale = d ** -0.5
    xs = [_inputs(1, H, L, d, dtype, 4100 + 13 * i + d, fox) for i, L in enumerate(lens)]
    dvs = [_dev(torch, x, dtype) for x in xs]
    names = ["q", "k", "v", "w", "beta", "dO"] + (["logf"] if fox else [])
    packed = {n: torch.cat([_to_blhd(dv[n])[0] for dv in dvs], dim=0).contiguous() for n in names}       # [T,H,d] / [T,H]
    o, lse = pa.path_attn_varlen_fwd(packed["q"], packed["k"], packed["v"], packed["w"], packed["beta"], cu,
                                     log_f=packed.get("logf"), scale=scale)
    g = pa.path_attn_varlen_bwd(packed["q"], packed["k"], packed["v"], packed["w"], packed["beta"], o, lse, packed["dO"], cu,
                                log_f=packed.get("logf"), scale=scale)
    torch.cuda.synchronize()
    for i, (dv, L) in enumerate(zip(dvs, lens)):
        sl = slice(cu[i], cu[i + 1])
        if fox:
            o1, lse1 = pa.path_attn_fox_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], dv["logf"], scale=scale)
            g1 = pa.path_attn_fox_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], dv["logf"], o1, lse1, dv["dO"], scale=scale)
        else:
            o1, lse1 = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
            g1 = pa.path_attn_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o1, lse1, dv["dO"], scale=scale)
        torch.cuda.synchronize()
        assert torch.equal(o[sl], _to_blhd(o1)[0]) and torch.equal(lse[sl], _to_blhd(lse1)[0]), i
        for j, (a, b) in enumerate(zip(g, g1)):
            if j < 5:
                assert torch.equal(a[sl], _to_blhd(b)[0]), (i, j)
            else:
                assert _close_dlogf(a[sl], _to_blhd(b)[0], dtype)
    # sequence 2 (1030 tokens: a ragged tail and, for d = 64, two super-blocks) against the oracle
    i = 2
    x = xs[i]
    sl = slice(cu[i], cu[i + 1])
    kw = {"logf": x["logf"]} if fox else {}
    o_ref, lse_ref = oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale, **kw)
    got_o = o[sl].float().cpu().numpy().astype(np.float64).transpose(1, 0, 2)[None]           # -> [1,H,L,d]
    got_lse = lse[sl].cpu().numpy().astype(np.float64).T[None]
    assert np.abs(got_o - o_ref).max() <= (1e-4 if dtype == "fp32" else 2e-2)
    assert np.abs(got_lse - lse_ref).max() <= 1e-3
    ref = oracle.bwd(x["q"], x["k"], x["v"], x["w"], x["beta"], x["dO"], scale, **kw)
    for a, r in zip(g, ref):
        a = a[sl].float().cpu().numpy().astype(np.float64)
        a = a.transpose(1, 0, 2)[None] if a.ndim == 3 else a.T[None]
        assert np.abs(a - r).max() / max(np.abs(r).max(), 1e-2) <= (1e-4 if dtype == "fp32" else 2e-2)


def test_layout_and_varlen_argument_checks(gpu):
    torch, pa = gpu
    lib = pa.load_library()
    x = _dev(torch, _inputs(1, 1, 64, 64, "fp32", 9, False), "fp32")
    with pytest.raises(pa.PathAttnError):
        pa.path_attn_fwd_layout(x["q"], x["k"], x["v"], x["w"], x["beta"], 7)                 # unknown layout
    assert pa.path_attn_varlen_workspace_bytes([0, 5, 5], 2, 64, pa.PATH_F32) == 0           # an empty sequence
    assert pa.path_attn_varlen_workspace_bytes([1, 5], 2, 64, pa.PATH_F32) == 0              # does not start at 0
    # one set of launches for the batch: the sequence table, then the arrays of a batch of two at the longest length
    assert pa.path_attn_varlen_workspace_bytes([0, 5, 70], 2, 64, pa.PATH_F32) == 256 + pa.path_attn_workspace_bytes(2, 2, 65, 64, pa.PATH_F32)
    assert lib is not None


def test_varlen_batch_of_many_short_sequences_in_one_set_of_launches(gpu):
    """64 sequences of 256..2048 tokens (bf16, H = 4, d = 64) as ONE problem: forward and backward are bit-equal
    (dlog_f aside: none here) to a loop over the sequences on [1,L,H,d] tensors, and the time of both is printed."""
    import time
    torch, pa = gpu
    rng = np.random.default_rng(77)
    H, d, nseq = 4, 64, 64
    lens = [int(v) for v in rng.integers(256, 2049, nseq)]
    lens[3], lens[17] = 256, 2048
    cu = [0]
    for n in lens:
        cu.append(cu[-1] + n)
    T = cu[-1]
    g = torch.Generator(device="cuda").manual_seed(5)
    rn = lambda *shape: torch.randn(*shape, device="cuda", generator=g)
    q, k, v, dO = (rn(T, H, d).to(torch.bfloat16) for _ in range(4))
    w = torch.nn.functional.normalize(rn(T, H, d), dim=-1).to(torch.bfloat16)
    beta = (2 * torch.sigmoid(rn(T, H))).to(torch.bfloat16)
    scale = d ** -0.5

    def one_grid():
        o, lse = pa.path_attn_varlen_fwd(q, k, v, w, beta, cu, scale=scale)
        return (o, lse) + tuple(pa.path_attn_varlen_bwd(q, k, v, w, beta, o, lse, dO, cu, scale=scale))

    def per_sequence():
        outs = [torch.empty_like(q), torch.empty((T, H), dtype=torch.float32, device="cuda")] + [torch.empty_like(q) for _ in range(4)] + [torch.empty_like(beta)]
        for i in range(nseq):
            sl = slice(cu[i], cu[i + 1])
            a = [t[sl][None] for t in (q, k, v, w, beta)]
            o1, l1 = pa.path_attn_fwd_layout(*a, pa.PATH_LAYOUT_BLHD, scale=scale)
            gr = pa.path_attn_bwd_layout(*a, o1, l1, dO[sl][None], pa.PATH_LAYOUT_BLHD, scale=scale)
            for dst, src in zip(outs, (o1, l1) + tuple(gr)):
                dst[sl] = src[0]
        return tuple(outs)

    a = one_grid()
    b = per_sequence()
    torch.cuda.synchronize()
    for i, (x, y) in enumerate(zip(a, b)):
        assert torch.equal(x, y), i
    times = {}
    for name, f in (("one set of launches", one_grid), ("loop over the sequences", per_sequence)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        times[name] = (time.perf_counter() - t0) / 3 * 1e3
    print(f"[varlen 64 sequences, {T} tokens, H={H} d={d}] forward+backward: " + ", ".join(f"{n} {t:.2f} ms" for n, t in times.items()), flush=True)
