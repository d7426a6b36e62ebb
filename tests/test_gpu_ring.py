"""GPU tests of the sequence-parallel forward (one device's share of the ring of paper Sec. 3.5), run with -m gpu.

One GPU plays every device in turn: each segment runs path_attn_ring_local, then one path_attn_ring_hop per
earlier segment (nearest first), then path_attn_ring_finish.  The concatenated result is held against the oracle's
forward of the WHOLE sequence (bars: o 1e-4 / 2e-2, lse 1e-3) and, where the segment lengths are multiples of the
second blocking level (1024 tokens), bit for bit against path_attn_fwd of the whole sequence.
"""
import numpy as np
import pytest

from paper_2505_16381_amd import synth_inputs as si

pytestmark = pytest.mark.gpu
TOL_O = {"fp32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2505_16381_amd as pa
    assert torch.cuda.is_available()
    pa.load_library()
    return torch, pa


def _ring_forward(torch, pa, dv, lengths, d, dt, scale):
    B, H = dv["q"].shape[:2]
    gates = "logf" in dv
    starts = np.concatenate([[0], np.cumsum(lengths)]).astype(int)
    ws, st, seg = [], [], []
    for r, Ls in enumerate(lengths):
        a, b = int(starts[r]), int(starts[r + 1])
        s = {n: dv[n][:, :, a:b].contiguous() for n in dv}
        seg.append(s)
        ws.append(torch.empty(pa.path_attn_workspace_bytes(B, H, Ls, d, dt, False), dtype=torch.uint8, device="cuda"))
        st.append(torch.empty(pa.path_attn_ring_state_bytes(B, H, Ls, d), dtype=torch.uint8, device="cuda"))
        pa.path_attn_ring_local(s["q"], s["k"], s["v"], s["w"], s["beta"], st[r], ws[r], log_f=s.get("logf"), scale=scale)
    outs, lses = [], []
    for r, Ls in enumerate(lengths):
        for s in range(r - 1, -1, -1):             # nearest earlier segment first
            pa.path_attn_ring_hop(st[r], B, H, Ls, ws[s], lengths[s], d, dt, with_gates=gates, scale=scale)
        o = torch.empty_like(seg[r]["q"])
        lse = torch.empty((B, H, Ls), dtype=torch.float32, device="cuda")
        pa.path_attn_ring_finish(st[r], o, lse, gates_workspace=ws[r] if gates else None)
        outs.append(o)
        lses.append(lse)
    torch.cuda.synchronize()
    return torch.cat(outs, dim=2), torch.cat(lses, dim=2)


@pytest.mark.parametrize("dtype,d,lengths", [
    ("bf16", 128, [1024, 1024, 1024]),          # super-block-aligned segments: bit-identical to the one-device forward
    ("fp32", 64, [2048, 1024]),
    ("bf16", 64, [1024, 2048, 700]),            # ragged last segment
    ("fp32", 128, [448, 320, 232]),             # segments shorter than a super-block, ragged last one
    ("bf16", 128, [1600, 64, 1]),               # one-chunk and one-token segments
])
def test_ring_of_segments_matches_the_whole_sequence(gpu, oracle, dtype, d, lengths):
    torch, pa = gpu
    B, H, L = 1, 3, int(sum(lengths))
    x = si.make_inputs(B, H, L, d, dtype, 4100 + L + d, 0.0)
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    dt = pa.PATH_F32 if dtype == "fp32" else pa.PATH_BF16
    scale = d ** -0.5
    dv = {n: torch.from_numpy(a).to("cuda").to(td).contiguous() for n, a in x.items()}
    print(f"[ring] {dtype} d={d} segments {lengths}", flush=True)
    o, lse = _ring_forward(torch, pa, dv, lengths, d, dt, scale)
    o_ref, lse_ref = oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale)
    eo = np.abs(o.float().cpu().numpy().astype(np.float64) - o_ref).max()
    el = np.abs(lse.cpu().numpy().astype(np.float64) - lse_ref).max()
    print(f"[ring] against the oracle: o {eo:.2e} lse {el:.2e}", flush=True)
    assert eo <= TOL_O[dtype] and el <= 1e-3
    o1, lse1 = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
    torch.cuda.synchronize()
    if all(n % 1024 == 0 for n in lengths[:-1]):
        # every segment starts on a super-block edge: the same tiles, the same products, the same order
        assert torch.equal(o, o1) and torch.equal(lse, lse1)
    else:
        assert (o.float() - o1.float()).abs().max().item() <= TOL_O[dtype]
        assert (lse - lse1).abs().max().item() <= 1e-3


def test_ring_at_the_headline_head_shape(gpu, oracle):
    """Four segments of 2048 tokens (the headline sequence split over four devices), d = 128, eight heads -- one per
    XCD: bit-identical to the one-device forward, and rows on both sides of every segment edge against the oracle."""
    torch, pa = gpu
    B, H, d, lengths = 1, 8, 128, [2048] * 4
    L = sum(lengths)
    x = si.make_inputs(B, H, L, d, "bf16", 4500, 0.0)
    dv = {n: torch.from_numpy(a).to("cuda").to(torch.bfloat16).contiguous() for n, a in x.items()}
    scale = d ** -0.5
    o, lse = _ring_forward(torch, pa, dv, lengths, d, pa.PATH_BF16, scale)
    o1, lse1 = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
    torch.cuda.synchronize()
    assert torch.equal(o, o1) and torch.equal(lse, lse1)
    rows = np.unique(np.concatenate([np.arange(e - 2, e + 3) for e in (2048, 4096, 6144)] + [[0, 1, 2047, 8190, 8191]]
                                    + [np.random.default_rng(45).integers(0, L, 40)]))
    o_ref, lse_ref = oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale, rows=rows)
    eo = np.abs(o[:, :, rows].float().cpu().numpy().astype(np.float64) - o_ref).max()
    el = np.abs(lse[:, :, rows].cpu().numpy().astype(np.float64) - lse_ref).max()
    print(f"[ring 4 x 2048, d=128, 8 heads] {len(rows)} rows against the oracle: o {eo:.2e} lse {el:.2e}", flush=True)
    assert eo <= 2e-2 and el <= 1e-3


@pytest.mark.parametrize("dtype,d,lengths", [("bf16", 128, [1024, 1088, 300]), ("fp32", 64, [320, 448, 130])])
def test_ring_with_forget_gates(gpu, oracle, dtype, d, lengths):
    """PaTH-FoX over the ring: every segment counts its gate sums from its own start; a hop adds the totals of the
    segments passed.  Held against the oracle's gated forward of the whole sequence and the one-device gated forward."""
    torch, pa = gpu
    B, H, L = 1, 2, int(sum(lengths))
    x = si.make_inputs(B, H, L, d, dtype, 4300 + L + d, 0.0)
    rng = np.random.default_rng(4300 + L)
    z = rng.normal(2.0, 1.0, size=(B, H, L)).astype(np.float32)
    logf = (-np.log1p(np.exp(-z))).astype(np.float32)
    x["logf"] = si.round_to_bf16(logf) if dtype == "bf16" else logf
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    dt = pa.PATH_F32 if dtype == "fp32" else pa.PATH_BF16
    scale = d ** -0.5
    dv = {n: torch.from_numpy(a).to("cuda").to(td).contiguous() for n, a in x.items()}
    o, lse = _ring_forward(torch, pa, dv, lengths, d, dt, scale)
    o_ref, lse_ref = oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale, logf=x["logf"])
    eo = np.abs(o.float().cpu().numpy().astype(np.float64) - o_ref).max()
    el = np.abs(lse.cpu().numpy().astype(np.float64) - lse_ref).max()
    print(f"[ring, gates] {dtype} d={d} segments {lengths}: o {eo:.2e} lse {el:.2e}", flush=True)
    assert eo <= TOL_O[dtype] and el <= 1e-3
    o1, lse1 = pa.path_attn_fox_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], dv["logf"], scale=scale)
    torch.cuda.synchronize()
    assert (o.float() - o1.float()).abs().max().item() <= TOL_O[dtype]
    assert (lse - lse1).abs().max().item() <= 1e-3


def test_hop_reads_only_the_regions_it_names(gpu):
    """What travels between devices: a receiving buffer that holds only the regions path_attn_ring_regions names
    (everything else poisoned) gives the same hop as the sender's whole workspace."""
    torch, pa = gpu
    B, H, d, Ls = 1, 2, 128, 1088
    x = si.make_inputs(B, H, 2 * Ls, d, "bf16", 4400, 0.0)
    dv = {n: torch.from_numpy(a).to("cuda").to(torch.bfloat16).contiguous() for n, a in x.items()}
    seg = [{n: dv[n][:, :, r * Ls:(r + 1) * Ls].contiguous() for n in dv} for r in range(2)]
    nbytes = pa.path_attn_workspace_bytes(B, H, Ls, d, pa.PATH_BF16, False)
    ws = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    st = [torch.empty(pa.path_attn_ring_state_bytes(B, H, Ls, d), dtype=torch.uint8, device="cuda") for _ in range(2)]
    for r in range(2):
        pa.path_attn_ring_local(seg[r]["q"], seg[r]["k"], seg[r]["v"], seg[r]["w"], seg[r]["beta"], st[r], ws[r])
    st_ref = st[1].clone()
    pa.path_attn_ring_hop(st_ref, B, H, Ls, ws[0], Ls, d, pa.PATH_BF16)
    recv = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")          # NaN patterns everywhere else
    regions = pa.path_attn_ring_regions(B, H, Ls, d, pa.PATH_BF16)
    for off, nb in regions[:3]:
        assert off % 256 == 0 and off + nb <= nbytes
        recv[off:off + nb].copy_(ws[0][off:off + nb])
    pa.path_attn_ring_hop(st[1], B, H, Ls, recv, Ls, d, pa.PATH_BF16)
    torch.cuda.synchronize()
    assert torch.equal(st[1], st_ref)
    assert sum(nb for _, nb in regions[:3]) == (2 * Ls * d + 2 * d * d) * 2 * B * H      # 2 L d + ceil(L/1024) d^2 elements per head


def test_ring_argument_checks(gpu):
    torch, pa = gpu
    B, H, d = 1, 2, 64
    st = torch.empty(pa.path_attn_ring_state_bytes(B, H, 128, d), dtype=torch.uint8, device="cuda")
    ws = torch.empty(pa.path_attn_workspace_bytes(B, H, 100, d, pa.PATH_F32, False), dtype=torch.uint8, device="cuda")
    with pytest.raises(pa.PathAttnError) as e:
        pa.path_attn_ring_hop(st, B, H, 128, ws, 100, d, pa.PATH_F32)          # a ragged earlier segment
    assert e.value.code == 2                                                    # PATH_ERR_SHAPE
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(pa.PathAttnError) as e:
        pa.path_attn_ring_hop(st, B, H, 128, small, 128, d, pa.PATH_F32)       # not a segment's workspace
    assert e.value.code == 5                                                    # PATH_ERR_WORKSPACE
    assert pa.path_attn_ring_state_bytes(B, H, 128, d) == B * H * 2 * 2 * (2 * (d // 32) * 1024 + 192) * 4
