"""GPU parity of the forward path against the fp64 oracle (run with -m gpu).

Tolerances are the benchmark's: max |o - o_oracle| <= 1e-4 (fp32 I/O) or
2e-2 (bf16 I/O); max |lse - lse_oracle| <= 1e-3.
"""
import numpy as np
import pytest

from paper_2505_16381_amd import synth_inputs as si

pytestmark = pytest.mark.gpu

TOL_O = {"fp32": 1e-4, "bf16": 2e-2}
TOL_LSE = 1e-3


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2505_16381_amd as pa
    assert torch.cuda.is_available(), "these tests need a GPU"
    pa.load_library()
    return torch, pa


def _to_dev(torch, x, dtype):
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    return {n: torch.from_numpy(a).to("cuda").to(td).contiguous() for n, a in x.items()}


def _run(gpu, x, dtype, scale):
    torch, pa = gpu
    dv = _to_dev(torch, x, dtype)
    o, lse = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
    torch.cuda.synchronize()
    return o.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)


def _check(gpu, oracle, x, dtype, scale, rows=None, tag=""):
    o, lse = _run(gpu, x, dtype, scale)
    o_ref, lse_ref = oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale, rows=rows)
    if rows is not None:
        o, lse = o[:, :, rows], lse[:, :, rows]
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    eo, el = np.abs(o - o_ref).max(), np.abs(lse - lse_ref).max()
    print(f"[{tag}] dtype={dtype} max|do|={eo:.3e} max|dlse|={el:.3e}", flush=True)
    assert eo <= TOL_O[dtype], (tag, eo)
    assert el <= TOL_LSE, (tag, el)


def test_prep_intermediates_fp32(gpu, oracle):
    """Chunk preprocessing outputs vs the NumPy block model (localises layout bugs)."""
    import blockwise_model as bm
    import ws_layout as wl
    torch, pa = gpu
    B, H, L, d = 1, 2, 200, 64
    x = si.make_inputs(B, H, L, d, "fp32", 101)
    dv = _to_dev(torch, x, "fp32")
    nbytes = pa.path_attn_workspace_bytes(B, H, L, d, pa.PATH_F32)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=0.125, workspace=ws)
    torch.cuda.synchronize()
    off = pa.path_attn_fwd_workspace_layout(B, H, L, d, pa.PATH_F32)
    raw = ws.cpu().numpy()
    NC = -(-L // 64)
    f32 = lambda a, b_: raw[a:b_].view(np.float32).astype(np.float64)
    kt = wl.unfrag(f32(off[0], off[1])[: B * H * NC * 64 * d].reshape(B * H, NC, 64 * d), 64, d, 4)
    # V^T tiles: [32-key half][...] -- each half is a fragment-order tile with d rows and 32 contraction indices
    vth = wl.unfrag(f32(off[1], off[2])[: B * H * NC * 64 * d].reshape(B * H, NC, 2, 32 * d), d, 32, 4)
    vt = np.concatenate([vth[:, :, 0], vth[:, :, 1]], axis=-1)
    dp = wl.unfrag(f32(off[2], off[3])[: B * H * NC * d * d].reshape(B * H, NC, d * d), d, d, 4)
    xi = wl.unacc(f32(off[3], off[4])[: B * H * NC * 64 * d].reshape(B * H, NC, 2, d // 32, 1024))
    sd = wl.unacc(f32(off[4], off[5])[: B * H * NC * 4096].reshape(B * H, NC, 2, 2, 1024))
    for bh in range(B * H):
        pad = lambda a: np.pad(a.astype(np.float64), [(0, NC * 64 - L)] + [(0, 0)] * (a.ndim - 1))
        q, k, v, w, beta = (pad(x[n].reshape((B * H, L) + x[n].shape[3:])[bh]) for n in ("q", "k", "v", "w", "beta"))
        for c in range(NC):
            s = slice(c * 64, (c + 1) * 64)
            pre = bm.chunk_prep(q[s], k[s], w[s], beta[s])
            err = {}
            err["Kb"] = np.abs(kt[bh, c] - pre["Kb"]).max()
            err["Vt"] = np.abs(vt[bh, c] - v[s].T).max()
            err["-dP^T"] = np.abs(dp[bh, c] + pre["dP"].T).max()
            # xinit block [tb][cb]: rows = d index within block, cols = query within block
            Qb = np.block([[xi[bh, c, tb, cb].T for cb in range(d // 32)] for tb in range(2)])
            err["Qb"] = np.abs(Qb - pre["Qb"]).max()
            # sd block [qb][kb]: rows = key, cols = query; only key <= query is defined
            Sd = np.block([[sd[bh, c, qb, kb].T for kb in range(2)] for qb in range(2)])
            nv = min(64, L - c * 64)
            err["Sd"] = np.abs(np.tril(Sd)[:nv, :nv] - pre["Sd"][:nv, :nv]).max()
            print(f"bh={bh} chunk={c} " + " ".join(f"{n}={e:.2e}" for n, e in err.items()), flush=True)
            for n, e in err.items():
                assert e < 2e-4, (bh, c, n, e)


def test_config0_tiny_fp32(gpu, oracle):
    x, c = si.make_config(0)
    _check(gpu, oracle, x, "fp32", c["d"] ** -0.5, tag="cfg0")


@pytest.mark.parametrize("L", [1, 2, 63, 64, 65, 130, 300])
@pytest.mark.parametrize("d", [64, 128])
def test_fp32_ragged_lengths(gpu, oracle, L, d):
    x = si.make_inputs(1, 3, L, d, "fp32", 200 + L + d)
    _check(gpu, oracle, x, "fp32", d ** -0.5, tag=f"fp32 L={L} d={d}")


@pytest.mark.parametrize("dtype,L,d", [("fp32", 2200, 64), ("fp32", 3300, 128), ("bf16", 2500, 64), ("bf16", 4100, 128)])
def test_several_superblocks(gpu, oracle, dtype, L, d):
    """Three to five super-blocks (16 chunks = 1024 tokens each), ragged: near chunks, far
    super-blocks and the far product all take part."""
    x = si.make_inputs(1, 2, L, d, dtype, 250 + L + d)
    _check(gpu, oracle, x, dtype, d ** -0.5, tag=f"superblocks {dtype} L={L} d={d}")


@pytest.mark.parametrize("L", [1, 77, 512, 1000])
@pytest.mark.parametrize("d", [64, 128])
def test_bf16_small(gpu, oracle, L, d):
    x = si.make_inputs(2, 2, L, d, "bf16", 300 + L + d)
    _check(gpu, oracle, x, "bf16", d ** -0.5, tag=f"bf16 L={L} d={d}")


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_special_betas(gpu, oracle, dtype):
    """beta exactly 0, 1 (singular H) and 2 (reflection) inside one sequence."""
    x = si.make_inputs(1, 2, 320, 64, dtype, 400)
    x["beta"][..., 0::3] = 0.0
    x["beta"][..., 1::3] = 1.0
    x["beta"][..., 2::3] = 2.0
    _check(gpu, oracle, x, dtype, 0.125, tag="special betas")


@pytest.mark.parametrize("L,d", [(1100, 128), (700, 64)])
def test_bf16_large_magnitude_inputs(gpu, oracle, L, d):
    """With bf16 I/O the transported operands (query state, boundary-adjusted keys, chunk products) travel as
    fp16, whose range ends at 65504; the header's rule is that the norms of q and k rows stay below that.  Here
    q and k are 64 times their usual size (row norms ~ 64 sqrt(d) ~ 700, far inside the bound but far outside the
    unit scale of the other cases), with `scale` reduced by 64^2 so that the logits are the usual ones."""
    x = si.make_inputs(1, 2, L, d, "bf16", 430 + L + d)
    x["q"] = (x["q"] * 64).astype(np.float32)       # powers of two: still exact bf16 values
    x["k"] = (x["k"] * 64).astype(np.float32)
    _check(gpu, oracle, x, "bf16", d ** -0.5 / 4096, tag=f"bf16 x64 inputs L={L} d={d}")


def test_swap_construction_on_gpu(gpu, oracle):
    """The paper's swap-tracking construction (App. A), zero-padded from d = 6 to 64, scale 1."""
    rng = np.random.default_rng(5)
    n = 99
    L, d = n + 1, 64
    q = np.zeros((1, 1, L, d), np.float32); k = np.zeros_like(q); v = np.zeros_like(q); w = np.zeros_like(q)
    q[..., :6] = 0.02 * np.array([1, 2, 3, 4, 5, 54.5])      # small "n" keeps exp() in range
    k[0, 0, 0, :6] = [1, 2, 3, 4, 5, -1]
    v[0, 0, 0, 0] = 1.0
    lst = [1, 2, 3, 4, 5]
    for t in range(1, L):
        a, b = rng.choice(5, size=2, replace=False)
        w[0, 0, t, a] = 2 ** -0.5; w[0, 0, t, b] = -(2 ** -0.5)
        lst[a], lst[b] = lst[b], lst[a]
    beta = np.full((1, 1, L), 2.0, np.float32)
    x = dict(q=q, k=k, v=v, w=w, beta=beta)
    o, lse = _run(gpu, x, "fp32", 1.0)
    s0 = 0.02 * (sum((i + 1) * lst[i] for i in range(5)) - 54.5)
    a0 = np.exp(s0) / (np.exp(s0) + n)
    assert abs(o[0, 0, n, 0] - a0) < 1e-5 and np.abs(o[0, 0, n, 1:]).max() < 1e-6
    _check(gpu, oracle, x, "fp32", 1.0, tag="swaps")


def test_config1_bf16_full_and_beta_zero(gpu, oracle):
    x, c = si.make_config(1)
    scale = c["d"] ** -0.5
    _check(gpu, oracle, x, "bf16", scale, tag="cfg1")
    # beta = 0 run: must equal plain causal softmax attention (computed here densely, fp64, 4 heads)
    x0 = dict(x); x0["beta"] = np.zeros_like(x["beta"])
    o, lse = _run(gpu, x0, "bf16", scale)
    L = c["L"]
    mask = np.tril(np.ones((L, L), dtype=bool))
    for (b, h) in [(0, 0), (3, 7), (7, 15), (5, 2)]:
        S = scale * x["q"][b, h].astype(np.float64) @ x["k"][b, h].astype(np.float64).T
        S = np.where(mask, S, -np.inf)
        m = S.max(-1, keepdims=True); e = np.exp(S - m); z = e.sum(-1, keepdims=True)
        assert np.abs(o[b, h] - (e / z) @ x["v"][b, h].astype(np.float64)).max() <= 2e-2
        assert np.abs(lse[b, h] - (m + np.log(z))[:, 0]).max() <= 1e-3


def _sample_rows(L, n, seed):
    """Seeded sample of query rows: the last 64 (longest products), random ones, the first chunk boundaries and
    the three rows around EVERY super-block boundary (multiples of 1024 tokens: last row that has no far block
    to its left in the new super-block, first row of it, and the one after)."""
    rng = np.random.default_rng(seed)
    edges = np.concatenate([[s - 1, s, s + 1] for s in range(1024, L, 1024)]) if L > 1024 else np.zeros(0, int)
    return np.unique(np.concatenate([np.arange(L - 64, L), rng.integers(0, L, n), [0, 1, 63, 64, 65, 127, 128], edges]).astype(int))


def test_config2_headline_sampled_rows(gpu, oracle):
    x, c = si.make_config(2)
    rows = _sample_rows(c["L"], 200, 7)
    _check(gpu, oracle, x, "bf16", c["d"] ** -0.5, rows=rows, tag="cfg2")


def test_config4_long_context_sampled_rows(gpu, oracle):
    x, c = si.make_config(4)
    rows = _sample_rows(c["L"], 130, 8)
    _check(gpu, oracle, x, "bf16", c["d"] ** -0.5, rows=rows, tag="cfg4")
