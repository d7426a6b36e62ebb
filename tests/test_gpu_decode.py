"""GPU parity of the decode path (key prefill, in-place key-cache update, decode step) against the
decode oracle (run with -m gpu).

Bars.  fp32 caches: keys 1e-4 (absolute, |k| ~ sqrt(d)... values O(1)), o 1e-4, lse 1e-3 -- the
forward's bars.  bf16 caches: every refresh rounds the stored keys to bf16 again (part of the
method as run); the oracle models exactly that rounding (``round_cache``), and the bars are the
forward's bf16 bars (o 2e-2, lse 1e-3 per step on a freshly rounded cache; keys within one bf16
rounding of the oracle's: 2^-8 relative to max|k|)."""
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


@pytest.fixture(scope="module")
def dec():
    from oracle import decode_oracle
    return decode_oracle


def _dev(gpu, x, dtype):
    torch, _ = gpu
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    return {n: torch.from_numpy(a).to("cuda").to(td).contiguous() for n, a in x.items()}, td


def _prefill(gpu, dv, td, L, Lmax):
    torch, pa = gpu
    B, H, _, d = dv["q"].shape
    dt = pa.PATH_F32 if td == torch.float32 else pa.PATH_BF16
    ws = torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, dt, False), dtype=torch.uint8, device="cuda")
    sl = lambda n: dv[n][:, :, :L].contiguous()
    pa.path_attn_fwd_prep(sl("q"), sl("k"), sl("v"), sl("w"), dv["beta"][:, :, :L].contiguous(), ws)
    kc = torch.zeros((B, H, Lmax, d), dtype=td, device="cuda")
    vc = torch.zeros((B, H, Lmax, d), dtype=td, device="cuda")
    pa.path_key_prefill(sl("v"), ws, kc, vc)
    torch.cuda.synchronize()
    return kc, vc


@pytest.mark.parametrize("dtype,L,d", [("fp32", 64, 64), ("fp32", 300, 128), ("fp32", 1100, 64), ("bf16", 200, 64),
                                       ("bf16", 1030, 128)])
def test_key_prefill_matches_the_oracle_cache(gpu, dec, dtype, L, d):
    x = si.make_inputs(1, 2, L, d, dtype, 900 + L + d, 0.0)
    dv, td = _dev(gpu, x, dtype)
    kc, vc = _prefill(gpu, dv, td, L, L + 7)
    want = dec.key_prefill(x["k"], x["w"], x["beta"])
    got = kc[:, :, :L].float().cpu().numpy().astype(np.float64)
    tol = 1e-4 if dtype == "fp32" else 2.0 ** -8 * np.abs(want).max() * 1.5      # storage rounding + fp16 transport
    err = np.abs(got - want).max()
    print(f"[prefill {dtype} L={L} d={d}] max|dk|={err:.2e} (bar {tol:.2e})", flush=True)
    assert err <= tol
    assert np.array_equal(vc[:, :, :L].float().cpu().numpy(), dv["v"].float().cpu().numpy())
    assert float(kc[:, :, L:].abs().max()) == 0.0 and float(vc[:, :, L:].abs().max()) == 0.0    # nothing past L


@pytest.mark.parametrize("dtype,L0,steps,d", [("fp32", 100, 12, 64), ("fp32", 1, 20, 128), ("bf16", 257, 10, 128),
                                               ("bf16", 700, 6, 64)])
def test_decode_steps_match_the_oracle(gpu, dec, dtype, L0, steps, d):
    torch, pa = gpu
    L = L0 + steps
    x = si.make_inputs(2, 2, L, d, dtype, 950 + L + d, 0.0)
    dv, td = _dev(gpu, x, dtype)
    scale = d ** -0.5
    kc, vc = _prefill(gpu, dv, td, L0, L)
    # the oracle continues from the SAME cache contents (what the prefill left, as stored)
    okc = kc[:, :, :L0].float().cpu().numpy().astype(np.float64)
    ovc = vc[:, :, :L0].float().cpu().numpy().astype(np.float64)
    rnd = None if dtype == "fp32" else (lambda a: si.round_to_bf16(a.astype(np.float32)).astype(np.float64))
    worst_o = worst_l = worst_k = 0.0
    for t in range(L0, L):
        o, lse = pa.path_decode_step(dv["q"][:, :, t].contiguous(), dv["k"][:, :, t].contiguous(), dv["v"][:, :, t].contiguous(),
                                     dv["w"][:, :, t].contiguous(), dv["beta"][:, :, t].contiguous(), kc, vc, t, scale)
        torch.cuda.synchronize()
        o_ref, lse_ref, okc, ovc = dec.decode_step(x["q"][:, :, t], x["k"][:, :, t], x["v"][:, :, t], x["w"][:, :, t],
                                                   x["beta"][:, :, t], okc, ovc, scale, round_cache=rnd)
        worst_o = max(worst_o, np.abs(o.float().cpu().numpy() - o_ref).max())
        worst_l = max(worst_l, np.abs(lse.cpu().numpy() - lse_ref).max())
        worst_k = max(worst_k, np.abs(kc[:, :, :t + 1].float().cpu().numpy() - okc).max())
    print(f"[decode {dtype} L0={L0} steps={steps} d={d}] max|do|={worst_o:.2e} max|dlse|={worst_l:.2e} max|dk|={worst_k:.2e}", flush=True)
    assert worst_o <= (1e-4 if dtype == "fp32" else 2e-2)
    assert worst_l <= 1e-3
    # bf16: a key whose fp32 value sits on a rounding boundary may round the other way on the GPU
    # (fp32 arithmetic) than in the oracle (fp64): allow one bf16 step on the keys
    kmax = np.abs(okc).max()
    assert worst_k <= (1e-4 if dtype == "fp32" else 2.0 ** -7 * kmax)


def test_prefill_then_decode_reproduces_the_forward_rows(gpu):
    """Consistency inside the library: the decode path continues the training-time forward."""
    torch, pa = gpu
    L0, steps, d = 192, 8, 64
    x = si.make_inputs(1, 2, L0 + steps, d, "fp32", 990, 0.0)
    dv, td = _dev(gpu, x, "fp32")
    scale = d ** -0.5
    o_full, lse_full = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
    kc, vc = _prefill(gpu, dv, td, L0, L0 + steps)
    for t in range(L0, L0 + steps):
        o, lse = pa.path_decode_step(dv["q"][:, :, t].contiguous(), dv["k"][:, :, t].contiguous(), dv["v"][:, :, t].contiguous(),
                                     dv["w"][:, :, t].contiguous(), dv["beta"][:, :, t].contiguous(), kc, vc, t, scale)
        assert float((o - o_full[:, :, t]).abs().max()) <= 1e-4
        assert float((lse - lse_full[:, :, t]).abs().max()) <= 1e-3


def test_decode_argument_checks(gpu):
    torch, pa = gpu
    B, H, d, Lmax = 1, 2, 64, 16
    z = torch.zeros((B, H, d), device="cuda")
    beta = torch.zeros((B, H), device="cuda")
    kc = torch.zeros((B, H, Lmax, d), device="cuda")
    with pytest.raises(pa.PathAttnError) as e:
        pa.path_decode_step(z, z, z, z, beta, kc, kc.clone(), Lmax, 0.125)       # cache full
    assert e.value.code == 2
    with pytest.raises(pa.PathAttnError) as e:
        pa.path_decode_step(z, z, z, z, beta, kc, kc.clone(), 0, 0.0)            # scale must be positive
    assert e.value.code == 4
