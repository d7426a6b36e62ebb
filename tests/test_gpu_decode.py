"""GPU parity of the decode path (key prefill, in-place key-cache update, decode step) against the
decode oracle (run with -m gpu).

The oracle never sees anything the GPU wrote: it prefills its own cache from the inputs.

Bars.  fp32 caches: keys 1e-4 (absolute, values O(1)), o 1e-4, lse 1e-3 -- the forward's bars.
bf16 caches: every refresh rounds the stored keys to bf16 again (part of the method as run).  The
first check holds them against the un-rounded fp64 recurrence over 64 and more steps, with the growth
law of that rounding as the bar (stated in the test); the second, over a few steps, against an oracle
that re-rounds its own cache the same way (o 2e-2, lse 1e-3, keys within four bf16 steps)."""
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


def _run_steps(gpu, dec, x, dv, kc, vc, L0, L, scale, okc, ovc, rnd):
    """Decode tokens L0..L-1 on the GPU and in the oracle (which starts from ITS OWN prefilled cache okc/ovc).
    Returns per step (n = steps done): max errors of o, lse and of the whole key cache."""
    torch, pa = gpu
    rows = []
    for t in range(L0, L):
        o, lse = pa.path_decode_step(dv["q"][:, :, t].contiguous(), dv["k"][:, :, t].contiguous(), dv["v"][:, :, t].contiguous(),
                                     dv["w"][:, :, t].contiguous(), dv["beta"][:, :, t].contiguous(), kc, vc, t, scale)
        torch.cuda.synchronize()
        o_ref, lse_ref, okc, ovc = dec.decode_step(x["q"][:, :, t], x["k"][:, :, t], x["v"][:, :, t], x["w"][:, :, t],
                                                   x["beta"][:, :, t], okc, ovc, scale, round_cache=rnd)
        rows.append((t - L0 + 1, np.abs(o.float().cpu().numpy() - o_ref).max(), np.abs(lse.cpu().numpy() - lse_ref).max(),
                     np.abs(kc[:, :, :t + 1].float().cpu().numpy() - okc).max(), np.abs(okc).max()))
    return rows


def _oracle_prefill(dec, x, L0):
    """The oracle's own cache after the prompt (fp64, nothing from the GPU)."""
    return (dec.key_prefill(x["k"][:, :, :L0], x["w"][:, :, :L0], x["beta"][:, :, :L0]),
            x["v"][:, :, :L0].astype(np.float64))


@pytest.mark.parametrize("dtype,L0,steps,d", [("fp32", 100, 12, 64), ("fp32", 1, 20, 128), ("fp32", 1100, 70, 64)])
def test_decode_steps_match_the_oracle(gpu, dec, dtype, L0, steps, d):
    """fp32 caches against the section's first equation in fp64; the oracle prefills its own cache."""
    L = L0 + steps
    x = si.make_inputs(2, 2, L, d, dtype, 950 + L + d, 0.0)
    dv, td = _dev(gpu, x, dtype)
    scale = d ** -0.5
    kc, vc = _prefill(gpu, dv, td, L0, L)
    okc, ovc = _oracle_prefill(dec, x, L0)
    rows = _run_steps(gpu, dec, x, dv, kc, vc, L0, L, scale, okc, ovc, None)
    wo, wl, wk = (max(r[i] for r in rows) for i in (1, 2, 3))
    print(f"[decode {dtype} L0={L0} steps={steps} d={d}] max|do|={wo:.2e} max|dlse|={wl:.2e} max|dk|={wk:.2e}", flush=True)
    assert wo <= 1e-4 and wl <= 1e-3 and wk <= 1e-4


@pytest.mark.parametrize("L0,steps,d", [(257, 72, 128), (700, 64, 64), (1, 96, 64)])
def test_bf16_cache_against_the_unrounded_recurrence(gpu, dec, L0, steps, d):
    """bf16 caches, refreshed in place n times, held against the UN-ROUNDED fp64 recurrence (paper Sec. 3.4,
    first equation; no model of the kernel's rounding on the oracle's side).  Every refresh rounds every
    stored key once more: an error uniform within half a bf16 step, 0.4 * 2^-9 relative (rms).  The transitions
    are contractions, so earlier errors are not amplified and the cache performs a random walk about the exact
    one: after n refreshes max|dk| = c 2^-9 sqrt(n+1) max|k| with c between 0.9 and 2 in a CPU simulation of
    the rounding (bar: c = 3).  A logit s = scale q.k with scale = d^-1/2, |q| ~ sqrt(d) then carries an error of
    about 0.4 * 2^-9 sqrt(n+1) (rms), and lse = log sum exp averages the logits' errors with the softmax
    weights, i.e. over the effective number of keys (a third of the L0 + n cached ones at these logit
    spreads): four standard deviations are 3 * 2^-9 sqrt((n+1) / (L0+n)), which is added to the forward's 1e-3
    (all of it when the cache holds two keys, a small part of it when it holds hundreds).  o stays far inside
    the forward's 2e-2."""
    L = L0 + steps
    x = si.make_inputs(2, 2, L, d, "bf16", 950 + L + d, 0.0)
    dv, td = _dev(gpu, x, "bf16")
    scale = d ** -0.5
    kc, vc = _prefill(gpu, dv, td, L0, L)
    okc, ovc = _oracle_prefill(dec, x, L0)
    rows = _run_steps(gpu, dec, x, dv, kc, vc, L0, L, scale, okc, ovc, None)
    for n, eo, el, ek, kmax in rows:
        if n in (1, 8, 32, steps):
            print(f"[bf16 cache vs exact recurrence L0={L0} d={d}] n={n}: max|do|={eo:.2e} max|dlse|={el:.2e} "
                  f"max|dk|/(2^-9 sqrt(n+1) max|k|)={ek / (2.0 ** -9 * np.sqrt(n + 1) * kmax):.2f}", flush=True)
        assert eo <= 2e-2
        assert el <= 1e-3 + 3.0 * 2.0 ** -9 * np.sqrt((n + 1) / (L0 + n))
        assert ek <= 3.0 * 2.0 ** -9 * np.sqrt(n + 1) * kmax


@pytest.mark.parametrize("L0,steps,d", [(257, 10, 128), (700, 6, 64)])
def test_bf16_cache_against_the_rounding_model(gpu, dec, L0, steps, d):
    """Second, tighter check over a few steps: the oracle re-rounds its own cache to bf16 at every step
    (``round_cache``, pinned on the CPU), starting from its own prefilled cache rounded once.  o and lse then
    agree far better than against the exact recurrence.  The keys themselves agree only to a few bf16 steps: a
    value near a rounding boundary falls one way on the GPU (fp32 arithmetic, fp16-transported prefill) and the
    other way in the oracle (fp64), after which the two copies are rounded independently at every refresh
    (bar: four steps of the largest binade, 2^-6 max|k|)."""
    L = L0 + steps
    x = si.make_inputs(2, 2, L, d, "bf16", 950 + L + d, 0.0)
    dv, td = _dev(gpu, x, "bf16")
    scale = d ** -0.5
    kc, vc = _prefill(gpu, dv, td, L0, L)
    rnd = lambda a: si.round_to_bf16(a.astype(np.float32)).astype(np.float64)
    okc, ovc = _oracle_prefill(dec, x, L0)
    rows = _run_steps(gpu, dec, x, dv, kc, vc, L0, L, scale, rnd(okc), ovc, rnd)
    wo, wl, wk = (max(r[i] for r in rows) for i in (1, 2, 3))
    kmax = rows[-1][4]
    print(f"[decode bf16 vs rounding model L0={L0} steps={steps} d={d}] max|do|={wo:.2e} max|dlse|={wl:.2e} max|dk|={wk:.2e}", flush=True)
    assert wo <= 2e-2 and wl <= 1e-3
    assert wk <= 2.0 ** -6 * kmax


def test_prefill_then_decode_reproduces_the_forward_rows(gpu, oracle):
    """The decode path continues the training-time forward: both are held against the forward ORACLE's rows
    (and, as a consistency check inside the library, against each other)."""
    torch, pa = gpu
    L0, steps, d = 192, 8, 64
    x = si.make_inputs(1, 2, L0 + steps, d, "fp32", 990, 0.0)
    dv, td = _dev(gpu, x, "fp32")
    scale = d ** -0.5
    o_full, lse_full = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
    kc, vc = _prefill(gpu, dv, td, L0, L0 + steps)
    o_ref, lse_ref = oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale)
    for t in range(L0, L0 + steps):
        o, lse = pa.path_decode_step(dv["q"][:, :, t].contiguous(), dv["k"][:, :, t].contiguous(), dv["v"][:, :, t].contiguous(),
                                     dv["w"][:, :, t].contiguous(), dv["beta"][:, :, t].contiguous(), kc, vc, t, scale)
        assert np.abs(o.cpu().numpy() - o_ref[:, :, t]).max() <= 1e-4
        assert np.abs(lse.cpu().numpy() - lse_ref[:, :, t]).max() <= 1e-3
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


@pytest.mark.parametrize("dtype,L0,steps,d", [("fp32", 130, 40, 64), ("fp32", 1, 24, 128), ("bf16", 600, 64, 128)])
def test_gated_decode_steps_match_the_oracle(gpu, dec, oracle, dtype, L0, steps, d):
    """PaTH-FoX at decode time: gate prefill + gated steps against the gated decode oracle (its own prefill, its own
    running sums) and, for the last step, against the gated FORWARD oracle's row.  fp32 caches: the forward's bars.
    bf16 caches: the drift law of the plain bf16 case, with one change.  There the log-sum-exp averages the logits'
    errors over all L0 + n cached keys; gates concentrate the attention on the recent ones, so the average runs over
    the effective number of keys of the gate profile g_i = exp(c_t - c_i), n_eff = (sum g)^2 / sum g^2 (here about 15),
    and the bar is 1e-3 + 3 * 2^-9 * sqrt((n + 1) / n_eff).  The sums themselves are kept in fp32 and add nothing."""
    torch, pa = gpu
    L = L0 + steps
    x = si.make_inputs(2, 2, L, d, dtype, 990 + L + d, 0.0)
    rng = np.random.default_rng(990 + L)
    logf = (-np.log1p(np.exp(-rng.normal(2.0, 1.0, size=(2, 2, L))))).astype(np.float32)
    x["logf"] = si.round_to_bf16(logf) if dtype == "bf16" else logf
    dv, td = _dev(gpu, x, dtype)
    scale = d ** -0.5
    kc, vc = _prefill(gpu, dv, td, L0, L)
    cc = torch.zeros((2, 2, L), dtype=torch.float32, device="cuda")
    pa.path_gate_prefill(dv["logf"][:, :, :L0].contiguous(), cc)
    torch.cuda.synchronize()
    occ = np.cumsum(x["logf"][:, :, :L0].astype(np.float64), axis=-1)
    assert np.abs(cc[:, :, :L0].cpu().numpy() - occ).max() <= 1e-4 and float(cc[:, :, L0:].abs().max()) == 0.0
    okc, ovc = _oracle_prefill(dec, x, L0)
    wo = wl = 0.0
    for t in range(L0, L):
        tok = [dv[n][:, :, t].contiguous() for n in ("q", "k", "v", "w")] + [dv["beta"][:, :, t].contiguous(), dv["logf"][:, :, t].contiguous()]
        o, lse = pa.path_decode_step_fox(*tok, kc, vc, cc, t, scale)
        torch.cuda.synchronize()
        o_ref, lse_ref, okc, ovc, occ = dec.decode_step(x["q"][:, :, t], x["k"][:, :, t], x["v"][:, :, t], x["w"][:, :, t], x["beta"][:, :, t],
                                                        okc, ovc, scale, logf_t=x["logf"][:, :, t], cc=occ)
        wo = max(wo, np.abs(o.float().cpu().numpy() - o_ref).max())
        el = np.abs(lse.cpu().numpy() - lse_ref).max()
        wl = max(wl, el)
        if dtype == "bf16":
            n = t - L0 + 1
            g = np.exp(occ[..., -1:] - occ)
            n_eff = min(float((g.sum(-1) ** 2 / (g ** 2).sum(-1)).min()), L0 + n)
            assert el <= 1e-3 + 3.0 * 2.0 ** -9 * np.sqrt((n + 1) / n_eff), (n, el, n_eff)
    assert np.abs(cc.cpu().numpy() - occ).max() <= 1e-4 * max(1.0, np.abs(occ).max())
    # the last step is the gated forward's last row
    o_fw, lse_fw = oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale, rows=np.array([L - 1]), logf=x["logf"])
    eo = np.abs(o.float().cpu().numpy() - o_fw[:, :, 0]).max()
    ef = np.abs(lse.cpu().numpy() - lse_fw[:, :, 0]).max()
    print(f"[gated decode {dtype} L0={L0} steps={steps} d={d}] max|do|={wo:.2e} max|dlse|={wl:.2e}; last step against the forward row: {eo:.2e} {ef:.2e}", flush=True)
    if dtype == "fp32":
        assert wo <= 1e-4 and wl <= 1e-3 and eo <= 1e-4 and ef <= 1e-3
    else:
        assert wo <= 2e-2 and eo <= 2e-2 and ef <= 1e-3 + 3.0 * 2.0 ** -9 * np.sqrt((steps + 1) / n_eff)


def test_gated_decode_argument_checks(gpu):
    torch, pa = gpu
    z = torch.zeros((1, 2, 64), device="cuda")
    cc = torch.zeros((1, 2, 8), device="cuda")
    kc = torch.zeros((1, 2, 8, 64), device="cuda")
    with pytest.raises(pa.PathAttnError) as e:
        pa.path_decode_step_fox(z, z, z, z, torch.zeros((1, 2), device="cuda"), torch.zeros((1, 2), device="cuda"), kc, kc.clone(), cc, 8, 0.125)
    assert e.value.code == 2                       # the cache is full: n must be < Lmax
    with pytest.raises(pa.PathAttnError) as e:
        pa.path_gate_prefill(torch.zeros((1, 2, 9), device="cuda"), cc)
    assert e.value.code == 2                       # a prompt longer than the cache
