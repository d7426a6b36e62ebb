"""The decode step that allocates nothing (path_decode_step_static: its split partials live in a device array
inside the library) against the ordinary decode step with a caller workspace, through the C ABI: same inputs,
same caches -> bit-identical o, lse and caches, on two calls in a row, the second with a smaller problem (fewer
heads, a shorter cache, so fewer splits), so that what the first call left in the shared array would show.
Named so that pytest collects it last."""
import ctypes

import numpy as np
import pytest

from paper_2505_16381_amd import synth_inputs as si

pytestmark = pytest.mark.gpu


def _case(torch, pa, lib, B, H, n, d, dtype, seed):
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    dt = pa.PATH_F32 if dtype == "fp32" else pa.PATH_BF16
    Lmax = n + 3
    x = si.make_inputs(B, H, Lmax, d, dtype, seed, 0.0)
    dev = {k_: torch.from_numpy(a).to("cuda").to(td).contiguous() for k_, a in x.items()}
    tok = {k_: dev[k_][:, :, n].contiguous() for k_ in ("q", "k", "v", "w")}
    beta = dev["beta"][:, :, n].contiguous()
    scale = d ** -0.5
    outs = []
    for static in (False, True):
        kc = dev["k"].clone(); vc = dev["v"].clone()       # any cache contents do: both variants start from the same
        kc[:, :, n:] = 0; vc[:, :, n:] = 0
        o = torch.full((B, H, d), 7.0, dtype=td, device="cuda")
        lse = torch.full((B, H), 7.0, dtype=torch.float32, device="cuda")
        p = lambda t: ctypes.c_void_p(t.data_ptr())
        if static:
            rc = lib.path_decode_step_static(p(tok["q"]), p(tok["k"]), p(tok["v"]), p(tok["w"]), p(beta), p(kc), p(vc), n, Lmax,
                                             p(o), p(lse), B, H, d, scale, dt, None)
        else:
            ws = torch.empty(pa.path_decode_workspace_bytes(B, H, d), dtype=torch.uint8, device="cuda")
            rc = lib.path_decode_step(p(tok["q"]), p(tok["k"]), p(tok["v"]), p(tok["w"]), p(beta), p(kc), p(vc), n, Lmax,
                                      p(o), p(lse), B, H, d, scale, dt, p(ws), ws.numel(), None)
        torch.cuda.synchronize()
        assert rc == 0, (static, rc, pa.path_attn_last_error())
        outs.append((o.float().cpu().numpy(), lse.cpu().numpy(), kc.float().cpu().numpy(), vc.float().cpu().numpy()))
    for a, b, name in zip(outs[0], outs[1], ("o", "lse", "kcache", "vcache")):
        assert np.isfinite(a).all() and np.array_equal(a, b), name
    return outs[1]


def test_static_decode_step_matches_the_workspace_variant_twice_in_a_row():
    import torch
    import paper_2505_16381_amd as pa
    assert torch.cuda.is_available()
    lib = pa.load_library()
    assert pa.path_decode_static_scratch_bytes() == 8 * 1024 * 1024
    print("[static decode] first call: B=4 H=16 n=5000 d=128 bf16", flush=True)
    _case(torch, pa, lib, 4, 16, 5000, 128, "bf16", 77)            # 16 splits per head
    print("[static decode] second call, smaller: B=1 H=3 n=300 d=64 fp32", flush=True)
    _case(torch, pa, lib, 1, 3, 300, 64, "fp32", 78)               # 3 splits per head, other record size
    print("[static decode] third call: n=0 (empty cache)", flush=True)
    _case(torch, pa, lib, 2, 2, 0, 64, "bf16", 79)


def test_static_decode_step_against_the_oracle_and_its_limit(oracle):
    import torch
    import paper_2505_16381_amd as pa
    from oracle import decode_oracle as dec
    lib = pa.load_library()
    B, H, n, d = 2, 4, 700, 128
    x = si.make_inputs(B, H, n + 1, d, "fp32", 80, 0.0)
    dev = {k_: torch.from_numpy(a).to("cuda").contiguous() for k_, a in x.items()}
    kc = dev["k"].clone(); vc = dev["v"].clone()
    o = torch.empty((B, H, d), device="cuda"); lse = torch.empty((B, H), device="cuda")
    pa.path_decode_step_static(*(dev[k_][:, :, n].contiguous() for k_ in ("q", "k", "v", "w")), dev["beta"][:, :, n].contiguous(),
                               kc, vc, n, d ** -0.5, o, lse)
    torch.cuda.synchronize()
    o_ref, lse_ref, kc_ref, _ = dec.decode_step(x["q"][:, :, n], x["k"][:, :, n], x["v"][:, :, n], x["w"][:, :, n], x["beta"][:, :, n],
                                                x["k"][:, :, :n], x["v"][:, :, :n], d ** -0.5)
    assert np.abs(o.cpu().numpy() - o_ref).max() <= 1e-4 and np.abs(lse.cpu().numpy() - lse_ref).max() <= 1e-3
    assert np.abs(kc.cpu().numpy() - kc_ref).max() <= 1e-4
    # beyond the array's size: a status code and a reason, nothing launched (the pointers are never touched)
    z = ctypes.c_void_p(0x1000)
    rc = lib.path_decode_step_static(z, z, z, z, z, z, z, 5, 16, z, z, 1, 253, 128, 0.1, pa.PATH_BF16, None)
    assert rc == 5 and "static scratch" in pa.path_attn_last_error()
    assert lib.path_decode_step_static(z, z, z, z, z, z, z, 5, 16, z, z, 1, 497, 64, 0.1, pa.PATH_BF16, None) == 5
