"""GPU parity on seeded random shapes (run with -m gpu): forward and backward against the oracle.

The fixed cases of the other files pick their shapes by hand; here batch, heads, length, head dimension, dtype
and scale come from a seeded generator, with the lengths drawn around the places where the kernels change
behaviour (chunk edges at multiples of 64, super-block edges at multiples of 1024) and head counts that are not
multiples of eight (the workgroup numbering deals heads to the eight XCDs in rounds of eight).
Bars as everywhere: o 1e-4 / 2e-2, lse 1e-3, gradients 1e-4 / 2e-2 of the tensor's maximum.
"""
import numpy as np
import pytest

from paper_2505_16381_amd import synth_inputs as si

pytestmark = pytest.mark.gpu
TOL_O = {"fp32": 1e-4, "bf16": 2e-2}
TOL_G = {"fp32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2505_16381_amd as pa
    assert torch.cuda.is_available()
    pa.load_library()
    return torch, pa


def _shapes():
    rng = np.random.default_rng(20250516)
    edges = [1, 63, 64, 65, 127, 128, 129, 1023, 1024, 1025, 1087, 1088, 2047, 2048, 2049]
    out = []
    for case in range(14):
        dtype = "fp32" if case % 2 == 0 else "bf16"
        d = int(rng.choice([64, 128]))
        B = int(rng.choice([1, 2, 3]))
        H = int(rng.choice([1, 3, 5, 9, 11]))
        if rng.random() < 0.6:
            L = int(rng.choice(edges))
        else:
            L = int(rng.integers(2, 2300))
        # keep the oracle's work per case bounded (pairs ~ B H L^2 / 2)
        while B * H * L * L > 3.0e7 and H > 1:
            H = max(1, H // 2)
        if B * H * L * L > 3.0e7:
            B = 1
        scale = float(rng.choice([d ** -0.5, 0.5 * d ** -0.5, 0.2]))
        out.append((case, dtype, B, H, L, d, scale))
    return out


@pytest.mark.parametrize("case,dtype,B,H,L,d,scale", _shapes())
def test_random_shape_forward_and_backward(gpu, oracle, case, dtype, B, H, L, d, scale):
    torch, pa = gpu
    x = si.make_inputs(B, H, L, d, dtype, 9000 + case, 0.0, with_do=True)
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    dv = {n: torch.from_numpy(a).to("cuda").to(td).contiguous() for n, a in x.items()}
    print(f"[random shape {case}] {dtype} B={B} H={H} L={L} d={d} scale={scale:.4f}", flush=True)
    o, lse = pa.path_attn_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], scale=scale)
    grads = pa.path_attn_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], scale=scale)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.fwd(x["q"], x["k"], x["v"], x["w"], x["beta"], scale)
    eo = np.abs(o.float().cpu().numpy().astype(np.float64) - o_ref).max()
    el = np.abs(lse.cpu().numpy().astype(np.float64) - lse_ref).max()
    assert eo <= TOL_O[dtype] and el <= 1e-3, (eo, el)
    ref = oracle.bwd(x["q"], x["k"], x["v"], x["w"], x["beta"], x["dO"], scale)
    worst = []
    for n, g, r in zip(("dq", "dk", "dv", "dw", "dbeta"), grads, ref):
        g = g.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(g).all(), n
        worst.append((np.abs(g - r).max() / max(np.abs(r).max(), 1e-2), n))
    print(f"[random shape {case}] o {eo:.2e} lse {el:.2e} grads " + " ".join(f"{n}={e:.2e}" for e, n in worst), flush=True)
    assert max(worst)[0] <= TOL_G[dtype], worst
