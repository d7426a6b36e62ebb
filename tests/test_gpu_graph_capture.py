"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset), so a
forward + backward step can be captured in a HIP graph and replayed (run with -m gpu).

The graph is replayed several times with new values in the same input buffers, with eager work and
synchronisations of the program between the replays, and every replay is held bit for bit against the eager
result for the same inputs.  A last test overlaps two steps on two streams, each with a workspace of its own.
"""
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


@pytest.mark.parametrize("dtype,B,H,L,d", [("bf16", 2, 3, 1100, 128), ("fp32", 1, 2, 300, 64)])
def test_training_step_replays_from_a_graph(gpu, dtype, B, H, L, d):
    torch, pa = gpu
    td = torch.float32 if dtype == "fp32" else torch.bfloat16
    dt = pa.PATH_F32 if dtype == "fp32" else pa.PATH_BF16
    scale = d ** -0.5
    names = ("q", "k", "v", "w", "beta", "dO")
    sets = []
    for seed in (3100, 3101, 3102):
        x = si.make_inputs(B, H, L, d, dtype, seed + L, 0.0, with_do=True)
        sets.append({n: torch.from_numpy(x[n]).to("cuda").to(td).contiguous() for n in names})
    buf = {n: torch.empty_like(sets[0][n]) for n in names}          # the graph's fixed input buffers
    ws = torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, dt, True), dtype=torch.uint8, device="cuda")

    def step():
        o, lse = pa.path_attn_train_fwd(buf["q"], buf["k"], buf["v"], buf["w"], buf["beta"], ws, scale=scale)
        grads = pa.path_attn_train_bwd(buf["q"], buf["k"], buf["v"], buf["w"], buf["beta"], o, lse, buf["dO"], ws, scale=scale)
        return (o, lse) + tuple(grads)

    def load(s):
        for n in names:
            buf[n].copy_(s[n])

    eager = []
    for s in sets:                                    # eager results (this also runs every kernel once before the capture)
        load(s)
        eager.append([t.clone() for t in step()])
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        outs = step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    other = si.make_inputs(1, 2, 130, 64, "fp32", 3200, 0.0)
    od = {n: torch.from_numpy(a).to("cuda") for n, a in other.items()}
    for rep, idx in enumerate((1, 0, 2, 2, 1)):
        load(sets[idx])
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs, eager[idx]):
            assert torch.equal(got, ref), (rep, idx)
        # eager work of the program between the replays
        pa.path_attn_fwd(od["q"], od["k"], od["v"], od["w"], od["beta"], scale=0.125)
        torch.cuda.synchronize()


def test_allocation_free_decode_step_replays_from_a_graph(gpu):
    """path_decode_step_static is for callers that cannot allocate -- code under graph capture is one.  The step
    refreshes the key cache in place, so every replay starts from a restored cache."""
    torch, pa = gpu
    B, H, n, d = 2, 8, 900, 128
    x = si.make_inputs(B, H, n + 2, d, "bf16", 3300, 0.0)
    dev = {k_: torch.from_numpy(a).to("cuda").to(torch.bfloat16).contiguous() for k_, a in x.items()}
    tok = [dev[k_][:, :, n].contiguous() for k_ in ("q", "k", "v", "w")] + [dev["beta"][:, :, n].contiguous()]
    kc0, vc0 = dev["k"].clone(), dev["v"].clone()
    kc0[:, :, n:] = 0
    vc0[:, :, n:] = 0
    kc, vc = kc0.clone(), vc0.clone()
    o = torch.empty((B, H, d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, H), dtype=torch.float32, device="cuda")
    scale = d ** -0.5
    pa.path_decode_step_static(*tok, kc, vc, n, scale, o, lse)            # eager (also looks the static array up, once per device)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (o, lse, kc, vc)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    kc.copy_(kc0); vc.copy_(vc0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        pa.path_decode_step_static(*tok, kc, vc, n, scale, o, lse)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(3):
        kc.copy_(kc0); vc.copy_(vc0); o.zero_(); lse.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((o, lse, kc, vc), ref):
            assert torch.equal(got, want), rep
        pa.path_attn_fwd(dev["q"][:, :, :200].contiguous(), dev["k"][:, :, :200].contiguous(), dev["v"][:, :, :200].contiguous(),
                         dev["w"][:, :, :200].contiguous(), dev["beta"][:, :, :200].contiguous())          # eager work in between
        torch.cuda.synchronize()


def test_two_streams_with_their_own_workspaces_do_not_disturb_each_other(gpu):
    """Calls that use distinct workspaces may overlap on different streams (the header's thread-safety rule): two
    forward + backward steps enqueued alternately on two streams give the bits of the same steps run one after the other."""
    torch, pa = gpu
    probs = []
    for i, (B, H, L, d) in enumerate(((1, 4, 1500, 128), (2, 3, 900, 64))):
        x = si.make_inputs(B, H, L, d, "bf16", 3400 + i, 0.0, with_do=True)
        dv = {n: torch.from_numpy(a).to("cuda").to(torch.bfloat16).contiguous() for n, a in x.items()}
        ws = torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, pa.PATH_BF16, True), dtype=torch.uint8, device="cuda")
        probs.append((dv, ws, d ** -0.5))

    def fwd(p, stream=None):
        dv, ws, sc = p
        return pa.path_attn_train_fwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], ws, scale=sc, stream=stream)

    def bwd(p, o, lse, stream=None):
        dv, ws, sc = p
        return pa.path_attn_train_bwd(dv["q"], dv["k"], dv["v"], dv["w"], dv["beta"], o, lse, dv["dO"], ws, scale=sc, stream=stream)

    serial = []
    for p in probs:
        o, lse = fwd(p)
        serial.append([t.clone() for t in (o, lse) + tuple(bwd(p, o, lse))])
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for s in streams:
        s.wait_stream(torch.cuda.current_stream())
    outs = [None, None]
    for rep in range(2):
        with torch.cuda.stream(streams[0]):
            f0 = fwd(probs[0], streams[0])
        with torch.cuda.stream(streams[1]):
            f1 = fwd(probs[1], streams[1])
        with torch.cuda.stream(streams[0]):
            outs[0] = f0 + tuple(bwd(probs[0], *f0, streams[0]))
        with torch.cuda.stream(streams[1]):
            outs[1] = f1 + tuple(bwd(probs[1], *f1, streams[1]))
        torch.cuda.synchronize()
        for i in range(2):
            for got, want in zip(outs[i], serial[i]):
                assert torch.equal(got, want), (rep, i)
