"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset), so a
forward + backward step can be captured in a HIP graph and replayed (run with -m gpu).

The graph is replayed several times with new values in the same input buffers, with eager work and
synchronisations of the program between the replays, and every replay is held bit for bit against the eager
result for the same inputs.
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
