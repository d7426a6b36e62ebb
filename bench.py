#!/usr/bin/env python3
"""Benchmark of the PaTH attention hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input
at the headline shape B=4, H=16, L=8192, d=128 (bf16 I/O): forward (chunk
transform + sweep) and, once the library provides it at this shape, backward.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

FLOP convention: attention-equivalent 4*d*L(L+1)/2*B*H for the forward and
2.5x that for the backward (FlashAttention convention, masked work not
counted); the PaTH-inclusive count (query-state updates at the blocking the
kernels use, the two transforms) is reported next to it, and every percentage of
the datasheet peak also against the MFMA rate measured in the same run.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "PaTH attn fwd+bwd TFLOP/s and % bf16 MFMA peak at B=4,H=16,L=8192,d=128"
PEAK_TFLOPS = 2500.0      # MI355X dense bf16/fp16 MFMA
CHUNK = 64                # tokens per chunk (the library's UT-transform block)
SBC = 16                  # chunks per super-block (second blocking level: one query-state update per 1024 keys)
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "fwd_bwd_headline_L8192_d128_hbm_traffic.txt")


def attn_flops(B, H, L, d):
    return 4.0 * d * (L * (L + 1) / 2.0) * B * H


def path_extra_flops(B, H, L, d):
    """PaTH-only work of the forward at the blocking the kernels use (chunk C = 64, super-block S = 16 chunks):
    the chunk transform, the second-level transform, and the query-state updates -- one 2*C*d*d update per
    (query chunk, key chunk of its own super-block left of it) and one per (query chunk, super-block further
    left), none after a head's first chunk / first super-block."""
    nc = -(-L // CHUNK)
    prep = (14.0 * CHUNK * CHUNK * d + 2.0 * CHUNK * d * d + 4.0 * CHUNK ** 3 + CHUNK ** 3 / 3.0) * nc
    prep2 = (2.0 * CHUNK * d * d + 2.0 * d ** 3) * nc          # keys carried to the super-block edge; running product
    upd = 0
    for c in range(nc):
        jsb = (c // SBC) * SBC
        near = sum(1 for j in range(jsb, c) if j > 0)
        far = max(0, c // SBC - 1)
        upd += near + far
    return (prep + prep2 + 2.0 * CHUNK * d * d * upd) * B * H


def pair_counts(L):
    """(near, far) query-key pairs per head of the backward's key-side kernels: near = keys in the query's own
    super-block but left of its chunk; far = keys in super-blocks left of the query's."""
    nc = -(-L // CHUNK)
    near = far = 0
    for c in range(nc):
        nq = min(CHUNK, L - c * CHUNK)
        jsb = (c // SBC) * SBC
        near += nq * (c - jsb) * CHUNK
        far += nq * jsb * CHUNK
    return near, far


def measured_mfma_peak(torch, pa, dev, random_operands=False):
    """TFLOP/s of a register-resident MFMA chain (two waves per SIMD, no memory traffic): what the matrix pipes
    deliver at the clock the chip holds under that load -- with smooth operands, or with operands of random sign
    and significand (the kind the kernels multiply: more power per product, lower clock)."""
    sink = torch.empty(1024 * 4 * 64, dtype=torch.float32, device=dev)
    pa.path_probe_mfma(sink, 2, 2000, random_operands=random_operands)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    flops = pa.path_probe_mfma(sink, 2, 20000, random_operands=random_operands)
    e1.record()
    torch.cuda.synchronize()
    return flops / (e0.elapsed_time(e1) * 1e-3) / 1e12


def profiled_traffic(kernel_key):
    """HBM bytes per launch of a kernel from the committed rocprofv3 counter profile (FETCH_SIZE / WRITE_SIZE runs
    of this same command), or None when the profile does not list it."""
    try:
        for line in open(TRAFFIC_PROFILE):
            if line.startswith("# json:"):
                rec = json.loads(line[len("# json:"):])
                if rec.get("kernel") == kernel_key:
                    return rec
    except OSError:
        pass
    return None


def cpu_baseline(x, cfg, scale, n_rows=3072):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload: its forward on a row sample of
    all heads and its backward (not separable by rows) on four whole heads."""
    import numpy as np
    from oracle import path_oracle
    rng = np.random.default_rng(0)
    L, d = cfg["L"], cfg["d"]
    n_heads = cfg["B"] * cfg["H"]
    rows = np.unique(rng.integers(0, L, n_rows))
    sub = {n: x[n].reshape((1, n_heads) + x[n].shape[2:]) for n in ("q", "k", "v", "w", "beta", "dO")}
    path_oracle.fwd(sub["q"], sub["k"], sub["v"], sub["w"], sub["beta"], scale, rows=rows[:2])  # warm
    t0 = time.perf_counter()
    path_oracle.fwd(sub["q"], sub["k"], sub["v"], sub["w"], sub["beta"], scale, rows=rows)
    t_f = time.perf_counter() - t0
    one = {n: a[:, :4] for n, a in sub.items()}
    t0 = time.perf_counter()
    path_oracle.bwd(one["q"], one["k"], one["v"], one["w"], one["beta"], one["dO"], scale)
    t_b = time.perf_counter() - t0
    pairs_f = float((rows + 1).sum()) * n_heads
    pairs_b = 4 * L * (L + 1) / 2.0
    return {
        "value": (pairs_f * 4.0 * d + pairs_b * 10.0 * d) / (t_f + t_b) / 1e12, "unit": "TFLOP/s", "cores": path_oracle.num_threads(),
        "kind": "oracle", "seconds": t_f + t_b, "fwd_seconds": t_f, "bwd_seconds": t_b,
        "sample": f"forward: all {n_heads} heads x {len(rows)} random query rows of the headline shape ({pairs_f:.3g} query-key "
                  f"pairs, 4d attention-equivalent flops each); backward (forward walk included): four whole heads "
                  f"({pairs_b:.3g} pairs, 2.5 x 4d each)",
    }


def bench_decode(args, torch, pa, si, dev):
    """One decoding step at the headline head shape over a cache of L tokens (paper Sec. 3.4):
    every cached key is refreshed in place, then q attends over the cache.  HBM-bound:
    algorithmic traffic = read K + write K + read V = 3 * L * d * 2 bytes per head."""
    cfg = dict(si.CONFIGS[args.config])
    if args.shape:
        cfg.update(dict(zip(("B", "H", "L", "d"), (int(v) for v in args.shape.split(",")))))
    B, H, L, d = cfg["B"], cfg["H"], cfg["L"], cfg["d"]
    g = torch.Generator(device="cuda").manual_seed(20250516)
    rn = lambda *shape: torch.randn(*shape, device=dev, generator=g)
    kc = rn(B, H, L + 64, d).to(torch.bfloat16)
    vc = rn(B, H, L + 64, d).to(torch.bfloat16)
    q, k, v = (rn(B, H, d).to(torch.bfloat16) for _ in range(3))
    w = torch.nn.functional.normalize(rn(B, H, d), dim=-1).to(torch.bfloat16)
    beta = (2 * torch.sigmoid(rn(B, H))).to(torch.bfloat16)
    ws = torch.empty(pa.path_decode_workspace_bytes(B, H, d), dtype=torch.uint8, device=dev)
    scale = d ** -0.5
    step = lambda: pa.path_decode_step(q, k, v, w, beta, kc, vc, L, scale, workspace=ws)   # same position every time
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = e0.elapsed_time(e1) / args.steps
    bytes_alg = 3.0 * L * d * 2 * B * H
    # key prefill of the same cache from a prompt's forward workspace (one-off, linear in L)
    pq, pk, pv = (rn(B, H, L, d).to(torch.bfloat16) for _ in range(3))
    pw = torch.nn.functional.normalize(rn(B, H, L, d), dim=-1).to(torch.bfloat16)
    pbeta = (2 * torch.sigmoid(rn(B, H, L))).to(torch.bfloat16)
    fws = torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, pa.PATH_BF16, False), dtype=torch.uint8, device=dev)
    pa.path_attn_fwd_prep(pq, pk, pv, pw, pbeta, fws)
    pa.path_key_prefill(pv, fws, kc, vc)
    torch.cuda.synchronize()
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    p0.record()
    for _ in range(5):
        pa.path_key_prefill(pv, fws, kc, vc)
    p1.record()
    torch.cuda.synchronize()
    prefill_ms = p0.elapsed_time(p1) / 5
    out = {
        "metric": "PaTH decode step: in-place key-cache refresh + attention, tokens/s", "value": B / (wall / args.steps),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16 caches, fp32 arithmetic",
        "data": "synthetic",
        "config": {"workload": f"decode step over a cache of L={L} tokens, B={B} H={H} d={d}"},
        "key_prefill_ms": prefill_ms,
        "roofline": {"kernel": "decode_partial_kernel + decode_combine_kernel", "bound": "hbm", "achieved": bytes_alg / (ms * 1e-3) / 1e9,
                     "peak": 8000.0, "unit": "GB/s", "frac": bytes_alg / (ms * 1e-3) / 1e9 / 8000.0, "traffic": None,
                     "note": "algorithmic bytes = read K + write K + read V = 3*L*d*2 per head; HIP-event time of one step"},
    }
    print(json.dumps(out))


def bench_ring(args, torch, pa, si, dev):
    """One device's share of the sequence-parallel forward (ring of paper Sec. 3.5) at the headline head shape: the
    device holds a segment of L tokens of a longer sequence; timed are its own segment (transforms + sweep) and one
    hop over an earlier segment of the same length (dense: every query attends every key, 4*d flops per pair)."""
    cfg = dict(si.CONFIGS[args.config])
    if args.shape:
        cfg.update(dict(zip(("B", "H", "L", "d"), (int(v) for v in args.shape.split(",")))))
    B, H, L, d = cfg["B"], cfg["H"], cfg["L"], cfg["d"]
    g = torch.Generator(device="cuda").manual_seed(20250516)
    rn = lambda *shape: torch.randn(*shape, device=dev, generator=g)
    segs = []
    for _ in range(2):                              # an earlier segment and the device's own
        q, k, v = (rn(B, H, L, d).to(torch.bfloat16) for _ in range(3))
        w = torch.nn.functional.normalize(rn(B, H, L, d), dim=-1).to(torch.bfloat16)
        beta = (2 * torch.sigmoid(rn(B, H, L))).to(torch.bfloat16)
        segs.append((q, k, v, w, beta))
    ws = [torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, pa.PATH_BF16, False), dtype=torch.uint8, device=dev) for _ in range(2)]
    st = [torch.empty(pa.path_attn_ring_state_bytes(B, H, L, d), dtype=torch.uint8, device=dev) for _ in range(2)]
    scale = d ** -0.5
    o = torch.empty_like(segs[1][0])
    lse = torch.empty((B, H, L), dtype=torch.float32, device=dev)
    pa.path_attn_ring_local(*segs[0], st[0], ws[0], scale=scale)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(marks=None):
        pa.path_attn_ring_local(*segs[1], st[1], ws[1], scale=scale)
        if marks: marks[1].record()
        pa.path_attn_ring_hop(st[1], B, H, L, ws[0], L, d, pa.PATH_BF16, scale=scale)
        if marks: marks[2].record()
        pa.path_attn_ring_finish(st[1], o, lse)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    allm = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        m = [ev() for _ in range(4)]
        m[0].record()
        step(m)
        m[3].record()
        allm.append(m)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    mean = lambda i, j: sum(m[i].elapsed_time(m[j]) for m in allm) / len(allm)
    local_ms, hop_ms, fin_ms = mean(0, 1), mean(1, 2), mean(2, 3)
    hop_fl = 4.0 * d * L * L * B * H
    es = 2
    hop_bytes = (2.0 * L * d + ((L + 1023) // 1024) * d * d) * es * B * H       # what the hop needs from the other device
    out = {
        "metric": "PaTH sequence-parallel forward, one device's share: own segment + one hop, attention-equivalent TFLOP/s",
        "value": (attn_flops(B, H, L, d) + hop_fl) / (wall / args.steps) / 1e12, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16 I/O, fp16+bf16 MFMA operands, fp32 accumulate", "data": "synthetic",
        "config": {"workload": f"segment of L={L} tokens per device, B={B} H={H} d={d}: own segment, one hop over an earlier segment, normalisation"},
        "own_segment_ms": local_ms, "hop_ms": hop_ms, "finish_ms": fin_ms,
        "hop_operand_bytes": hop_bytes,
        "hop_link_ms_at_153GBps": hop_bytes / 153e9 * 1e3,
        "roofline": {"kernel": "attn_fwd2_kernel<hop> (every query of the segment against every key of an earlier segment)", "bound": "mfma",
                     "achieved": hop_fl / (hop_ms * 1e-3) / 1e12, "peak": PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": hop_fl / (hop_ms * 1e-3) / 1e12 / PEAK_TFLOPS, "traffic": None,
                     "note": "4*d flops per (query, key) pair, all pairs; HIP-event time of the hop"},
    }
    print(json.dumps(out))


def bench_fox(args, torch, pa, si, dev):
    """PaTH-FoX (forget gates on the logits, paper Sec. 2.2 extension) forward + backward at the
    chosen configuration's shape; same FLOP convention as the headline line."""
    cfg = dict(si.CONFIGS[args.config])
    if args.shape:
        cfg.update(dict(zip(("B", "H", "L", "d"), (int(v) for v in args.shape.split(",")))))
    B, H, L, d = cfg["B"], cfg["H"], cfg["L"], cfg["d"]
    g = torch.Generator(device="cuda").manual_seed(20250516)
    rn = lambda *shape: torch.randn(*shape, device=dev, generator=g)
    q, k, v, dO = (rn(B, H, L, d).to(torch.bfloat16) for _ in range(4))
    w = torch.nn.functional.normalize(rn(B, H, L, d), dim=-1).to(torch.bfloat16)
    beta = (2 * torch.sigmoid(rn(B, H, L))).to(torch.bfloat16)
    logf = torch.nn.functional.logsigmoid(rn(B, H, L) + 2.0).to(torch.bfloat16)
    ws_f = torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, pa.PATH_BF16, False), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, pa.PATH_BF16, True), dtype=torch.uint8, device=dev)
    scale = d ** -0.5
    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []

    def step(record):
        e0, e1, e2 = (ev(), ev(), ev()) if record else (None,) * 3
        if record: e0.record()
        o, lse = pa.path_attn_train_fwd(q, k, v, w, beta, ws_b, log_f=logf, scale=scale)      # the training pair, with gates
        if record: e1.record()
        pa.path_attn_train_bwd(q, k, v, w, beta, o, lse, dO, ws_b, log_f=logf, scale=scale)
        if record:
            e2.record()
            marks.append((e0, e1, e2))

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    fwd_ms = sum(a.elapsed_time(b) for a, b, _ in marks) / len(marks)
    bwd_ms = sum(b.elapsed_time(c) for _, b, c in marks) / len(marks)
    fl = attn_flops(B, H, L, d)
    value = 3.5 * fl / (ms_step * 1e-3) / 1e12
    print(json.dumps({
        "metric": "PaTH-FoX attn fwd+bwd TFLOP/s (attention-equivalent)", "value": value, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 I/O, fp16+bf16 MFMA operands, fp32 accumulate", "data": "synthetic",
        "config": {"workload": f"PaTH-FoX forward+backward (training pair, shared workspace), B={B} H={H} L={L} d={d} causal"},
        "fwd": {"ms": fwd_ms, "attn_equiv_tflops": fl / (fwd_ms * 1e-3) / 1e12},
        "bwd": {"ms": bwd_ms, "attn_equiv_tflops": 2.5 * fl / (bwd_ms * 1e-3) / 1e12},
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration index (default: headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fwd-only", action="store_true")
    ap.add_argument("--shape", type=str, default=None, help="override B,H,L,d of the chosen configuration (exploration only)")
    ap.add_argument("--workload", choices=["train", "decode", "fox", "ring"], default="train",
                    help="train (default): the headline forward+backward step; decode: one decoding step "
                         "(in-place key-cache refresh + attention) over a cache of L tokens; fox: PaTH-FoX forward+backward; ring: one "
                         "device's share of the sequence-parallel forward (own segment + one hop); each its own JSON line")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (each (batch, head) is independent; "
              "multi-GPU runs would shard heads with no communication). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2505_16381_amd as pa
    from paper_2505_16381_amd import synth_inputs as si

    pa.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.workload == "decode":
        return bench_decode(args, torch, pa, si, dev)
    if args.workload == "ring":
        return bench_ring(args, torch, pa, si, dev)
    if args.workload == "fox":
        return bench_fox(args, torch, pa, si, dev)
    over = {}
    if args.shape:
        over = dict(zip(("B", "H", "L", "d"), (int(v) for v in args.shape.split(","))))
    x, cfg = si.make_config(args.config, with_do=True, **over)
    if over:
        cfg["name"] += "_shape_override"

    B, H, L, d = cfg["B"], cfg["H"], cfg["L"], cfg["d"]
    td = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    dt_code = pa.PATH_BF16 if cfg["dtype"] == "bf16" else pa.PATH_F32
    scale = d ** -0.5
    t = {n: torch.from_numpy(a).to(dev).to(td).contiguous() for n, a in x.items()}
    o = torch.empty_like(t["q"])
    lse = torch.empty((B, H, L), dtype=torch.float32, device=dev)
    ws_f = torch.empty(pa.path_attn_workspace_bytes(B, H, L, d, dt_code, False), dtype=torch.uint8, device=dev)
    bwd_bytes = pa.path_attn_workspace_bytes(B, H, L, d, dt_code, True)
    do_bwd = bwd_bytes > 0 and not args.fwd_only
    ws_b = torch.empty(max(bwd_bytes, 256), dtype=torch.uint8, device=dev) if do_bwd else None

    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []

    # One training step = the training pair: forward and backward share the backward-sized workspace, so the
    # chunk transform runs once per step (forward-only runs use the plain forward and its smaller workspace).
    BWD_STAGES = (("scan", pa.PATH_BWD_STAGE_SCAN), ("keys_near", pa.PATH_BWD_STAGE_KEYS_NEAR), ("keys_far", pa.PATH_BWD_STAGE_KEYS_FAR),
                  ("ddp", pa.PATH_BWD_STAGE_DDP), ("chunk", pa.PATH_BWD_STAGE_CHUNK))
    grads = [torch.empty_like(t["q"]) for _ in range(4)] + [torch.empty_like(t["beta"])] if do_bwd else None

    def step(record):
        es = [ev() for _ in range(3 + len(BWD_STAGES))] if record else None
        if record: es[0].record()
        if do_bwd:
            pa.path_attn_train_fwd_prep(t["q"], t["k"], t["v"], t["w"], t["beta"], ws_b)
        else:
            pa.path_attn_fwd_prep(t["q"], t["k"], t["v"], t["w"], t["beta"], ws_f)
        if record: es[1].record()
        if do_bwd:
            pa.path_attn_train_fwd_sweep(o, lse, scale, ws_b)
        else:
            pa.path_attn_fwd_sweep(o, lse, scale, ws_f)
        if record: es[2].record()
        if do_bwd:
            # the backward of the pair, stage by stage (together exactly path_attn_train_bwd), an event after each
            for i, (_, bit) in enumerate(BWD_STAGES):
                pa.path_attn_train_bwd_stages(bit, t["q"], t["k"], t["v"], t["w"], t["beta"], o, lse, t["dO"], grads, ws_b, scale=scale)
                if record: es[3 + i].record()
        if record:
            marks.append(es)

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_step = wall * 1e3 / args.steps
    mean = lambda i, j: sum(es[i].elapsed_time(es[j]) for es in marks) / len(marks)
    prep_ms, sweep_ms = mean(0, 1), mean(1, 2)
    stage_ms = {name: mean(2 + i, 3 + i) for i, (name, _) in enumerate(BWD_STAGES)} if do_bwd else {}
    bwd_ms = mean(2, 2 + len(BWD_STAGES)) if do_bwd else None

    # for the record, outside the timed region: the stand-alone calls (each runs the transform itself)
    alone = None
    if do_bwd:
        a0, a1, a2 = ev(), ev(), ev()
        for i in range(3):
            if i == 1: a0.record()
            pa.path_attn_fwd(t["q"], t["k"], t["v"], t["w"], t["beta"], scale=scale, o=o, lse=lse, workspace=ws_f)
        a1.record()
        for i in range(2):
            pa.path_attn_bwd(t["q"], t["k"], t["v"], t["w"], t["beta"], o, lse, t["dO"], scale=scale, workspace=ws_b)
        a2.record()
        torch.cuda.synchronize()
        alone = {"path_attn_fwd_ms": a0.elapsed_time(a1) / 2, "path_attn_bwd_ms": a1.elapsed_time(a2) / 2}
    peak_meas = measured_mfma_peak(torch, pa, dev)
    peak_rand = measured_mfma_peak(torch, pa, dev, random_operands=True)

    fl_f = attn_flops(B, H, L, d)
    fl_step = fl_f * (3.5 if do_bwd else 1.0)
    value = fl_step / (ms_step * 1e-3) / 1e12
    fwd_tflops = fl_f / ((prep_ms + sweep_ms) * 1e-3) / 1e12
    sweep_tflops = fl_f / (sweep_ms * 1e-3) / 1e12
    # Roofline of the dominant kernel of the timed step.  The stages that are ONE kernel launch each are the sweep
    # and the two key-side passes; their algorithmic flops: sweep 4d per (query, key <= query) pair; key-side 8d
    # per pair of its range (logit and dP recomputed, dV and dK accumulated: four d-long dot products).
    near_pairs, far_pairs = pair_counts(L)
    single = {"attn_fwd2_kernel (forward sweep" + ("; in the training pair it also writes the backward's query states)" if do_bwd else ")"):
              (sweep_ms, fl_f, "4*d flops per (query, key <= query) pair")}
    if do_bwd:
        single["bwd_keyside2_kernel<FAR> (key-side sums over the queries right of the key's super-block)"] = (
            stage_ms["keys_far"], 8.0 * d * far_pairs * B * H, "8*d flops per (query, key) pair with the key in a super-block left of the query's")
        single["bwd_keyside2_kernel<near> (key-side sums inside the key's super-block; also the near product gradients)"] = (
            stage_ms["keys_near"], 8.0 * d * near_pairs * B * H, "8*d flops per (query, key) pair of one super-block, key chunk left of the query chunk")
    dom = max(single, key=lambda kname: single[kname][0])
    dom_ms, dom_fl, dom_note = single[dom]
    traffic = profiled_traffic(dom.split(" ")[0]) if (args.config == 2 and not args.shape) else None
    out = {
        "metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 I/O, fp16+bf16 MFMA operands, fp32 accumulate" if cfg["dtype"] == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg['name']}: B={B} H={H} L={L} d={d} causal, "
                               f"{'forward+backward' if do_bwd else 'forward only'}",
                   "passes": "fwd+bwd (training pair: path_attn_train_fwd + path_attn_train_bwd in its stages, shared workspace)" if do_bwd else "fwd"},
        "pct_of_mfma_peak": 100.0 * value / PEAK_TFLOPS,
        "mfma_peak_measured_tflops": peak_meas,
        "pct_of_measured_clock_peak": 100.0 * value / peak_meas,
        "mfma_peak_measured_random_operands_tflops": peak_rand,
        "pct_of_measured_random_operand_peak": 100.0 * value / peak_rand,
        "tokens_per_s": B * L / (ms_step * 1e-3),
        "fwd": {"ms": prep_ms + sweep_ms, "prep_ms": prep_ms, "sweep_ms": sweep_ms,
                "attn_equiv_tflops": fwd_tflops, "pct_of_mfma_peak": 100.0 * fwd_tflops / PEAK_TFLOPS,
                "pct_of_measured_clock_peak": 100.0 * fwd_tflops / peak_meas,
                "sweep_pct_of_measured_random_operand_peak": 100.0 * sweep_tflops / peak_rand,
                "sweep_attn_equiv_tflops": sweep_tflops, "sweep_frac_of_mfma_peak": sweep_tflops / PEAK_TFLOPS,
                "path_inclusive_tflops": (fl_f + path_extra_flops(B, H, L, d)) / ((prep_ms + sweep_ms) * 1e-3) / 1e12,
                "path_inclusive_note": "adds the chunk transform, the second-level transform and the query-state updates at the "
                                       "blocking used: chunk 64, one update per key chunk of the own super-block and one per 1024 keys further left"},
        "bwd": ({"ms": bwd_ms, "attn_equiv_tflops": 2.5 * fl_f / (bwd_ms * 1e-3) / 1e12, "stages_ms": stage_ms} if do_bwd else None),
        "standalone_calls": alone,
        "roofline": {"kernel": dom, "bound": "mfma", "achieved": dom_fl / (dom_ms * 1e-3) / 1e12,
                     "peak": PEAK_TFLOPS, "unit": "TFLOP/s", "frac": dom_fl / (dom_ms * 1e-3) / 1e12 / PEAK_TFLOPS,
                     "traffic": (traffic["fetch_bytes"] + traffic["write_bytes"]) if traffic else None,
                     "launch_ms": dom_ms, "flops_per_launch": dom_fl,
                     "note": "the kernel with the longest launch among the single-kernel stages of the timed step; achieved = its "
                             "algorithmic flops (" + dom_note + ") / its HIP-event time inside the timed region; traffic = HBM bytes "
                             "per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE profile of this command "
                             "(profiles/fwd_bwd_headline_L8192_d128_hbm_traffic.txt), null if that profile does not list the kernel"},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(x, cfg, scale)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
