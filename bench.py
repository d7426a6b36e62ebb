#!/usr/bin/env python3
"""Benchmark of the PaTH attention hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input
at the headline shape B=4, H=16, L=8192, d=128 (bf16 I/O): forward (chunk
transform + sweep) and, once the library provides it at this shape, backward.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

FLOP convention: attention-equivalent 4*d*L(L+1)/2*B*H for the forward and
2.5x that for the backward (FlashAttention convention, masked work not
counted); the PaTH-inclusive count (query-state updates, chunk transform) is
reported next to it.
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
SWEEP_HBM_BYTES = 4.69e9  # measured HBM traffic of one launch of the pair's sweep at the headline shape (see profiles/)
CHUNK = 64


def attn_flops(B, H, L, d):
    return 4.0 * d * (L * (L + 1) / 2.0) * B * H


def path_extra_flops(B, H, L, d):
    """PaTH-only work at the blocking used (chunk 64, one query-state update per key chunk)."""
    nc = -(-L // CHUNK)
    prep = (14.0 * CHUNK * CHUNK * d + 2.0 * CHUNK * d * d + 4.0 * CHUNK ** 3 + CHUNK ** 3 / 3.0) * nc
    # one (32 queries x d x d) update per (query block, key chunk strictly left of it, except chunk 0)
    upd = 0.0
    for c in range(nc):
        upd += 2.0 * CHUNK * d * d * max(0, c - 1)
    return (prep + upd) * B * H


def cpu_baseline(x, cfg, scale, n_rows=6144):
    """The fp64 oracle, as it stands, on a bounded row sample of the same workload."""
    import numpy as np
    from oracle import path_oracle
    rng = np.random.default_rng(0)
    L, d = cfg["L"], cfg["d"]
    n_heads = cfg["B"] * cfg["H"]
    rows = np.unique(rng.integers(0, L, n_rows))
    sub = {n: x[n].reshape((1, n_heads) + x[n].shape[2:]) for n in ("q", "k", "v", "w", "beta")}
    path_oracle.fwd(sub["q"], sub["k"], sub["v"], sub["w"], sub["beta"], scale, rows=rows[:2])  # warm
    t0 = time.perf_counter()
    path_oracle.fwd(sub["q"], sub["k"], sub["v"], sub["w"], sub["beta"], scale, rows=rows)
    dt = time.perf_counter() - t0
    pairs = float((rows + 1).sum()) * n_heads
    return {
        "value": pairs * 4.0 * d / dt / 1e12, "unit": "TFLOP/s", "cores": path_oracle.num_threads(),
        "kind": "oracle", "seconds": dt,
        "sample": f"forward only, all {n_heads} heads x {len(rows)} random query rows of the headline shape "
                  f"({pairs:.3g} query-key pairs), attention-equivalent flops 4d per pair",
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
    ap.add_argument("--workload", choices=["train", "decode", "fox"], default="train",
                    help="train (default): the headline forward+backward step; decode: one decoding step "
                         "(in-place key-cache refresh + attention) over a cache of L tokens, its own JSON line")
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
    def step(record):
        e0, e1, e2, e3 = (ev(), ev(), ev(), ev()) if record else (None,) * 4
        if record: e0.record()
        if do_bwd:
            pa.path_attn_train_fwd_prep(t["q"], t["k"], t["v"], t["w"], t["beta"], ws_b)
        else:
            pa.path_attn_fwd_prep(t["q"], t["k"], t["v"], t["w"], t["beta"], ws_f)
        if record: e1.record()
        if do_bwd:
            pa.path_attn_train_fwd_sweep(o, lse, scale, ws_b)
        else:
            pa.path_attn_fwd_sweep(o, lse, scale, ws_f)
        if record: e2.record()
        if do_bwd:
            pa.path_attn_train_bwd(t["q"], t["k"], t["v"], t["w"], t["beta"], o, lse, t["dO"], ws_b, scale=scale)
        if record:
            e3.record()
            marks.append((e0, e1, e2, e3))

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_step = wall * 1e3 / args.steps
    prep_ms = sum(a.elapsed_time(b) for a, b, _, _ in marks) / len(marks)
    sweep_ms = sum(b.elapsed_time(c) for _, b, c, _ in marks) / len(marks)
    bwd_ms = sum(c.elapsed_time(e) for _, _, c, e in marks) / len(marks) if do_bwd else None

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

    fl_f = attn_flops(B, H, L, d)
    fl_step = fl_f * (3.5 if do_bwd else 1.0)
    value = fl_step / (ms_step * 1e-3) / 1e12
    fwd_tflops = fl_f / ((prep_ms + sweep_ms) * 1e-3) / 1e12
    sweep_tflops = fl_f / (sweep_ms * 1e-3) / 1e12
    out = {
        "metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 I/O, fp16+bf16 MFMA operands, fp32 accumulate" if cfg["dtype"] == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg['name']}: B={B} H={H} L={L} d={d} causal, "
                               f"{'forward+backward' if do_bwd else 'forward only (no backward at this shape yet)'}",
                   "passes": "fwd+bwd (training pair: path_attn_train_fwd + path_attn_train_bwd, shared workspace)" if do_bwd else "fwd"},
        "pct_of_mfma_peak": 100.0 * value / PEAK_TFLOPS,
        "tokens_per_s": B * L / (ms_step * 1e-3),
        "fwd": {"ms": prep_ms + sweep_ms, "prep_ms": prep_ms, "sweep_ms": sweep_ms,
                "attn_equiv_tflops": fwd_tflops, "pct_of_mfma_peak": 100.0 * fwd_tflops / PEAK_TFLOPS,
                "path_inclusive_tflops": (fl_f + path_extra_flops(B, H, L, d)) / ((prep_ms + sweep_ms) * 1e-3) / 1e12},
        "bwd": ({"ms": bwd_ms, "attn_equiv_tflops": 2.5 * fl_f / (bwd_ms * 1e-3) / 1e12} if do_bwd else None),
        "standalone_calls": alone,
        "roofline": {"kernel": "attn_fwd2_kernel (sweep; in the training pair it also writes the backward's query states)"
                               if do_bwd else "attn_fwd2_kernel (sweep)", "bound": "mfma", "achieved": sweep_tflops,
                     "peak": PEAK_TFLOPS, "unit": "TFLOP/s", "frac": sweep_tflops / PEAK_TFLOPS,
                     "traffic": SWEEP_HBM_BYTES if (args.config == 2 and not args.shape) else None,
                     "note": "achieved = attention-equivalent flops of the launch / HIP-event time of the sweep kernel; "
                             "traffic = HBM bytes per launch from rocprofv3 FETCH_SIZE/WRITE_SIZE "
                             "(profiles/fwd_bwd_headline_L8192_d128_hbm_traffic.txt): 2.57e9 in + 2.12e9 out (the fetched bytes vary between runs, 2.4-2.6e9), of which "
                             "1.96e9 are the query states kept for the backward; the forward alone needs 1.2e9 "
                             "(the stand-alone forward's sweep, without that output: 1.4-1.5 ms, frac 0.29-0.31, same profile)"},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(x, cfg, scale)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
