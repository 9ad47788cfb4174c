#!/usr/bin/env python3
"""Throughput of the PyramidInfer prefill layer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 64x2k]

A step is one pass of the whole hot path over one synthetic batch that already sits in
HBM: causal attention -> recent-window scores -> per-sequence top-k -> gather of K and V
-> gather of the hidden rows.  The default workload is the shape throughput is quoted on:
64 prompts of 2048 tokens on a LLaMA-7B-shaped layer (32 heads, d 128, hidden 4096,
window 64, 1905 of 2048 tokens kept), i.e. the first layer of the 32-layer pyramid.

The timed region calls the per-step entry points of the C ABI back to back on one stream
(the same launches pyr_prefill_layer issues) with HIP events between them, so the line
also carries the average duration of every kernel and the roofline fraction of the
dominant one.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published

# HBM bytes per launch at the default workload, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this script, scaled by what the same counters read for the hidden-row gather (a plain copy of known
# size); the counter summary is profiles/layer_step_64x2k_pmc.txt.
MEASURED_TRAFFIC = {
    ("64x2k", "attention"): 6.55e9,       # 5.34 GB read + 1.21 GB written (algorithmic 4.31 GB)
    ("64x2k", "gather"): 5.99e9,          # read = written = algorithmic after calibration
}


def attention_flops(seq_lens, n_q_heads, head_dim):
    """QK^T and PV over the causal lower triangle only: 2*d*S*(S+1) per head and sequence."""
    return float(sum(2 * head_dim * S * (S + 1) * n_q_heads for S in seq_lens))


def score_flops(seq_lens, n_q_heads, head_dim, w):
    return float(sum(2 * head_dim * min(w, S) * S * n_q_heads for S in seq_lens))


def cpu_baseline(wl, n_seqs_sample):
    """The float64 oracle, as it stands, on the first n_seqs_sample sequences of the workload."""
    import numpy as np
    from oracle import pyr_oracle as orc
    from paper_2405_12532_amd import synth
    sub = synth.shrunk(wl, wl.seq_lens[:n_seqs_sample])
    x = synth.make_inputs(sub)
    num, den, floor = sub.schedule_args()
    keep = np.asarray([orc.schedule_next(S, sub.w, num, den, floor) for S in sub.seq_lens], dtype=np.int32)
    f = synth.bf16_bits_to_f64
    q, k, v = f(x["q"]), f(x["k"]), f(x["v"])
    hid = x.get("hidden")
    t0 = time.perf_counter()
    orc.prefill_layer(q, k, v, x["seq_offsets"], sub.w, keep, hidden=hid)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    return {
        "value": sub.total_tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
        "sample": f"{n_seqs_sample} of {wl.n_seqs} sequences ({sub.total_tokens} tokens, all heads, all rows), "
                  f"{dt:.2f} s wall, numpy float64",
        "seconds": dt,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="64x2k", help="64x2k (default), cfg1, cfg2, cfg4, cfg5")
    ap.add_argument("--cpu-seqs", type=int, default=12, help="sequences the CPU oracle is timed on (0: skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
    from paper_2405_12532_amd import binding as pyr, synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    pyr.load()
    wl = synth.workload(args.workload)
    x = synth.make_inputs(wl)
    T, Hq, Hkv, d, D = wl.total_tokens, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.hidden_dim

    q, k, v = (pyr.to_device_bf16(x[n]) for n in ("q", "k", "v"))
    hidden = pyr.to_device_bf16(x["hidden"]) if D > 0 else None
    off_h = torch.from_numpy(np.ascontiguousarray(x["seq_offsets"], dtype=np.int32))
    num, den, floor = wl.schedule_args()       # the retention rule of the workload, evaluated by the library's schedule
    keep_h = torch.tensor([pyr.schedule_next(S, wl.w, num, den, floor) for S in wl.seq_lens], dtype=torch.int32)
    off_d, keep_d = off_h.cuda(), keep_h.cuda()
    n_kept = int(keep_h.sum())
    shape = pyr.make_shape(wl.n_seqs, T, max(wl.seq_lens), Hq, Hkv, d)
    ws_bytes = pyr.workspace_bytes(shape, wl.w)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    lse = ws[: T * Hq * 4].view(torch.float32)
    tile_map = ws[ws_bytes - (((wl.n_seqs + 1) * 4 + 255) // 256 * 256):].view(torch.int32)
    out = torch.empty_like(q)
    scores = torch.empty(T, dtype=torch.float32, device="cuda")
    kept = torch.empty(n_kept, dtype=torch.int32, device="cuda")
    out_off = torch.empty(wl.n_seqs + 1, dtype=torch.int32, device="cuda")
    k_out = torch.empty((n_kept, Hkv, d), dtype=torch.bfloat16, device="cuda")
    v_out = torch.empty_like(k_out)
    hidden_out = torch.empty((n_kept, D), dtype=torch.bfloat16, device="cuda") if D > 0 else None
    kv_row = Hkv * d * 2

    names = ["attention", "score", "select", "gather_kv", "gather_hidden"]

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        pyr.attention(q, k, v, off_d, off_h, shape, 0.0, out, lse, tile_map)
        mark(1)
        pyr.score(q, k, lse, off_d, off_h, shape, wl.w, 0.0, scores)
        mark(2)
        pyr.select(scores, off_d, off_h, keep_d, keep_h, wl.n_seqs, wl.w, kept, out_off)
        mark(3)
        pyr.compact2(k, k_out, v, v_out, kv_row, kept, n_kept)
        mark(4)
        if D > 0:
            pyr.compact(hidden, D * 2, kept, n_kept, hidden_out)
        mark(5)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    kernel_ms = {n: float(np.mean([e[i].elapsed_time(e[i + 1]) for e in evs])) for i, n in enumerate(names)}

    # the same step through the single entry point, as a cross-check of the decomposed timing
    def fused_step():
        pyr.prefill_layer(q, k, v, off_d, off_h, shape, wl.w, 0.0, keep_d, keep_h, out, scores, kept, out_off,
                          k_out, v_out, ws, ws_bytes)
        if D > 0:
            pyr.compact(hidden, D * 2, kept, n_kept, hidden_out)
    fused_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        fused_step()
    torch.cuda.synchronize()
    fused_ms = (time.perf_counter() - t1) * 1e3 / args.steps

    # the optional extras of the step, timed on their own (not part of `value`): recency-weighted
    # score pass and the gather of the kept tokens' position ids
    rw = torch.linspace(0.25, 1.0, wl.w, dtype=torch.float32, device="cuda")
    pos = torch.arange(T, dtype=torch.int32, device="cuda")
    pos_out = torch.empty(n_kept, dtype=torch.int32, device="cuda")
    ex = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for i in range(-1, args.steps):
        e = ex[max(i, 0)]
        e[0].record()
        pyr.score_weighted(q, k, lse, off_d, off_h, shape, wl.w, 0.0, rw, scores)
        e[1].record()
        pyr.gather_positions(pos, kept, n_kept, pos_out)
        e[2].record()
    torch.cuda.synchronize()
    extras_ms = {"score_weighted": float(np.mean([e[0].elapsed_time(e[1]) for e in ex])),
                 "gather_positions": float(np.mean([e[1].elapsed_time(e[2]) for e in ex]))}
    # generation-phase update of a cache of the same size: the window's queries in their own buffer,
    # row statistics + fold + score + select + gathers in one call
    q_win = torch.stack([q[int(off_h[b + 1]) - wl.w:int(off_h[b + 1])] for b in range(wl.n_seqs)]).contiguous() \
        if min(wl.seq_lens) >= wl.w else None
    if q_win is not None:
        dws_bytes = pyr.decode_workspace_bytes(shape, wl.w)
        dws = torch.empty(dws_bytes, dtype=torch.uint8, device="cuda")
        de = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
        for i in range(-1, args.steps):
            e = de[max(i, 0)]
            e[0].record()
            pyr.decode_update(q_win, k, v, off_d, off_h, shape, wl.w, 0.0, keep_d, keep_h, None, pos, scores, kept,
                              out_off, k_out, v_out, pos_out, dws, dws_bytes)
            e[1].record()
        torch.cuda.synchronize()
        extras_ms["decode_update"] = float(np.mean([e[0].elapsed_time(e[1]) for e in de]))

    fl = attention_flops(wl.seq_lens, Hq, d)
    att_tflops = fl / (kernel_ms["attention"] * 1e-3) / 1e12
    compact_bytes = 2.0 * n_kept * (2 * kv_row + D * 2) + 4.0 * n_kept * (2 if D > 0 else 1)
    select_bytes = 4.0 * T + 4.0 * n_kept
    sc_ms = kernel_ms["select"] + kernel_ms["gather_kv"] + kernel_ms["gather_hidden"]
    gather_ms = kernel_ms["gather_kv"] + kernel_ms["gather_hidden"]

    line = {
        "metric": "prefill tokens/s through attention + PvC select + compact (one layer step)",
        "value": T * args.steps / wall, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.n_seqs} seqs x {max(wl.seq_lens)} tokens (T={T}), Hq={Hq}, Hkv={Hkv}, "
                               f"d={d}, hidden={D}, w={wl.w}, kept={n_kept}",
                   "tokens_per_step": T, "kept_rows": n_kept},
        "kernel_ms": kernel_ms, "extras_ms": extras_ms, "ms_per_step_single_entry_point": fused_ms,
        "roofline": {"kernel": "attention", "bound": "mfma", "achieved": att_tflops, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": att_tflops / PEAK_BF16_TFLOPS,
                     "traffic": MEASURED_TRAFFIC.get((wl.name, "attention")),
                     "flops_per_launch": fl},
        "roofline_select_compact": {
            "kernel": "select + gather_kv + gather_hidden", "bound": "hbm",
            "achieved": (compact_bytes + select_bytes) / (sc_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": (compact_bytes + select_bytes) / (sc_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "gather_only_GBs": compact_bytes / (gather_ms * 1e-3) / 1e9,
            "traffic": MEASURED_TRAFFIC.get((wl.name, "gather")), "bytes_per_step": compact_bytes + select_bytes},
        "score_tflops": score_flops(wl.seq_lens, Hq, d, wl.w) / (kernel_ms["score"] * 1e-3) / 1e12,
    }
    if args.cpu_seqs > 0:
        line["cpu_baseline"] = cpu_baseline(wl, min(args.cpu_seqs, wl.n_seqs))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
