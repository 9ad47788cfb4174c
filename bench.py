#!/usr/bin/env python3
"""Throughput of the PyramidInfer prefill layer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 64x2k] [--no-extras]

A step is one pass of the whole hot path over one synthetic batch that already sits in
HBM: causal attention -> recent-window scores -> per-sequence top-k -> gather of K and V
-> gather of the hidden rows.  The default workload is the shape throughput is quoted on:
64 prompts of 2048 tokens on a LLaMA-7B-shaped layer (32 heads, d 128, hidden 4096,
window 64, 1905 of 2048 tokens kept), i.e. the first layer of the 32-layer pyramid.

The timed region calls the per-step entry points of the C ABI back to back on one stream
with HIP events between them, so the line also carries the duration of every kernel
(mean, median, minimum) and the roofline fraction of the dominant one.  Beside `value`
the line reports, as extras that are not part of it: the same step through the merged
entry point (pyr_prefill_layer_fused), a whole 32-layer pyramid pass at batch 64, the
small-batch workloads (separate calls against the merged call), the optional parts of the
step, ceilings measured on this very GPU (MFMA-only loop, device-to-device copy), and the
float64 oracle timed on the machine's host cores.  Prints ONE JSON line.
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
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_64x2k.json")   # HBM bytes per launch from rocprofv3 --pmc runs


def attention_flops(seq_lens, n_q_heads, head_dim):
    """QK^T and PV over the causal lower triangle only: 2*d*S*(S+1) per head and sequence."""
    return float(sum(2 * head_dim * S * (S + 1) * n_q_heads for S in seq_lens))


def score_flops(seq_lens, n_q_heads, head_dim, w):
    return float(sum(2 * head_dim * min(w, S) * S * n_q_heads for S in seq_lens))


def measured_traffic(workload_name):
    """HBM bytes per launch of the attention kernel and of the gathers, measured with hardware counters at the
    commit the file names (see profiles/); None for a workload the file does not cover."""
    try:
        t = json.load(open(TRAFFIC_FILE))
    except OSError:
        return {}
    return t.get("bytes_per_launch", {}) if t.get("workload") == workload_name else {}


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(wl, n_seqs_sample, reps=3):
    """The float64 oracle, as it stands, on the first n_seqs_sample sequences of the workload:
    one warm-up run, then the median of `reps` runs."""
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
    times = []
    for _ in range(reps + 1):
        t0 = time.perf_counter()
        orc.prefill_layer(q, k, v, x["seq_offsets"], sub.w, keep, hidden=hid)
        times.append(time.perf_counter() - t0)
    dt = float(np.median(times[1:]))
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    return {
        "value": sub.total_tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
        "sample": f"{n_seqs_sample} of {wl.n_seqs} sequences ({sub.total_tokens} tokens, all heads, all rows), numpy float64, "
                  f"1 warm-up + median of {reps} runs ({', '.join('%.2f' % t for t in times[1:])} s; warm-up {times[0]:.2f} s)",
        "seconds": dt, "cpu": cpu_model(),
    }


class Step:
    """Device buffers of one workload and the two ways to run its layer step."""

    def __init__(self, pyr, synth, wl, x=None):
        import numpy as np
        import torch
        self.pyr, self.wl, self.torch = pyr, wl, torch
        x = synth.make_inputs(wl) if x is None else x
        T, Hq, Hkv, d, D = wl.total_tokens, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.hidden_dim
        self.T, self.D = T, D
        self.q, self.k, self.v = (pyr.to_device_bf16(x[n]) for n in ("q", "k", "v"))
        self.hidden = pyr.to_device_bf16(x["hidden"]) if D > 0 else None
        self.off_h = torch.from_numpy(np.ascontiguousarray(x["seq_offsets"], dtype=np.int32))
        num, den, floor = wl.schedule_args()       # the retention rule of the workload, evaluated by the library's schedule
        self.keep_h = torch.tensor([pyr.schedule_next(S, wl.w, num, den, floor) for S in wl.seq_lens], dtype=torch.int32)
        self.off_d, self.keep_d = self.off_h.cuda(), self.keep_h.cuda()
        self.n_kept = int(self.keep_h.sum())
        self.shape = pyr.make_shape(wl.n_seqs, T, max(wl.seq_lens), Hq, Hkv, d)
        self.ws_bytes = pyr.workspace_bytes(self.shape, wl.w)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        self.lse = torch.empty((T, Hq), dtype=torch.float32, device="cuda")
        self.tile_map = torch.empty(wl.n_seqs + 1, dtype=torch.int32, device="cuda")
        self.out = torch.empty_like(self.q)
        self.scores = torch.empty(T, dtype=torch.float32, device="cuda")
        self.kept = torch.empty(self.n_kept, dtype=torch.int32, device="cuda")
        self.out_off = torch.empty(wl.n_seqs + 1, dtype=torch.int32, device="cuda")
        self.k_out = torch.empty((self.n_kept, Hkv, d), dtype=torch.bfloat16, device="cuda")
        self.v_out = torch.empty_like(self.k_out)
        self.hidden_out = torch.empty((self.n_kept, D), dtype=torch.bfloat16, device="cuda") if D > 0 else None
        self.kv_row = Hkv * d * 2
        self.names = ["attention", "score", "select", "gather_kv", "gather_hidden"]

    def separate(self, events=None):
        """attention, score, select, K+V gather, hidden gather: the per-step entry points, five launches"""
        pyr, wl = self.pyr, self.wl

        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        pyr.attention(self.q, self.k, self.v, self.off_d, self.off_h, self.shape, 0.0, self.out, self.lse, self.tile_map)
        mark(1)
        pyr.score(self.q, self.k, self.lse, self.off_d, self.off_h, self.shape, wl.w, 0.0, self.scores)
        mark(2)
        pyr.select(self.scores, self.off_d, self.off_h, self.keep_d, self.keep_h, wl.n_seqs, wl.w, self.kept, self.out_off)
        mark(3)
        pyr.compact2(self.k, self.k_out, self.v, self.v_out, self.kv_row, self.kept, self.n_kept)
        mark(4)
        if self.D > 0:
            pyr.compact(self.hidden, self.D * 2, self.kept, self.n_kept, self.hidden_out)
        mark(5)

    def fused(self):
        """the same step through pyr_prefill_layer_fused: four launches"""
        self.pyr.prefill_layer_fused(self.q, self.k, self.v, self.off_d, self.off_h, self.shape, self.wl.w, 0.0, self.keep_d,
                                     self.keep_h, None, self.hidden, self.D * 2, None, self.out, self.scores, self.kept,
                                     self.out_off, self.k_out, self.v_out, self.hidden_out, None, self.ws, self.ws_bytes)

    def static(self):
        """the step through pyr_prefill_layer_static (K and V only, scratch memory inside the library: nothing allocated)"""
        self.pyr.prefill_layer_static(self.q, self.k, self.v, self.off_d, self.off_h, self.shape, self.wl.w, 0.0, self.keep_d,
                                      self.keep_h, self.out, self.scores, self.kept, self.out_off, self.k_out, self.v_out)

    def time_ms(self, fn, steps, warmup=2):
        torch = self.torch
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps


def stats(v):
    import numpy as np
    return {"mean": float(np.mean(v)), "median": float(np.median(v)), "min": float(np.min(v))}


def pyramid_pass(pyr, synth, st, steps):
    """All 32 layers of the pyramid at batch 64 on device-resident inputs: layer l runs the merged step on the first
    64*S_l rows of the layer-0 Q/K/V buffers (same value distribution, surviving length S_l from the library's
    schedule) and on the hidden rows the layer before it gathered, so hidden rows really travel through 32 gathers."""
    import torch
    wl = st.wl
    B, S0 = wl.n_seqs, wl.seq_lens[0]
    num, den, floor = wl.schedule_args()
    lens = [S0]
    for _ in range(32):
        lens.append(pyr.schedule_next(lens[-1], wl.w, num, den, floor))
    layers = []
    for l in range(32):
        S, k_next = lens[l], lens[l + 1]
        off_h = torch.arange(0, B * S + 1, S, dtype=torch.int32)
        keep_h = torch.full((B,), k_next, dtype=torch.int32)
        layers.append(dict(S=S, T=B * S, n_kept=B * k_next, off_h=off_h, off_d=off_h.cuda(), keep_h=keep_h, keep_d=keep_h.cuda(),
                           shape=pyr.make_shape(B, B * S, S, wl.n_q_heads, wl.n_kv_heads, wl.head_dim)))
    hid = [st.hidden, torch.empty_like(st.hidden)]

    def one_pass():
        src = 0
        for L in layers:
            T, nk = L["T"], L["n_kept"]
            pyr.prefill_layer_fused(st.q[:T], st.k[:T], st.v[:T], L["off_d"], L["off_h"], L["shape"], wl.w, 0.0, L["keep_d"],
                                    L["keep_h"], None, hid[src][:T], st.D * 2, None, st.out[:T], st.scores[:T], st.kept[:nk],
                                    st.out_off, st.k_out[:nk], st.v_out[:nk], hid[1 - src][:nk], None, st.ws, st.ws_bytes)
            src = 1 - src
        # (layer 0 reads st.hidden and writes the second buffer, layer 1 reads that and overwrites st.hidden, and so on:
        #  after the first pass the hidden values are no longer the originals, which does not change what is timed)
    ms = st.time_ms(one_pass, steps, warmup=1)
    layer_tokens = B * sum(lens[:32])
    return {"ms_per_pass": ms, "layer_tokens_per_pass": layer_tokens, "prompt_tokens_per_pass": B * S0,
            "layer_tokens_per_s": layer_tokens / (ms * 1e-3), "prompt_tokens_per_s": B * S0 / (ms * 1e-3),
            "lengths": lens, "entry_point": "pyr_prefill_layer_fused, 32 calls"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="64x2k", help="64x2k (default), cfg1, cfg2, cfg4, cfg5, 1x2k, 1x8k")
    ap.add_argument("--cpu-seqs", type=int, default=8, help="sequences the CPU oracle is timed on (0: skip)")
    ap.add_argument("--no-extras", action="store_true", help="only the timed step (for profiler runs)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one device-to-device copy of 1 GiB with torch (a copy of known size that is not this "
                         "library's, to scale the profiler's FETCH_SIZE / WRITE_SIZE counters by)")
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
    st = Step(pyr, synth, wl)
    T, Hq, Hkv, d, D = wl.total_tokens, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.hidden_dim
    n_kept = st.n_kept

    for _ in range(args.warmup):
        st.separate()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        st.separate(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    per_kernel = {n: stats([e[i].elapsed_time(e[i + 1]) for e in evs]) for i, n in enumerate(st.names)}
    kernel_ms = {n: per_kernel[n]["mean"] for n in st.names}

    fused_ms = st.time_ms(st.fused, args.steps)

    fl = attention_flops(wl.seq_lens, Hq, d)
    att_tflops = fl / (kernel_ms["attention"] * 1e-3) / 1e12
    compact_bytes = 2.0 * n_kept * (2 * st.kv_row + D * 2) + 4.0 * n_kept * (2 if D > 0 else 1)
    select_bytes = 4.0 * T + 4.0 * n_kept
    sc_ms = kernel_ms["select"] + kernel_ms["gather_kv"] + kernel_ms["gather_hidden"]
    gather_ms = kernel_ms["gather_kv"] + kernel_ms["gather_hidden"]
    traffic = measured_traffic(wl.name)

    line = {
        "metric": "prefill tokens/s through attention + PvC select + compact (one layer step)",
        "value": T * args.steps / wall, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.n_seqs} seqs x {max(wl.seq_lens)} tokens (T={T}), Hq={Hq}, Hkv={Hkv}, "
                               f"d={d}, hidden={D}, w={wl.w}, kept={n_kept}",
                   "tokens_per_step": T, "kept_rows": n_kept},
        "kernel_ms": kernel_ms, "kernel_ms_median": {n: per_kernel[n]["median"] for n in st.names},
        "kernel_ms_min": {n: per_kernel[n]["min"] for n in st.names},
        "ms_per_step_single_entry_point": fused_ms,
        "roofline": {"kernel": "attention", "bound": "mfma", "achieved": att_tflops, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": att_tflops / PEAK_BF16_TFLOPS,
                     "traffic": traffic.get("attention"), "flops_per_launch": fl,
                     "achieved_at_min_ms": fl / (per_kernel["attention"]["min"] * 1e-3) / 1e12},
        "roofline_select_compact": {
            "kernel": "select + gather_kv + gather_hidden", "bound": "hbm",
            "achieved": (compact_bytes + select_bytes) / (sc_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": (compact_bytes + select_bytes) / (sc_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "gather_only_GBs": compact_bytes / (gather_ms * 1e-3) / 1e9,
            "traffic": traffic.get("gather"), "bytes_per_step": compact_bytes + select_bytes},
        "score_tflops": score_flops(wl.seq_lens, Hq, d, wl.w) / (kernel_ms["score"] * 1e-3) / 1e12,
    }

    if args.calibration_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if not args.no_extras:
        # ---- ceilings of this very GPU, beside the published peaks
        sink = torch.zeros(1, dtype=torch.float32, device="cuda")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        pyr.diag_mfma_only(200, sink)
        torch.cuda.synchronize()
        e0.record()
        mf = pyr.diag_mfma_only(4000, sink)
        e1.record()
        torch.cuda.synchronize()
        mfma_tflops = mf / (e0.elapsed_time(e1) * 1e-3) / 1e12
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 10 * 2.0 * src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del dst
        isink = torch.zeros(1, dtype=torch.int32, device="cuda")
        read_gbs = {}
        for name, k_layout in (("consecutive", 0), ("k_layout", 1)):
            pyr.diag_read_stream(src, src.numel(), k_layout, isink)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(10):
                pyr.diag_read_stream(src, src.numel(), k_layout, isink)
            e1.record()
            torch.cuda.synchronize()
            read_gbs[name] = 10 * src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src
        k_bytes = 2.0 * T * Hkv * d
        line["measured_ceilings"] = {
            "mfma_only_bf16_TFLOPs": mfma_tflops, "published_bf16_TFLOPs": PEAK_BF16_TFLOPS,
            "attention_frac_of_measured_mfma": att_tflops / mfma_tflops,
            "copy_GBs_read_plus_write": copy_gbs, "published_hbm_GBs": PEAK_HBM_GBS,
            "gather_frac_of_measured_copy": compact_bytes / (gather_ms * 1e-3) / 1e9 / copy_gbs,
            "read_only_GBs": read_gbs["consecutive"], "read_only_k_layout_GBs": read_gbs["k_layout"],
            "score_pass_k_read_at_that_rate_ms": k_bytes / read_gbs["k_layout"] / 1e6,
            "score_pass_ms": kernel_ms["score"],
            "how": "MFMA: pyr_diag_mfma_only, 64000 v_mfma_f32_32x32x16_bf16 per wavefront, 2 wavefronts per SIMD on every "
                   "compute unit; copy: torch copy_ of 1 GiB device to device, 10 times; read only: pyr_diag_read_stream over 1 GiB, "
                   "10 times (LDS-direct loads as the score pass issues them for K, consecutive tiles or K's strided "
                   "layout at 32 heads of 128), against which the score pass's own K read is priced"}

        # ---- the optional parts of the step, timed on their own
        rw = torch.linspace(0.25, 1.0, wl.w, dtype=torch.float32, device="cuda")
        pos = torch.arange(T, dtype=torch.int32, device="cuda")
        pos_out = torch.empty(n_kept, dtype=torch.int32, device="cuda")
        extras_ms = {
            "score_weighted": st.time_ms(lambda: pyr.score_weighted(st.q, st.k, st.lse, st.off_d, st.off_h, st.shape, wl.w, 0.0,
                                                                    rw, st.scores), args.steps),
            "gather_positions": st.time_ms(lambda: pyr.gather_positions(pos, st.kept, n_kept, pos_out), args.steps)}
        if min(wl.seq_lens) >= wl.w:
            q_win = torch.stack([st.q[int(st.off_h[b + 1]) - wl.w:int(st.off_h[b + 1])] for b in range(wl.n_seqs)]).contiguous()
            dws_bytes = pyr.decode_workspace_bytes(st.shape, wl.w)
            dws = torch.empty(dws_bytes, dtype=torch.uint8, device="cuda")
            extras_ms["decode_update"] = st.time_ms(
                lambda: pyr.decode_update(q_win, st.k, st.v, st.off_d, st.off_h, st.shape, wl.w, 0.0, st.keep_d, st.keep_h, None,
                                          pos, st.scores, st.kept, st.out_off, st.k_out, st.v_out, pos_out, dws, dws_bytes),
                args.steps)
            del dws, q_win
        line["extras_ms"] = extras_ms

        # ---- the whole 32-layer pyramid at batch 64 (the default workload is its first layer)
        if wl.name == "64x2k":
            line["pyramid_32_layers"] = pyramid_pass(pyr, synth, st, max(2, args.steps // 5))

        # ---- small batch (Appendix A.1: where the selection overhead shows): separate calls against the merged call
        small = {}
        for name in ("cfg1", "1x2k", "1x8k"):
            s2 = Step(pyr, synth, synth.workload(name))
            evs2 = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(50)]
            for _ in range(5):
                s2.separate()
            torch.cuda.synchronize()
            for e in evs2:
                s2.separate(e)
            torch.cuda.synchronize()
            km = {n: float(np.median([e[i].elapsed_time(e[i + 1]) for e in evs2])) for i, n in enumerate(s2.names)}
            small[name] = {"kernel_ms_median_separate_calls": km, "select_over_attention": km["select"] / km["attention"],
                           "ms_per_step_separate_calls": s2.time_ms(s2.separate, 200, warmup=10),
                           "ms_per_step_fused_call": s2.time_ms(s2.fused, 200, warmup=10)}
            # the launch-bound end of the range once more without the host in the loop: the step that allocates nothing
            # (K and V only), eagerly and replayed from a HIP graph
            small[name]["ms_per_step_static_call_kv_only"] = s2.time_ms(s2.static, 200, warmup=10)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                s2.static()
            small[name]["ms_per_step_static_call_graph_replay"] = s2.time_ms(graph.replay, 200, warmup=10)
            del graph, s2
        line["small_batch"] = small

    if args.cpu_seqs > 0:
        line["cpu_baseline"] = cpu_baseline(wl, min(args.cpu_seqs, wl.n_seqs))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
