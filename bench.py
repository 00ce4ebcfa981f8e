"""Benchmark of the query-aware decode hot path on one MI355X.

A step = one decode step of one attention layer over one synthetic batch: one
new token per sequence is appended (K/V slot write + incremental min/max), then
all pages are scored, the top-K selected and sparse attention run over them.  By
default that is ONE launch of ts_append_and_decode; --step separate times the
two-call form (ts_append_token_meta, then ts_query_aware_decode) instead.  Consecutive steps rotate over several
independent layers (own KV pool, metadata and query), as a model's decode step
does, so each step finds its metadata and KV pages in HBM rather than in the
256 MB memory-side cache left warm by the previous step.

Prints ONE JSON line: metric, value (us/step), roofline of the dominant kernel, CPU-oracle baseline.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "query-aware decode attention µs/step and effective HBM GB/s (% of peak)"
HBM_PEAK = 8.0e12   # MI355X published HBM3E bandwidth, B/s

# HBM bytes per fused launch from rocprofv3 counters (FETCH_SIZE and WRITE_SIZE, one run each,
# eager launches over cold data, each scaled by what the same counter reads for a plain
# 256 MiB copy: x1.9997 and x1.0000).  Counters cannot be read from inside this process, so the
# figures are carried here from the committed summaries under profiles/.
MEASURED_TRAFFIC_BYTES = {
    "tinyllama": int((26954.1 * 1.9997 + 1818.1) * 1024),
    "longctx": int((19619.5 * 1.9997 + 1892.6) * 1024),
    "gpt2_345m": int((25656.6 * 1.9997 + 1136.1) * 1024),
    "tiny": int((371.0 * 1.9997 + 9.6) * 1024),
    "ragged": int((2383591.8 * 1.9997 + 1104.1) * 1024),
}

WORKLOAD_DESC = {
    "tiny": "configs[0] tiny single-head: B1 1q/1kv d64 L4096 S16 K32",
    "gpt2_345m": "configs[1] GPT2-345M-shaped MHA: B8 16q/16kv d64 L8192 S16 K64, permuted pool",
    "tinyllama": "configs[2] TinyLLaMA-shaped GQA: B16 32q/4kv d64 L16384 S16 K128, outlier channels",
    "longctx": "configs[3] long-context GQA: B4 32q/4kv d64 L131072 S32 K128, random-walk keys",
    "ragged": "configs[4] ragged serving batch: 64 seqs L~U[1024,32768] 32q/32kv d128 S16 budget 25%",
}


class Layer:
    """One attention layer's device state + pre-marshalled C arguments."""

    def __init__(self, ts, wl, spec, seed, dev, n_q):
        import torch
        self.w = w = wl.make_workload(spec, dev, seed=seed, n_q=n_q, n_new=1, poison=0.0)
        self.page_min = torch.zeros((spec.B, spec.Hkv, w.P_max, spec.d),
                                    dtype=torch.float16 if spec.kv == "fp16" else torch.bfloat16,
                                    device=dev)
        self.page_max = torch.zeros_like(self.page_min)
        self.seq_lens = w.seq_lens.clone()
        self.layout = ts.make_layout(spec.B, spec.Hq, spec.Hkv, spec.d, spec.S, w.P_max, w.k_pool,
                                     w.v_pool, w.block_table, self.seq_lens, self.page_min,
                                     self.page_max, k_scale=w.k_scale, v_scale=w.v_scale)
        self.out = torch.zeros((spec.B, spec.Hq, spec.d), dtype=torch.float32, device=dev)
        self.ws = ts.new_workspace(self.layout, w.K_max, dev)
        ts.build_page_meta(self.layout)
        lib = ts.lib()
        vp = ctypes.c_void_p
        lay = ctypes.byref(self.layout)
        scale = 1.0 / math.sqrt(spec.d)
        tps = None if w.topk_per_seq is None else vp(w.topk_per_seq.data_ptr())
        self._append = (lib.ts_append_token_meta, (lay, vp(w.k_new[0].data_ptr()),
                                                   vp(w.v_new[0].data_ptr()), 1))
        self._both = [(lib.ts_append_and_decode,
                       (lay, vp(w.k_new[0].data_ptr()), vp(w.v_new[0].data_ptr()),
                        vp(w.q[i].data_ptr()), w.topk, tps, w.K_max, scale,
                        vp(self.out.data_ptr()), None, None, None, vp(self.ws.data_ptr()),
                        self.ws.numel())) for i in range(n_q)]
        self._fused = [(lib.ts_query_aware_decode,
                        (lay, vp(w.q[i].data_ptr()), w.topk, tps, w.K_max, scale,
                         vp(self.out.data_ptr()), None, None, None, vp(self.ws.data_ptr()),
                         self.ws.numel())) for i in range(n_q)]

    def append(self, stream):
        f, a = self._append
        st = f(*a, stream)
        if st != 0:
            raise RuntimeError(f"ts_append_token_meta -> {st}")

    def fused(self, stream, qi=0):
        f, a = self._fused[qi % len(self._fused)]
        st = f(*a, stream)
        if st != 0:
            raise RuntimeError(f"ts_query_aware_decode -> {st}")

    def both(self, stream, qi=0):
        f, a = self._both[qi % len(self._both)]
        st = f(*a, stream)
        if st != 0:
            raise RuntimeError(f"ts_append_and_decode -> {st}")

    def reset_lengths(self):
        self.seq_lens.copy_(self.w.seq_lens)


def time_region(torch, fn, n):
    """Host wall time and HIP-event time of n calls of fn(i), synchronised on both sides."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(n):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0), e0.elapsed_time(e1) * 1e-3


def capture_graph(torch, layers, body, per_graph):
    """Capture per_graph calls of body(layer, stream), rotating over the layers (kernel
    nodes only, no memset nodes)."""
    n_layers = len(layers)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gstream = ctypes.c_void_p(side.cuda_stream)
        for i in range(n_layers):       # warm the kernels on the capture stream
            body(layers[i], gstream)
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for i in range(per_graph):
                body(layers[i % n_layers], gstream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    return g


def cpu_baseline(spec, layer, wl, budget_s=20.0):
    """The CPU oracle, as it stands, on the same step (score + select + attend over
    the layer's metadata and KV) for a bounded number of sequences / repetitions."""
    import numpy as np
    from oracle import ts_oracle as oracle
    w = layer.w
    lens_all = layer.seq_lens.cpu()
    # bound host memory / time: at most ~1 GiB of logical KV per tensor
    per_seq = spec.Hkv * int(lens_all.max()) * spec.d * 2
    n_seq = max(1, min(spec.B, (1 << 30) // max(per_seq, 1)))
    seqs = list(range(n_seq))
    L = lens_all[:n_seq].numpy().astype(np.int32)
    qb = wl.bits(w.q[0][:n_seq])
    pmin, pmax = wl.bits(layer.page_min[:n_seq]), wl.bits(layer.page_max[:n_seq])
    tps = None if w.topk_per_seq is None else w.topk_per_seq[:n_seq].cpu().numpy()
    scale = 1.0 / math.sqrt(spec.d)
    if spec.kv == "int8":
        kv = [t.cpu().numpy() for t in wl.logical_kv_i8(w, seqs=seqs, seq_lens=lens_all)]

        def step():
            oracle.query_aware_decode_i8(qb, *kv, pmin, pmax, L, spec.S, w.topk, w.K_max, scale,
                                         topk_per_seq=tps)
    else:
        K, V = wl.logical_kv(w, seqs=seqs, seq_lens=lens_all)
        Kb, Vb = wl.bits(K), wl.bits(V)

        def step():
            with oracle.element_format(spec.kv):
                oracle.query_aware_decode(qb, Kb, Vb, pmin, pmax, L, spec.S, w.topk, w.K_max, scale,
                                          topk_per_seq=tps)
    times = []
    t_start = time.perf_counter()
    while True:
        t0 = time.perf_counter()
        step()
        times.append(time.perf_counter() - t0)
        if len(times) >= 3 and time.perf_counter() - t_start > 0.5 * budget_s:
            break
        if time.perf_counter() - t_start > budget_s:
            break
    med = sorted(times)[len(times) // 2]
    us_step = med * 1e6 * spec.B / n_seq
    cores = oracle.max_threads()
    # the same on one thread (a few runs, at most a fifth of the budget again)
    oracle.set_num_threads(1)
    single, t_start = [], time.perf_counter()
    while len(single) < 3 and (not single or time.perf_counter() - t_start < 0.2 * budget_s):
        t0 = time.perf_counter()
        step()
        single.append(time.perf_counter() - t0)
    oracle.set_num_threads(0)
    return {"value": round(us_step, 1), "unit": "us/step", "cores": cores,
            "single_thread_value": round(sorted(single)[len(single) // 2] * 1e6 * spec.B / n_seq, 1),
            "kind": "oracle",
            "sample": f"{n_seq} of {spec.B} sequences (all KV heads), score+select+attend (the append "
                      f"of one token, microseconds on a CPU, is not in the timed loop), "
                      f"median of {len(times)} runs scaled by {spec.B}/{n_seq}; attention loop "
                      f"OpenMP over query heads, scoring and selection single-threaded"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="tinyllama", choices=list(WORKLOAD_DESC))
    ap.add_argument("--layers", type=int, default=0, help="independent layers rotated (0 = auto)")
    ap.add_argument("--launch", default="graph", choices=["graph", "eager"])
    ap.add_argument("--step", default="one_launch", choices=["one_launch", "separate"],
                    help="one_launch: ts_append_and_decode; separate: ts_append_token_meta + "
                         "ts_query_aware_decode")
    ap.add_argument("--kv-format", default="bf16", choices=["bf16", "fp16", "int8"],
                    help="format of the cache (fp16: every 16-bit tensor IEEE half; int8: codes + "
                         "one fp32 scale per token and head)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true",
                    help="skip timing the dense (whole-cache) attention beside the step")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the per-launch percentiles, the warm figure and the plain copy")
    ap.add_argument("--cpu-budget", type=float, default=20.0)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (a known size against which "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_12211_amd import tinyserve as ts
    from paper_2509_12211_amd import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    spec = wl.scaled(wl.SPECS[args.workload], kv=args.kv_format)
    lens_nom = torch.full((spec.B,), spec.L, dtype=torch.int32)
    nominal = wl.algorithmic_bytes(spec, lens_nom) if not spec.L_min else None

    # enough layers that one rotation touches >= 768 MiB (3x the memory-side cache)
    step_bytes_guess = (nominal["total"] if nominal else 5 << 30)
    n_layers = args.layers or int(min(16, max(1, math.ceil((768 << 20) / step_bytes_guess))))
    steps, warmup = args.steps, args.warmup
    appends_per_layer = (steps + warmup) // n_layers + 2
    spec = wl.scaled(spec, headroom=max(16, appends_per_layer * 3 + 8))
    n_q = 4
    layers = [Layer(ts, wl, spec, 1000 + 17 * i, dev, n_q) for i in range(n_layers)]
    torch.cuda.synchronize()
    by = wl.algorithmic_bytes(spec, layers[0].seq_lens, layers[0].w.topk_per_seq)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if args.calibration_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    one_launch = args.step == "one_launch"
    # large batches: ts_append_and_decode enqueues the append as a kernel of its own; the
    # dominant kernel timed alone for the roofline is then the plain fused one
    single_kernel = one_launch and ts.append_and_decode_launches(layers[0].layout,
                                                                 layers[0].w.K_max) == 1

    def step(i):
        ly = layers[i % n_layers]
        if one_launch:
            ly.both(stream, i // n_layers)
        else:
            ly.append(stream)
            ly.fused(stream, i // n_layers)

    def fused_only(i):   # the dominant kernel alone: with a single-kernel step it IS the step
        if single_kernel:
            layers[i % n_layers].both(stream, i // n_layers)
        else:
            layers[i % n_layers].fused(stream, i // n_layers)

    launch = args.launch

    # steps per captured graph: whole rotations over the layers, at least 8 steps (a
    # graph of one or two kernels would be timed by its own launch overhead)
    per_graph = n_layers * max(1, -(-8 // n_layers))

    def capture(body):
        return capture_graph(torch, layers, body, per_graph)

    def body_step(ly, st):
        if one_launch:
            ly.both(st, 0)
        else:
            ly.append(st)
            ly.fused(st, 0)

    def body_fused(ly, st):
        if single_kernel:
            ly.both(st, 0)
        else:
            ly.fused(st, 0)

    graph = graph_fused = None
    if launch == "graph":
        try:
            graph = capture(body_step)
            graph_fused = capture(body_fused)
        except Exception as e:   # fall back to eager launches, and say so
            print(f"bench.py: graph capture failed ({e}); using eager launches", file=sys.stderr)
            graph = graph_fused = None
            launch = "eager"

    # ---- timed region: exactly `steps` steps -------------------------------------
    if graph is not None:
        reps_w = max(1, warmup // per_graph)
        reps = max(1, steps // per_graph)
        steps, warmup = reps * per_graph, reps_w * per_graph
        for _ in range(reps_w):
            graph.replay()
        wall, ev = time_region(torch, lambda i: graph.replay(), reps)
    else:
        for i in range(warmup):
            step(i)
        wall, ev = time_region(torch, step, steps)
    us_step = wall / steps * 1e6
    for ly in layers:
        assert ts.workspace_status(ly.ws) == 0, "a bounded wait expired inside the fused kernel"

    # ---- roofline leg: the fused kernel alone, HIP events on its stream -----------
    n_roof = steps
    if graph_fused is not None:
        graph_fused.replay()
        _, ev_fused = time_region(torch, lambda i: graph_fused.replay(), n_roof // per_graph)
    else:
        for i in range(min(warmup, 2 * n_layers)):
            fused_only(i)
        _, ev_fused = time_region(torch, fused_only, n_roof)
    fused_us = ev_fused / n_roof * 1e6
    achieved = by["total"] / (fused_us * 1e-6) / 1e9

    # ---- distribution of single launches, the same step on data left warm, and a plain
    # ---- copy of the same number of bytes ------------------------------------------
    extra = {}
    if not args.no_extras:
        # (1) every launch bracketed by its own pair of events (eager, cold rotation); the
        # pair adds its own few microseconds, so these sit above the graph figure
        n_one = min(steps, 200)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(n_one)]
        for i in range(2 * n_layers):
            fused_only(i)
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(evs):
            a.record()
            fused_only(i)
            b.record()
        torch.cuda.synchronize()
        one = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
        extra["single_launch_event_us"] = {
            "p10": round(one[n_one // 10], 2), "p50": round(one[n_one // 2], 2),
            "p90": round(one[(9 * n_one) // 10], 2), "launches": n_one,
            "note": "dominant kernel, eager, one event pair per launch (adds its own overhead)"}
        # (2) warm: the same layer again and again, so metadata and KV pages are found in
        # the caches left by the previous launch
        n_warm = 64
        for i in range(8):
            (layers[0].both if single_kernel else layers[0].fused)(stream, 0)
        _, ev_w = time_region(
            torch, lambda i: (layers[0].both if single_kernel else layers[0].fused)(stream, 0),
            n_warm)
        extra["warm_us_per_launch"] = round(ev_w / n_warm * 1e6, 2)
        # (3) a plain device copy that moves as many bytes as the step's algorithmic bytes
        # (half read, half written), rotating over buffers so that it is cold as well
        half = max(by["total"] // 2 // 4, 1)
        n_buf = max(2, min(32, (1 << 30) // max(by["total"], 1)))
        srcs = [torch.ones(half, dtype=torch.float32, device=dev) for _ in range(n_buf)]
        dsts = [torch.empty_like(t) for t in srcs]
        for i in range(n_buf):
            dsts[i].copy_(srcs[i])
        g_copy = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g_copy, stream=side):
                for i in range(n_buf):
                    dsts[i].copy_(srcs[i])
        torch.cuda.current_stream().wait_stream(side)
        g_copy.replay()
        reps_c = max(2, 256 // n_buf)
        _, ev_c = time_region(torch, lambda i: g_copy.replay(), reps_c)
        copy_us = ev_c / (reps_c * n_buf) * 1e6
        extra["copy_same_bytes"] = {
            "us": round(copy_us, 2), "GBps": round(2 * half * 4 / (copy_us * 1e-6) / 1e9, 1),
            "kernel_pct_of_copy_bandwidth": round(100.0 * copy_us / fused_us, 1),
            "note": "torch device-to-device copy kernel, bytes read + written = algorithmic bytes "
                    "of the step, cold buffers, HIP graph"}
        del srcs, dsts, g_copy

    # ---- other entry points, for the record ---------------------------------------
    _, ev_b = time_region(torch, lambda i: ts.build_page_meta(layers[i % n_layers].layout),
                          2 * n_layers)
    build_us = ev_b / (2 * n_layers) * 1e6
    for ly in layers:
        ly.reset_lengths()
        ts.build_page_meta(ly.layout)
    _, ev_a = time_region(torch, lambda i: layers[i % n_layers].append(stream), 2 * n_layers)
    append_us = ev_a / (2 * n_layers) * 1e6

    # ---- the comparison the paper reports: attention over the whole cache ---------
    dense = None
    if not args.no_dense:
        dws = [ts.new_dense_workspace(ly.layout, dev) for ly in layers]
        scale = 1.0 / math.sqrt(spec.d)

        def dense_call(i):
            ly = layers[i % n_layers]
            ts.dense_decode_attention(ly.layout, ly.w.q[0], scale, ly.out, dws[i % n_layers])

        for i in range(n_layers):
            dense_call(i)
        n_dense = max(2 * n_layers, 4)
        _, ev_d = time_region(torch, dense_call, n_dense)
        dense_us = ev_d / n_dense * 1e6
        dense = {"kernel": "ts_dense_decode_attention (every cached token, same pool and block table)",
                 "us_per_launch": round(dense_us, 2),
                 "GBps": round(by["dense"] / (dense_us * 1e-6) / 1e9, 1),
                 "speedup_of_step_over_dense": round(dense_us / us_step, 2),
                 "bytes_fraction_of_dense": round(by["total"] / by["dense"], 4)}

    result = {
        "metric": METRIC,
        "value": round(us_step, 3),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(us_step * 1e-3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"bf16": "bf16", "fp16": "fp16",
                  "int8": "int8 KV expanded to bf16 for the MFMA"}[args.kv_format],
        "data": "synthetic",
        "effective_GBps": round(by["total"] / (us_step * 1e-6) / 1e9, 1),
        "pct_of_hbm_peak": round(100.0 * by["total"] / (us_step * 1e-6) / HBM_PEAK, 2),
        "config": {
            "workload": WORKLOAD_DESC[args.workload] + {"bf16": "", "fp16": ", FP16 tensors",
                                                          "int8": ", INT8 KV pool"}[args.kv_format],
            "step": ("ts_append_and_decode (append + score + select + attend in one launch), one layer"
                     if single_kernel else
                     "ts_append_and_decode (large batch: append kernel + fused decode kernel), one layer"
                     if one_launch else
                     "ts_append_token_meta + fused ts_query_aware_decode, one layer"),
            "layers_rotated": n_layers,
            "launch": launch,
            "softmax_scale": "1/sqrt(d)",
            "bytes_per_step": by,
            "device_event_us_per_step": round(ev / steps * 1e6, 3),
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "query_aware_decode_kernel",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK / 1e9,
            "unit": "GB/s",
            "frac": round(achieved * 1e9 / HBM_PEAK, 4),
            "traffic": (MEASURED_TRAFFIC_BYTES.get(args.workload)
                        if args.kv_format == "bf16" else None),
            "us_per_launch": round(fused_us, 3),
            "launches": n_roof,
        },
        "other_kernels_us": {"ts_build_page_meta": round(build_us, 2),
                             "ts_append_token_meta": round(append_us, 2)},
    }
    result.update(extra)
    if dense is not None:
        result["dense_baseline"] = dense
    if not args.no_cpu_baseline:
        layers[0].reset_lengths()
        ts.build_page_meta(layers[0].layout)
        torch.cuda.synchronize()
        result["cpu_baseline"] = cpu_baseline(spec, layers[0], wl, args.cpu_budget)
    print(json.dumps(result, ensure_ascii=False), flush=True)


if __name__ == "__main__":
    main()
