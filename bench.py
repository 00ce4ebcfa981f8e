"""Benchmark of the query-aware decode hot path on one MI355X.

A step = one decode step of one attention layer over one synthetic batch: one
new token per sequence is appended (K/V slot write + incremental min/max), then
all pages are scored, the top-K selected and sparse attention run over them.  By
default that is ONE launch of ts_append_and_decode; --step separate times the
two-call form (ts_append_token_meta, then ts_query_aware_decode) instead.
Consecutive steps rotate over several independent layers (own KV pool, metadata
and queries), as a model's decode step does, so each step finds its metadata and
KV pages in HBM rather than in the 256 MB memory-side cache left warm by the
previous step, and every pass over the layers uses the next of 16 queries.

Prints ONE JSON line: metric, value (us/step) and roofline of the headline
workload (--workload, default the TinyLLaMA-shaped one), the CPU-oracle baseline,
and a compact `all_workloads` map with the same measurement of the other four.

--phase-marks prints, instead, where the microseconds of the fused kernel go
(timestamps taken inside the kernel by the tuning build of the library).
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
N_QUERIES = 16      # queries a layer cycles through
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")

WORKLOAD_DESC = {
    "tiny": "configs[0] tiny single-head: B1 1q/1kv d64 L4096 S16 K32",
    "gpt2_345m": "configs[1] GPT2-345M-shaped MHA: B8 16q/16kv d64 L8192 S16 K64, permuted pool",
    "tinyllama": "configs[2] TinyLLaMA-shaped GQA: B16 32q/4kv d64 L16384 S16 K128, outlier channels",
    "longctx": "configs[3] long-context GQA: B4 32q/4kv d64 L131072 S32 K128, random-walk keys",
    "ragged": "configs[4] ragged serving batch: 64 seqs L~U[1024,32768] 32q/32kv d128 S16 budget 25%",
}


def measured_traffic(workload, kv_format):
    """HBM bytes per fused launch from rocprofv3 counters (FETCH_SIZE and WRITE_SIZE, one run
    each, scaled by what the same counter reads for a plain copy of known size).  Counters
    cannot be read from inside this process: the figures come from a tracked file that names
    the commit they were taken at, so a stale figure shows in the JSON line."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
        row = t["workloads"][workload]
        if kv_format != "bf16":
            return None, None
        b = (row["fetch_kib"] * t["fetch_scale"] + row["write_kib"] * t["write_scale"]) * 1024
        return int(b), t.get("measured_at_commit")
    except (OSError, KeyError, ValueError):
        return None, None


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
        self._ts = ts

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

    def rewind(self):
        """Back to the generated lengths (the appended tokens are written again by the next
        leg) with the metadata rebuilt from the pool."""
        self.seq_lens.copy_(self.w.seq_lens)
        self._ts.build_page_meta(self.layout)


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
    """Capture per_graph calls of body(layer, stream, query index): step i goes to layer
    i mod n_layers with query i div n_layers (kernel nodes only, no memset nodes)."""
    n_layers = len(layers)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gstream = ctypes.c_void_p(side.cuda_stream)
        for i in range(n_layers):       # warm the kernels on the capture stream
            body(layers[i], gstream, 0)
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for i in range(per_graph):
                body(layers[i % n_layers], gstream, i // n_layers)
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
    # scaled to the whole batch by the tokens the sample holds (the sequences differ in
    # length in the ragged batch, and the oracle's work goes with the tokens)
    tok_all, tok_sample = int(lens_all.sum()), int(lens_all[:n_seq].sum())
    up = tok_all / max(tok_sample, 1)
    us_step = med * 1e6 * up
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
            "single_thread_value": round(sorted(single)[len(single) // 2] * 1e6 * up, 1),
            "kind": "oracle",
            "sample": f"{n_seq} of {spec.B} sequences (all KV heads; {tok_sample} of {tok_all} cached "
                      f"tokens), score+select+attend (the append of one token, microseconds on a "
                      f"CPU, is not in the timed loop), median of {len(times)} runs scaled by the "
                      f"token ratio {up:.3f}; attention loop OpenMP over query heads, scoring and "
                      f"selection single-threaded"}


class Bench:
    """The layers of one workload, the captured graphs of its step, and the timing legs."""

    def __init__(self, torch, ts, wl, name, kv_format, step_mode, launch, n_layers_arg, dev):
        self.torch, self.ts, self.wl, self.name, self.dev = torch, ts, wl, name, dev
        spec = wl.scaled(wl.SPECS[name], kv=kv_format)
        lens_nom = torch.full((spec.B,), spec.L, dtype=torch.int32)
        nominal = wl.algorithmic_bytes(spec, lens_nom) if not spec.L_min else None
        # enough layers that one rotation touches >= 768 MiB (3x the memory-side cache)
        guess = nominal["total"] if nominal else 5 << 30
        self.n_layers = n_layers_arg or int(min(16, max(1, math.ceil((768 << 20) / guess))))
        # a graph holds one pass over the layers per query; the lengths advance with every
        # step and every leg starts from the generated lengths again, so the pool's headroom
        # has to cover one whole leg (build)
        self.per_graph = self.n_layers * N_QUERIES
        self.spec0 = spec
        self.one_launch = step_mode == "one_launch"
        self.launch = launch
        self.layers = None
        self.graph = self.graph_fused = None

    def build(self, steps_total):
        """steps_total: the most steps any single leg runs (sets the append headroom)."""
        torch, ts, wl = self.torch, self.ts, self.wl
        per_layer = -(-steps_total // self.n_layers) + 100
        spec = wl.scaled(self.spec0, headroom=max(16, per_layer))
        self.spec = spec
        self.layers = [Layer(ts, wl, spec, 1000 + 17 * i, self.dev, N_QUERIES)
                       for i in range(self.n_layers)]
        torch.cuda.synchronize()
        ly0 = self.layers[0]
        self.bytes = wl.algorithmic_bytes(spec, ly0.seq_lens, ly0.w.topk_per_seq)
        # large batches: ts_append_and_decode enqueues the append as a kernel of its own; the
        # dominant kernel timed alone for the roofline is then the plain fused one
        self.single_kernel = self.one_launch and ts.append_and_decode_launches(ly0.layout,
                                                                               ly0.w.K_max) == 1
        self.stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        if self.launch == "graph":
            try:
                self.graph = capture_graph(torch, self.layers, self.body_step, self.per_graph)
                self.rewind()
                self.graph_fused = capture_graph(torch, self.layers, self.body_fused, self.per_graph)
                self.rewind()
            except Exception as e:   # fall back to eager launches, and say so
                print(f"bench.py: graph capture failed ({e}); using eager launches", file=sys.stderr)
                self.graph = self.graph_fused = None
                self.launch = "eager"

    def rewind(self):
        for ly in self.layers:
            ly.rewind()
        self.torch.cuda.synchronize()

    def body_step(self, ly, st, qi):
        if self.one_launch:
            ly.both(st, qi)
        else:
            ly.append(st)
            ly.fused(st, qi)

    def body_fused(self, ly, st, qi):   # the dominant kernel alone: with a single-kernel step it IS the step
        if self.single_kernel:
            ly.both(st, qi)
        else:
            ly.fused(st, qi)

    def eager(self, body):
        return lambda i: body(self.layers[i % self.n_layers], self.stream, i // self.n_layers)

    def rounds(self, steps):
        """Steps rounded UP to whole graphs (one graph = one pass over the layers per query)."""
        return max(1, -(-steps // self.per_graph))

    def time_steps(self, body, graph, steps, warmup):
        """(wall s, event s, steps run, warm-up steps run) of the step `body`."""
        torch = self.torch
        if graph is not None:
            rw, rt = self.rounds(warmup), self.rounds(steps)
            for _ in range(rw):
                graph.replay()
            wall, ev = time_region(torch, lambda i: graph.replay(), rt)
            return wall, ev, rt * self.per_graph, rw * self.per_graph
        fn = self.eager(body)
        for i in range(warmup):
            fn(i)
        wall, ev = time_region(torch, fn, steps)
        return wall, ev, steps, warmup

    def check(self):
        for ly in self.layers:
            assert self.ts.workspace_status(ly.ws) == 0, "a bounded wait expired inside the fused kernel"

    def dense(self, n_launches=None):
        torch, ts = self.torch, self.ts
        dws = [ts.new_dense_workspace(ly.layout, self.dev) for ly in self.layers]
        scale = 1.0 / math.sqrt(self.spec.d)

        def dense_call(i):
            ly = self.layers[i % self.n_layers]
            ts.dense_decode_attention(ly.layout, ly.w.q[0], scale, ly.out, dws[i % self.n_layers])

        for i in range(self.n_layers):
            dense_call(i)
        n = n_launches or max(2 * self.n_layers, 4)
        _, ev = time_region(torch, dense_call, n)
        return ev / n * 1e6

    def free(self):
        self.layers = None
        self.graph = self.graph_fused = None
        import gc
        gc.collect()
        self.torch.cuda.empty_cache()


def compact_measurement(torch, ts, wl, name, args, dev):
    """us/step, the fused kernel alone, its roofline fraction and the dense baseline of one
    of the workloads that is not the headline (no CPU baseline, no extras)."""
    b = Bench(torch, ts, wl, name, args.kv_format, args.step, args.launch, 0, dev)
    steps = b.per_graph * (2 if name != "ragged" else 1)
    b.build(2 * steps)
    wall, ev, n, nw = b.time_steps(b.body_step, b.graph, steps, b.per_graph)
    b.check()
    b.rewind()
    _, evf, nf, _ = b.time_steps(b.body_fused, b.graph_fused, steps, b.per_graph)
    b.rewind()
    us, fused_us = wall / n * 1e6, evf / nf * 1e6
    dense_us = None if args.no_dense else b.dense(max(4, min(2 * b.n_layers, 16)))
    traffic, _ = measured_traffic(name, args.kv_format)
    r = {"us_per_step": round(us, 3), "kernel_us": round(fused_us, 3),
         "frac": round(b.bytes["total"] / (fused_us * 1e-6) / HBM_PEAK, 4),
         "achieved_GBps": round(b.bytes["total"] / (fused_us * 1e-6) / 1e9, 1),
         "dense_us": None if dense_us is None else round(dense_us, 2),
         "algorithmic_bytes": b.bytes["total"], "traffic": traffic,
         "steps": n, "layers_rotated": b.n_layers, "launch": b.launch}
    b.free()
    return r


def phase_marks(torch, ts, wl, args, dev):
    """Timestamps taken inside the fused kernel (tuning build): where a launch spends its
    microseconds, in the regime the benchmark times (the last launch of a back-to-back
    rotation over the layers) and on data left in the caches (the same layer again)."""
    import numpy as np
    lib = ts.lib()
    if not hasattr(lib, "ts_debug_set_profile_buffer"):
        raise SystemExit("bench.py --phase-marks needs the tuning build")
    lib.ts_debug_set_profile_buffer.argtypes = [ctypes.c_void_p]
    names = {22: "kernel entry", 23: "first loads issued", 20: "query rows arrived",
             16: "query sums ready", 1: "own pages scored", 3: "all members' scores in",
             4: "barrier after the exchange", 12: "cut-off bin found", 13: "ties at the cut resolved",
             14: "ranks known", 5: "selection done (list in LDS)", 27: "attention prologue done",
             28: "page ids read", 17: "first ring of page loads issued", 18: "last page consumed",
             24: "waves merged (barrier)", 25: "partial handed on / output written",
             6: "workgroup done"}
    order = [22, 23, 20, 16, 1, 3, 4, 12, 13, 14, 5, 27, 28, 17, 18, 24, 25, 6]
    b = Bench(torch, ts, wl, args.workload, args.kv_format, args.step, "eager", 0, dev)
    b.build(6 * b.n_layers + 64)
    buf = torch.zeros((8192, 64), dtype=torch.int64, device=dev)
    fn = b.eager(b.body_fused)
    print(f"phase marks of {WORKLOAD_DESC[args.workload]}; microseconds after the first workgroup "
          f"enters the kernel; percentiles over the workgroups of one launch, median over 5 launches")
    for regime in ("rotating", "same layer"):
        acc = []
        for rep in range(5):
            b.rewind()
            for i in range(b.n_layers):
                fn(i)
            torch.cuda.synchronize()
            buf.zero_()
            torch.cuda.synchronize()
            assert lib.ts_debug_set_profile_buffer(ctypes.c_void_p(buf.data_ptr())) == 0
            if regime == "rotating":
                for i in range(3 * b.n_layers):
                    fn(i)
            else:
                for i in range(8):
                    fn(0)
            torch.cuda.synchronize()
            assert lib.ts_debug_set_profile_buffer(None) == 0
            t = buf.cpu().numpy().astype(np.float64)
            acc.append(t[t[:, 22] > 0])
        b.check()
        n_wg = len(acc[0])
        print(f"== {regime} ({'last of %d back-to-back launches over %d layers' % (3 * b.n_layers, b.n_layers) if regime == 'rotating' else 'last of 8 launches on one layer: data left in the caches'}), "
              f"{n_wg} workgroups")

        def stat(fn_):
            return float(np.median([fn_(t, t[:, 22].min()) for t in acc]))
        for m in order:
            if not (acc[0][:, m] > 0).any():
                continue

            def pct(q, m=m):
                return stat(lambda t, t0: np.percentile((t[:, m][t[:, m] > 0] - t0) / 100.0, q))
            print(f"   {names[m]:34s} min {pct(0):6.2f}  p50 {pct(50):6.2f}  p90 {pct(90):6.2f}  max {pct(100):6.2f}")
        for base, nm in ((32, "own pages scored"), (40, "all members' scores in"),
                         (48, "first ring of loads issued"), (56, "last page consumed")):
            def waves(t, t0, base=base):
                blk = t[:, base:base + 8]
                blk = blk[(blk > 0).all(axis=1)]
                if not len(blk):
                    return [float("nan")] * 4
                us = (blk - t0) / 100.0
                return [np.median(us.min(axis=1)), np.median(us.max(axis=1)), us.max(),
                        np.median(us.max(axis=1) - us.min(axis=1))]
            r = np.median(np.array([waves(t, t[:, 22].min()) for t in acc]), axis=0)
            print(f"   by wave, {nm:28s} fastest wave p50 {r[0]:6.2f}  slowest wave p50 {r[1]:6.2f}  "
                  f"max {r[2]:6.2f}  spread inside a workgroup p50 {r[3]:5.2f}")
    b.free()


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
    ap.add_argument("--no-all-workloads", action="store_true",
                    help="time the headline workload only (skip the compact map of the others)")
    ap.add_argument("--cpu-budget", type=float, default=20.0)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (a known size against which "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled)")
    ap.add_argument("--phase-marks", action="store_true",
                    help="print the phase timeline of the fused kernel (loads the tuning build, "
                         "libtinyserve_prof.so: python paper_2509_12211_amd/build.py --profile)")
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
    if args.phase_marks:
        from paper_2509_12211_amd import build as hip_build
        if not os.path.exists(hip_build.PROFILE_LIB):
            raise SystemExit("bench.py --phase-marks: build the tuning library first "
                             "(python paper_2509_12211_amd/build.py --profile)")
        ts.LIB_PATH = hip_build.PROFILE_LIB
        phase_marks(torch, ts, wl, args, dev)
        return

    b = Bench(torch, ts, wl, args.workload, args.kv_format, args.step, args.launch, args.layers, dev)
    steps_req, warmup_req = args.steps, args.warmup
    n_layers = b.n_layers
    if args.launch == "graph":
        most = max(b.rounds(steps_req), b.rounds(warmup_req)) * b.per_graph * 2
    else:
        most = steps_req + warmup_req
    b.build(max(most, 400))
    spec, layers, by = b.spec, b.layers, b.bytes
    stream = b.stream
    if args.calibration_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    single_kernel, launch = b.single_kernel, b.launch
    one_launch = b.one_launch
    fused_only = b.eager(b.body_fused)

    # ---- timed region: the requested steps, rounded up to whole graphs ---------------
    wall, ev, steps, warmup = b.time_steps(b.body_step, b.graph, steps_req, warmup_req)
    us_step = wall / steps * 1e6
    b.check()
    b.rewind()

    # ---- roofline leg: the fused kernel alone, HIP events on its stream -----------
    _, ev_fused, n_roof, _ = b.time_steps(b.body_fused, b.graph_fused, steps_req, b.per_graph)
    fused_us = ev_fused / n_roof * 1e6
    achieved = by["total"] / (fused_us * 1e-6) / 1e9
    b.rewind()

    # ---- distribution of single launches, the same step on data left warm, and a plain
    # ---- copy of the same number of bytes ------------------------------------------
    extra = {}
    if not args.no_extras:
        # (1) every launch bracketed by its own pair of events (eager, cold rotation); the
        # pair adds its own few microseconds, so these sit above the graph figure
        n_one = 200
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(n_one)]
        for i in range(2 * n_layers):
            fused_only(i)
        torch.cuda.synchronize()
        for i, (a, c) in enumerate(evs):
            a.record()
            fused_only(i)
            c.record()
        torch.cuda.synchronize()
        one = sorted(a.elapsed_time(c) * 1e3 for a, c in evs)
        extra["single_launch_event_us"] = {
            "p10": round(one[n_one // 10], 2), "p50": round(one[n_one // 2], 2),
            "p90": round(one[(9 * n_one) // 10], 2), "launches": n_one,
            "note": "dominant kernel, eager, one event pair per launch (adds its own overhead)"}
        b.rewind()
        # (2) warm: the same layer again and again, so metadata and KV pages are found in
        # the caches left by the previous launch
        n_warm = 64
        warm = (layers[0].both if single_kernel else layers[0].fused)
        for i in range(8):
            warm(stream, 0)
        _, ev_w = time_region(torch, lambda i: warm(stream, 0), n_warm)
        extra["warm_us_per_launch"] = round(ev_w / n_warm * 1e6, 2)
        b.rewind()
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
    n_other = max(2 * n_layers, 8)
    _, ev_b = time_region(torch, lambda i: ts.build_page_meta(layers[i % n_layers].layout), n_other)
    build_us = ev_b / n_other * 1e6
    pool_bytes = by["dense"] // 2 + by["meta"]     # every cached key read once, every box written
    b.rewind()
    _, ev_a = time_region(torch, lambda i: layers[i % n_layers].append(stream), n_other)
    append_us = ev_a / n_other * 1e6
    b.rewind()

    # ---- the comparison the paper reports: attention over the whole cache ---------
    dense = None
    if not args.no_dense:
        dense_us = b.dense()
        dense = {"kernel": "ts_dense_decode_attention (every cached token, same pool and block table)",
                 "us_per_launch": round(dense_us, 2),
                 "GBps": round(by["dense"] / (dense_us * 1e-6) / 1e9, 1),
                 "speedup_of_step_over_dense": round(dense_us / us_step, 2),
                 "bytes_fraction_of_dense": round(by["total"] / by["dense"], 4)}

    traffic, traffic_commit = measured_traffic(args.workload, args.kv_format)
    result = {
        "metric": METRIC,
        "value": round(us_step, 3),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "steps_requested": steps_req,
        "warmup_requested": warmup_req,
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
            "queries_cycled": N_QUERIES,
            "launch": launch,
            "steps_per_graph": b.per_graph if launch == "graph" else None,
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
            "traffic": traffic,
            "traffic_measured_at_commit": traffic_commit,
            "us_per_launch": round(fused_us, 3),
            "launches": n_roof,
        },
        "other_kernels_us": {"ts_build_page_meta": round(build_us, 2),
                             "ts_build_page_meta_GBps": round(pool_bytes / (build_us * 1e-6) / 1e9, 1),
                             "ts_build_page_meta_frac_of_hbm_peak":
                                 round(pool_bytes / (build_us * 1e-6) / HBM_PEAK, 4),
                             "ts_append_token_meta": round(append_us, 2)},
    }
    result.update(extra)
    if dense is not None:
        result["dense_baseline"] = dense
    if not args.no_cpu_baseline:
        b.rewind()
        result["cpu_baseline"] = cpu_baseline(spec, layers[0], wl, args.cpu_budget)
    b.free()
    if not args.no_all_workloads:
        allw = {}
        for name in WORKLOAD_DESC:
            if name == args.workload:
                allw[name] = {"us_per_step": round(us_step, 3), "kernel_us": round(fused_us, 3),
                              "frac": round(achieved * 1e9 / HBM_PEAK, 4),
                              "achieved_GBps": round(achieved, 1),
                              "dense_us": None if dense is None else dense["us_per_launch"],
                              "algorithmic_bytes": by["total"], "traffic": traffic,
                              "steps": steps, "layers_rotated": n_layers, "launch": launch}
            else:
                allw[name] = compact_measurement(torch, ts, wl, name, args, dev)
        result["all_workloads"] = allw
    print(json.dumps(result, ensure_ascii=False), flush=True)


if __name__ == "__main__":
    main()
