"""Page-size / selection-ratio sweep of the query-aware decode step on one MI355X.

The paper's page-size ablation (Table 7: 16K context, budget 2048 tokens, page
size 4..64) and its selection-ratio ablation (K/P in {0.1, 0.2, 0.3, 0.5}) need
a trained model for their accuracy columns.  What can be reproduced on synthetic
inputs of the same shape is reported here, per configuration:
  - the latency of one decode step (ts_append_and_decode, cold data, HIP graph,
    measured exactly as bench.py does) and of dense attention over the whole
    cache (ts_dense_decode_attention);
  - the algorithmic bytes and the memory fraction 1/S + K*S/L of Section 3.6;
  - the share of the dense softmax mass that the selected pages capture,
    exp(lse_selected - lse_dense) averaged over (sequence, query head), next to
    K*S/L, the share a query-blind choice of K pages captures on average.
Workloads: the TinyLLaMA-shaped batch (B16, 32q/4kv, d64, L16384; grouped-query
attention, one selection shared by 8 query heads) and the GPT2-345M-shaped one
(B8, 16q/16kv, d64, L8192; one selection per head), each with the two key
recipes of the benchmark set: N(0,1) keys with outlier channels, and temporally
correlated random-walk keys.  The token budget is the one of the named
benchmark configuration (2048 and 1024 tokens).

Prints one JSON line per configuration, then a table.

--reuse measures instead the overlap of the page sets selected by consecutive
decode steps, |S_t and S_t+1| / K (the reuse of Section 3.6's cost model), on
the long-context random-walk workload, for query sequences of different
step-to-step correlation, with and without always-kept first / last pages.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench  # noqa: E402  (Layer, capture_graph, time_region)

PAGE_SIZES = [4, 8, 16, 32, 64]
RATIOS = [0.1, 0.2, 0.3, 0.5]


def measure(torch, ts, wl, spec, steps, dev):
    by_nom = wl.algorithmic_bytes(spec, torch.full((spec.B,), spec.L, dtype=torch.int32))
    n_layers = int(min(16, max(2, math.ceil((768 << 20) / by_nom["total"]))))
    per_graph = n_layers * max(1, -(-8 // n_layers))
    reps = max(1, steps // per_graph)
    spec = wl.scaled(spec, headroom=max(64, 3 * (reps + 3) * (per_graph // n_layers) + 8))
    layers = [bench.Layer(ts, wl, spec, 1000 + 17 * i, dev, 1) for i in range(n_layers)]
    g = bench.capture_graph(torch, layers, lambda ly, st, qi: ly.both(st, 0), per_graph)
    g.replay()
    wall, _ = bench.time_region(torch, lambda i: g.replay(), reps)
    step_us = wall / (reps * per_graph) * 1e6
    for ly in layers:
        assert ts.workspace_status(ly.ws) == 0
    # dense attention over the whole cache, same layers
    scale = 1.0 / math.sqrt(spec.d)
    dws = [ts.new_dense_workspace(ly.layout, dev) for ly in layers]
    lse_d = torch.empty((spec.B, spec.Hq), dtype=torch.float32, device=dev)

    def dense_call(i):
        ly = layers[i % n_layers]
        ts.dense_decode_attention(ly.layout, ly.w.q[0], scale, ly.out, dws[i % n_layers])

    for i in range(n_layers):
        dense_call(i)
    n_dense = max(2 * n_layers, 8)
    _, ev_d = bench.time_region(torch, dense_call, n_dense)
    dense_us = ev_d / n_dense * 1e6
    # captured softmax mass on layer 0 (staged calls; same kernels' arithmetic)
    ly = layers[0]
    w = ly.w
    scores = torch.empty((spec.B, spec.Hkv, w.P_max), dtype=torch.float32, device=dev)
    sel = torch.empty((spec.B, spec.Hkv, w.K_max), dtype=torch.int32, device=dev)
    cnt = torch.empty((spec.B,), dtype=torch.int32, device=dev)
    lse_s = torch.empty_like(lse_d)
    ts.score_pages(ly.layout, w.q[0], scores)
    ts.select_topk_pages(ly.layout, scores, w.topk, w.K_max, sel, cnt, topk_per_seq=w.topk_per_seq)
    ts.sparse_decode_attention(ly.layout, w.q[0], sel, cnt, w.K_max, scale, ly.out, ly.ws,
                               lse_out=lse_s)
    ts.dense_decode_attention(ly.layout, w.q[0], scale, ly.out, dws[0], lse_out=lse_d)
    torch.cuda.synchronize()
    mass = torch.exp(lse_s - lse_d).double()
    by = wl.algorithmic_bytes(spec, ly.seq_lens, w.topk_per_seq)
    P = -(-int(ly.seq_lens[0]) // spec.S)
    return {
        "shape": spec.name, "keys": spec.keys, "S": spec.S, "K": spec.topk, "P": P,
        "K_over_P": round(spec.topk / P, 3),
        "step_us": round(step_us, 2), "dense_us": round(dense_us, 2),
        "speedup_vs_dense": round(dense_us / step_us, 2),
        "algorithmic_MB": round(by["total"] / 1e6, 1),
        "effective_GBps": round(by["total"] / step_us / 1e3, 1),
        "memory_fraction_model": round(1.0 / spec.S + spec.topk * spec.S / spec.L, 4),
        "bytes_fraction_measured": round(by["total"] / by["dense"], 4),
        "mass_captured_mean": round(float(mass.mean()), 4),
        "mass_captured_p10": round(float(mass.flatten().quantile(0.1)), 4),
        "mass_query_blind": round(min(1.0, spec.topk * spec.S / spec.L), 4),
        "layers_rotated": n_layers,
    }


def reuse(torch, ts, wl, steps, dev):
    """Overlap of consecutive selections.  The query of step t+1 is
    a * q_t + sqrt(1 - a^2) * noise (a = 0: independent queries)."""
    base = wl.SPECS["longctx"]
    rows = []
    for keep in [(0, 0), (1, 2)]:
        for a in [0.0, 0.9, 0.99, 0.999]:
            spec = wl.scaled(base, headroom=steps + 64)
            w = wl.make_workload(spec, dev, seed=1003, n_q=1, n_new=steps, poison=0.0)
            pmin = torch.zeros((spec.B, spec.Hkv, w.P_max, spec.d), dtype=torch.bfloat16, device=dev)
            pmax = torch.zeros_like(pmin)
            lens = w.seq_lens.clone()
            lay = ts.make_layout(spec.B, spec.Hq, spec.Hkv, spec.d, spec.S, w.P_max, w.k_pool,
                                 w.v_pool, w.block_table, lens, pmin, pmax,
                                 keep_first_pages=keep[0], keep_last_pages=keep[1])
            ts.build_page_meta(lay)
            ws = ts.new_workspace(lay, w.K_max, dev)
            out = torch.empty((spec.B, spec.Hq, spec.d), dtype=torch.float32, device=dev)
            sel = torch.empty((spec.B, spec.Hkv, w.K_max), dtype=torch.int32, device=dev)
            g = torch.Generator(device=dev)
            g.manual_seed(77)
            q = torch.randn((spec.B, spec.Hq, spec.d), generator=g, device=dev)
            prev, overlaps = None, []
            scale = 1.0 / math.sqrt(spec.d)
            for t in range(steps):
                ts.append_and_decode(lay, w.k_new[t], w.v_new[t], q.to(torch.bfloat16), w.topk,
                                     w.K_max, scale, out, ws, sel_out=sel)
                cur = sel.clone()
                if prev is not None:
                    # both lists ascending, no padding (K < P): count common ids per unit
                    common = (cur[:, :, :, None] == prev[:, :, None, :]).any(-1).sum(-1)
                    overlaps.append(common.double().mean().item() / w.K_max)
                prev = cur
                q = a * q + math.sqrt(1.0 - a * a) * torch.randn(q.shape, generator=g, device=dev)
            torch.cuda.synchronize()
            assert ts.workspace_status(ws) == 0
            o = sum(overlaps) / len(overlaps)
            frac_new = 1.0 / spec.S + (1.0 - o) * spec.topk * spec.S / spec.L
            r = {"workload": "longctx", "query_correlation": a, "keep_first": keep[0],
                 "keep_last": keep[1], "steps": steps, "K": spec.topk,
                 "overlap_mean": round(o, 4), "overlap_min": round(min(overlaps), 4),
                 "overlap_query_blind": round(spec.topk * spec.S / spec.L, 4),
                 "memory_fraction_no_reuse": round(1.0 / spec.S + spec.topk * spec.S / spec.L, 4),
                 "memory_fraction_new_pages_only": round(frac_new, 4)}
            rows.append(r)
            print(json.dumps(r), flush=True)
            del w, pmin, pmax, ws
            torch.cuda.empty_cache()
    hdr = ("query_correlation", "keep_first", "keep_last", "overlap_mean", "overlap_min",
           "overlap_query_blind", "memory_fraction_no_reuse", "memory_fraction_new_pages_only")
    print("| " + " | ".join(hdr) + " |")
    print("|" + "---|" * len(hdr))
    for r in rows:
        print("| " + " | ".join(str(r[h]) for h in hdr) + " |")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reuse", action="store_true",
                    help="measure the overlap of consecutive steps' selections instead")
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--keys", default="offset,walk")
    ap.add_argument("--shapes", default="tinyllama,gpt2_345m")
    ap.add_argument("--only", default="", help="'budget' or 'ratio' to run one half of the sweep")
    args = ap.parse_args()
    import torch
    from paper_2509_12211_amd import tinyserve as ts
    from paper_2509_12211_amd import workloads as wl
    if not torch.cuda.is_available():
        print("sweep.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.reuse:
        reuse(torch, ts, wl, min(args.steps, 48), dev)
        return
    rows = []
    for shape, keys in [(s, k) for s in args.shapes.split(",") for k in args.keys.split(",")]:
        base = wl.SPECS[shape]
        budget = base.topk * base.S
        configs = []
        if args.only != "ratio":
            configs += [("budget", S, budget // S) for S in PAGE_SIZES]
        if args.only != "budget":
            configs += [("ratio", S, max(1, round(r * base.L / S)))
                        for S in PAGE_SIZES for r in RATIOS]
        for kind, S, K in configs:
            spec = wl.scaled(base, S=S, topk=K, keys=keys)
            print(f"[sweep] {kind} {shape} keys={keys} S={S} K={K}", file=sys.stderr, flush=True)
            r = measure(torch, ts, wl, spec, args.steps, dev)
            r["sweep"] = kind
            rows.append(r)
            print(json.dumps(r), flush=True)
            torch.cuda.empty_cache()
    hdr = ("sweep", "shape", "keys", "S", "K", "K_over_P", "step_us", "dense_us", "speedup_vs_dense",
           "algorithmic_MB", "memory_fraction_model", "mass_captured_mean", "mass_captured_p10",
           "mass_query_blind")
    print("| " + " | ".join(hdr) + " |")
    print("|" + "---|" * len(hdr))
    for r in rows:
        print("| " + " | ".join(str(r[h]) for h in hdr) + " |")


if __name__ == "__main__":
    main()
