"""Shared test plumbing: runs the CPU oracle on (a sample of) a synthetic
workload and compares HIP results against it with the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

from paper_2509_12211_amd import workloads as wl

SCORE_RTOL = 1e-5     # fp32 page scores vs the fp64 oracle, relative
OUT_ATOL = 2e-3       # attention output, absolute (bf16 inputs, fp32 accumulation)
GAP_RTOL = 1e-5       # selections may differ only where the oracle's K-th / (K+1)-th
                      # scores are closer than this (relative)


def oracle_unit_inputs(w, b, h, q_idx=0, seq_lens=None):
    """Logical inputs of one (sequence, KV head) as numpy bit patterns."""
    G = w.spec.Hq // w.spec.Hkv
    lens = (w.seq_lens if seq_lens is None else seq_lens).cpu()
    K, V = wl.logical_kv(w, seqs=[b], heads=[h], seq_lens=lens)
    q = w.q[q_idx, b, h * G:(h + 1) * G][None]            # [1][G][d]
    L = np.array([int(lens[b])], dtype=np.int32)
    return wl.bits(q), wl.bits(K), wl.bits(V), L


def oracle_unit(oracle, w, b, h, scale, q_idx=0, seq_lens=None, topk=None, keep=(0, 0)):
    """Full oracle step for one unit; returns its dict plus the metadata."""
    q, K, V, L = oracle_unit_inputs(w, b, h, q_idx, seq_lens)
    S = w.spec.S
    pmin, pmax = oracle.build_page_meta(K, L, S, w.P_max)
    if topk is None:
        topk = int(w.topk_per_seq[b]) if w.topk_per_seq is not None else w.topk
    r = oracle.query_aware_decode(q, K, V, pmin, pmax, L, S, topk, w.K_max, scale,
                                  keep_first=keep[0], keep_last=keep[1])
    r.update(pmin=pmin, pmax=pmax, q=q, K=K, V=V, L=L)
    return r


def oracle_sequence(oracle, w, b, heads, scale, q_idx=0, seq_lens=None, keep=(0, 0)):
    """Full oracle step for several KV heads of one sequence in ONE oracle call (the
    heads become the oracle's KV heads, in the order given); works for the 16-bit and
    the INT8 cache.  Returns the oracle's dict plus its inputs and the metadata."""
    sp = w.spec
    G = sp.Hq // sp.Hkv
    lens = (w.seq_lens if seq_lens is None else seq_lens).cpu()
    heads = list(heads)
    qh = torch.cat([w.q[q_idx, b, h * G:(h + 1) * G] for h in heads])[None]   # [1][n*G][d]
    q = wl.bits(qh)
    L = np.array([int(lens[b])], dtype=np.int32)
    topk = int(w.topk_per_seq[b]) if w.topk_per_seq is not None else w.topk
    if sp.kv == "int8":
        Kq, ks, Vq, vs = (t.cpu().numpy() for t in
                          wl.logical_kv_i8(w, seqs=[b], heads=heads, seq_lens=lens))
        pmin, pmax = oracle.build_page_meta_i8(Kq, ks, L, sp.S, w.P_max)
        r = oracle.query_aware_decode_i8(q, Kq, ks, Vq, vs, pmin, pmax, L, sp.S, topk, w.K_max,
                                         scale, keep_first=keep[0], keep_last=keep[1])
        r.update(kv=(Kq, ks, Vq, vs))
    else:
        K, V = wl.logical_kv(w, seqs=[b], heads=heads, seq_lens=lens)
        K, V = wl.bits(K), wl.bits(V)
        pmin, pmax = oracle.build_page_meta(K, L, sp.S, w.P_max)
        r = oracle.query_aware_decode(q, K, V, pmin, pmax, L, sp.S, topk, w.K_max, scale,
                                      keep_first=keep[0], keep_last=keep[1])
        r.update(kv=(K, V))
    r.update(pmin=pmin, pmax=pmax, q=q, L=L)
    return r


def head_view(r, i, G):
    """The entries of oracle_sequence's result that belong to its i-th head, shaped like
    a single-unit result (what check_selection expects)."""
    v = dict(scores=r["scores"][:, i:i + 1], sel=r["sel"][:, i:i + 1], sel_count=r["sel_count"],
             gap=r["gap"][:, i:i + 1], out=r["out"][:, i * G:(i + 1) * G],
             q=r["q"][:, i * G:(i + 1) * G], L=r["L"],
             pmin=r["pmin"][:, i:i + 1], pmax=r["pmax"][:, i:i + 1])
    v["kv"] = tuple(t[:, i:i + 1] for t in r["kv"])
    return v


def attention_on_set(oracle, w, v, sel_row, count, scale):
    """Oracle attention of one unit (a head_view) over a GIVEN page list: what the output
    is compared with when the selection differs from the oracle's at a near-tie."""
    sel = np.ascontiguousarray(np.asarray(sel_row)[None, None])
    cnt = np.array([int(count)], dtype=np.int32)
    if w.spec.kv == "int8":
        Kq, ks, Vq, vs = (np.ascontiguousarray(t) for t in v["kv"])
        return oracle.sparse_decode_attention_i8(np.ascontiguousarray(v["q"]), Kq, ks, Vq, vs, sel,
                                                 cnt, v["L"], w.spec.S, scale)[0]
    K, V = (np.ascontiguousarray(t) for t in v["kv"])
    return oracle.sparse_decode_attention(np.ascontiguousarray(v["q"]), K, V, sel, cnt, v["L"],
                                          w.spec.S, scale)[0]


def by_sequence(units):
    """[(b, h), ...] -> {b: [h, ...]} in ascending order."""
    groups = {}
    for b, h in sorted(set(units)):
        groups.setdefault(b, []).append(h)
    return groups


def assert_scores_close(gpu_scores, oracle_scores, Pb, what=""):
    g = np.asarray(gpu_scores, dtype=np.float64)
    o = np.asarray(oracle_scores, dtype=np.float64)
    assert np.all(np.isneginf(g[Pb:])), f"{what}: pages >= P_b must score -inf"
    err = np.abs(g[:Pb] - o[:Pb])
    tol = SCORE_RTOL * np.maximum(np.abs(o[:Pb]), 1e-30)
    bad = np.nonzero(err > tol)[0]
    assert bad.size == 0, (f"{what}: {bad.size} scores off, worst rel "
                           f"{np.max(err / np.maximum(np.abs(o[:Pb]), 1e-30)):.3e} at page {bad[:5]}")


def check_selection(gpu_sel, gpu_count, r, what=""):
    """Bit-exact against the oracle's set, except at a near-tie of the cut: then
    the sets may differ only in pages whose oracle scores sit at the cut.
    Returns True when the sets are identical."""
    n = int(r["sel_count"][0])
    assert int(gpu_count) == n, f"{what}: sel_count {gpu_count} != {n}"
    g = np.asarray(gpu_sel)
    assert np.all(g[n:] == -1), f"{what}: padding must be -1"
    assert np.all(np.diff(g[:n]) > 0), f"{what}: ids must be strictly ascending"
    o = r["sel"][0, 0]
    if np.array_equal(g[:n], o[:n]):
        return True
    gap = float(r["gap"][0, 0])
    assert gap <= GAP_RTOL, f"{what}: selection differs but the oracle's cut gap is {gap:.3e}"
    s = r["scores"][0, 0]
    cut = np.sort(s[o[:n]])[0]
    diff = np.setxor1d(g[:n], o[:n])
    rel = np.abs(s[diff] - cut) / max(abs(cut), 1e-30)
    assert np.all(rel <= 10 * GAP_RTOL), f"{what}: swapped pages are not at the cut ({rel.max():.3e})"
    return False


def assert_out_close(gpu_out, oracle_out, what=""):
    g = np.asarray(gpu_out, dtype=np.float64)
    err = np.abs(g - oracle_out)
    assert np.all(np.isfinite(g)), f"{what}: non-finite output"
    assert err.max() <= OUT_ATOL, f"{what}: max abs err {err.max():.3e} > {OUT_ATOL}"
    return float(err.max())


def full_size_units(w, name):
    """Units compared at full size: every (sequence, KV head) of the small batches; of the
    ragged batch all KV heads of the 8 shortest and the 8 longest sequences and of the
    sequences that hold the first unit, the units on either side of the first hand-out
    of tickets beyond the resident workgroups (255, 256) and the last unit."""
    B, Hkv = w.spec.B, w.spec.Hkv
    if name != "ragged":
        return [(b, h) for b in range(B) for h in range(Hkv)]
    order = torch.argsort(w.seq_lens.cpu(), stable=True).tolist()
    seqs = set(order[:8]) | set(order[-8:]) | {0, 255 // Hkv, 256 // Hkv, B - 1}
    return [(b, h) for b in sorted(seqs) for h in range(Hkv)]


def unit_samples(w, n, seed=0):
    """A deterministic sample of (sequence, KV head) units, always including the
    first and last unit, the shortest and the longest sequence."""
    B, Hkv = w.spec.B, w.spec.Hkv
    lens = w.seq_lens.cpu()
    picks = {(0, 0), (B - 1, Hkv - 1), (int(lens.argmin()), 0), (int(lens.argmax()), Hkv - 1)}
    rng = np.random.default_rng(seed)
    while len(picks) < min(n, B * Hkv):
        picks.add((int(rng.integers(B)), int(rng.integers(Hkv))))
    return sorted(picks)
