"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded
inputs.  Reduced shapes are compared for every (sequence, KV head); the five
full-size workloads are compared on every unit (the ragged batch: on every unit of
20 of its 64 sequences), in the launch configuration bench.py times."""
import math

import numpy as np
import pytest
import torch

from paper_2509_12211_amd import tinyserve as ts
from paper_2509_12211_amd import workloads as wl

from helpers import (assert_out_close, assert_scores_close, attention_on_set, by_sequence,
                     check_selection, full_size_units, head_view, oracle_sequence, unit_samples)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


class Session:
    """Device buffers + layout struct for one workload."""

    def __init__(self, w, poison_meta=True, keep=(0, 0), cluster_size=0, wait_limit=0):
        self.w = w
        self.keep = keep      # pages kept whatever their score: (first, last)
        sp = w.spec
        fill = float("nan") if poison_meta else 0.0
        self.page_min = torch.full((sp.B, sp.Hkv, w.P_max, sp.d), fill, dtype=w.k_pool.dtype,
                                   device=DEV)
        self.page_max = torch.full_like(self.page_min, fill)
        self.seq_lens = w.seq_lens.clone()
        self.layout = ts.make_layout(sp.B, sp.Hq, sp.Hkv, sp.d, sp.S, w.P_max, w.k_pool, w.v_pool,
                                     w.block_table, self.seq_lens, self.page_min, self.page_max,
                                     keep_first_pages=keep[0], keep_last_pages=keep[1],
                                     cluster_size=cluster_size, wait_limit=wait_limit)
        self.scores = torch.full((sp.B, sp.Hkv, w.P_max), float("nan"), dtype=torch.float32,
                                 device=DEV)
        self.sel = torch.full((sp.B, sp.Hkv, w.K_max), -7, dtype=torch.int32, device=DEV)
        self.sel_count = torch.full((sp.B,), -7, dtype=torch.int32, device=DEV)
        self.out = torch.full((sp.B, sp.Hq, sp.d), float("nan"), dtype=torch.float32, device=DEV)
        self.ws = ts.new_workspace(self.layout, w.K_max, DEV)

    def fused(self, scale, q_idx=0, report=True):
        w = self.w
        ts.query_aware_decode(self.layout, w.q[q_idx], w.topk, w.K_max, scale, self.out, self.ws,
                              topk_per_seq=w.topk_per_seq,
                              scores_out=self.scores if report else None,
                              sel_out=self.sel if report else None,
                              sel_count_out=self.sel_count if report else None)

    def staged(self, scale, q_idx=0):
        w = self.w
        ts.score_pages(self.layout, w.q[q_idx], self.scores)
        ts.select_topk_pages(self.layout, self.scores, w.topk, w.K_max, self.sel, self.sel_count,
                             topk_per_seq=w.topk_per_seq)
        ts.sparse_decode_attention(self.layout, w.q[q_idx], self.sel, self.sel_count, w.K_max,
                                   scale, self.out, self.ws)


def compare_units(oracle, sess, units, scale, q_idx=0, what=""):
    """Compare the session's current scores / sel / out with the oracle."""
    w = sess.w
    sp = w.spec
    G = sp.Hq // sp.Hkv
    torch.cuda.synchronize()
    assert ts.workspace_status(sess.ws) == 0
    scores = sess.scores.cpu().numpy()
    sel = sess.sel.cpu().numpy()
    cnt = sess.sel_count.cpu().numpy()
    out = sess.out.cpu().numpy()
    lens = sess.seq_lens.cpu()
    worst = 0.0
    mdt = sess.page_min.dtype
    with oracle.element_format(sp.kv):
        worst = _compare_units(oracle, sess, units, scale, q_idx, what, w, sp, G, scores, sel, cnt,
                               out, lens, mdt)
    return worst


def _compare_units(oracle, sess, units, scale, q_idx, what, w, sp, G, scores, sel, cnt, out, lens,
                   mdt):
    """One oracle call per sequence (all the wanted KV heads of it at once)."""
    worst = 0.0
    for b, heads in by_sequence(units).items():
        r = oracle_sequence(oracle, w, b, heads, scale, q_idx=q_idx, seq_lens=lens, keep=sess.keep)
        Pb = int(oracle.num_pages(int(lens[b]), sp.S))
        for i, h in enumerate(heads):
            tag = f"{what} unit(b={b},h={h})"
            v = head_view(r, i, G)
            omin = wl.from_bits(v["pmin"], dtype=mdt).to(torch.float64).numpy()[0, 0]
            omax = wl.from_bits(v["pmax"], dtype=mdt).to(torch.float64).numpy()[0, 0]
            gmin = sess.page_min[b, h, :Pb].to(torch.float64).cpu().numpy()
            gmax = sess.page_max[b, h, :Pb].to(torch.float64).cpu().numpy()
            assert np.array_equal(gmin, omin[:Pb]), f"{tag}: page_min"
            assert np.array_equal(gmax, omax[:Pb]), f"{tag}: page_max"
            assert_scores_close(scores[b, h], v["scores"][0, 0], Pb, tag)
            same = check_selection(sel[b, h], cnt[b], v, tag)
            ref = v["out"][0]
            if not same:   # near-tie at the cut: attention is checked on the GPU's own set
                ref = attention_on_set(oracle, w, v, sel[b, h], cnt[b], scale)
            worst = max(worst, assert_out_close(out[b, h * G:(h + 1) * G], ref, tag))
    return worst


REDUCED = {
    # several score slices, several splits, a ragged last page
    "mha_d64_s16": wl.WorkloadSpec("mha_d64_s16", 3, 4, 4, 64, 16, 2000, 24, headroom=40),
    "gqa8_d64_s16_offset": wl.WorkloadSpec("gqa8", 2, 16, 2, 64, 16, 4101, 40, keys="offset"),
    "gqa8_d64_s32_walk": wl.WorkloadSpec("walk", 2, 16, 2, 64, 32, 6007, 20, keys="walk"),
    "mha_d128_s16_ragged": wl.WorkloadSpec("ragged", 6, 4, 4, 128, 16, 3000, 0, L_min=1,
                                           budget_frac=0.25),
    "gqa4_d128_s32": wl.WorkloadSpec("gqa4_d128_s32", 2, 8, 2, 128, 32, 2500, 9),
    "gqa16_d64_s16": wl.WorkloadSpec("gqa16", 1, 16, 1, 64, 16, 1030, 70),
    "k_exceeds_p": wl.WorkloadSpec("k_exceeds_p", 2, 2, 2, 64, 16, 100, 32),
    # pages smaller than an MFMA tile (four / two pages per 16-token fragment; list lengths
    # that are no multiple of the group, a one-token last page)
    "gqa8_d64_s4": wl.WorkloadSpec("s4", 2, 16, 2, 64, 4, 1501, 90, keys="offset"),
    "gqa2_d128_s4": wl.WorkloadSpec("s4b", 2, 4, 2, 128, 4, 703, 33),
    "mha_d128_s8": wl.WorkloadSpec("s8", 3, 4, 4, 128, 8, 1003, 37),
    "mha_d64_s8_ragged": wl.WorkloadSpec("s8r", 5, 4, 4, 64, 8, 900, 0, L_min=1, budget_frac=0.25),
    # 64-token pages (two 32-token fragments each); last page 8 and 40 tokens long
    "gqa4_d64_s64": wl.WorkloadSpec("s64", 2, 8, 2, 64, 64, 5000, 11, keys="walk"),
    "mha_d128_s64": wl.WorkloadSpec("s64b", 2, 4, 4, 128, 64, 3048, 7),
}


@pytest.fixture(scope="module")
def built():
    ts.lib()
    assert torch.cuda.is_available()
    return True


@pytest.fixture
def splits(request):
    """Workgroups per (sequence, KV head): 0 = the library's own choice (a single
    workgroup for sequences this short), otherwise a forced cluster size."""
    ts.set_tuning(0, request.param, 0)
    yield request.param
    ts.set_tuning(0, 0, 0)


FORMATS = ["bf16", "fp16"]    # 16-bit element formats of the cache (the INT8 one has its own file)


@pytest.mark.parametrize("name", list(REDUCED))
@pytest.mark.parametrize("scale_mode,splits", [("rsqrt_d", 0), ("one", 3), ("rsqrt_d", 8)],
                         indirect=["splits"])
@pytest.mark.parametrize("fmt", FORMATS)
def test_reduced_all_units(oracle, built, name, scale_mode, splits, fmt):
    spec = wl.scaled(REDUCED[name], kv=fmt)
    print(f"[case] reduced {name} {fmt} scale={scale_mode} splits={splits}", flush=True)
    # paper-literal scale runs on two dense pools, the usual one on the interleaved K|V pool
    w = wl.make_workload(spec, DEV, seed=2000 + len(name), n_q=2,
                         interleave=(scale_mode == "rsqrt_d"))
    scale = 1.0 / math.sqrt(spec.d) if scale_mode == "rsqrt_d" else 1.0
    if scale_mode == "one":      # paper-literal softmax(q.k): keep logits in a sane range
        w.q.mul_(0.25)
    sess = Session(w)
    ts.build_page_meta(sess.layout)
    units = [(b, h) for b in range(spec.B) for h in range(spec.Hkv)]
    # staged path
    sess.staged(scale, q_idx=1)
    compare_units(oracle, sess, units, scale, q_idx=1, what=f"{name}/staged")
    staged = (sess.scores.clone(), sess.sel.clone(), sess.sel_count.clone(), sess.out.clone())
    # fused path, reporting its intermediates
    for t in (sess.scores, sess.out):
        t.fill_(float("nan"))
    sess.sel.fill_(-7)
    sess.sel_count.fill_(-7)
    sess.fused(scale, q_idx=1)
    compare_units(oracle, sess, units, scale, q_idx=1, what=f"{name}/fused")
    # fused == staged: same kernels' arithmetic, so selections identical, outputs to 1e-6
    assert torch.equal(sess.scores, staged[0])
    assert torch.equal(sess.sel, staged[1]) and torch.equal(sess.sel_count, staged[2])
    assert (sess.out - staged[3]).abs().max().item() <= 1e-6
    # fused without reporting buffers, twice: same bits (determinism, workspace re-armed)
    first = sess.out.clone()
    sess.out.fill_(float("nan"))
    sess.fused(scale, q_idx=1, report=False)
    torch.cuda.synchronize()
    assert torch.equal(sess.out, first)


def test_select_on_given_scores_is_exact(oracle, built):
    """ts_select_topk_pages on fp32 scores the oracle also sees: bit-exact sets,
    including heavy ties (quantised scores), -0/+0, and K >= P."""
    print("[case] select exact", flush=True)
    B, Hkv, S, Pmax, Kmax = 6, 3, 16, 1500, 300
    rng = np.random.default_rng(77)
    lens = np.array([1500 * 16, 777 * 16 + 3, 16, 0, 299 * 16, 1200 * 16], dtype=np.int32)
    sc = rng.standard_normal((B, Hkv, Pmax)).astype(np.float32)
    sc[0, 1] = np.round(sc[0, 1] * 2) / 2                 # many exact ties
    sc[0, 2] = 0.0
    sc[0, 2, ::3] = -0.0                                   # signed zeros rank equal
    sc[1, 0] = np.float32(1e-30) * sc[1, 0]                # tiny magnitudes
    sc[1, 1] = -np.abs(sc[1, 1]) * 1e20                    # all negative, large
    sc[5, 0] = np.round(sc[5, 0] * 64) / 64               # small tie groups at the cut
    sc[5, 1] = np.round(sc[5, 1] * 8) / 8                 # tie groups of a few dozen
    sc[5, 2] = np.round(sc[5, 2] * 512) / 512             # mostly pairs
    topk_ps = np.array([300, 100, 5, 7, 299, 200], dtype=np.int32)
    lens_d = torch.from_numpy(lens).to(DEV)
    for per_seq, (kf, kl) in [(False, (0, 0)), (True, (0, 0)), (False, (1, 2)), (True, (3, 0)),
                              (True, (0, 4)), (False, (200, 150)), (True, (2, 1))]:
        lay = ts.make_layout(B, Hkv, Hkv, 64, S, Pmax, None, None, None, lens_d, None, None,
                             keep_first_pages=kf, keep_last_pages=kl)
        lay.num_phys_pages = 1      # no pool is read by the selection
        d_sc = torch.from_numpy(sc).to(DEV)
        sel = torch.full((B, Hkv, Kmax), -7, dtype=torch.int32, device=DEV)
        cnt = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        tps = torch.from_numpy(topk_ps).to(DEV) if per_seq else None
        ts.select_topk_pages(lay, d_sc, 123, Kmax, sel, cnt, topk_per_seq=tps)
        torch.cuda.synchronize()
        osel, ocnt, _ = oracle.select_topk_pages(sc.astype(np.float64), lens, S, 123, Kmax,
                                                 topk_per_seq=topk_ps if per_seq else None,
                                                 keep_first=kf, keep_last=kl)
        assert np.array_equal(cnt.cpu().numpy(), ocnt), (per_seq, kf, kl)
        assert np.array_equal(sel.cpu().numpy(), osel), (per_seq, kf, kl)


@pytest.mark.parametrize("crowd", [2, 9, 24, 32, 33, 200])
def test_select_with_a_crowded_cut_off_bin(oracle, built, crowd):
    """The cut falls into a bin that holds `crowd` pages with distinct scores a hair apart
    (up to 32 are listed and ranked, more go through the exact passes), owned by threads
    of several waves and, some of them, by one thread; every rank offset behind them must
    still come out right: the lists are the oracle's, bit for bit."""
    print(f"[case] crowded cut-off bin {crowd}", flush=True)
    B, Hkv, S, Pmax, Kmax = 3, 2, 16, 4096, 512
    rng = np.random.default_rng(1000 + crowd)
    lens = np.array([4096 * 16, 3000 * 16 + 5, 4096 * 16], dtype=np.int32)
    sc = (rng.random((B, Hkv, Pmax)) * 0.8).astype(np.float32)
    n_sure = 150
    need = max(1, crowd // 3)
    for b in range(B):
        Pb = -(-int(lens[b]) // S)
        for h in range(Hkv):
            pages = rng.permutation(Pb)
            sure, rest = pages[:n_sure], pages[n_sure:]
            sc[b, h, sure] = (0.95 + 0.05 * rng.random(n_sure)).astype(np.float32)
            # the crowd: a run of consecutive pages (one thread owns several), the rest scattered
            start = int(rest[0]) // 8 * 8
            run = [p for p in range(start, min(start + 6, Pb)) if p not in set(sure.tolist())]
            others = [int(p) for p in rest[1:] if p not in run][:max(0, crowd - len(run))]
            members = (run + others)[:crowd]
            sc[b, h, members] = (0.9 + 1e-6 * rng.permutation(len(members))).astype(np.float32)
    topk = n_sure + need
    lens_d = torch.from_numpy(lens).to(DEV)
    lay = ts.make_layout(B, Hkv, Hkv, 64, S, Pmax, None, None, None, lens_d, None, None)
    lay.num_phys_pages = 1      # no pool is read by the selection
    sel = torch.full((B, Hkv, Kmax), -7, dtype=torch.int32, device=DEV)
    cnt = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    ts.select_topk_pages(lay, torch.from_numpy(sc).to(DEV), topk, Kmax, sel, cnt)
    torch.cuda.synchronize()
    osel, ocnt, _ = oracle.select_topk_pages(sc.astype(np.float64), lens, S, topk, Kmax)
    assert np.array_equal(cnt.cpu().numpy(), ocnt)
    assert np.array_equal(sel.cpu().numpy(), osel)


@pytest.mark.parametrize("name,keep", [("mha_d64_s16", (1, 2)), ("gqa8_d64_s32_walk", (2, 0)),
                                       ("mha_d128_s16_ragged", (0, 3)), ("gqa8_d64_s4", (4, 8)),
                                       ("gqa4_d64_s64", (1, 1)), ("k_exceeds_p", (3, 3)),
                                       ("gqa16_d64_s16", (40, 40))])
@pytest.mark.parametrize("splits", [0, 4], indirect=True)
def test_always_kept_pages(oracle, built, name, keep, splits):
    """Selection with always-kept first / last pages (an option outside the paper),
    staged and fused, against the oracle; the last pair asks for more such pages
    than the budget holds."""
    spec = REDUCED[name]
    print(f"[case] always-kept {name} keep={keep} splits={splits}", flush=True)
    w = wl.make_workload(spec, DEV, seed=99, n_q=1, n_new=1)
    sess = Session(w, keep=keep)
    ts.build_page_meta(sess.layout)
    scale = 1.0 / math.sqrt(spec.d)
    units = [(b, h) for b in range(spec.B) for h in range(spec.Hkv)]
    sess.staged(scale)
    compare_units(oracle, sess, units, scale, what=f"{name}/kept/staged")
    staged_sel = sess.sel.clone()
    sess.sel.fill_(-7)
    sess.fused(scale)
    compare_units(oracle, sess, units, scale, what=f"{name}/kept/fused")
    assert torch.equal(staged_sel, sess.sel)
    # the kept pages are there (when the budget holds them)
    sel = sess.sel.cpu().numpy()
    lens = sess.seq_lens.cpu().numpy()
    for (b, h) in units:
        Pb = -(-int(lens[b]) // spec.S)
        kept = [j for j in range(Pb) if j < keep[0] or j >= Pb - keep[1]]
        n = int(sess.sel_count[b])
        if len(kept) <= n:
            assert set(kept) <= set(sel[b, h, :n].tolist())
    # and through the launch that appends: the newest page is the appended token's
    ts.append_and_decode(sess.layout, w.k_new[0], w.v_new[0], w.q[0], w.topk, w.K_max, scale,
                         sess.out, sess.ws, topk_per_seq=w.topk_per_seq, scores_out=sess.scores,
                         sel_out=sess.sel, sel_count_out=sess.sel_count)
    compare_units(oracle, sess, units, scale, what=f"{name}/kept/append")


def test_append_matches_oracle_and_rebuild(oracle, built):
    """Appends crossing page boundaries: metadata equals the oracle's incremental
    update and a from-scratch rebuild; the appended K/V are visible to the fused step."""
    print("[case] append", flush=True)
    spec = wl.WorkloadSpec("app", 4, 8, 2, 64, 16, 200, 6, L_min=1, headroom=48)
    n_new = 40
    w = wl.make_workload(spec, DEV, seed=31, n_q=n_new, n_new=n_new)
    sess = Session(w)
    ts.build_page_meta(sess.layout)
    scale = 0.125
    lens0 = w.seq_lens.cpu().numpy().copy()
    units = [(b, h) for b in range(spec.B) for h in range(spec.Hkv)]
    for i in range(n_new):
        ts.append_token_meta(sess.layout, w.k_new[i], w.v_new[i], advance_seq_lens=True)
        if i % 13 == 0 or i == n_new - 1:
            sess.fused(scale, q_idx=i)
            torch.cuda.synchronize()
            assert np.array_equal(sess.seq_lens.cpu().numpy(), lens0 + i + 1)
            # compare_units rebuilds the logical K/V from the pool (so it sees the
            # appended tokens) and the oracle's metadata from scratch
            compare_units(oracle, sess, units, scale, q_idx=i, what=f"append step {i}")
    # metadata-only append (v_new = NULL) without advancing
    before = sess.seq_lens.clone()
    ts.append_token_meta(sess.layout, w.k_new[0], None, advance_seq_lens=False)
    torch.cuda.synchronize()
    assert torch.equal(before, sess.seq_lens)
    # oracle incremental update on host copies of the same metadata
    lens = before.cpu().numpy()
    pmin = wl.bits(sess.page_min)
    pmax = wl.bits(sess.page_max)
    # undo: rebuild on device, run the oracle's append on the rebuilt rows, compare
    ts.build_page_meta(sess.layout)
    torch.cuda.synchronize()
    omin, omax = wl.bits(sess.page_min).copy(), wl.bits(sess.page_max).copy()
    oracle.append_token_meta(wl.bits(w.k_new[0]), lens, spec.S, omin, omax)
    for b in range(spec.B):
        j = int(lens[b]) // spec.S
        a = wl.from_bits(pmin[b, :, j]).float().numpy()
        o = wl.from_bits(omin[b, :, j]).float().numpy()
        assert np.array_equal(a, o)
        a = wl.from_bits(pmax[b, :, j]).float().numpy()
        o = wl.from_bits(omax[b, :, j]).float().numpy()
        assert np.array_equal(a, o)


APPEND_FUSED = {
    # clusters of two workgroups per unit
    "gqa4_d64_s16": wl.WorkloadSpec("af1", 4, 8, 2, 64, 16, 200, 6, L_min=1, headroom=48),
    # more units than workgroups: one workgroup per unit, units handed out by ticket
    "mha_d128_s16_many": wl.WorkloadSpec("af2", 72, 4, 4, 128, 16, 300, 5, L_min=1, headroom=48),
    "gqa8_d64_s32": wl.WorkloadSpec("af3", 3, 16, 2, 64, 32, 700, 7, keys="walk", headroom=80),
    "gqa2_d128_s32": wl.WorkloadSpec("af4", 2, 4, 2, 128, 32, 500, 4, headroom=80),
    "gqa4_d64_s4": wl.WorkloadSpec("af5", 3, 8, 2, 64, 4, 150, 9, L_min=1, headroom=48),
    "mha_d128_s8": wl.WorkloadSpec("af6", 2, 4, 4, 128, 8, 300, 6, headroom=80),
    "gqa2_d64_s64": wl.WorkloadSpec("af7", 2, 4, 2, 64, 64, 1000, 4, headroom=128),
    "mha_d128_s64": wl.WorkloadSpec("af8", 3, 2, 2, 128, 64, 700, 3, L_min=1, headroom=128),
}


def _bits_equal(a, b):
    return torch.equal(a.contiguous().view(torch.int16), b.contiguous().view(torch.int16))


@pytest.mark.parametrize("name", list(APPEND_FUSED))
@pytest.mark.parametrize("splits", [0, 2, 5], indirect=True)
@pytest.mark.parametrize("fmt", FORMATS)
def test_append_and_decode_equals_separate_calls(oracle, built, name, splits, fmt):
    """ts_append_and_decode == ts_append_token_meta followed by ts_query_aware_decode:
    same outputs, same metadata, same pool contents, same lengths, step after step
    across page boundaries, including a sequence that runs out of room."""
    spec = wl.scaled(APPEND_FUSED[name], kv=fmt)
    print(f"[case] append+decode {name} {fmt} splits={splits}", flush=True)
    n_new = 36
    scale = 1.0 / math.sqrt(spec.d)
    sessions = []
    for _ in range(2):
        w = wl.make_workload(spec, DEV, seed=77, n_q=n_new, n_new=n_new, poison=0.0)
        sess = Session(w, poison_meta=False)
        if not spec.L_min:
            # every sequence owns all P_max pages here: sequence 0 is put two tokens
            # short of its capacity, so the third append must be refused
            sess.seq_lens[0] = w.P_max * spec.S - 2
        ts.build_page_meta(sess.layout)
        sessions.append(sess)
    a, f = sessions
    single = spec.B * spec.Hkv * max(splits, 1) <= 256
    assert ts.append_and_decode_launches(f.layout, f.w.K_max) == (1 if single else 2)
    units = [(b, h) for b in range(min(spec.B, 6)) for h in range(spec.Hkv)]
    for i in range(n_new):
        ts.append_token_meta(a.layout, a.w.k_new[i], a.w.v_new[i], advance_seq_lens=True)
        a.fused(scale, q_idx=i)
        w = f.w
        ts.append_and_decode(f.layout, w.k_new[i], w.v_new[i], w.q[i], w.topk, w.K_max, scale, f.out,
                             f.ws, topk_per_seq=w.topk_per_seq, scores_out=f.scores,
                             sel_out=f.sel, sel_count_out=f.sel_count)
        torch.cuda.synchronize()
        assert ts.workspace_status(f.ws) == 0 and ts.workspace_status(a.ws) == 0
        what = f"{name} step {i}"
        assert torch.equal(a.seq_lens, f.seq_lens), what
        assert torch.equal(a.sel_count, f.sel_count) and torch.equal(a.sel, f.sel), what
        assert _bits_equal(a.page_min, f.page_min) and _bits_equal(a.page_max, f.page_max), what
        assert _bits_equal(a.w.k_pool, f.w.k_pool) and _bits_equal(a.w.v_pool, f.w.v_pool), what
        assert torch.equal(a.scores, f.scores), what
        assert (a.out - f.out).abs().max().item() <= 1e-6, what
        if i in (0, 17, n_new - 1):
            compare_units(oracle, f, units, scale, q_idx=i, what=what)
    if not spec.L_min:
        assert int(f.seq_lens[0]) == f.w.P_max * spec.S      # stopped at capacity


MANY_UNITS = {
    # more units than resident workgroups: the build of the fused kernel that loops over
    # units (one workgroup per unit, units handed out by ticket), every (d, S) instance
    "d64_s16": wl.WorkloadSpec("mu1", 80, 4, 4, 64, 16, 700, 9, L_min=1, headroom=32),
    "d64_s32": wl.WorkloadSpec("mu2", 40, 16, 8, 64, 32, 900, 6, L_min=1, headroom=64),
    "d128_s16": wl.WorkloadSpec("mu3", 70, 4, 4, 128, 16, 500, 0, L_min=1, budget_frac=0.3,
                                headroom=32),
    "d128_s32": wl.WorkloadSpec("mu4", 36, 16, 8, 128, 32, 800, 5, L_min=1, headroom=64),
    "d64_s4": wl.WorkloadSpec("mu5", 80, 4, 4, 64, 4, 300, 11, L_min=1, headroom=32),
    "d64_s8": wl.WorkloadSpec("mu6", 40, 16, 8, 64, 8, 500, 0, L_min=1, budget_frac=0.2,
                              headroom=32),
    "d64_s64": wl.WorkloadSpec("mu7", 40, 16, 8, 64, 64, 1500, 5, L_min=1, headroom=128),
    "d128_s4": wl.WorkloadSpec("mu8", 36, 16, 8, 128, 4, 250, 14, L_min=1, headroom=32),
    "d128_s8": wl.WorkloadSpec("mu9", 70, 4, 4, 128, 8, 400, 0, L_min=1, budget_frac=0.3,
                               headroom=32),
    "d128_s64": wl.WorkloadSpec("mu10", 72, 4, 4, 128, 64, 1200, 4, L_min=1, headroom=128),
}


@pytest.mark.parametrize("name", list(MANY_UNITS))
@pytest.mark.parametrize("fmt", FORMATS)
def test_many_units_loop_build(oracle, built, name, fmt):
    spec = wl.scaled(MANY_UNITS[name], kv=fmt)
    print(f"[case] many units {name} {fmt}", flush=True)
    w = wl.make_workload(spec, DEV, seed=404, n_q=3, n_new=3)
    sess = Session(w)
    ts.build_page_meta(sess.layout)
    scale = 1.0 / math.sqrt(spec.d)
    n_units = spec.B * spec.Hkv
    assert n_units > 256
    assert ts.append_and_decode_launches(sess.layout, w.K_max) == 2   # append runs on its own
    rng = np.random.default_rng(9)
    picks = sorted(set(rng.integers(0, n_units, 10).tolist()) | {0, 255, 256, n_units - 1})
    units = [(u // spec.Hkv, u % spec.Hkv) for u in picks]
    for i in range(3):
        if i == 1:      # one step through the launch that also appends
            ts.append_and_decode(sess.layout, w.k_new[i], w.v_new[i], w.q[i], w.topk, w.K_max, scale,
                                 sess.out, sess.ws, topk_per_seq=w.topk_per_seq,
                                 scores_out=sess.scores, sel_out=sess.sel,
                                 sel_count_out=sess.sel_count)
        else:
            sess.fused(scale, q_idx=i)
        compare_units(oracle, sess, units, scale, q_idx=i, what=f"{name} launch {i}")
        # units are handed out longest sequence first: every one of them must have been
        # (the buffers start out as NaN / -7)
        assert torch.isfinite(sess.out).all() and int(sess.sel[:, :, 0].min()) >= 0
        sess.out.fill_(float("nan"))
        sess.sel.fill_(-7)


CLUSTER_LOOP = {
    # 129 to 255 units in clusters of two or more workgroups (forced: the library's own
    # plan keeps a launch resident and would give these batches one workgroup per unit):
    # more clusters than fit on the device at once, so each works through several units
    "d64_s16": wl.WorkloadSpec("cl1", 40, 16, 4, 64, 16, 1800, 20, L_min=1, headroom=32),
    "d128_s32": wl.WorkloadSpec("cl2", 22, 16, 8, 128, 32, 2600, 0, L_min=1, budget_frac=0.2,
                                headroom=64),
    "d64_s4_walk": wl.WorkloadSpec("cl3", 36, 8, 4, 64, 4, 700, 30, keys="walk", L_min=1,
                                   headroom=32),
}


@pytest.mark.parametrize("name,splits", [("d64_s16", 2), ("d128_s32", 2), ("d64_s4_walk", 3),
                                         ("d64_s16", 5)], indirect=["splits"])
@pytest.mark.parametrize("fmt", FORMATS)
def test_clusters_that_work_through_several_units(oracle, built, name, splits, fmt):
    """The looping build of the fused kernel WITH clusters: more clusters than the device
    holds at once, so each takes several units in turn (score exchange, bin counting and
    the tagged partials once per unit, the launch tag fixed at the first).  Three launches
    in a row, the middle one with the append in front; sampled units against the oracle,
    and every unit must have been written."""
    spec = wl.scaled(CLUSTER_LOOP[name], kv=fmt)
    print(f"[case] cluster loop {name} splits={splits} {fmt}", flush=True)
    w = wl.make_workload(spec, DEV, seed=505, n_q=3, n_new=3)
    sess = Session(w)
    ts.build_page_meta(sess.layout)
    scale = 1.0 / math.sqrt(spec.d)
    n_units = spec.B * spec.Hkv
    assert 128 < n_units < 256
    assert ts.append_and_decode_launches(sess.layout, w.K_max) == 2   # not all resident at once
    rng = np.random.default_rng(10)
    picks = sorted(set(rng.integers(0, n_units, 10).tolist()) | {0, 127, 128, n_units - 1})
    units = [(u // spec.Hkv, u % spec.Hkv) for u in picks]
    for i in range(3):
        if i == 1:
            ts.append_and_decode(sess.layout, w.k_new[i], w.v_new[i], w.q[i], w.topk, w.K_max, scale,
                                 sess.out, sess.ws, topk_per_seq=w.topk_per_seq,
                                 scores_out=sess.scores, sel_out=sess.sel,
                                 sel_count_out=sess.sel_count)
        else:
            sess.fused(scale, q_idx=i)
        compare_units(oracle, sess, units, scale, q_idx=i, what=f"{name} launch {i}")
        assert torch.isfinite(sess.out).all() and int(sess.sel[:, :, 0].min()) >= 0
        sess.out.fill_(float("nan"))
        sess.sel.fill_(-7)


def test_query_sums_read_back_through_one_hot_boxes(built):
    """Boxes are overwritten so that page c has max = unit vector c and min = 0: the
    score of page c then equals Qp_c = sum over the group's heads of max(q_c, 0), read
    back exactly.  More units than workgroups, many launches: every workgroup scores
    several units in a row, and any mix-up of one unit's query staging with the
    next phase of another wave shows as a wrong or zero channel."""
    print("[case] one-hot probe", flush=True)
    spec = wl.WorkloadSpec("probe", 72, 8, 4, 128, 16, 2100, 8, headroom=64)
    n = 12
    w = wl.make_workload(spec, DEV, seed=5, n_q=n, n_new=n, poison=0.0)
    sess = Session(w, poison_meta=False)
    ts.build_page_meta(sess.layout)
    sess.page_min[:, :, :128] = 0
    sess.page_max[:, :, :128] = torch.eye(128, dtype=torch.bfloat16, device=DEV)[None, None]
    G = spec.Hq // spec.Hkv
    scale = 1.0 / math.sqrt(spec.d)
    for i in range(n):
        if i % 2:
            sess.fused(scale, q_idx=i)
        else:
            ts.append_and_decode(sess.layout, w.k_new[i], w.v_new[i], w.q[i], w.topk, w.K_max, scale,
                                 sess.out, sess.ws, scores_out=sess.scores, sel_out=sess.sel,
                                 sel_count_out=sess.sel_count)
        torch.cuda.synchronize()
        assert ts.workspace_status(sess.ws) == 0
        qp = w.q[i].float().clamp(min=0).view(spec.B, spec.Hkv, G, spec.d).sum(2)
        assert torch.equal(sess.scores[:, :, :128], qp), f"launch {i}"


LSE_ATOL = 2e-3   # log of the softmax denominator, absolute (fp32 sums of bf16 products)


@pytest.mark.parametrize("name", ["mha_d64_s16", "gqa8_d64_s32_walk", "mha_d128_s16_ragged",
                                  "gqa4_d128_s32", "k_exceeds_p", "gqa8_d64_s4", "mha_d128_s8",
                                  "gqa4_d64_s64", "mha_d128_s64"])
@pytest.mark.parametrize("fmt", FORMATS)
def test_dense_baseline_matches_oracle(oracle, built, name, fmt):
    """ts_dense_decode_attention (attention over the whole cache, the comparison the
    paper measures against) against the oracle's dense softmax attention, output and
    log-denominator."""
    spec = wl.scaled(REDUCED[name], kv=fmt)
    print(f"[case] dense {name} {fmt}", flush=True)
    w = wl.make_workload(spec, DEV, seed=11, n_q=1)
    sess = Session(w)
    scale = 1.0 / math.sqrt(spec.d)
    ws = ts.new_dense_workspace(sess.layout, DEV)
    lse = torch.full((spec.B, spec.Hq), float("nan"), dtype=torch.float32, device=DEV)
    ts.dense_decode_attention(sess.layout, w.q[0], scale, sess.out, ws, lse_out=lse)
    torch.cuda.synchronize()
    K, V = wl.logical_kv(w)
    with oracle.element_format(fmt):
        ref, ref_lse = oracle.dense_decode_attention(wl.bits(w.q[0]), wl.bits(K), wl.bits(V),
                                                     w.seq_lens.cpu().numpy(), scale,
                                                     return_lse=True)
    err = np.abs(sess.out.cpu().numpy().astype(np.float64) - ref).max()
    assert err <= 2e-3, f"dense attention off by {err}"
    err = np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse).max()
    assert err <= LSE_ATOL, f"dense log-denominator off by {err}"
    # a second call on the same workspace (counters left re-armed), without the extra output
    first = sess.out.clone()
    ts.dense_decode_attention(sess.layout, w.q[0], scale, sess.out, ws)
    torch.cuda.synchronize()
    assert torch.equal(first, sess.out)


@pytest.mark.parametrize("name", ["gqa8_d64_s16_offset", "gqa8_d64_s32_walk", "mha_d128_s16_ragged",
                                  "gqa2_d128_s4", "mha_d64_s8_ragged", "gqa4_d64_s64"])
@pytest.mark.parametrize("splits", [0, 3], indirect=True)
def test_selected_mass_matches_oracle(oracle, built, name, splits):
    """The log-denominator of ts_sparse_decode_attention over the selected pages, and
    from it the share of the dense softmax mass the selection captures,
    exp(lse_selected - lse_dense), against the oracle on the same selection."""
    spec = REDUCED[name]
    print(f"[case] selected mass {name} splits={splits}", flush=True)
    w = wl.make_workload(spec, DEV, seed=13, n_q=1)
    sess = Session(w)
    ts.build_page_meta(sess.layout)
    scale = 1.0 / math.sqrt(spec.d)
    ts.score_pages(sess.layout, w.q[0], sess.scores)
    ts.select_topk_pages(sess.layout, sess.scores, w.topk, w.K_max, sess.sel, sess.sel_count,
                         topk_per_seq=w.topk_per_seq)
    lse_s = torch.full((spec.B, spec.Hq), float("nan"), dtype=torch.float32, device=DEV)
    lse_d = torch.full_like(lse_s, float("nan"))
    ts.sparse_decode_attention(sess.layout, w.q[0], sess.sel, sess.sel_count, w.K_max, scale,
                               sess.out, sess.ws, lse_out=lse_s)
    dws = ts.new_dense_workspace(sess.layout, DEV)
    dense_out = torch.empty_like(sess.out)
    ts.dense_decode_attention(sess.layout, w.q[0], scale, dense_out, dws, lse_out=lse_d)
    torch.cuda.synchronize()
    K, V = wl.logical_kv(w)
    args = (wl.bits(w.q[0]), wl.bits(K), wl.bits(V))
    lens = w.seq_lens.cpu().numpy()
    o_out, o_lse = oracle.sparse_decode_attention(*args, sess.sel.cpu().numpy(),
                                                  sess.sel_count.cpu().numpy(), lens, spec.S, scale,
                                                  return_lse=True)
    _, o_dense = oracle.dense_decode_attention(*args, lens, scale, return_lse=True)
    assert np.abs(sess.out.cpu().numpy() - o_out).max() <= 2e-3
    assert np.abs(lse_s.cpu().numpy() - o_lse).max() <= LSE_ATOL
    mass = torch.exp(lse_s - lse_d).cpu().numpy().astype(np.float64)
    o_mass = np.exp(o_lse - o_dense)
    assert np.all(mass <= 1.0 + 1e-2) and np.abs(mass - o_mass).max() <= 5e-3


@pytest.mark.parametrize("name", ["gqa8_d64_s16_offset", "mha_d128_s16_ragged", "gqa8_d64_s4",
                                  "gqa4_d64_s64"])
@pytest.mark.parametrize("splits", [0, 3], indirect=True)
def test_bf16_output_is_the_rounded_fp32_output(built, name, splits):
    """out_format = TS_OUT_BF16: every attention entry point writes its fp32 result (the
    one the oracle comparisons above cover) rounded to bf16, nearest even: bit-equal to
    torch's conversion of the fp32 output of the same call."""
    spec = REDUCED[name]
    print(f"[case] bf16 out {name} splits={splits}", flush=True)
    w = wl.make_workload(spec, DEV, seed=17, n_q=1, n_new=1)
    a = Session(w)
    ts.build_page_meta(a.layout)
    lay16 = ts.make_layout(spec.B, spec.Hq, spec.Hkv, spec.d, spec.S, w.P_max, w.k_pool, w.v_pool,
                           w.block_table, a.seq_lens, a.page_min, a.page_max,
                           out_format=ts.TS_OUT_BF16)
    out16 = torch.full((spec.B, spec.Hq, spec.d), float("nan"), dtype=torch.bfloat16, device=DEV)
    scale = 1.0 / math.sqrt(spec.d)
    a.fused(scale)
    ts.query_aware_decode(lay16, w.q[0], w.topk, w.K_max, scale, out16, a.ws,
                          topk_per_seq=w.topk_per_seq)
    torch.cuda.synchronize()
    assert _bits_equal(out16, a.out.to(torch.bfloat16)), "fused"
    out16.fill_(float("nan"))
    ts.sparse_decode_attention(a.layout, w.q[0], a.sel, a.sel_count, w.K_max, scale, a.out, a.ws)
    ts.sparse_decode_attention(lay16, w.q[0], a.sel, a.sel_count, w.K_max, scale, out16, a.ws)
    torch.cuda.synchronize()
    assert _bits_equal(out16, a.out.to(torch.bfloat16)), "staged"
    dws = ts.new_dense_workspace(a.layout, DEV)
    ts.dense_decode_attention(a.layout, w.q[0], scale, a.out, dws)
    ts.dense_decode_attention(lay16, w.q[0], scale, out16, dws)
    torch.cuda.synchronize()
    assert _bits_equal(out16, a.out.to(torch.bfloat16)), "dense"


@pytest.mark.parametrize("splits", [0, 4], indirect=True)
def test_graph_replays_match_eager(built, splits):
    """A captured HIP graph of decode steps (the form bench.py times) replayed several
    times, with eager work and synchronisations in between: every replay must equal
    the same steps issued eagerly on a twin.  The launch tag of the score exchange is
    device state for exactly this reason (kernel arguments are frozen in a graph)."""
    print(f"[case] graph replay splits={splits}", flush=True)
    spec = wl.WorkloadSpec("graph", 3, 8, 2, 64, 16, 1200, 10, keys="offset", headroom=160)
    scale = 1.0 / math.sqrt(spec.d)
    twins = []
    for _ in range(2):
        w = wl.make_workload(spec, DEV, seed=21, n_q=2, n_new=2, poison=0.0)
        sess = Session(w, poison_meta=False)
        ts.build_page_meta(sess.layout)
        twins.append(sess)
    e, g = twins

    def steps(sess):     # two decode steps: one launch each, then a plain fused call
        w = sess.w
        ts.append_and_decode(sess.layout, w.k_new[0], w.v_new[0], w.q[0], w.topk, w.K_max, scale,
                             sess.out, sess.ws)
        ts.append_and_decode(sess.layout, w.k_new[1], w.v_new[1], w.q[1], w.topk, w.K_max, scale,
                             sess.out, sess.ws)
        ts.query_aware_decode(sess.layout, w.q[0], w.topk, w.K_max, scale, sess.out, sess.ws,
                              scores_out=sess.scores, sel_out=sess.sel,
                              sel_count_out=sess.sel_count)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        steps(g)                       # warm-up on the capture stream (also advances g)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            steps(g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    steps(e)                           # e catches up with the warm-up
    for r in range(5):
        graph.replay()
        steps(e)
        torch.cuda.synchronize()
        assert ts.workspace_status(g.ws) == 0 and ts.workspace_status(e.ws) == 0
        assert torch.equal(e.seq_lens, g.seq_lens), f"replay {r}"
        assert torch.equal(e.sel, g.sel) and torch.equal(e.scores, g.scores), f"replay {r}"
        assert _bits_equal(e.page_min, g.page_min) and _bits_equal(e.w.k_pool, g.w.k_pool)
        assert (e.out - g.out).abs().max().item() <= 1e-6, f"replay {r}"
        # unrelated eager work between replays
        torch.empty(1 << 20, device=DEV).normal_().sum().item()


@pytest.mark.parametrize("profile", ["outlier_group", "hidden_peak", "ramp", "all_equal"])
@pytest.mark.parametrize("splits", [4, 16], indirect=True)
def test_selection_where_a_member_misjudges_the_score_range(oracle, built, splits, profile):
    """With a cluster, every member bins the scores over a range estimated from its own
    share of the pages (every g-th group of eight).  Boxes are overwritten so that page
    j scores exactly G * s_j, with profiles chosen so that some members misjudge the
    range badly: one group of very large scores that a single member sees (its bins
    then lump all other pages together, with heavy ties at the cut); forty large scores
    in groups only two members see (for the others they crowd into the top bin, and the
    cut falls inside it); a ramp; all scores equal.  Every member must still arrive at
    the exact top-K (ties to the lower page), or pages would be attended twice or not
    at all: scores, selection and output are compared with the oracle's."""
    print(f"[case] misjudged range {profile} splits={splits}", flush=True)
    spec = wl.WorkloadSpec("range", 2, 4, 2, 64, 16, 16 * 600, 32, headroom=0)
    w = wl.make_workload(spec, DEV, seed=31, n_q=1, n_new=1, poison=0.0)
    sess = Session(w, poison_meta=False)
    ts.build_page_meta(sess.layout)
    P, G, g = w.P_max, spec.Hq // spec.Hkv, splits
    rng = np.random.default_rng(3)
    s = rng.integers(-8, 9, size=P).astype(np.float32)           # heavy ties
    topk = 32
    if profile == "outlier_group":
        first = 8 * (g - 1)                                       # one group of the last member's
        s[first:first + 8] = 200 + np.arange(8)
    elif profile == "hidden_peak":
        groups = [gi for gi in range(P // 8) if gi % g in (0, 1)][3:8]   # five groups, two members
        for gi in groups:
            s[8 * gi:8 * gi + 8] = 100 + (np.arange(8) % 7)
        topk = 20
    elif profile == "ramp":
        s = (np.arange(P) // 3).astype(np.float32)               # top pages all at the end
    else:
        s[:] = 3.0
    box = torch.zeros((P, spec.d), dtype=torch.float32)
    box[:, 0] = torch.from_numpy(s)
    box = box.to(sess.page_min.dtype).to(DEV)
    sess.page_min[:] = box[None, None]
    sess.page_max[:] = box[None, None]
    q = w.q[0].clone()
    q[:, :, 0] = 1.0                                             # score = sum over the group of s_j
    scale = 1.0 / math.sqrt(spec.d)
    ts.query_aware_decode(sess.layout, q, topk, w.K_max, scale, sess.out, sess.ws,
                          scores_out=sess.scores, sel_out=sess.sel, sel_count_out=sess.sel_count)
    torch.cuda.synchronize()
    assert ts.workspace_status(sess.ws) == 0
    lens = sess.seq_lens.cpu().numpy()
    scores = sess.scores.cpu().numpy()
    assert np.array_equal(scores, np.broadcast_to(G * s, scores.shape)), "scores"
    sel, cnt, _ = oracle.select_topk_pages(scores.astype(np.float64), lens, spec.S, topk, w.K_max)
    assert np.array_equal(sess.sel_count.cpu().numpy(), cnt)
    assert np.array_equal(sess.sel.cpu().numpy(), sel), "selection"
    K, V = wl.logical_kv(w)
    ref = oracle.sparse_decode_attention(wl.bits(q), wl.bits(K), wl.bits(V), sel, cnt, lens, spec.S,
                                         scale)
    assert_out_close(sess.out.cpu().numpy(), ref, what=profile)


@pytest.mark.parametrize("splits", [4], indirect=True)
def test_launch_tag_wraps_past_zero(built, splits):
    """The words a cluster exchanges carry a 32-bit launch count as their tag, and 0
    marks a word nobody has written since the workspace was initialised.  A workspace
    whose count is about to wrap (set by hand here: word 16 of the control block at the
    head of the workspace) must carry on across the wrap like a fresh one."""
    print("[case] launch tag wrap", flush=True)
    spec = wl.WorkloadSpec("wrap", 2, 8, 2, 64, 16, 1500, 12, keys="offset", headroom=64)
    scale = 1.0 / math.sqrt(spec.d)
    twins = []
    for _ in range(2):
        w = wl.make_workload(spec, DEV, seed=77, n_q=6, n_new=1, poison=0.0)
        sess = Session(w, poison_meta=False)
        ts.build_page_meta(sess.layout)
        twins.append(sess)
    fresh, old = twins
    old.ws.view(torch.int32)[16] = -3          # three launches before 2^32
    torch.cuda.synchronize()
    for i in range(6):
        for sess in twins:
            w = sess.w
            ts.query_aware_decode(sess.layout, w.q[i], w.topk, w.K_max, scale, sess.out, sess.ws,
                                  scores_out=sess.scores, sel_out=sess.sel,
                                  sel_count_out=sess.sel_count)
        torch.cuda.synchronize()
        assert ts.workspace_status(fresh.ws) == 0 and ts.workspace_status(old.ws) == 0, f"launch {i}"
        assert torch.equal(fresh.sel, old.sel) and torch.equal(fresh.scores, old.scores), f"launch {i}"
        assert torch.equal(fresh.out, old.out), f"launch {i}"
    assert int(old.ws.view(torch.int32)[16]) == 4 and int(fresh.ws.view(torch.int32)[16]) == 6


def test_fused_agrees_with_staged_on_random_shapes(built):
    """150 random shapes (head_dim, page size, group size, lengths, K, key structure,
    always-kept pages, coarsely quantised boxes for heavy ties) with random cluster
    sizes: the fused kernel's selection must equal, entry for entry, what the staged
    selection (itself bit-exact against the oracle in the tests above) makes of the
    fused kernel's scores, and its output must agree with the staged attention over that
    selection.  Every member of a cluster bins the scores in its own way; this is the
    test that they still agree whatever the shape."""
    rng = np.random.default_rng(2024)
    for case in range(150):
        d = int(rng.choice([64, 128]))
        S = int(rng.choice([4, 8, 16, 32, 64]))
        Hkv, G, B = int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 4, 8])), int(rng.integers(1, 4))
        L = int(rng.integers(S * 3, S * 400))
        K = min(int(rng.integers(1, max(2, (L + S - 1) // S))), 200)
        keys = str(rng.choice(["normal", "offset", "walk"]))
        splits = int(rng.choice([0, 0, 2, 3, 4, 8, 16]))
        keep = (int(rng.integers(0, 3)), int(rng.integers(0, 3))) if rng.random() < 0.3 else (0, 0)
        if case % 10 == 9:    # one or two long units, many kept pages: the library's largest clusters
            B, Hkv, splits = 1, int(rng.choice([1, 2])), 0
            L = int(rng.integers(S * 300, S * 3000))
            K = int(rng.integers(64, 600))
        spec = wl.WorkloadSpec("rand", B, Hkv * G, Hkv, d, S, L, K, keys=keys,
                               L_min=(1 if rng.random() < 0.5 else 0), headroom=S)
        what = f"case {case}: {spec} splits={splits} keep={keep}"
        print(f"[case] random shape {case}", flush=True)
        w = wl.make_workload(spec, DEV, seed=int(rng.integers(1 << 30)), n_q=1, n_new=1, poison=0.0)
        a = Session(w, poison_meta=False, keep=keep)
        ts.build_page_meta(a.layout)
        if rng.random() < 0.3:
            a.page_min.copy_((a.page_min.float() * 2).round() / 2)
            a.page_max.copy_((a.page_max.float() * 2).round() / 2)
        scale = 1.0 / math.sqrt(d)
        ts.set_tuning(0, splits, 0)
        try:
            ws = ts.new_workspace(a.layout, w.K_max, DEV)
            ts.query_aware_decode(a.layout, w.q[0], w.topk, w.K_max, scale, a.out, ws,
                                  topk_per_seq=w.topk_per_seq, scores_out=a.scores, sel_out=a.sel,
                                  sel_count_out=a.sel_count)
            sel2, cnt2, out2 = torch.full_like(a.sel, -7), torch.full_like(a.sel_count, -7), torch.full_like(a.out, float("nan"))
            ts.select_topk_pages(a.layout, a.scores, w.topk, w.K_max, sel2, cnt2,
                                 topk_per_seq=w.topk_per_seq)
            ts.sparse_decode_attention(a.layout, w.q[0], sel2, cnt2, w.K_max, scale, out2, ws)
            torch.cuda.synchronize()
            assert ts.workspace_status(ws) == 0, what
        finally:
            ts.set_tuning(0, 0, 0)
        assert torch.equal(a.sel_count, cnt2) and torch.equal(a.sel, sel2), what
        assert torch.isfinite(a.out).all() and (a.out - out2).abs().max().item() <= 2e-5, what


def test_append_and_decode_agrees_with_two_calls_on_random_shapes(built):
    """90 random shapes in all three cache formats, three decode steps each:
    ts_append_and_decode on one twin, ts_append_token_meta + ts_query_aware_decode on the
    other.  Pool, scales, metadata, lengths and selection must come out bit-equal and the
    outputs agree (the in-launch append splices the token into registers, and for the
    INT8 cache quantises it in three different waves)."""
    rng = np.random.default_rng(77)

    def twin(spec, seed):
        w = wl.make_workload(spec, DEV, seed=seed, n_q=3, n_new=3, poison=0.0)
        meta_dtype = torch.bfloat16 if spec.kv == "int8" else w.k_pool.dtype
        pmin = torch.zeros((spec.B, spec.Hkv, w.P_max, spec.d), dtype=meta_dtype, device=DEV)
        pmax = torch.zeros_like(pmin)
        lens = w.seq_lens.clone()
        lay = ts.make_layout(spec.B, spec.Hq, spec.Hkv, spec.d, spec.S, w.P_max, w.k_pool, w.v_pool,
                             w.block_table, lens, pmin, pmax, k_scale=w.k_scale, v_scale=w.v_scale)
        ts.build_page_meta(lay)
        out = torch.full((spec.B, spec.Hq, spec.d), float("nan"), dtype=torch.float32, device=DEV)
        sel = torch.full((spec.B, spec.Hkv, w.K_max), -7, dtype=torch.int32, device=DEV)
        return w, lay, pmin, pmax, lens, out, sel, ts.new_workspace(lay, w.K_max, DEV)

    for case in range(90):
        d, S = int(rng.choice([64, 128])), int(rng.choice([4, 8, 16, 32, 64]))
        Hkv, G, B = int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 4, 8])), int(rng.integers(1, 4))
        L = int(rng.integers(S * 3, S * 300))
        K = min(int(rng.integers(1, max(2, (L + S - 1) // S))), 150)
        fmt, splits = str(rng.choice(["bf16", "fp16", "int8"])), int(rng.choice([0, 0, 2, 4, 8]))
        spec = wl.WorkloadSpec("rand", B, Hkv * G, Hkv, d, S, L, K,
                               keys=str(rng.choice(["normal", "offset", "walk"])),
                               L_min=(1 if rng.random() < 0.5 else 0), headroom=3 * S, kv=fmt)
        seed = int(rng.integers(1 << 30))
        print(f"[case] random append {case} {fmt}", flush=True)
        scale = 1.0 / math.sqrt(d)
        ts.set_tuning(0, splits, 0)
        try:
            wa, la, amin, amax, alens, aout, asel, aws = twin(spec, seed)
            wf, lf, fmin, fmax, flens, fout, fsel, fws = twin(spec, seed)
            for i in range(3):
                what = f"case {case} step {i}: {spec} splits={splits}"
                ts.append_token_meta(la, wa.k_new[i], wa.v_new[i], advance_seq_lens=True)
                ts.query_aware_decode(la, wa.q[i], wa.topk, wa.K_max, scale, aout, aws,
                                      topk_per_seq=wa.topk_per_seq, sel_out=asel)
                ts.append_and_decode(lf, wf.k_new[i], wf.v_new[i], wf.q[i], wf.topk, wf.K_max, scale,
                                     fout, fws, topk_per_seq=wf.topk_per_seq, sel_out=fsel)
                torch.cuda.synchronize()
                assert ts.workspace_status(aws) == 0 and ts.workspace_status(fws) == 0, what
                assert torch.equal(alens, flens), what
                assert torch.equal(wa.k_pool, wf.k_pool) and torch.equal(wa.v_pool, wf.v_pool), what
                assert _bits_equal(amin, fmin) and _bits_equal(amax, fmax), what
                if fmt == "int8":
                    assert torch.equal(wa.k_scale, wf.k_scale) and torch.equal(wa.v_scale, wf.v_scale), what
                assert torch.equal(asel, fsel), what
                assert torch.isfinite(fout).all() and (aout - fout).abs().max().item() <= 2e-5, what
        finally:
            ts.set_tuning(0, 0, 0)


def test_workgroups_are_dealt_out_to_the_xcds_in_turn(built):
    """The fused kernel puts the workgroups of one cluster on ids that are congruent modulo
    the number of XCDs, on the understanding that the hardware deals consecutive ids out to
    the XCDs in turn (starting wherever the previous launch left off).  Nothing but speed
    depends on it; this is the check that it holds here."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    xcds = cus // 32 if cus >= 64 and cus % 32 == 0 else 1
    for n in (16, 256, 1024):
        ids = ts.debug_xcc_ids(n, DEV)
        torch.cuda.synchronize()
        want = (torch.arange(n, dtype=torch.int32, device=DEV) + ids[0]) % xcds
        assert torch.equal(ids, want), f"{n} workgroups: XCDs {ids[:16].tolist()} ..."


@pytest.mark.parametrize("name", ["gqa8_d64_s16_offset", "mha_d64_s16"])
def test_one_workgroup_per_unit_on_request(oracle, built, name):
    """ts_layout.cluster_size = 1 (a device shared with other kernels): no workgroup waits for
    another, whatever the batch; results as always.  cluster_size = 3 overrides the plan the
    other way."""
    spec = REDUCED[name]
    w = wl.make_workload(spec, DEV, seed=77, n_q=1, n_new=1)
    units = [(b, h) for b in range(spec.B) for h in range(spec.Hkv)]
    scale = 1.0 / math.sqrt(spec.d)
    try:
        ts.set_tuning(0, 8, 0)       # the layout's own value must win over the process-wide one
        for cs in (1, 3):
            print(f"[case] cluster_size={cs} {name}", flush=True)
            sess = Session(w, cluster_size=cs)
            ts.build_page_meta(sess.layout)
            sess.fused(scale)
            compare_units(oracle, sess, units, scale, what=f"cluster_size={cs}/{name}")
    finally:
        ts.set_tuning(0, 0, 0)


@pytest.mark.parametrize("topk", [3, 12, 31, 32, 33, 64, 72, 130, 257])
@pytest.mark.parametrize("cluster", [1, 2])
def test_every_length_of_a_wave_s_fragment_list(oracle, built, topk, cluster):
    """The attention's ring of buffers is laid out by how many of them are in use: fewer
    fragments than buffers, exactly a ring, whole rounds, a round refilled in part, a last
    partial ring.  With one or two workgroups per unit and these budgets a wave gets 0 to
    33 fragments, which walks through every one of those paths (S = 16, one page a fragment)."""
    print(f"[case] ring topk={topk} cluster={cluster}", flush=True)
    spec = wl.WorkloadSpec("ring", 2, 8, 2, 64, 16, 6000, topk, keys="walk", headroom=40)
    w = wl.make_workload(spec, DEV, seed=500 + topk, n_q=1, n_new=1)
    units = [(b, h) for b in range(spec.B) for h in range(spec.Hkv)]
    scale = 1.0 / math.sqrt(spec.d)
    sess = Session(w, cluster_size=cluster)
    ts.build_page_meta(sess.layout)
    sess.fused(scale)
    compare_units(oracle, sess, units, scale, what=f"ring/topk={topk}/cluster={cluster}")
    fused_out = sess.out.clone()
    sess.staged(scale)     # the staged attention kernel walks the same ring
    compare_units(oracle, sess, units, scale, what=f"ring/topk={topk}/staged")
    assert torch.equal(sess.out, fused_out) or float((sess.out - fused_out).abs().max()) <= 2e-3


@pytest.mark.parametrize("cluster", [5, 6, 9, 17, 18, 24, 40])
@pytest.mark.parametrize("shape", ["d64_g4", "d128_g8"])
def test_cluster_merge_in_batches(oracle, built, cluster, shape):
    """The cluster's last member takes the other members' partial results four at a time
    (up to five members) or sixteen at a time: cluster sizes on either side of both limits,
    two and three batches, members that have no page at all, a head handled by one wave
    (d = 64) and by two (d = 128, where a thread also works through two channels' worth of
    the unit's G * d outputs)."""
    print(f"[case] merge batches cluster={cluster} {shape}", flush=True)
    spec = (wl.WorkloadSpec("merge64", 2, 8, 2, 64, 16, 5000, 48, keys="walk", headroom=40) if shape == "d64_g4"
            else wl.WorkloadSpec("merge128", 1, 16, 2, 128, 16, 4000, 36, keys="offset", headroom=40))
    w = wl.make_workload(spec, DEV, seed=700 + cluster, n_q=1, n_new=1)
    units = [(b, h) for b in range(spec.B) for h in range(spec.Hkv)]
    scale = 1.0 / math.sqrt(spec.d)
    sess = Session(w, cluster_size=cluster)
    ts.build_page_meta(sess.layout)
    for step in range(2):     # the second launch finds the first one's words in the workspace
        sess.out.fill_(float("nan"))
        sess.fused(scale)
        compare_units(oracle, sess, units, scale, what=f"merge/cluster={cluster}/{shape}/launch {step}")


def test_an_expired_wait_raises_the_sticky_word_and_the_launch_still_ends(oracle, built):
    """ts_layout.wait_limit = 1 lets a workgroup give up on its partners after two looks.  Such a
    launch must still run to its end (nothing hangs, nothing is read out of bounds) and
    report itself through ts_workspace_status; after ts_workspace_init the same workspace
    serves a normal launch again.  The limit is made to bite from the host: with 33 pages to
    keep out of a list laid out for 40 and clusters of eight, the cluster's last member, the
    one that merges, has no page of its own and looks for its partners' partial results
    while they are still fetching theirs."""
    spec = REDUCED["gqa8_d64_s16_offset"]      # topk (= the list's stride) is 40
    w = wl.make_workload(spec, DEV, seed=91, n_q=1, n_new=1)
    assert w.K_max == 40
    units = [(b, h) for b in range(spec.B) for h in range(spec.Hkv)]
    scale = 1.0 / math.sqrt(spec.d)
    hasty = Session(w, cluster_size=8, wait_limit=1)
    ts.build_page_meta(hasty.layout)
    expired = 0
    for attempt in range(8):
        print(f"[case] expiring wait, try {attempt}", flush=True)
        ts.query_aware_decode(hasty.layout, w.q[0], 33, w.K_max, scale, hasty.out, hasty.ws)
        torch.cuda.synchronize()
        if ts.workspace_status(hasty.ws) != 0:
            expired += 1
            ts.workspace_init(hasty.ws)
            torch.cuda.synchronize()
            assert ts.workspace_status(hasty.ws) == 0
    assert expired > 0, "no launch ran into a two-look limit"
    # the same workspace, patient again
    patient = Session(w, cluster_size=8)
    ts.build_page_meta(patient.layout)
    patient.ws = hasty.ws
    patient.fused(scale)
    compare_units(oracle, patient, units, scale, what="after an expired launch")


@pytest.mark.parametrize("B,Hkv", [(40, 4), (25, 4), (24, 8), (50, 4), (16, 4), (4, 4)])
def test_plan_keeps_the_launch_resident(built, B, Hkv):
    """Up to 256 units the library sizes its clusters so that every workgroup of the
    launch is resident at once (the members of a cluster wait for each other; clusters
    that do not fit would take the units in turns, which measured up to 40 % slower):
    ts_append_and_decode is then a single launch."""
    spec = wl.WorkloadSpec("plan", B, Hkv * 4, Hkv, 64, 16, 2048, 32, headroom=32)
    w = wl.make_workload(spec, DEV, seed=1, n_q=1, n_new=1, poison=0.0)
    sess = Session(w, poison_meta=False)
    assert ts.append_and_decode_launches(sess.layout, w.K_max) == 1


def test_degenerate_lengths(oracle, built):
    """Empty sequence, single token, exactly one page, one token past a page."""
    print("[case] degenerate", flush=True)
    spec = wl.WorkloadSpec("deg", 5, 4, 2, 64, 16, 40, 2, headroom=8)
    w = wl.make_workload(spec, DEV, seed=5)
    sess = Session(w)
    sess.seq_lens.copy_(torch.tensor([0, 1, 16, 17, 40], dtype=torch.int32))
    ts.build_page_meta(sess.layout)
    units = [(b, h) for b in range(spec.B) for h in range(spec.Hkv)]
    sess.fused(0.125)
    compare_units(oracle, sess, units, 0.125, what="degenerate/fused")
    assert torch.all(sess.out[0] == 0)          # no token: zeros
    sess.staged(0.125)
    compare_units(oracle, sess, units, 0.125, what="degenerate/staged")


@pytest.mark.parametrize("S", [4, 8, 64])
def test_full_size_other_page_sizes(oracle, built, S):
    """The TinyLLaMA-shaped workload with the page size of the paper's page-size
    ablation (Table 7: 16K context, budget 2048 tokens), default launch shape,
    sampled units; one step through the launch that appends."""
    spec = wl.scaled(wl.SPECS["tinyllama"], S=S, topk=2048 // S)
    print(f"[case] full tinyllama S={S}", flush=True)
    w = wl.make_workload(spec, DEV, seed=1200 + S, n_q=2, n_new=1)
    sess = Session(w)
    ts.build_page_meta(sess.layout)
    scale = 1.0 / math.sqrt(spec.d)
    units = full_size_units(w, "tinyllama")
    sess.fused(scale, q_idx=1)
    compare_units(oracle, sess, units, scale, q_idx=1, what=f"full/S{S}")
    ts.append_and_decode(sess.layout, w.k_new[0], w.v_new[0], w.q[0], w.topk, w.K_max, scale,
                         sess.out, sess.ws, scores_out=sess.scores, sel_out=sess.sel,
                         sel_count_out=sess.sel_count)
    compare_units(oracle, sess, units, scale, q_idx=0, what=f"full/S{S}/append")


@pytest.mark.parametrize("name", ["tinyllama", "ragged"])
def test_full_size_fp16(oracle, built, name):
    """Benchmark workloads at full size with IEEE-half tensors, default launch shapes: one
    step through ts_append_and_decode, the same units as test_full_size_sampled."""
    spec = wl.scaled(wl.SPECS[name], kv="fp16")
    print(f"[case] full fp16 {name}", flush=True)
    w = wl.make_workload(spec, DEV, seed=1700, n_q=2, n_new=1)
    sess = Session(w, poison_meta=(name != "ragged"))
    ts.build_page_meta(sess.layout)
    scale = 1.0 / math.sqrt(spec.d)
    ts.append_and_decode(sess.layout, w.k_new[0], w.v_new[0], w.q[1], w.topk, w.K_max, scale,
                         sess.out, sess.ws, topk_per_seq=w.topk_per_seq, scores_out=sess.scores,
                         sel_out=sess.sel, sel_count_out=sess.sel_count)
    compare_units(oracle, sess, full_size_units(w, name), scale, q_idx=1, what=f"full fp16/{name}")


FULL = ["tiny", "gpt2_345m", "tinyllama", "longctx", "ragged"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_sampled(oracle, built, name):
    """The five benchmark workloads at full size, default launch shapes: EVERY unit of the four
    small batches, and of the ragged batch every KV head of 20 sequences (shortest, longest, the
    ticket boundaries), against the oracle."""
    spec = wl.SPECS[name]
    print(f"[case] full {name}", flush=True)
    w = wl.make_workload(spec, DEV, seed=1000 + FULL.index(name), n_q=2, n_new=1)
    sess = Session(w, poison_meta=(name != "ragged"))
    ts.build_page_meta(sess.layout)
    scale = 1.0 / math.sqrt(spec.d)
    if name == "ragged":      # the serving step: append one token per sequence, then decode
        ts.append_token_meta(sess.layout, w.k_new[0], w.v_new[0], advance_seq_lens=True)
    sess.fused(scale, q_idx=1)
    units = full_size_units(w, name)
    worst = compare_units(oracle, sess, units, scale, q_idx=1, what=f"full/{name}")
    print(f"[full {name}] {len(units)} of {spec.B * spec.Hkv} units compared", flush=True)
    print(f"[full {name}] worst |out - oracle| = {worst:.3e}", flush=True)
    # properties that hold for every unit: counts, ordering, finite outputs
    torch.cuda.synchronize()
    lens = sess.seq_lens.to(torch.int64)
    P = (lens + spec.S - 1) // spec.S
    K = w.topk_per_seq.to(torch.int64) if w.topk_per_seq is not None else torch.full_like(P, w.topk)
    expect = torch.minimum(torch.minimum(K, P), torch.full_like(P, w.K_max))
    assert torch.equal(sess.sel_count.to(torch.int64), expect)
    sel = sess.sel.to(torch.int64)
    idx = torch.arange(w.K_max, device=DEV)[None, None, :]
    live = idx < expect[:, None, None]
    assert torch.all(sel[~live.expand_as(sel)] == -1)
    assert torch.all((sel < P[:, None, None])[live.expand_as(sel)])
    inc = (sel[..., 1:] > sel[..., :-1]) | ~live.expand_as(sel)[..., 1:]
    assert torch.all(inc)
    assert torch.all(torch.isfinite(sess.out))
    # staged path on the same inputs agrees with the fused one
    fused_out, fused_sel = sess.out.clone(), sess.sel.clone()
    sess.staged(scale, q_idx=1)
    torch.cuda.synchronize()
    assert torch.equal(sess.sel, fused_sel)
    assert (sess.out - fused_out).abs().max().item() <= 1e-6
    # the step bench.py times: one call of ts_append_and_decode (for the small batches a
    # single launch of the kernel build with the append folded in), first with the
    # reporting buffers for the comparison, then as bench.py calls it (outputs only)
    if name != "ragged":       # (ragged has already appended its one spare token above)
        args = (sess.layout, w.k_new[0], w.v_new[0], w.q[0], w.topk, w.K_max, scale, sess.out,
                sess.ws)
        ts.append_and_decode(*args, topk_per_seq=w.topk_per_seq, scores_out=sess.scores,
                             sel_out=sess.sel, sel_count_out=sess.sel_count)
        compare_units(oracle, sess, units, scale, q_idx=0, what=f"full/{name}/append+decode")
        reported = sess.out.clone()
        sess.seq_lens.sub_(1)                       # the same step again, nothing reported
        sess.out.fill_(float("nan"))
        ts.append_and_decode(*args, topk_per_seq=w.topk_per_seq)
        torch.cuda.synchronize()
        assert ts.workspace_status(sess.ws) == 0
        assert torch.equal(sess.out, reported)
