"""GPU parity of the INT8 KV cache format (int8 codes, one fp32 scale per token and
KV head, bf16 metadata rounded outwards) against the CPU oracle's INT8 functions:
metadata build, append with quantisation, staged and fused decode, dense baseline."""
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


class Session8:
    def __init__(self, w):
        self.w = w
        sp = w.spec
        assert sp.kv == "int8"
        self.page_min = torch.full((sp.B, sp.Hkv, w.P_max, sp.d), float("nan"), dtype=torch.bfloat16,
                                   device=DEV)
        self.page_max = torch.full_like(self.page_min, float("nan"))
        self.seq_lens = w.seq_lens.clone()
        self.layout = ts.make_layout(sp.B, sp.Hq, sp.Hkv, sp.d, sp.S, w.P_max, w.k_pool, w.v_pool,
                                     w.block_table, self.seq_lens, self.page_min, self.page_max,
                                     k_scale=w.k_scale, v_scale=w.v_scale)
        assert self.layout.kv_format == ts.TS_KV_INT8
        self.scores = torch.full((sp.B, sp.Hkv, w.P_max), float("nan"), dtype=torch.float32,
                                 device=DEV)
        self.sel = torch.full((sp.B, sp.Hkv, w.K_max), -7, dtype=torch.int32, device=DEV)
        self.sel_count = torch.full((sp.B,), -7, dtype=torch.int32, device=DEV)
        self.out = torch.full((sp.B, sp.Hq, sp.d), float("nan"), dtype=torch.float32, device=DEV)
        self.ws = ts.new_workspace(self.layout, w.K_max, DEV)

    def fused(self, scale, q_idx=0):
        w = self.w
        ts.query_aware_decode(self.layout, w.q[q_idx], w.topk, w.K_max, scale, self.out, self.ws,
                              topk_per_seq=w.topk_per_seq, scores_out=self.scores,
                              sel_out=self.sel, sel_count_out=self.sel_count)

    def staged(self, scale, q_idx=0):
        w = self.w
        ts.score_pages(self.layout, w.q[q_idx], self.scores)
        ts.select_topk_pages(self.layout, self.scores, w.topk, w.K_max, self.sel, self.sel_count,
                             topk_per_seq=w.topk_per_seq)
        ts.sparse_decode_attention(self.layout, w.q[q_idx], self.sel, self.sel_count, w.K_max,
                                   scale, self.out, self.ws)


def unit_inputs(w, b, h, q_idx, lens):
    G = w.spec.Hq // w.spec.Hkv
    Kq, ks, Vq, vs = wl.logical_kv_i8(w, seqs=[b], heads=[h], seq_lens=lens)
    q = wl.bits(w.q[q_idx, b, h * G:(h + 1) * G][None])
    L = np.array([int(lens[b])], dtype=np.int32)
    return q, Kq.cpu().numpy(), ks.cpu().numpy(), Vq.cpu().numpy(), vs.cpu().numpy(), L


def compare_units(oracle, sess, units, scale, q_idx=0, what=""):
    """One oracle call per sequence (all the wanted KV heads of it at once)."""
    w = sess.w
    sp = w.spec
    G = sp.Hq // sp.Hkv
    torch.cuda.synchronize()
    assert ts.workspace_status(sess.ws) == 0
    scores, sel = sess.scores.cpu().numpy(), sess.sel.cpu().numpy()
    cnt, out = sess.sel_count.cpu().numpy(), sess.out.cpu().numpy()
    lens = sess.seq_lens.cpu()
    for b, heads in by_sequence(units).items():
        r = oracle_sequence(oracle, w, b, heads, scale, q_idx=q_idx, seq_lens=lens)
        Pb = int(oracle.num_pages(int(lens[b]), sp.S))
        for i, h in enumerate(heads):
            tag = f"{what} unit(b={b},h={h})"
            v = head_view(r, i, G)
            assert np.array_equal(wl.bits(sess.page_min[b, h, :Pb]), v["pmin"][0, 0, :Pb]), f"{tag}: page_min"
            assert np.array_equal(wl.bits(sess.page_max[b, h, :Pb]), v["pmax"][0, 0, :Pb]), f"{tag}: page_max"
            assert_scores_close(scores[b, h], v["scores"][0, 0], Pb, tag)
            same = check_selection(sel[b, h], cnt[b], v, tag)
            ref = v["out"][0]
            if not same:
                ref = attention_on_set(oracle, w, v, sel[b, h], cnt[b], scale)
            assert_out_close(out[b, h * G:(h + 1) * G], ref, tag)


def spec8(name, *a, **kw):
    return wl.WorkloadSpec(name, *a, kv="int8", **kw)


REDUCED8 = {
    "mha_d64_s16": spec8("i1", 3, 4, 4, 64, 16, 2000, 24, headroom=40),
    "gqa8_d64_s32_walk": spec8("i2", 2, 16, 2, 64, 32, 6007, 20, keys="walk"),
    "mha_d128_s16_ragged": spec8("i3", 6, 4, 4, 128, 16, 3000, 0, L_min=1, budget_frac=0.25),
    "gqa4_d128_s32": spec8("i4", 2, 8, 2, 128, 32, 2500, 9),
    "gqa8_d64_s4": spec8("i5", 2, 16, 2, 64, 4, 1501, 90, keys="offset"),
    "mha_d128_s8": spec8("i6", 3, 4, 4, 128, 8, 1003, 37),
    "gqa4_d64_s64": spec8("i7", 2, 8, 2, 64, 64, 5000, 11, keys="walk"),
    "mha_d128_s64": spec8("i8", 2, 4, 4, 128, 64, 3048, 7),
    "gqa2_d128_s4": spec8("i9", 2, 4, 2, 128, 4, 703, 33),
    "mha_d64_s8": spec8("i10", 2, 2, 2, 64, 8, 500, 21),
}


@pytest.fixture
def splits(request):
    ts.set_tuning(0, request.param, 0)
    yield request.param
    ts.set_tuning(0, 0, 0)


@pytest.mark.parametrize("name", list(REDUCED8))
@pytest.mark.parametrize("splits", [0, 3], indirect=True)
def test_int8_reduced_all_units(oracle, name, splits):
    spec = REDUCED8[name]
    print(f"[case] int8 reduced {name} splits={splits}", flush=True)
    w = wl.make_workload(spec, DEV, seed=3000 + len(name), n_q=2, interleave=(splits == 0))
    scale = 1.0 / math.sqrt(spec.d)
    sess = Session8(w)
    ts.build_page_meta(sess.layout)
    units = [(b, h) for b in range(spec.B) for h in range(spec.Hkv)]
    sess.staged(scale, q_idx=1)
    compare_units(oracle, sess, units, scale, q_idx=1, what=f"{name}/staged")
    staged = (sess.scores.clone(), sess.sel.clone(), sess.sel_count.clone(), sess.out.clone())
    sess.out.fill_(float("nan"))
    sess.sel.fill_(-7)
    sess.fused(scale, q_idx=1)
    compare_units(oracle, sess, units, scale, q_idx=1, what=f"{name}/fused")
    assert torch.equal(sess.scores, staged[0]) and torch.equal(sess.sel, staged[1])
    assert (sess.out - staged[3]).abs().max().item() <= 1e-6
    # dense baseline and the log-denominators
    dws = ts.new_dense_workspace(sess.layout, DEV)
    lse = torch.full((spec.B, spec.Hq), float("nan"), dtype=torch.float32, device=DEV)
    ts.dense_decode_attention(sess.layout, w.q[1], scale, sess.out, dws, lse_out=lse)
    torch.cuda.synchronize()
    Kq, ks, Vq, vs = (t.cpu().numpy() for t in wl.logical_kv_i8(w))
    ref, ref_lse = oracle.sparse_decode_attention_i8(wl.bits(w.q[1]), Kq, ks, Vq, vs, None, None,
                                                     w.seq_lens.cpu().numpy(), spec.S, scale,
                                                     return_lse=True)
    assert np.abs(sess.out.cpu().numpy() - ref).max() <= 2e-3
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= 2e-3


APPEND8 = {
    "gqa4_d64_s16": spec8("a1", 4, 8, 2, 64, 16, 200, 6, L_min=1, headroom=48),
    "mha_d128_s32": spec8("a2", 3, 4, 4, 128, 32, 500, 4, headroom=80),
    "gqa2_d64_s4": spec8("a3", 3, 4, 2, 64, 4, 150, 9, L_min=1, headroom=48),
    "mha_d128_s64": spec8("a4", 2, 2, 2, 128, 64, 700, 3, L_min=1, headroom=128),
}


@pytest.mark.parametrize("name", list(APPEND8))
def test_int8_append_quantises_like_the_oracle(oracle, name):
    """ts_append_token_meta on the INT8 cache: codes, scales and the widened boxes are
    the oracle's, bit for bit; the boxes equal a rebuild; ts_append_and_decode (one
    launch that quantises the token itself) equals the two calls; decode results match
    the oracle."""
    spec = APPEND8[name]
    print(f"[case] int8 append {name}", flush=True)
    n_new = 36
    scale = 1.0 / math.sqrt(spec.d)
    twins = []
    for _ in range(2):
        w = wl.make_workload(spec, DEV, seed=55, n_q=n_new, n_new=n_new, poison=0.0)
        sess = Session8(w)
        if not spec.L_min:
            sess.seq_lens[0] = w.P_max * spec.S - 2     # runs out of room at the third append
        ts.build_page_meta(sess.layout)
        twins.append(sess)
    a, f = twins
    assert ts.append_and_decode_launches(f.layout, f.w.K_max) == 1
    units = [(b, h) for b in range(spec.B) for h in range(spec.Hkv)]
    B, Hkv, S, d = spec.B, spec.Hkv, spec.S, spec.d
    spliced = 0     # (unit, step) pairs whose selection holds the page of the token just appended
    for i in range(n_new):
        lens = a.seq_lens.cpu().numpy().copy()
        omin, omax = wl.bits(a.page_min).copy(), wl.bits(a.page_max).copy()
        ts.append_token_meta(a.layout, a.w.k_new[i], a.w.v_new[i], advance_seq_lens=True)
        a.fused(scale, q_idx=i)
        w = f.w
        ts.append_and_decode(f.layout, w.k_new[i], w.v_new[i], w.q[i], w.topk, w.K_max, scale, f.out,
                             f.ws, topk_per_seq=w.topk_per_seq, scores_out=f.scores,
                             sel_out=f.sel, sel_count_out=f.sel_count)
        torch.cuda.synchronize()
        what = f"{name} step {i}"
        # the oracle's quantiser and incremental box update on the state before the step
        kq, ksc = oracle.quantize_rows_i8(wl.bits(a.w.k_new[i]))
        vq, vsc = oracle.quantize_rows_i8(wl.bits(a.w.v_new[i]))
        oracle.append_token_meta_i8(kq, ksc, lens, S, omin, omax)
        bt = a.w.block_table.cpu().numpy()
        for b in range(B):
            j, slot = int(lens[b]) // S, int(lens[b]) % S
            if j >= a.w.P_max:
                assert int(a.seq_lens[b]) == lens[b], what          # refused, nothing advanced
                continue
            assert int(a.seq_lens[b]) == lens[b] + 1, what
            phys = int(bt[b, j])
            assert np.array_equal(a.w.k_pool[phys, :, slot, :].cpu().numpy(), kq[b]), what
            assert np.array_equal(a.w.v_pool[phys, :, :, slot].cpu().numpy(), vq[b]), what
            assert np.array_equal(a.w.k_scale[phys, :, slot].cpu().numpy(), ksc[b]), what
            assert np.array_equal(a.w.v_scale[phys, :, slot].cpu().numpy(), vsc[b]), what
            assert np.array_equal(wl.bits(a.page_min[b, :, j]), omin[b, :, j]), what
            assert np.array_equal(wl.bits(a.page_max[b, :, j]), omax[b, :, j]), what
        # one launch == two calls
        assert torch.equal(a.seq_lens, f.seq_lens), what
        assert torch.equal(a.w.k_pool, f.w.k_pool) and torch.equal(a.w.v_pool, f.w.v_pool), what
        assert torch.equal(a.w.k_scale, f.w.k_scale) and torch.equal(a.w.v_scale, f.w.v_scale), what
        assert np.array_equal(wl.bits(a.page_min), wl.bits(f.page_min)), what
        assert np.array_equal(wl.bits(a.page_max), wl.bits(f.page_max)), what
        assert torch.equal(a.sel, f.sel) and torch.equal(a.scores, f.scores), what
        assert (a.out - f.out).abs().max().item() <= 1e-6, what
        sel = f.sel.cpu().numpy().reshape(B, Hkv, -1)
        spliced += sum(int((sel[b] == int(lens[b]) // S).any(axis=-1).sum())
                       for b in range(B) if int(lens[b]) // S < f.w.P_max)
        if i in (0, 17, n_new - 1):
            compare_units(oracle, f, units, scale, q_idx=i, what=what)     # includes box == rebuild
    if not spec.L_min:
        assert int(f.seq_lens[0]) == f.w.P_max * S
    assert spliced > 0      # the attention did take the token from the caller's arrays


MANY8 = {
    "d128_s16": spec8("m1", 70, 4, 4, 128, 16, 500, 0, L_min=1, budget_frac=0.3, headroom=32),
    "d64_s32": spec8("m2", 40, 16, 8, 64, 32, 900, 6, L_min=1, headroom=64),
    "d64_s4": spec8("m3", 80, 4, 4, 64, 4, 300, 11, L_min=1, headroom=32),
    "d128_s64": spec8("m4", 72, 4, 4, 128, 64, 1200, 4, L_min=1, headroom=128),
}


@pytest.mark.parametrize("name", list(MANY8))
def test_int8_many_units_loop_build(oracle, name):
    spec = MANY8[name]
    print(f"[case] int8 many units {name}", flush=True)
    w = wl.make_workload(spec, DEV, seed=404, n_q=2, n_new=1)
    sess = Session8(w)
    ts.build_page_meta(sess.layout)
    scale = 1.0 / math.sqrt(spec.d)
    n_units = spec.B * spec.Hkv
    assert n_units > 256
    rng = np.random.default_rng(9)
    picks = sorted(set(rng.integers(0, n_units, 8).tolist()) | {0, 255, 256, n_units - 1})
    units = [(u // spec.Hkv, u % spec.Hkv) for u in picks]
    sess.fused(scale, q_idx=0)
    compare_units(oracle, sess, units, scale, q_idx=0, what=f"{name} launch 0")
    ts.append_and_decode(sess.layout, w.k_new[0], w.v_new[0], w.q[1], w.topk, w.K_max, scale, sess.out,
                         sess.ws, topk_per_seq=w.topk_per_seq, scores_out=sess.scores,
                         sel_out=sess.sel, sel_count_out=sess.sel_count)
    compare_units(oracle, sess, units, scale, q_idx=1, what=f"{name} launch 1")


@pytest.mark.parametrize("name", ["tinyllama", "ragged"])
def test_int8_full_size_sampled(oracle, name):
    """Benchmark workloads at full size with the INT8 cache, default launch shapes; the same
    units as the bf16 full-size test (all of tinyllama's, 20 sequences of ragged's)."""
    spec = wl.scaled(wl.SPECS[name], kv="int8")
    print(f"[case] int8 full {name}", flush=True)
    w = wl.make_workload(spec, DEV, seed=1500, n_q=2, n_new=1)
    sess = Session8(w)
    ts.build_page_meta(sess.layout)
    scale = 1.0 / math.sqrt(spec.d)
    ts.append_and_decode(sess.layout, w.k_new[0], w.v_new[0], w.q[1], w.topk, w.K_max, scale, sess.out,
                         sess.ws, topk_per_seq=w.topk_per_seq, scores_out=sess.scores,
                         sel_out=sess.sel, sel_count_out=sess.sel_count)
    compare_units(oracle, sess, full_size_units(w, name), scale, q_idx=1, what=f"int8 full/{name}")
