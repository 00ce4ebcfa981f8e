"""Pins for the CPU oracle (no GPU): the oracle is checked against things other
than itself -- a hand-worked example, the upper-bound invariant of Eq. 2, the
K = P special case against a library attention routine, brute force over all
page subsets on tiny inputs, closed forms, and append == rebuild."""
import itertools
import json
import os

import numpy as np
import pytest
import torch

from paper_2509_12211_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "two_page_example.json")


def bf16_bits(x):
    """float array (values exactly representable or to be rounded) -> uint16 bf16 bits."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return wl.bits(t)


def bf16_val(bits):
    return wl.from_bits(bits).to(torch.float64).numpy()


def rand_bf16(rng, shape, scale=1.0):
    return bf16_bits(rng.standard_normal(shape) * scale)


# ----------------------------------------------------------------------------
# hand-worked example (tests/golden/two_page_example.json)
# ----------------------------------------------------------------------------
def _golden():
    with open(GOLDEN) as f:
        return json.load(f)


def test_golden_metadata(oracle):
    g = _golden()
    K = bf16_bits(g["keys"]).reshape(1, 1, 4, 2)
    pmin, pmax = oracle.build_page_meta(K, [4], g["S"], 2)
    assert np.array_equal(bf16_val(pmin)[0, 0], np.array(g["page_min"], dtype=np.float64))
    assert np.array_equal(bf16_val(pmax)[0, 0], np.array(g["page_max"], dtype=np.float64))


@pytest.mark.parametrize("case", range(4))
def test_golden_cases(oracle, case):
    g = _golden()
    c = g["cases"][case]
    S = g["S"]
    K = bf16_bits(g["keys"]).reshape(1, 1, 4, 2)
    V = bf16_bits(g["values"]).reshape(1, 1, 4, 2)
    q = bf16_bits(c["q"]).reshape(1, -1, 2)
    pmin, pmax = oracle.build_page_meta(K, [4], S, 2)
    for form in (0, 1):
        s = oracle.score_pages(q, pmin, pmax, [4], S, form=form)
        assert np.array_equal(s[0, 0], np.array(c["scores"], dtype=np.float64))
    best = oracle.true_page_max(q, K, [4], S, 2)
    assert np.array_equal(best[0], np.array(c["true_page_max"], dtype=np.float64))
    r = oracle.query_aware_decode(q, K, V, pmin, pmax, [4], S, 1, 1, c["scale"])
    assert r["sel"][0, 0].tolist() == c["top1"]
    assert r["sel_count"].tolist() == [1]
    np.testing.assert_allclose(r["out"][0], np.array(c["out_top1"]), rtol=0, atol=1e-12)
    if "out_top2" in c:
        r2 = oracle.query_aware_decode(q, K, V, pmin, pmax, [4], S, 2, 2, c["scale"])
        assert r2["sel"][0, 0].tolist() == [0, 1]
        np.testing.assert_allclose(r2["out"][0], np.array(c["out_top2"]), rtol=0, atol=1e-12)


def test_golden_append(oracle):
    g = _golden()
    S = g["S"]
    K = bf16_bits(g["keys"]).reshape(1, 1, 4, 2)
    pmin, pmax = oracle.build_page_meta(K, [4], S, 3)
    L = 4
    for step in g["append"]:
        oracle.append_token_meta(bf16_bits(step["k_new"]).reshape(1, 1, 2), [L], S, pmin, pmax)
        L += 1
        j = step["page"]
        assert bf16_val(pmin)[0, 0, j].tolist() == step["page_min"]
        assert bf16_val(pmax)[0, 0, j].tolist() == step["page_max"]
    # pages 0 and 1 untouched
    assert bf16_val(pmin)[0, 0, :2].tolist() == g["page_min"]
    assert bf16_val(pmax)[0, 0, :2].tolist() == g["page_max"]


# ----------------------------------------------------------------------------
# invariant: Eq. 2 is an upper bound on max_{k in page} q.k  (Section 3.5)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("seed,keys_scale", [(0, 1.0), (1, 4.0), (2, 0.1)])
def test_bound_invariant_per_head(oracle, seed, keys_scale):
    rng = np.random.default_rng(seed)
    B, H, d, S = 3, 2, 16, 8
    lens = np.array([64, 37, 1], dtype=np.int32)   # full pages, ragged tail, single token
    Lmax, Pmax = 64, 8
    K = rand_bf16(rng, (B, H, Lmax, d), keys_scale)
    q = rand_bf16(rng, (B, H, d))
    pmin, pmax = oracle.build_page_meta(K, lens, S, Pmax)
    s = oracle.score_pages(q, pmin, pmax, lens, S)           # G = 1: one bound per head
    best = oracle.true_page_max(q, K, lens, S, Pmax)
    P = oracle.num_pages(lens, S)
    for b in range(B):
        assert np.all(s[b, :, :P[b]] >= best[b, :, :P[b]])    # zero slack: same summation order
        assert np.all(np.isneginf(s[b, :, P[b]:]))
        assert np.all(np.isfinite(s[b, :, :P[b]]))
    # the bound is not vacuous: on random data it is strictly loose on most pages
    assert np.mean(s[0] > best[0]) > 0.9


def test_bound_invariant_group(oracle):
    """GQA: the group score is >= the sum of the heads' true page maxima
    >= the page maximum of the summed logits."""
    rng = np.random.default_rng(5)
    B, Hq, Hkv, d, S, L = 2, 8, 2, 8, 4, 40
    K = rand_bf16(rng, (B, Hkv, L, d))
    q = rand_bf16(rng, (B, Hq, d))
    lens = np.array([40, 22], dtype=np.int32)
    pmin, pmax = oracle.build_page_meta(K, lens, S, 10)
    s = oracle.score_pages(q, pmin, pmax, lens, S)
    best = oracle.true_page_max(q, K, lens, S, 10)           # [B][Hq][P]
    G = Hq // Hkv
    for b in range(B):
        Pb = int(oracle.num_pages(lens[b], S))
        for h in range(Hkv):
            tot = best[b, h * G:(h + 1) * G, :Pb].sum(axis=0)
            assert np.all(s[b, h, :Pb] >= tot - 1e-12 * np.abs(tot))


def test_two_score_forms_agree(oracle):
    rng = np.random.default_rng(7)
    K = rand_bf16(rng, (2, 2, 48, 32))
    q = rand_bf16(rng, (2, 4, 32))
    q[0, 0, :4] = 0                       # exact zeros in the query: both branches give 0
    lens = np.array([48, 30], dtype=np.int32)
    pmin, pmax = oracle.build_page_meta(K, lens, 16, 3)
    a = oracle.score_pages(q, pmin, pmax, lens, 16, form=0)
    b = oracle.score_pages(q, pmin, pmax, lens, 16, form=1)
    assert np.array_equal(a, b)


# ----------------------------------------------------------------------------
# closed forms
# ----------------------------------------------------------------------------
def test_constant_pages_bound_is_tight(oracle):
    """All keys of a page equal => m = M = k => score = q.k exactly."""
    rng = np.random.default_rng(11)
    d, S, P = 8, 4, 5
    page_keys = rand_bf16(rng, (P, d))
    K = np.repeat(page_keys[:, None, :], S, axis=1).reshape(1, 1, P * S, d)
    q = rand_bf16(rng, (1, 1, d))
    pmin, pmax = oracle.build_page_meta(K, [P * S], S, P)
    assert np.array_equal(pmin, pmax)
    s = oracle.score_pages(q, pmin, pmax, [P * S], S)
    qv, kv = bf16_val(q)[0, 0], bf16_val(page_keys)
    expect = np.array([sum(qv[c] * kv[j, c] for c in range(d)) for j in range(P)])
    assert np.array_equal(s[0, 0], expect)


def test_single_key_uniform_values(oracle):
    """Equal logits => uniform weights => output is the plain mean of the values."""
    d, S = 4, 4
    K = np.tile(bf16_bits([[0.5, -1.0, 2.0, 0.25]]), (8, 1)).reshape(1, 1, 8, d)
    V = bf16_bits(np.arange(32).reshape(8, 4)).reshape(1, 1, 8, d)
    q = bf16_bits([[1.0, 2.0, -1.0, 4.0]]).reshape(1, 1, d)
    sel = np.array([[[1]]], dtype=np.int32)
    out = oracle.sparse_decode_attention(q, K, V, sel, [1], [8], S, 0.7)
    np.testing.assert_allclose(out[0, 0], bf16_val(V)[0, 0, 4:8].mean(axis=0), atol=1e-13)


# ----------------------------------------------------------------------------
# log of the softmax denominator (reported next to the attention output)
# ----------------------------------------------------------------------------
def test_lse_closed_form_equal_logits(oracle):
    """n tokens with the same logit a: the denominator is n * exp(a)."""
    d, S = 4, 4
    K = np.tile(bf16_bits([[0.5, -1.0, 2.0, 0.25]]), (8, 1)).reshape(1, 1, 8, d)
    V = rand_bf16(np.random.default_rng(0), (1, 1, 8, d))
    q = bf16_bits([[1.0, 2.0, -1.0, 4.0]]).reshape(1, 1, d)
    logit = 0.7 * (0.5 * 1.0 - 1.0 * 2.0 - 2.0 * 1.0 + 0.25 * 4.0)
    _, lse = oracle.sparse_decode_attention(q, K, V, np.array([[[1]]], dtype=np.int32), [1], [7], S,
                                            0.7, return_lse=True)
    assert lse[0, 0] == pytest.approx(logit + np.log(3.0), abs=1e-13)   # tokens 4, 5, 6
    _, lse = oracle.dense_decode_attention(q, K, V, [7], 0.7, return_lse=True)
    assert lse[0, 0] == pytest.approx(logit + np.log(7.0), abs=1e-13)
    _, lse = oracle.sparse_decode_attention(q, K, V, np.array([[[0]]], dtype=np.int32), [0], [7], S,
                                            0.7, return_lse=True)
    assert lse[0, 0] == -np.inf


def test_lse_against_library_and_partition(oracle):
    """Against scipy's logsumexp of independently computed logits; and the softmax
    mass of disjoint page sets adds up to that of their union (the whole cache: 1)."""
    from scipy.special import logsumexp
    rng = np.random.default_rng(11)
    B, Hq, Hkv, d, S = 2, 4, 2, 8, 4
    lens = np.array([22, 13], dtype=np.int32)
    Lmax, G = 24, Hq // Hkv
    K = rand_bf16(rng, (B, Hkv, Lmax, d))
    V = rand_bf16(rng, (B, Hkv, Lmax, d))
    q = rand_bf16(rng, (B, Hq, d), 2.0)
    scale = 0.3
    _, dense = oracle.dense_decode_attention(q, K, V, lens, scale, return_lse=True)
    Kv, qv = bf16_val(K), bf16_val(q)
    for b in range(B):
        for g in range(Hq):
            a = scale * (Kv[b, g // G, :lens[b]] @ qv[b, g])
            assert dense[b, g] == pytest.approx(logsumexp(a), abs=1e-12)
    # pages {0, 2, 4} and {1, 3, 5} partition every sequence (absent pages hold no token)
    even = np.tile(np.array([0, 2, 4], dtype=np.int32), (B, Hkv, 1))
    odd = np.tile(np.array([1, 3, 5], dtype=np.int32), (B, Hkv, 1))
    # sequence 1 has 4 pages: its lists are {0, 2} and {1, 3}
    even[1, :, 2] = -1
    odd[1, :, 2] = -1
    cnt_b = np.array([3, 2], dtype=np.int32)
    _, le = oracle.sparse_decode_attention(q, K, V, even, cnt_b, lens, S, scale, return_lse=True)
    _, lo = oracle.sparse_decode_attention(q, K, V, odd, cnt_b, lens, S, scale, return_lse=True)
    np.testing.assert_allclose(np.exp(le - dense) + np.exp(lo - dense), 1.0, rtol=0, atol=1e-12)
    for b in range(B):
        for g in range(Hq):
            toks = [t for j in even[b, g // G, :cnt_b[b]] for t in range(j * S, min((j + 1) * S, lens[b]))]
            a = scale * (Kv[b, g // G, toks] @ qv[b, g])
            assert le[b, g] == pytest.approx(logsumexp(a), abs=1e-12)


# ----------------------------------------------------------------------------
# K = P  ==>  dense softmax attention, against torch's SDPA (a library routine)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("scale", [1.0, 0.125])
def test_all_pages_equals_dense_library(oracle, scale):
    rng = np.random.default_rng(3)
    B, Hq, Hkv, d, S = 2, 4, 2, 16, 8
    lens = np.array([40, 29], dtype=np.int32)
    Lmax = 40
    K = rand_bf16(rng, (B, Hkv, Lmax, d))
    V = rand_bf16(rng, (B, Hkv, Lmax, d))
    q = rand_bf16(rng, (B, Hq, d), 0.5)
    pmin, pmax = oracle.build_page_meta(K, lens, S, 5)
    r = oracle.query_aware_decode(q, K, V, pmin, pmax, lens, S, 99, 5, scale)
    assert r["sel_count"].tolist() == [5, 4]
    assert r["sel"][1, 0].tolist() == [0, 1, 2, 3, -1]
    dense = oracle.dense_decode_attention(q, K, V, lens, scale)
    np.testing.assert_allclose(r["out"], dense, rtol=0, atol=1e-13)
    G = Hq // Hkv
    Kt, Vt, qt = (torch.from_numpy(bf16_val(x)) for x in (K, V, q))
    for b in range(B):
        L = int(lens[b])
        kk = Kt[b, :, :L].repeat_interleave(G, dim=0)          # [Hq][L][d]
        vv = Vt[b, :, :L].repeat_interleave(G, dim=0)
        ref = torch.nn.functional.scaled_dot_product_attention(
            qt[b][:, None, :], kk, vv, scale=scale)[:, 0]
        np.testing.assert_allclose(r["out"][b], ref.numpy(), rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------
# brute force on tiny inputs (independent numpy, enumerates every page subset)
# ----------------------------------------------------------------------------
def _brute(qv, Kv, Vv, L, S, Ksel, scale):
    """qv [G][d], Kv/Vv [L][d] float64.  Returns (best subset, out [G][d])."""
    P = -(-L // S)
    pages = [range(j * S, min((j + 1) * S, L)) for j in range(P)]
    score = []
    for toks in pages:
        lo = Kv[list(toks)].min(axis=0)
        hi = Kv[list(toks)].max(axis=0)
        score.append(sum(max(qg[c] * lo[c], qg[c] * hi[c]) for qg in qv for c in range(len(lo))))
    kk = min(Ksel, P)
    # the chosen set maximises the total score; among maximisers, the lexicographically
    # smallest id tuple (what "ties go to the lower page id" means for a set)
    best = max(itertools.combinations(range(P), kk),
               key=lambda c: (sum(score[j] for j in c), tuple(-j for j in c)))
    toks = [t for j in best for t in pages[j]]
    out = []
    for qg in qv:
        a = np.array([scale * float(np.dot(qg, Kv[t])) for t in toks])
        w = np.exp(a - a.max())
        w /= w.sum()
        out.append((w[:, None] * Vv[toks]).sum(axis=0))
    return list(best), np.array(out), np.array(score)


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_tiny(oracle, seed):
    rng = np.random.default_rng(100 + seed)
    d = int(rng.integers(1, 5))
    S = int(rng.integers(1, 5))
    G = int(rng.integers(1, 4))
    B, Hkv = 2, 2
    lens = rng.integers(1, 6 * S + 1, size=B).astype(np.int32)
    Lmax = int(lens.max())
    Pmax = -(-Lmax // S)
    Ksel = int(rng.integers(1, Pmax + 2))
    # small integer-valued keys make equal scores (ties) common
    K = bf16_bits(rng.integers(-2, 3, size=(B, Hkv, Lmax, d)))
    V = rand_bf16(rng, (B, Hkv, Lmax, d))
    q = bf16_bits(rng.integers(-2, 3, size=(B, Hkv * G, d)))
    pmin, pmax = oracle.build_page_meta(K, lens, S, Pmax)
    r = oracle.query_aware_decode(q, K, V, pmin, pmax, lens, S, Ksel, Pmax, 0.5)
    Kv, Vv, qv = bf16_val(K), bf16_val(V), bf16_val(q)
    for b in range(B):
        for h in range(Hkv):
            L = int(lens[b])
            best, out, score = _brute(qv[b, h * G:(h + 1) * G], Kv[b, h, :L], Vv[b, h, :L], L, S,
                                      Ksel, 0.5)
            Pb = -(-L // S)
            assert np.array_equal(r["scores"][b, h, :Pb], score)   # small integers: exact
            n = int(r["sel_count"][b])
            assert n == min(Ksel, Pb)
            assert r["sel"][b, h, :n].tolist() == best
            assert np.all(r["sel"][b, h, n:] == -1)
            np.testing.assert_allclose(r["out"][b, h * G:(h + 1) * G], out, rtol=0, atol=1e-12)


def test_tie_break_prefers_lower_page_id(oracle):
    scores = np.array([[[1.0, 3.0, 3.0, 3.0, 0.5, 3.0]]])
    sel, cnt, gap = oracle.select_topk_pages(scores, [6 * 4], 4, 3, 4)
    assert sel[0, 0].tolist() == [1, 2, 3, -1] and cnt.tolist() == [3]
    assert gap[0, 0] == 0.0                       # the first dropped page ties the last kept one
    sel, cnt, gap = oracle.select_topk_pages(scores, [6 * 4], 4, 4, 4)
    assert sel[0, 0].tolist() == [1, 2, 3, 5]
    assert gap[0, 0] == pytest.approx(2.0 / 3.0)
    # per-sequence budgets override the scalar; K > P is clipped to P
    scores2 = np.concatenate([scores, scores], axis=0)
    sel, cnt, _ = oracle.select_topk_pages(scores2, [24, 7], 4, 1, 6, topk_per_seq=[2, 6])
    assert sel[0, 0].tolist() == [1, 2, -1, -1, -1, -1]
    assert sel[1, 0].tolist() == [0, 1, -1, -1, -1, -1] and cnt.tolist() == [2, 2]


# ----------------------------------------------------------------------------
# incremental metadata == metadata rebuilt from scratch, after every append
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(8))
def test_always_kept_pages(oracle, seed):
    """Optional always-kept pages (first keep_first, last keep_last of each sequence):
    against an independent numpy ranking in which those pages get +inf, on random
    scores with ties; with both counts zero the plain selection is unchanged."""
    rng = np.random.default_rng(500 + seed)
    B, Hkv, S, Pmax = 3, 2, 4, 40
    lens = rng.integers(0, Pmax * S + 1, size=B).astype(np.int32)
    lens[0] = Pmax * S
    sc = np.round(rng.standard_normal((B, Hkv, Pmax)) * 4) / 4        # ties are common
    kf, kl = int(rng.integers(0, 4)), int(rng.integers(0, 5))
    K = int(rng.integers(1, 12))
    Kmax = 12
    sel, cnt, gap = oracle.select_topk_pages(sc, lens, S, K, Kmax, keep_first=kf, keep_last=kl)
    for b in range(B):
        Pb = -(-int(lens[b]) // S)
        Kb = min(K, Pb)
        assert cnt[b] == Kb
        for h in range(Hkv):
            s = sc[b, h, :Pb].copy()
            forced = np.array([j < kf or j >= Pb - kl for j in range(Pb)], dtype=bool)
            s[forced] = np.inf
            order = np.lexsort((np.arange(Pb), -s))          # score descending, then id ascending
            expect = sorted(order[:Kb].tolist())
            assert sel[b, h, :Kb].tolist() == expect
            assert np.all(sel[b, h, Kb:] == -1)
            if forced.sum() <= Kb:                            # every always-kept page is in
                assert set(np.nonzero(forced)[0].tolist()) <= set(expect)
    plain = oracle.select_topk_pages(sc, lens, S, K, Kmax)
    zero = oracle.select_topk_pages(sc, lens, S, K, Kmax, keep_first=0, keep_last=0)
    assert all(np.array_equal(a, b) for a, b in zip(plain, zero))


# ----------------------------------------------------------------------------
# IEEE half inputs (the paper's experiments run in FP16)
# ----------------------------------------------------------------------------
def test_fp16_decoder_against_numpy(oracle):
    """Every one of the 65536 bit patterns decodes as numpy's float16 does."""
    bits = np.arange(65536, dtype=np.uint16)
    with oracle.element_format("fp16"):
        got = oracle.decode_elements(bits)
    ref = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))
    # and the default is untouched afterwards
    assert oracle.decode_elements(bf16_bits([1.5, -2.0])).tolist() == [1.5, -2.0]


def test_fp16_all_pages_equals_dense_library(oracle):
    """The whole step in fp16 mode: metadata, Eq. 2 against a direct evaluation, and
    K = P against torch's attention on the same half-precision values."""
    rng = np.random.default_rng(21)
    B, Hq, Hkv, d, S = 2, 4, 2, 16, 8
    lens = np.array([37, 24], dtype=np.int32)
    Lmax, Pmax = 40, 5

    def h16(x):
        return np.asarray(x, dtype=np.float16).view(np.uint16)

    K, V = h16(rng.standard_normal((B, Hkv, Lmax, d))), h16(rng.standard_normal((B, Hkv, Lmax, d)))
    q = h16(rng.standard_normal((B, Hq, d)) * 0.5)
    Kf, Vf, qf = (x.view(np.float16).astype(np.float64) for x in (K, V, q))
    with oracle.element_format("fp16"):
        pmin, pmax = oracle.build_page_meta(K, lens, S, Pmax)
        r = oracle.query_aware_decode(q, K, V, pmin, pmax, lens, S, 99, Pmax, 0.25)
    G = Hq // Hkv
    for b in range(B):
        L = int(lens[b])
        for h in range(Hkv):
            for j in range(-(-L // S)):
                blk = Kf[b, h, j * S:min((j + 1) * S, L)]
                assert np.array_equal(pmin[b, h, j].view(np.float16).astype(np.float64), blk.min(0))
                assert np.array_equal(pmax[b, h, j].view(np.float16).astype(np.float64), blk.max(0))
                want = sum(max(qf[b, g, c] * blk[:, c].min(), qf[b, g, c] * blk[:, c].max())
                           for g in range(h * G, (h + 1) * G) for c in range(d))
                assert r["scores"][b, h, j] == pytest.approx(want, rel=1e-13, abs=1e-13)
        kk = torch.from_numpy(Kf[b, :, :L]).repeat_interleave(G, dim=0)
        vv = torch.from_numpy(Vf[b, :, :L]).repeat_interleave(G, dim=0)
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(qf[b])[:, None, :], kk, vv, scale=0.25)[:, 0]
        np.testing.assert_allclose(r["out"][b], ref.numpy(), rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------
# INT8 KV cache (an extension; format in oracle/ts_oracle.c)
# ----------------------------------------------------------------------------
def test_i8_quantisation_hand_worked(oracle):
    """scale = max|x| / 127, codes = round-half-even(x / scale), in fp32."""
    x = bf16_bits([[1.0, -0.5, 0.25, 0.0], [0.0, 0.0, 0.0, 0.0], [-3.0, 3.0, 1.5, -0.75]])
    xq, sc = oracle.quantize_rows_i8(x)
    assert sc[0] == np.float32(1.0) / np.float32(127.0)
    # 0.5 * 127 = 63.5 and 0.25 * 127 = 31.75 up to the rounding of 1/127 in fp32:
    # x / scale is evaluated in fp32 and comes out as exactly -63.5 and 31.75
    assert xq[0].tolist() == [127, -64, 32, 0]
    assert sc[1] == 1.0 and xq[1].tolist() == [0, 0, 0, 0]
    assert sc[2] == np.float32(3.0) / np.float32(127.0)
    assert xq[2].tolist() == [-127, 127, 64, -32]      # 63.5 -> 64 (even), 31.75 -> 32
    # the largest entry always maps to +-127 and the error is at most half a step
    rng = np.random.default_rng(5)
    y = rand_bf16(rng, (50, 16), 3.0)
    yq, ys = oracle.quantize_rows_i8(y)
    assert np.all(np.abs(yq).max(axis=1) == 127)
    err = np.abs(yq.astype(np.float64) * ys[:, None].astype(np.float64) - bf16_val(y))
    assert np.all(err <= 0.5 * ys[:, None].astype(np.float64) * (1 + 1e-6))


def test_i8_box_is_rounded_outwards(oracle):
    """Metadata of an INT8 page: min rounded down, max rounded up to bf16, so the box
    contains the dequantised keys; values that are bf16 numbers stay as they are."""
    # one page of two tokens, d = 4, scale chosen so that products need > 8 bits
    Kq = np.array([[[[3, -3, 64, 1], [5, -5, 64, -1]]]], dtype=np.int8)
    ks = np.array([[[1.0 + 2.0 ** -10, 1.0 + 2.0 ** -10]]], dtype=np.float32)
    pmin, pmax = oracle.build_page_meta_i8(Kq, ks, [2], 2, 1)
    lo, hi = bf16_val(pmin)[0, 0, 0], bf16_val(pmax)[0, 0, 0]
    s = 1.0 + 2.0 ** -10
    true_lo = np.array([3 * s, -5 * s, 64 * s, -1 * s])
    true_hi = np.array([5 * s, -3 * s, 64 * s, 1 * s])
    assert np.all(lo <= true_lo) and np.all(hi >= true_hi)
    # and tightly: the next bf16 number inwards would cut the value off
    assert lo.tolist() == [3.0, -5.03125, 64.0, -1.0078125]
    assert hi.tolist() == [5.03125, -3.0, 64.5, 1.0078125]
    # exactly representable products are not moved
    ks1 = np.ones((1, 1, 2), dtype=np.float32) * 0.5
    pmin, pmax = oracle.build_page_meta_i8(Kq, ks1, [2], 2, 1)
    assert bf16_val(pmin)[0, 0, 0].tolist() == [1.5, -2.5, 32.0, -0.5]
    assert bf16_val(pmax)[0, 0, 0].tolist() == [2.5, -1.5, 32.0, 0.5]


@pytest.mark.parametrize("seed", range(3))
def test_i8_equals_bf16_path_for_power_of_two_scales(oracle, seed):
    """With power-of-two scales the dequantised keys and values are bf16 numbers: every
    INT8 function must then reproduce the (pinned) bf16 functions on the dequantised cache."""
    rng = np.random.default_rng(40 + seed)
    B, Hq, Hkv, d, S = 2, 4, 2, 8, 4
    lens = np.array([27, 14], dtype=np.int32)
    Lmax, Pmax, Kmax = 28, 7, 3
    Kq = rng.integers(-127, 128, size=(B, Hkv, Lmax, d)).astype(np.int8)
    Vq = rng.integers(-127, 128, size=(B, Hkv, Lmax, d)).astype(np.int8)
    ks = (2.0 ** rng.integers(-8, -3, size=(B, Hkv, Lmax))).astype(np.float32)
    vs = (2.0 ** rng.integers(-8, -3, size=(B, Hkv, Lmax))).astype(np.float32)
    Kb = bf16_bits(Kq.astype(np.float64) * ks[..., None])
    Vb = bf16_bits(Vq.astype(np.float64) * vs[..., None])
    assert np.array_equal(bf16_val(Kb), Kq.astype(np.float64) * ks[..., None])   # exact
    q = rand_bf16(rng, (B, Hq, d), 0.5)
    pmin, pmax = oracle.build_page_meta(Kb, lens, S, Pmax)
    qmin, qmax = oracle.build_page_meta_i8(Kq, ks, lens, S, Pmax)
    for b in range(B):
        Pb = -(-int(lens[b]) // S)
        assert np.array_equal(pmin[b, :, :Pb], qmin[b, :, :Pb])
        assert np.array_equal(pmax[b, :, :Pb], qmax[b, :, :Pb])
    r = oracle.query_aware_decode(q, Kb, Vb, pmin, pmax, lens, S, 2, Kmax, 0.4)
    ri = oracle.query_aware_decode_i8(q, Kq, ks, Vq, vs, qmin, qmax, lens, S, 2, Kmax, 0.4)
    assert np.array_equal(r["sel"], ri["sel"]) and np.array_equal(r["scores"], ri["scores"])
    np.testing.assert_allclose(ri["out"], r["out"], rtol=0, atol=1e-13)
    dense, dl = oracle.dense_decode_attention(q, Kb, Vb, lens, 0.4, return_lse=True)
    di, dli = oracle.sparse_decode_attention_i8(q, Kq, ks, Vq, vs, None, None, lens, S, 0.4,
                                                return_lse=True)
    np.testing.assert_allclose(di, dense, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dli, dl, rtol=0, atol=1e-12)
    # append == rebuild, bit for bit
    kq_new = rng.integers(-127, 128, size=(B, Hkv, d)).astype(np.int8)
    ks_new = (1.0 + rng.random((B, Hkv))).astype(np.float32) * 0.01        # not powers of two
    Kq2, ks2 = Kq.copy(), ks.copy()
    for b in range(B):
        Kq2[b, :, lens[b]] = kq_new[b]
        ks2[b, :, lens[b]] = ks_new[b]
    amin, amax = qmin.copy(), qmax.copy()
    oracle.append_token_meta_i8(kq_new, ks_new, lens, S, amin, amax)
    rmin, rmax = oracle.build_page_meta_i8(Kq2, ks2, lens + 1, S, Pmax)
    for b in range(B):
        Pb = -(-int(lens[b] + 1) // S)
        assert np.array_equal(amin[b, :, :Pb], rmin[b, :, :Pb])
        assert np.array_equal(amax[b, :, :Pb], rmax[b, :, :Pb])


def test_i8_bound_invariant(oracle):
    """Eq. 2 on the outward-rounded box bounds q.k for every dequantised key, zero slack."""
    rng = np.random.default_rng(8)
    B, Hq, Hkv, d, S = 1, 2, 2, 16, 8
    L, Pmax = 61, 8
    Kq = rng.integers(-127, 128, size=(B, Hkv, L, d)).astype(np.int8)
    ks = (0.005 + 0.03 * rng.random((B, Hkv, L))).astype(np.float32)
    q = rand_bf16(rng, (B, Hq, d))
    pmin, pmax = oracle.build_page_meta_i8(Kq, ks, [L], S, Pmax)
    sc = oracle.score_pages(q, pmin, pmax, [L], S)
    qv = bf16_val(q)
    for h in range(Hkv):
        kd = Kq[0, h].astype(np.float64) * ks[0, h][:, None].astype(np.float64)
        for j in range(Pmax):
            toks = range(j * S, min((j + 1) * S, L))
            best = max(sum(qv[0, h, c] * kd[t, c] for c in range(d)) for t in toks)
            assert sc[0, h, j] >= best


def test_append_equals_rebuild(oracle):
    rng = np.random.default_rng(21)
    B, Hkv, d, S = 3, 2, 8, 4
    start = np.array([0, 5, 8], dtype=np.int32)      # empty, mid-page, page boundary
    n_app = 11
    Lmax = int(start.max()) + n_app
    Pmax = -(-Lmax // S)
    K = rand_bf16(rng, (B, Hkv, Lmax, d))
    pmin, pmax = oracle.build_page_meta(K, start, S, Pmax)
    lens = start.copy()
    for _ in range(n_app):
        k_new = np.stack([K[b, :, lens[b]] for b in range(B)])      # [B][Hkv][d]
        oracle.append_token_meta(k_new, lens, S, pmin, pmax)
        lens = lens + 1
        rmin, rmax = oracle.build_page_meta(K, lens, S, Pmax)
        for b in range(B):
            Pb = int(oracle.num_pages(lens[b], S))
            assert np.array_equal(pmin[b, :, :Pb], rmin[b, :, :Pb])
            assert np.array_equal(pmax[b, :, :Pb], rmax[b, :, :Pb])


def test_empty_sequence(oracle):
    rng = np.random.default_rng(2)
    K = rand_bf16(rng, (1, 1, 4, 4))
    q = rand_bf16(rng, (1, 2, 4))
    pmin, pmax = oracle.build_page_meta(K, [0], 2, 2)
    r = oracle.query_aware_decode(q, K, K, pmin, pmax, [0], 2, 2, 2, 1.0)
    assert r["sel_count"].tolist() == [0] and np.all(r["sel"] == -1)
    assert np.all(np.isneginf(r["scores"])) and np.all(r["out"] == 0.0)


# ----------------------------------------------------------------------------
# byte model of the paper's memory analysis (rho = 1): fraction = 1/S + K*S/L
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("name,frac", [("tiny", 0.1875), ("gpt2_345m", 0.1875),
                                       ("tinyllama", 0.1875), ("longctx", 0.0625)])
def test_byte_model_fraction(name, frac):
    spec = wl.SPECS[name]
    lens = torch.full((spec.B,), spec.L, dtype=torch.int32)
    by = wl.algorithmic_bytes(spec, lens)
    assert by["total"] / by["dense"] == frac == 1 / spec.S + spec.topk * spec.S / spec.L
