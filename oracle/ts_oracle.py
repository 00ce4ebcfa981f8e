"""ctypes front end of the CPU oracle (oracle/ts_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product path (paper_2509_12211_amd) never
imports this module.

Every array is a C-contiguous numpy array: bf16 tensors travel as uint16 bit
patterns, lengths / selections as int32, results as float64.  Shapes follow the
header comment of ts_oracle.c (logical [B][Hkv][Lmax][d] keys and values; no
block table).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ts_oracle.c")
_LIB = os.path.join(_HERE, "libts_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP for the timed attention loop)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.tso_version.restype = ctypes.c_int
        _lib.tso_max_threads.restype = ctypes.c_int
    return _lib


import contextlib


@contextlib.contextmanager
def element_format(fmt: str):
    """fmt = "bf16" (default) or "fp16": how the 16-bit inputs of the functions of the
    paper's path are decoded inside the block."""
    assert fmt in ("bf16", "fp16")
    _load().tso_set_element_format(1 if fmt == "fp16" else 0)
    try:
        yield
    finally:
        _load().tso_set_element_format(0)


def decode_elements(bits):
    bits = _u16(bits)
    out = np.empty(bits.shape, dtype=np.float64)
    _load().tso_decode_elements(_p(bits), bits.size, _p(out))
    return out


def max_threads() -> int:
    return int(_load().tso_max_threads())


def set_num_threads(n: int) -> None:
    """Threads for the OpenMP attention loop (n <= 0: the default again).  Timing only."""
    _load().tso_set_num_threads(int(n))


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_pages(seq_lens, S):
    return (np.asarray(seq_lens, dtype=np.int64) + S - 1) // S


def build_page_meta(K, seq_lens, S, Pmax):
    K = _u16(K)
    B, Hkv, Lmax, d = K.shape
    seq_lens = _i32(seq_lens)
    pmin = np.zeros((B, Hkv, Pmax, d), dtype=np.uint16)
    pmax = np.zeros((B, Hkv, Pmax, d), dtype=np.uint16)
    _load().tso_build_page_meta(_p(K), _p(seq_lens), B, Hkv, Lmax, d, S, Pmax, _p(pmin), _p(pmax))
    return pmin, pmax


def append_token_meta(k_new, seq_lens, S, page_min, page_max):
    """In place on page_min / page_max; seq_lens are the lengths BEFORE the append."""
    k_new = _u16(k_new)
    B, Hkv, d = k_new.shape
    seq_lens = _i32(seq_lens)
    assert page_min.flags.c_contiguous and page_max.flags.c_contiguous
    Pmax = page_min.shape[2]
    _load().tso_append_token_meta(_p(k_new), _p(seq_lens), B, Hkv, d, S, Pmax, _p(page_min),
                                  _p(page_max))


def score_pages(q, page_min, page_max, seq_lens, S, form=0):
    q = _u16(q)
    page_min, page_max = _u16(page_min), _u16(page_max)
    B, Hq, d = q.shape
    _, Hkv, Pmax, _ = page_min.shape
    seq_lens = _i32(seq_lens)
    scores = np.empty((B, Hkv, Pmax), dtype=np.float64)
    _load().tso_score_pages(_p(q), _p(page_min), _p(page_max), _p(seq_lens), B, Hq, Hkv, d, S,
                            Pmax, int(form), _p(scores))
    return scores


def select_topk_pages(scores, seq_lens, S, topk, Kmax, topk_per_seq=None, keep_first=0,
                      keep_last=0):
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    B, Hkv, Pmax = scores.shape
    seq_lens = _i32(seq_lens)
    tps = None if topk_per_seq is None else _i32(topk_per_seq)
    sel = np.empty((B, Hkv, Kmax), dtype=np.int32)
    cnt = np.empty((B,), dtype=np.int32)
    gap = np.empty((B, Hkv), dtype=np.float64)
    _load().tso_select_topk_pages(_p(scores), _p(seq_lens), B, Hkv, S, Pmax, int(topk), _p(tps),
                                  Kmax, int(keep_first), int(keep_last), _p(sel), _p(cnt), _p(gap))
    return sel, cnt, gap


def sparse_decode_attention(q, K, V, sel, sel_count, seq_lens, S, scale, return_lse=False):
    q, K, V = _u16(q), _u16(K), _u16(V)
    B, Hq, d = q.shape
    _, Hkv, Lmax, _ = K.shape
    sel, sel_count, seq_lens = _i32(sel), _i32(sel_count), _i32(seq_lens)
    Kmax = sel.shape[2]
    out = np.empty((B, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64) if return_lse else None
    _load().tso_sparse_decode_attention(_p(q), _p(K), _p(V), _p(sel), _p(sel_count), _p(seq_lens),
                                        B, Hq, Hkv, Lmax, d, S, Kmax, ctypes.c_double(scale),
                                        _p(out), _p(lse))
    return (out, lse) if return_lse else out


def dense_decode_attention(q, K, V, seq_lens, scale, return_lse=False):
    q, K, V = _u16(q), _u16(K), _u16(V)
    B, Hq, d = q.shape
    _, Hkv, Lmax, _ = K.shape
    seq_lens = _i32(seq_lens)
    out = np.empty((B, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64) if return_lse else None
    _load().tso_dense_decode_attention(_p(q), _p(K), _p(V), _p(seq_lens), B, Hq, Hkv, Lmax, d,
                                       ctypes.c_double(scale), _p(out), _p(lse))
    return (out, lse) if return_lse else out


def query_aware_decode(q, K, V, page_min, page_max, seq_lens, S, topk, Kmax, scale,
                       topk_per_seq=None, keep_first=0, keep_last=0):
    """score -> select -> attend.  Returns dict(scores, sel, sel_count, gap, out)."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    page_min, page_max = _u16(page_min), _u16(page_max)
    B, Hq, d = q.shape
    _, Hkv, Lmax, _ = K.shape
    Pmax = page_min.shape[2]
    seq_lens = _i32(seq_lens)
    tps = None if topk_per_seq is None else _i32(topk_per_seq)
    scores = np.empty((B, Hkv, Pmax), dtype=np.float64)
    sel = np.empty((B, Hkv, Kmax), dtype=np.int32)
    cnt = np.empty((B,), dtype=np.int32)
    gap = np.empty((B, Hkv), dtype=np.float64)
    out = np.empty((B, Hq, d), dtype=np.float64)
    _load().tso_query_aware_decode(_p(q), _p(K), _p(V), _p(page_min), _p(page_max), _p(seq_lens),
                                   B, Hq, Hkv, Lmax, d, S, Pmax, int(topk), _p(tps), Kmax,
                                   int(keep_first), int(keep_last), ctypes.c_double(scale), _p(scores), _p(sel), _p(cnt), _p(gap),
                                   _p(out))
    return dict(scores=scores, sel=sel, sel_count=cnt, gap=gap, out=out)


def true_page_max(q, K, seq_lens, S, Pmax):
    q, K = _u16(q), _u16(K)
    B, Hq, d = q.shape
    _, Hkv, Lmax, _ = K.shape
    seq_lens = _i32(seq_lens)
    best = np.empty((B, Hq, Pmax), dtype=np.float64)
    _load().tso_true_page_max(_p(q), _p(K), _p(seq_lens), B, Hq, Hkv, Lmax, d, S, Pmax, _p(best))
    return best


# ---------------------------------------------------------------------------
# INT8 KV cache (format defined in ts_oracle.c)
# ---------------------------------------------------------------------------
def _i8(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.int8, a.dtype
    return a


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def quantize_rows_i8(x):
    """bf16 bits [..., d] -> (int8 [..., d], float32 scale [...])."""
    x = _u16(x)
    d = x.shape[-1]
    n = x.size // d
    xq = np.empty(x.shape, dtype=np.int8)
    sc = np.empty(x.shape[:-1], dtype=np.float32)
    _load().tso_quantize_rows_i8(_p(x), n, d, _p(xq), _p(sc))
    return xq, sc


def build_page_meta_i8(Kq, ks, seq_lens, S, Pmax):
    Kq, ks = _i8(Kq), _f32(ks)
    B, Hkv, Lmax, d = Kq.shape
    seq_lens = _i32(seq_lens)
    pmin = np.zeros((B, Hkv, Pmax, d), dtype=np.uint16)
    pmax = np.zeros((B, Hkv, Pmax, d), dtype=np.uint16)
    _load().tso_build_page_meta_i8(_p(Kq), _p(ks), _p(seq_lens), B, Hkv, Lmax, d, S, Pmax, _p(pmin),
                                   _p(pmax))
    return pmin, pmax


def append_token_meta_i8(kq_new, ks_new, seq_lens, S, page_min, page_max):
    """In-place update of page_min / page_max (uint16 arrays) for one appended token."""
    kq_new, ks_new = _i8(kq_new), _f32(ks_new)
    B, Hkv, d = kq_new.shape
    assert page_min.dtype == np.uint16 and page_min.flags["C_CONTIGUOUS"]
    assert page_max.dtype == np.uint16 and page_max.flags["C_CONTIGUOUS"]
    Pmax = page_min.shape[2]
    seq_lens = _i32(seq_lens)
    _load().tso_append_token_meta_i8(_p(kq_new), _p(ks_new), _p(seq_lens), B, Hkv, d, S, Pmax,
                                     _p(page_min), _p(page_max))


def sparse_decode_attention_i8(q, Kq, ks, Vq, vs, sel, sel_count, seq_lens, S, scale,
                               return_lse=False):
    """sel = None: attention over every cached token (the dense baseline)."""
    q, Kq, Vq, ks, vs = _u16(q), _i8(Kq), _i8(Vq), _f32(ks), _f32(vs)
    B, Hq, d = q.shape
    _, Hkv, Lmax, _ = Kq.shape
    seq_lens = _i32(seq_lens)
    Kmax = 0
    if sel is not None:
        sel, sel_count = _i32(sel), _i32(sel_count)
        Kmax = sel.shape[2]
    out = np.empty((B, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64) if return_lse else None
    _load().tso_sparse_decode_attention_i8(
        _p(q), _p(Kq), _p(ks), _p(Vq), _p(vs), _p(sel), _p(sel_count) if sel is not None else None,
        _p(seq_lens), B, Hq, Hkv, Lmax, d, S, Kmax, ctypes.c_double(scale), _p(out), _p(lse))
    return (out, lse) if return_lse else out


def query_aware_decode_i8(q, Kq, ks, Vq, vs, page_min, page_max, seq_lens, S, topk, Kmax, scale,
                          topk_per_seq=None, keep_first=0, keep_last=0):
    q, Kq, Vq, ks, vs = _u16(q), _i8(Kq), _i8(Vq), _f32(ks), _f32(vs)
    page_min, page_max = _u16(page_min), _u16(page_max)
    B, Hq, d = q.shape
    _, Hkv, Lmax, _ = Kq.shape
    Pmax = page_min.shape[2]
    seq_lens = _i32(seq_lens)
    tps = None if topk_per_seq is None else _i32(topk_per_seq)
    scores = np.empty((B, Hkv, Pmax), dtype=np.float64)
    sel = np.empty((B, Hkv, Kmax), dtype=np.int32)
    cnt = np.empty((B,), dtype=np.int32)
    gap = np.empty((B, Hkv), dtype=np.float64)
    out = np.empty((B, Hq, d), dtype=np.float64)
    _load().tso_query_aware_decode_i8(
        _p(q), _p(Kq), _p(ks), _p(Vq), _p(vs), _p(page_min), _p(page_max), _p(seq_lens), B, Hq, Hkv,
        Lmax, d, S, Pmax, int(topk), _p(tps), Kmax, int(keep_first), int(keep_last),
        ctypes.c_double(scale), _p(scores), _p(sel), _p(cnt), _p(gap), _p(out))
    return dict(scores=scores, sel=sel, sel_count=cnt, gap=gap, out=out)
