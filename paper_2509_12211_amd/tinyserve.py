"""Thin ctypes binding over libtinyserve_hip.so (C ABI in include/tinyserve.h).

Argument marshalling only: every step of the decode path runs in the HIP
kernels.  Tensors are torch CUDA(ROCm) tensors used purely as device buffers;
the launch goes to torch's current stream.  There is no fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtinyserve_hip.so")

TS_OK = 0
TS_ERR_NULL = -1
TS_ERR_SHAPE = -2
TS_ERR_UNSUPPORTED = -3
TS_ERR_WORKSPACE = -4
TS_ERR_LAUNCH = -5
TS_ERR_DEVICE = -6
TS_OUT_F32 = 0
TS_OUT_BF16 = 1
TS_KV_BF16 = 0
TS_KV_INT8 = 1
TS_KV_FP16 = 2

EXPORTS = [
    "ts_build_page_meta", "ts_append_token_meta", "ts_score_pages", "ts_select_topk_pages",
    "ts_sparse_decode_attention", "ts_query_aware_decode", "ts_append_and_decode",
    "ts_append_and_decode_launches", "ts_dense_workspace_bytes", "ts_dense_decode_attention", "ts_workspace_bytes",
    "ts_workspace_init", "ts_workspace_status", "ts_set_tuning", "ts_strerror", "ts_version",
    "ts_debug_xcc_ids", "ts_query_aware_decode_static",
]


class TsLayout(ctypes.Structure):
    _fields_ = [
        ("num_seqs", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("max_pages_per_seq", ctypes.c_int32),
        ("num_phys_pages", ctypes.c_int32), ("kv_tile_stride", ctypes.c_int32),
        ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p),
        ("block_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
        ("page_min", ctypes.c_void_p), ("page_max", ctypes.c_void_p),
        ("keep_first_pages", ctypes.c_int32), ("keep_last_pages", ctypes.c_int32),
        ("out_format", ctypes.c_int32), ("kv_format", ctypes.c_int32),
        ("cluster_size", ctypes.c_int32), ("wait_limit", ctypes.c_int32),
        ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
    ]


class TinyServeError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


_lib = None


def lib():
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first "
                "(python -c 'import __graft_entry__ as g; g.build()'); there is no CPU fallback")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t, ctypes.c_float
        lp = ctypes.POINTER(TsLayout)
        L.ts_build_page_meta.argtypes = [lp, vp]
        L.ts_append_token_meta.argtypes = [lp, vp, vp, ctypes.c_int, vp]
        L.ts_score_pages.argtypes = [lp, vp, vp, vp]
        L.ts_select_topk_pages.argtypes = [lp, vp, i32, vp, i32, vp, vp, vp]
        L.ts_sparse_decode_attention.argtypes = [lp, vp, vp, vp, i32, f32, vp, vp, vp, sz, vp]
        L.ts_query_aware_decode.argtypes = [lp, vp, i32, vp, i32, f32, vp, vp, vp, vp, vp, sz, vp]
        L.ts_query_aware_decode_static.argtypes = [lp, vp, i32, vp, i32, f32, vp, vp, vp, vp, vp]
        L.ts_append_and_decode.argtypes = [lp, vp, vp, vp, i32, vp, i32, f32, vp, vp, vp, vp, vp, sz, vp]
        L.ts_append_and_decode_launches.argtypes = [lp, i32]
        L.ts_dense_workspace_bytes.argtypes = [lp]
        L.ts_dense_workspace_bytes.restype = sz
        L.ts_dense_decode_attention.argtypes = [lp, vp, f32, vp, vp, vp, sz, vp]
        L.ts_workspace_bytes.argtypes = [lp, i32]
        L.ts_workspace_bytes.restype = sz
        L.ts_workspace_init.argtypes = [vp, sz, vp]
        L.ts_workspace_status.argtypes = [vp, ctypes.POINTER(ctypes.c_int32)]
        L.ts_set_tuning.argtypes = [i32, i32, i32]
        L.ts_debug_xcc_ids.argtypes = [vp, i32, vp]
        L.ts_strerror.argtypes = [ctypes.c_int]
        L.ts_strerror.restype = ctypes.c_char_p
        L.ts_version.restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().ts_strerror(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, where):
    if status != TS_OK:
        raise TinyServeError(status, where)


def make_layout(B, Hq, Hkv, d, S, P_max, k_pool, v_pool, block_table, seq_lens, page_min,
                page_max, keep_first_pages=0, keep_last_pages=0, out_format=TS_OUT_F32,
                k_scale=None, v_scale=None, cluster_size=0, wait_limit=0) -> TsLayout:
    """Fill the C struct; tensors must stay alive while calls using it are in flight.
    int8 pools (with k_scale / v_scale) select the INT8 cache format, float16 pools the
    FP16 one (q, new tokens and metadata must then be float16 too)."""
    n_phys = 0 if k_pool is None else k_pool.shape[0]
    tile_stride = 0
    if k_pool is not None and Hkv > 1:
        # [n_phys][Hkv][...]: distance between the tiles of two heads (S*d for dense pools,
        # 2*S*d when the K and V tiles of a page are interleaved in one allocation)
        tile_stride = int(k_pool.stride(1))
        assert k_pool.stride(0) == Hkv * tile_stride and v_pool.stride(1) == tile_stride
    elif k_pool is not None:
        tile_stride = int(k_pool.stride(0))
    lay = TsLayout(B, Hq, Hkv, d, S, P_max, n_phys, tile_stride,
                   None if k_pool is None else k_pool.data_ptr(),
                   None if v_pool is None else v_pool.data_ptr(),
                   None if block_table is None else block_table.data_ptr(),
                   None if seq_lens is None else seq_lens.data_ptr(),
                   None if page_min is None else page_min.data_ptr(),
                   None if page_max is None else page_max.data_ptr(),
                   int(keep_first_pages), int(keep_last_pages), int(out_format),
                   (TS_KV_BF16 if k_pool is None else
                    {torch.int8: TS_KV_INT8, torch.float16: TS_KV_FP16}.get(k_pool.dtype, TS_KV_BF16)),
                   int(cluster_size), int(wait_limit),
                   None if k_scale is None else k_scale.data_ptr(),
                   None if v_scale is None else v_scale.data_ptr())
    return lay


def build_page_meta(layout):
    _check(lib().ts_build_page_meta(ctypes.byref(layout), _stream()), "ts_build_page_meta")


def append_token_meta(layout, k_new, v_new=None, advance_seq_lens=True):
    _check(lib().ts_append_token_meta(ctypes.byref(layout), _ptr(k_new), _ptr(v_new),
                                      1 if advance_seq_lens else 0, _stream()),
           "ts_append_token_meta")


def score_pages(layout, q, scores):
    _check(lib().ts_score_pages(ctypes.byref(layout), _ptr(q), _ptr(scores), _stream()),
           "ts_score_pages")


def select_topk_pages(layout, scores, topk, max_topk, sel, sel_count, topk_per_seq=None):
    _check(lib().ts_select_topk_pages(ctypes.byref(layout), _ptr(scores), int(topk),
                                      _ptr(topk_per_seq), int(max_topk), _ptr(sel),
                                      _ptr(sel_count), _stream()), "ts_select_topk_pages")


def workspace_bytes(layout, max_topk) -> int:
    return int(lib().ts_workspace_bytes(ctypes.byref(layout), int(max_topk)))


def workspace_init(workspace):
    _check(lib().ts_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream()), "ts_workspace_init")


def workspace_status(workspace) -> int:
    v = ctypes.c_int32(0)
    _check(lib().ts_workspace_status(_ptr(workspace), ctypes.byref(v)), "ts_workspace_status")
    return int(v.value)


def new_workspace(layout, max_topk, device) -> torch.Tensor:
    """Allocate (with torch) and initialise a workspace for this layout."""
    n = workspace_bytes(layout, max_topk)
    if n == 0:
        raise TinyServeError(TS_ERR_SHAPE, "ts_workspace_bytes")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    workspace_init(ws)
    return ws


def sparse_decode_attention(layout, q, sel, sel_count, max_topk, softmax_scale, out, workspace,
                            lse_out=None):
    _check(lib().ts_sparse_decode_attention(
        ctypes.byref(layout), _ptr(q), _ptr(sel), _ptr(sel_count), int(max_topk),
        float(softmax_scale), _ptr(out), _ptr(lse_out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream()), "ts_sparse_decode_attention")


def query_aware_decode(layout, q, topk, max_topk, softmax_scale, out, workspace,
                       topk_per_seq=None, scores_out=None, sel_out=None, sel_count_out=None):
    _check(lib().ts_query_aware_decode(
        ctypes.byref(layout), _ptr(q), int(topk), _ptr(topk_per_seq), int(max_topk),
        float(softmax_scale), _ptr(out), _ptr(scores_out), _ptr(sel_out), _ptr(sel_count_out),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
        "ts_query_aware_decode")


STATIC_WORKSPACE_BYTES = 4 << 20


def query_aware_decode_static(layout, q, topk, max_topk, softmax_scale, out, topk_per_seq=None,
                              scores_out=None, sel_out=None, sel_count_out=None):
    """ts_query_aware_decode on the library's own fixed workspace (allocates nothing)."""
    _check(lib().ts_query_aware_decode_static(
        ctypes.byref(layout), _ptr(q), int(topk), _ptr(topk_per_seq), int(max_topk),
        float(softmax_scale), _ptr(out), _ptr(scores_out), _ptr(sel_out), _ptr(sel_count_out),
        _stream()), "ts_query_aware_decode_static")


def append_and_decode(layout, k_new, v_new, q, topk, max_topk, softmax_scale, out, workspace,
                      topk_per_seq=None, scores_out=None, sel_out=None, sel_count_out=None):
    _check(lib().ts_append_and_decode(
        ctypes.byref(layout), _ptr(k_new), _ptr(v_new), _ptr(q), int(topk), _ptr(topk_per_seq),
        int(max_topk), float(softmax_scale), _ptr(out), _ptr(scores_out), _ptr(sel_out),
        _ptr(sel_count_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
        _stream()), "ts_append_and_decode")


def new_dense_workspace(layout, device) -> torch.Tensor:
    n = int(lib().ts_dense_workspace_bytes(ctypes.byref(layout)))
    if n == 0:
        raise TinyServeError(TS_ERR_SHAPE, "ts_dense_workspace_bytes")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    workspace_init(ws)
    return ws


def dense_decode_attention(layout, q, softmax_scale, out, workspace, lse_out=None):
    _check(lib().ts_dense_decode_attention(
        ctypes.byref(layout), _ptr(q), float(softmax_scale), _ptr(out), _ptr(lse_out),
        _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream()), "ts_dense_decode_attention")


def append_and_decode_launches(layout, max_topk) -> int:
    n = int(lib().ts_append_and_decode_launches(ctypes.byref(layout), int(max_topk)))
    if n < 0:
        raise TinyServeError(n, "ts_append_and_decode_launches")
    return n


def debug_xcc_ids(num_workgroups, device) -> torch.Tensor:
    """int32 [num_workgroups]: the XCD each workgroup of a probe launch ran on."""
    ids = torch.full((int(num_workgroups),), -1, dtype=torch.int32, device=device)
    _check(lib().ts_debug_xcc_ids(_ptr(ids), int(num_workgroups), _stream()), "ts_debug_xcc_ids")
    return ids


def set_tuning(reserved=0, num_splits=0, workgroups_per_cu=0):
    _check(lib().ts_set_tuning(int(reserved), int(num_splits),
                               int(workgroups_per_cu)), "ts_set_tuning")
