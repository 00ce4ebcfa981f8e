"""CPU-only checks of the C-ABI boundary: the library loads, exports every
symbol include/tinyserve.h declares, and validates arguments on the host
(error codes come back without any device work)."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2509_12211_amd import tinyserve as ts

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    with open(os.path.join(ROOT, "include", "tinyserve.h")) as f:
        text = f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ts_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ts.lib()
    names = declared_symbols()
    assert set(names) == set(ts.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    assert lib.ts_version() >= 1
    assert ts.strerror(ts.TS_OK) == "ok"
    assert "workspace" in ts.strerror(ts.TS_ERR_WORKSPACE)


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "tinyserve.h"\nint main(void) { ts_layout l; (void)l; return TS_OK; }\n')
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)


def _layout(**kw):
    base = dict(num_seqs=2, num_q_heads=8, num_kv_heads=2, head_dim=64, page_size=16,
                max_pages_per_seq=64, num_phys_pages=128, kv_tile_stride=0,
                k_pool=0x1000, v_pool=0x1000, block_table=0x1000, seq_lens=0x1000,
                page_min=0x1000, page_max=0x1000)
    base.update(kw)
    return ts.TsLayout(**base)


def test_struct_layout_matches_the_header(tmp_path):
    """The ctypes mirror of ts_layout has the size and field offsets the C compiler
    gives the struct in the header."""
    fields = [n for n, _ in ts.TsLayout._fields_]
    src = tmp_path / "lay.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "tinyserve.h"\n'
        'int main(void) {\n  printf("%zu", sizeof(ts_layout));\n'
        + "".join(f'  printf(" %zu", offsetof(ts_layout, {n}));\n' for n in fields)
        + "  return 0;\n}\n")
    exe = tmp_path / "lay"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True,
                                          text=True).stdout.split()]
    assert got[0] == ctypes.sizeof(ts.TsLayout)
    assert got[1:] == [getattr(ts.TsLayout, n).offset for n in fields]


def test_workspace_bytes_is_host_only_and_monotone():
    lay = _layout()
    n1 = ts.workspace_bytes(lay, 8)
    n2 = ts.workspace_bytes(lay, 64)
    assert 0 < n1 <= n2
    assert ts.workspace_bytes(lay, 0) == 0
    assert ts.workspace_bytes(_layout(head_dim=96), 8) == 0


@pytest.mark.parametrize("kw,code", [
    (dict(num_seqs=0), ts.TS_ERR_SHAPE),
    (dict(num_q_heads=7), ts.TS_ERR_SHAPE),
    (dict(keep_first_pages=-1), ts.TS_ERR_SHAPE),
    (dict(out_format=7), ts.TS_ERR_UNSUPPORTED),
    (dict(keep_last_pages=-2), ts.TS_ERR_SHAPE),
    (dict(cluster_size=-1), ts.TS_ERR_SHAPE),
    (dict(wait_limit=-1), ts.TS_ERR_SHAPE),
    (dict(max_pages_per_seq=-1), ts.TS_ERR_SHAPE),
    (dict(kv_tile_stride=512), ts.TS_ERR_SHAPE),      # smaller than one S*d tile
    (dict(kv_tile_stride=2052), ts.TS_ERR_SHAPE),     # tiles must stay 16-byte aligned
    (dict(head_dim=96), ts.TS_ERR_UNSUPPORTED),
    (dict(page_size=12), ts.TS_ERR_UNSUPPORTED),
    (dict(num_q_heads=64, num_kv_heads=2), ts.TS_ERR_UNSUPPORTED),
    (dict(max_pages_per_seq=1 << 20), ts.TS_ERR_UNSUPPORTED),
    (dict(page_min=None), ts.TS_ERR_NULL),
    (dict(seq_lens=None), ts.TS_ERR_NULL),
])
def test_layout_validation(kw, code):
    lib = ts.lib()
    lay = _layout(**kw)
    q = ctypes.c_void_p(0x1000)
    assert lib.ts_score_pages(ctypes.byref(lay), q, q, None) == code
    assert lib.ts_build_page_meta(ctypes.byref(lay), None) == code
    assert lib.ts_query_aware_decode(ctypes.byref(lay), q, 4, None, 4, 1.0, q, None, None, None, q,
                                     1 << 30, None) == code


def test_argument_validation():
    lib = ts.lib()
    lay = _layout()
    p = ctypes.c_void_p(0x1000)
    big = 1 << 30
    assert lib.ts_score_pages(None, p, p, None) == ts.TS_ERR_NULL
    assert lib.ts_score_pages(ctypes.byref(lay), None, p, None) == ts.TS_ERR_NULL
    assert lib.ts_append_token_meta(ctypes.byref(lay), None, None, 1, None) == ts.TS_ERR_NULL
    assert lib.ts_select_topk_pages(ctypes.byref(lay), p, 0, None, 8, p, p, None) == ts.TS_ERR_SHAPE
    assert lib.ts_select_topk_pages(ctypes.byref(lay), p, 9, None, 8, p, p, None) == ts.TS_ERR_SHAPE
    assert lib.ts_select_topk_pages(ctypes.byref(lay), p, 4, None, 8, None, p, None) == ts.TS_ERR_NULL
    assert lib.ts_sparse_decode_attention(ctypes.byref(lay), p, p, p, 8, 1.0, p, None, p, 16,
                                          None) == ts.TS_ERR_WORKSPACE
    assert lib.ts_sparse_decode_attention(ctypes.byref(lay), p, p, p, 8, 1.0, None, None, p, big,
                                          None) == ts.TS_ERR_NULL
    assert lib.ts_query_aware_decode(ctypes.byref(lay), p, 4, None, 8, 1.0, p, None, None, None, p,
                                     16, None) == ts.TS_ERR_WORKSPACE
    assert lib.ts_query_aware_decode(ctypes.byref(lay), p, 0, None, 8, 1.0, p, None, None, None, p,
                                     big, None) == ts.TS_ERR_SHAPE
    assert lib.ts_query_aware_decode(ctypes.byref(lay), p, 9, None, 8, 1.0, p, None, None, None, p,
                                     big, None) == ts.TS_ERR_SHAPE
    assert lib.ts_append_and_decode(ctypes.byref(lay), None, p, p, 4, None, 8, 1.0, p, None, None,
                                    None, p, big, None) == ts.TS_ERR_NULL
    assert lib.ts_append_and_decode(ctypes.byref(lay), p, p, p, 4, None, 8, 1.0, p, None, None,
                                    None, p, 16, None) == ts.TS_ERR_WORKSPACE
    assert lib.ts_dense_decode_attention(ctypes.byref(lay), p, 1.0, p, None, p, 16,
                                         None) == ts.TS_ERR_WORKSPACE
    assert lib.ts_dense_decode_attention(ctypes.byref(lay), None, 1.0, p, None, p, big,
                                         None) == ts.TS_ERR_NULL
    assert lib.ts_dense_workspace_bytes(ctypes.byref(lay)) > 0
    assert lib.ts_dense_workspace_bytes(ctypes.byref(_layout(head_dim=96))) == 0
    assert lib.ts_workspace_init(None, 1024, None) == ts.TS_ERR_NULL
    assert lib.ts_workspace_init(p, 8, None) == ts.TS_ERR_WORKSPACE
    assert lib.ts_workspace_status(None, None) == ts.TS_ERR_NULL
    assert lib.ts_set_tuning(-1, 0, 0) == ts.TS_ERR_SHAPE
    assert lib.ts_set_tuning(1, 0, 0) == ts.TS_ERR_SHAPE      # reserved must be 0
    assert lib.ts_set_tuning(0, -1, 0) == ts.TS_ERR_SHAPE


@pytest.mark.parametrize("missing", ["k_scale", "v_scale"])
def test_int8_cache_needs_both_scale_arrays(missing):
    """Every call that reads or writes an INT8 pool dereferences the per-token scales on
    the device: a forgotten array is a host-side error, not a GPU fault."""
    lib = ts.lib()
    scales = dict(k_scale=0x1000, v_scale=0x1000)
    scales[missing] = None
    lay = _layout(kv_format=ts.TS_KV_INT8, kv_tile_stride=1024, **scales)
    good = _layout(kv_format=ts.TS_KV_INT8, kv_tile_stride=1024, k_scale=0x1000, v_scale=0x1000)
    p = ctypes.c_void_p(0x1000)
    big = 1 << 30
    L = ctypes.byref(lay)
    assert lib.ts_query_aware_decode(L, p, 4, None, 8, 1.0, p, None, None, None, p, big,
                                     None) == ts.TS_ERR_NULL
    assert lib.ts_append_and_decode(L, p, p, p, 4, None, 8, 1.0, p, None, None, None, p, big,
                                    None) == ts.TS_ERR_NULL
    assert lib.ts_sparse_decode_attention(L, p, p, p, 8, 1.0, p, None, p, big, None) == ts.TS_ERR_NULL
    assert lib.ts_dense_decode_attention(L, p, 1.0, p, None, p, big, None) == ts.TS_ERR_NULL
    assert lib.ts_append_token_meta(L, p, p, 1, None) == ts.TS_ERR_NULL
    if missing == "k_scale":
        assert lib.ts_build_page_meta(L, None) == ts.TS_ERR_NULL
    # with both arrays the same calls get past the pointer checks (and stop at the workspace size)
    assert lib.ts_query_aware_decode(ctypes.byref(good), p, 4, None, 8, 1.0, p, None, None, None, p,
                                     16, None) == ts.TS_ERR_WORKSPACE


def test_cluster_size_changes_workspace_plan():
    lay1 = _layout(num_seqs=16, max_pages_per_seq=1024, cluster_size=1)
    lay8 = _layout(num_seqs=16, max_pages_per_seq=1024, cluster_size=8)
    assert 0 < ts.workspace_bytes(lay1, 128) < ts.workspace_bytes(lay8, 128)
    try:   # the layout's own value wins over the process-wide override
        ts.set_tuning(0, 32, 0)
        assert ts.workspace_bytes(lay1, 128) < ts.workspace_bytes(lay8, 128)
    finally:
        ts.set_tuning(0, 0, 0)


def test_tuning_changes_workspace_plan():
    lay = _layout(num_seqs=16, max_pages_per_seq=1024)
    try:
        ts.set_tuning(0, 1, 0)
        small = ts.workspace_bytes(lay, 128)
        ts.set_tuning(0, 32, 0)
        large = ts.workspace_bytes(lay, 128)
        assert large > small
    finally:
        ts.set_tuning(0, 0, 0)


def test_static_workspace_entry_rejects_what_does_not_fit():
    """ts_query_aware_decode_static has a fixed region to work in: a layout that needs more is
    turned away on the host (before the region is even looked up)."""
    lay = _layout(num_seqs=8, num_q_heads=16, num_kv_heads=4, max_pages_per_seq=16384,
                  num_phys_pages=1 << 20)
    assert ts.workspace_bytes(lay, 512) > ts.STATIC_WORKSPACE_BYTES
    p = ctypes.c_void_p(0x1000)
    call = ts.lib().ts_query_aware_decode_static
    assert call(ctypes.byref(lay), p, 512, None, 512, 1.0, p, None, None, None,
                None) == ts.TS_ERR_WORKSPACE
    assert call(ctypes.byref(_layout(head_dim=96)), p, 4, None, 4, 1.0, p, None, None, None,
                None) == ts.TS_ERR_UNSUPPORTED
    assert call(None, p, 4, None, 4, 1.0, p, None, None, None, None) == ts.TS_ERR_NULL


def test_binding_raises_without_library(monkeypatch):
    """No silent fallback: a missing library is an error."""
    monkeypatch.setattr(ts, "_lib", None)
    monkeypatch.setattr(ts, "LIB_PATH", os.path.join(ROOT, "does_not_exist.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        ts.lib()
