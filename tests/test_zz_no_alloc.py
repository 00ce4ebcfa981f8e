"""The allocation-free entry point, ts_query_aware_decode_static, against
ts_query_aware_decode on the same inputs: two calls in a row on the library's own
workspace, the second on a smaller input, then the first again."""
import math

import pytest
import torch

from paper_2509_12211_amd import tinyserve as ts
from paper_2509_12211_amd import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def run_both(spec, seed, cluster_size=0):
    """(static, reference) outputs / scores / selections of one workload."""
    w = wl.make_workload(spec, DEV, seed=seed, n_q=1, n_new=1)
    pmin = torch.zeros((spec.B, spec.Hkv, w.P_max, spec.d), dtype=w.k_pool.dtype, device=DEV)
    pmax = torch.zeros_like(pmin)
    lens = w.seq_lens.clone()
    lay = ts.make_layout(spec.B, spec.Hq, spec.Hkv, spec.d, spec.S, w.P_max, w.k_pool, w.v_pool,
                         w.block_table, lens, pmin, pmax, cluster_size=cluster_size)
    ts.build_page_meta(lay)
    scale = 1.0 / math.sqrt(spec.d)
    res = []
    for static in (True, False):
        out = torch.full((spec.B, spec.Hq, spec.d), float("nan"), dtype=torch.float32, device=DEV)
        scores = torch.full((spec.B, spec.Hkv, w.P_max), float("nan"), dtype=torch.float32, device=DEV)
        sel = torch.full((spec.B, spec.Hkv, w.K_max), -7, dtype=torch.int32, device=DEV)
        cnt = torch.full((spec.B,), -7, dtype=torch.int32, device=DEV)
        kw = dict(topk_per_seq=w.topk_per_seq, scores_out=scores, sel_out=sel, sel_count_out=cnt)
        if static:
            assert ts.workspace_bytes(lay, w.K_max) <= ts.STATIC_WORKSPACE_BYTES
            ts.query_aware_decode_static(lay, w.q[0], w.topk, w.K_max, scale, out, **kw)
        else:
            ws = ts.new_workspace(lay, w.K_max, DEV)
            ts.query_aware_decode(lay, w.q[0], w.topk, w.K_max, scale, out, ws, **kw)
            torch.cuda.synchronize()
            assert ts.workspace_status(ws) == 0
        torch.cuda.synchronize()
        res.append((out, scores, sel, cnt))
    return res


def same(a, b, what):
    for x, y, n in zip(a, b, ("out", "scores", "sel", "sel_count")):
        assert torch.equal(x.view(torch.int32), y.view(torch.int32)), f"{what}: {n} differs"
    assert torch.isfinite(a[0]).all(), what


def test_static_workspace_entry_matches_the_workspace_one():
    ts.lib()
    big = wl.WorkloadSpec("na_big", 4, 16, 2, 64, 16, 9000, 48, keys="offset")       # 8 units in clusters of 12
    small = wl.WorkloadSpec("na_small", 2, 4, 4, 128, 32, 1500, 6, L_min=300)
    many = wl.WorkloadSpec("na_many", 70, 4, 4, 64, 16, 700, 5, L_min=100)          # one workgroup per unit
    for rnd in range(2):
        for spec, seed in ((big, 11), (small, 12), (many, 13), (small, 14)):
            print(f"[case] static workspace, round {rnd}, {spec.name}", flush=True)
            s, r = run_both(spec, seed)
            same(s, r, f"{spec.name} round {rnd}")
    print("[case] static workspace, forced single workgroup", flush=True)
    s, r = run_both(big, 15, cluster_size=1)
    same(s, r, "cluster_size=1")
