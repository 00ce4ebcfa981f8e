"""Seeded synthetic decode workloads (input generation and page packing only).

This module draws random tensors and moves bytes between the logical view of a
KV cache ([token][channel] per sequence and KV head) and the paged pool layout
the HIP library reads.  It contains none of the method's arithmetic (no
min/max metadata, no scores, no selection, no attention), so both the HIP path
and the CPU oracle can be fed from it.

Pool layout (shared with include/tinyserve.h):
    k_pool  bf16 [num_phys_pages][Hkv][S][d]     one (page, head) K tile is S*d contiguous
    v_pool  bf16 [num_phys_pages][Hkv][d][S]     V tile stored channel-major (transposed)
    block_table int32 [B][P_max]                 logical page -> physical page
By default the two pools are strided views of ONE allocation
[num_phys_pages][Hkv][2][S*d], so the K and V tiles of a page are adjacent
(interleave=False gives two dense pools instead).
The five named workloads follow the shapes of the paper's small-model decoding
(GPT2-345M and TinyLLaMA head geometry, contexts 4K-128K, page size 16/32,
token budgets of 1/8 .. 1/4 of the pages); values are synthetic.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import torch


@dataclasses.dataclass(frozen=True)
class WorkloadSpec:
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    S: int
    L: int                     # context length (max length when ragged)
    topk: int                  # pages kept per (sequence, KV head); ignored if budget_frac
    keys: str = "normal"       # "normal" | "offset" | "walk"
    permute: bool = True       # physical pages randomly permuted in the shared pool
    L_min: int = 0             # ragged: lengths uniform in [L_min, L]; 0 = all equal L
    budget_frac: float = 0.0   # ragged: K_b = ceil(budget_frac * P_b)
    headroom: int = 64         # tokens of append room per sequence
    kv: str = "bf16"           # "bf16" | "fp16" (every 16-bit tensor IEEE half) |
                               # "int8" (int8 codes + one fp32 scale per token and head)


SPECS = {
    # batch 1, 1 q head / 1 KV head, 256 contiguous pages, keep 32
    "tiny": WorkloadSpec("tiny", 1, 1, 1, 64, 16, 4096, 32, permute=False),
    # GPT2-345M-shaped MHA: 16 heads x 64, 8K context, budget 1024 tokens
    "gpt2_345m": WorkloadSpec("gpt2_345m", 8, 16, 16, 64, 16, 8192, 64),
    # TinyLLaMA-shaped GQA 32/4, 16K context, outlier channels
    "tinyllama": WorkloadSpec("tinyllama", 16, 32, 4, 64, 16, 16384, 128, keys="offset"),
    # long-context GQA, 128K tokens, page 32, random-walk keys
    "longctx": WorkloadSpec("longctx", 4, 32, 4, 64, 32, 131072, 128, keys="walk"),
    # ragged serving batch, 64 sequences 1K..32K, d 128, budget 25 % of pages
    "ragged": WorkloadSpec("ragged", 64, 32, 32, 128, 16, 32768, 0, L_min=1024,
                           budget_frac=0.25),
}


def scaled(spec: WorkloadSpec, **kw) -> WorkloadSpec:
    """A copy of a named workload with some fields overridden (reduced test sizes)."""
    return dataclasses.replace(spec, **kw)


@dataclasses.dataclass
class Workload:
    spec: WorkloadSpec
    seq_lens: torch.Tensor        # int32 [B]   (device)
    P_max: int
    K_max: int
    topk: int
    topk_per_seq: Optional[torch.Tensor]   # int32 [B] or None
    num_phys_pages: int
    k_pool: torch.Tensor          # bf16 (or int8) [n_phys][Hkv][S][d]
    v_pool: torch.Tensor          # bf16 (or int8) [n_phys][Hkv][d][S]
    block_table: torch.Tensor     # int32 [B][P_max]
    q: torch.Tensor               # bf16 [n_q][B][Hq][d]
    k_new: torch.Tensor           # bf16 [n_new][B][Hkv][d]
    v_new: torch.Tensor           # bf16 [n_new][B][Hkv][d]
    k_scale: Optional[torch.Tensor] = None   # int8 cache: fp32 [n_phys][Hkv][S]
    v_scale: Optional[torch.Tensor] = None

    @property
    def device(self):
        return self.k_pool.device


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def budget_pages(spec: WorkloadSpec, seq_lens: torch.Tensor) -> torch.Tensor:
    """Per-sequence page budget of the ragged workload: max(1, ceil(frac * P_b))."""
    P = (seq_lens.to(torch.int64) + spec.S - 1) // spec.S
    kb = torch.ceil(P.to(torch.float64) * spec.budget_frac).to(torch.int64).clamp_(min=1)
    return torch.minimum(kb, P).to(torch.int32)


def _draw_keys(spec, g, Hkv, L, d, device, offset):
    """One sequence's keys, fp32 [Hkv][L][d], by the workload's recipe."""
    if spec.keys == "walk":
        steps = torch.randn((Hkv, L, d), generator=g, device=device, dtype=torch.float32) * 0.05
        k = torch.cumsum(steps, dim=1)
        k += torch.randn((Hkv, L, d), generator=g, device=device, dtype=torch.float32) * 0.5
        return k
    k = torch.randn((Hkv, L, d), generator=g, device=device, dtype=torch.float32)
    if spec.keys == "offset":
        k += offset[:, None, :]
    return k


def make_workload(spec: WorkloadSpec, device="cpu", seed=1000, n_q=1, n_new=1,
                  poison: float = float("nan"), interleave: bool = True) -> Workload:
    """Generate a workload on `device`.  Slots that hold no token (the tail of a
    partly filled page, the append headroom) are filled with `poison`."""
    device = torch.device(device)
    B, Hq, Hkv, d, S = spec.B, spec.Hq, spec.Hkv, spec.d, spec.S
    if spec.L_min:
        gl = torch.Generator(device="cpu")
        gl.manual_seed(int(seed) + 70)
        lens = torch.randint(spec.L_min, spec.L + 1, (B,), generator=gl, dtype=torch.int64)
    else:
        lens = torch.full((B,), spec.L, dtype=torch.int64)
    P_max = (spec.L + spec.headroom + S - 1) // S
    pages_alloc = (lens + spec.headroom + S - 1) // S          # per sequence, incl. headroom
    n_phys = int(pages_alloc.sum())
    if spec.permute:
        gp = torch.Generator(device="cpu")
        gp.manual_seed(int(seed) + 50)
        perm = torch.randperm(n_phys, generator=gp, dtype=torch.int64)
    else:
        perm = torch.arange(n_phys, dtype=torch.int64)
    block_table = torch.full((B, P_max), -1, dtype=torch.int32)
    start = 0
    for b in range(B):
        n = int(pages_alloc[b])
        block_table[b, :n] = perm[start:start + n].to(torch.int32)
        start += n

    int8 = spec.kv == "int8"
    e16 = torch.float16 if spec.kv == "fp16" else torch.bfloat16     # 16-bit element type
    dt = torch.int8 if int8 else e16
    fill = -128 if int8 else poison          # code -128 is never generated
    if interleave:
        kv = torch.full((n_phys, Hkv, 2, S * d), fill, dtype=dt, device=device)
        k_pool = kv[:, :, 0].view(n_phys, Hkv, S, d)
        v_pool = kv[:, :, 1].view(n_phys, Hkv, d, S)
    else:
        k_pool = torch.full((n_phys, Hkv, S, d), fill, dtype=dt, device=device)
        v_pool = torch.full((n_phys, Hkv, d, S), fill, dtype=dt, device=device)
    k_scale = v_scale = None
    if int8:
        k_scale = torch.full((n_phys, Hkv, S), poison, dtype=torch.float32, device=device)
        v_scale = torch.full((n_phys, Hkv, S), poison, dtype=torch.float32, device=device)
    g = _gen(device, seed)
    offset = torch.randn((Hkv, d), generator=g, device=device, dtype=torch.float32) * 2.0
    bt_dev = block_table.to(device)

    def codes_of(x):
        """int8 codes and per-token scales carrying the structure of the fp32 draw x
        [Hkv][L][d].  (A way to get int8 data of the workload's shape; it is not the
        library's quantiser, which only ts_append_token_meta exercises.)"""
        jitter = 1.0 + 0.05 * torch.rand(x.shape[:2], generator=g, device=device)
        sc = (x.abs().amax(dim=-1).clamp_(min=1e-6) / 120.0) * jitter
        return torch.round(x / sc[..., None]).clamp_(-127, 127).to(torch.int8), sc

    for b in range(B):
        L = int(lens[b])
        Pb = (L + S - 1) // S
        k = _draw_keys(spec, g, Hkv, L, d, device, offset)
        v = torch.randn((Hkv, L, d), generator=g, device=device, dtype=torch.float32)
        phys = bt_dev[b, :Pb].to(torch.int64)
        if int8:
            k, ks = codes_of(k)
            v, vs = codes_of(v)
            ksp = torch.full((Hkv, Pb * S), poison, dtype=torch.float32, device=device)
            vsp = torch.full((Hkv, Pb * S), poison, dtype=torch.float32, device=device)
            ksp[:, :L] = ks
            vsp[:, :L] = vs
            k_scale[phys] = ksp.view(Hkv, Pb, S).permute(1, 0, 2)
            v_scale[phys] = vsp.view(Hkv, Pb, S).permute(1, 0, 2)
        else:
            k, v = k.to(e16), v.to(e16)
        kp = torch.full((Hkv, Pb * S, d), fill, dtype=dt, device=device)
        vp = torch.full((Hkv, Pb * S, d), fill, dtype=dt, device=device)
        kp[:, :L] = k
        vp[:, :L] = v
        k_pool[phys] = kp.view(Hkv, Pb, S, d).permute(1, 0, 2, 3)
        v_pool[phys] = vp.view(Hkv, Pb, S, d).permute(1, 0, 3, 2)
        del k, v, kp, vp
    q = torch.randn((n_q, B, Hq, d), generator=g, device=device,
                    dtype=torch.float32).to(e16)
    k_new = torch.randn((n_new, B, Hkv, d), generator=g, device=device, dtype=torch.float32)
    if spec.keys == "offset":
        k_new += offset[None, None]
    k_new = k_new.to(e16)
    v_new = torch.randn((n_new, B, Hkv, d), generator=g, device=device,
                        dtype=torch.float32).to(e16)

    seq_lens = lens.to(torch.int32).to(device)
    if spec.budget_frac > 0:
        # budget counted on the page count after the step's append
        tps = budget_pages(spec, (lens + 1).to(torch.int32)).to(device)
        K_max = int(math.ceil(spec.budget_frac * ((spec.L + spec.headroom + S - 1) // S))) + 1
        topk = K_max
    else:
        tps = None
        K_max = spec.topk
        topk = spec.topk
    return Workload(spec, seq_lens, P_max, K_max, topk, tps, n_phys, k_pool, v_pool, bt_dev, q,
                    k_new, v_new, k_scale, v_scale)


def logical_kv(w: Workload, seqs=None, heads=None, seq_lens=None):
    """Gather the logical keys / values [len(seqs)][len(heads)][Lmax][d] (bf16, zero
    padded past each sequence's length) out of the paged pool, through the block
    table.  `seq_lens` overrides the workload's lengths (after appends)."""
    spec = w.spec
    S, d = spec.S, spec.d
    lens = (w.seq_lens if seq_lens is None else seq_lens).to("cpu", torch.int64)
    seqs = list(range(spec.B)) if seqs is None else list(seqs)
    heads = list(range(spec.Hkv)) if heads is None else list(heads)
    Lmax = max(int(lens[b]) for b in seqs)
    Lmax = max(Lmax, 1)
    hidx = torch.tensor(heads, dtype=torch.int64, device=w.device)
    K = torch.zeros((len(seqs), len(heads), Lmax, d), dtype=w.k_pool.dtype, device=w.device)
    V = torch.zeros_like(K)
    for i, b in enumerate(seqs):
        L = int(lens[b])
        Pb = (L + S - 1) // S
        if Pb == 0:
            continue
        phys = w.block_table[b, :Pb].to(torch.int64)
        kp = w.k_pool[phys][:, hidx]                    # [Pb][nh][S][d]
        vp = w.v_pool[phys][:, hidx]                    # [Pb][nh][d][S]
        K[i, :, :L] = kp.permute(1, 0, 2, 3).reshape(len(heads), Pb * S, d)[:, :L]
        V[i, :, :L] = vp.permute(1, 0, 3, 2).reshape(len(heads), Pb * S, d)[:, :L]
    return K, V


def logical_kv_i8(w: Workload, seqs=None, heads=None, seq_lens=None):
    """INT8 cache: logical codes [n][nh][Lmax][d] (int8, zero padded) and scales
    [n][nh][Lmax] (fp32, one padded) of keys and values: (Kq, ks, Vq, vs)."""
    spec = w.spec
    S, d = spec.S, spec.d
    lens = (w.seq_lens if seq_lens is None else seq_lens).to("cpu", torch.int64)
    seqs = list(range(spec.B)) if seqs is None else list(seqs)
    heads = list(range(spec.Hkv)) if heads is None else list(heads)
    Lmax = max(max(int(lens[b]) for b in seqs), 1)
    hidx = torch.tensor(heads, dtype=torch.int64, device=w.device)
    Kq = torch.zeros((len(seqs), len(heads), Lmax, d), dtype=torch.int8, device=w.device)
    Vq = torch.zeros_like(Kq)
    ks = torch.ones((len(seqs), len(heads), Lmax), dtype=torch.float32, device=w.device)
    vs = torch.ones_like(ks)
    for i, b in enumerate(seqs):
        L = int(lens[b])
        Pb = (L + S - 1) // S
        if Pb == 0:
            continue
        phys = w.block_table[b, :Pb].to(torch.int64)
        kp = w.k_pool[phys][:, hidx]
        vp = w.v_pool[phys][:, hidx]
        Kq[i, :, :L] = kp.permute(1, 0, 2, 3).reshape(len(heads), Pb * S, d)[:, :L]
        Vq[i, :, :L] = vp.permute(1, 0, 3, 2).reshape(len(heads), Pb * S, d)[:, :L]
        ks[i, :, :L] = w.k_scale[phys][:, hidx].permute(1, 0, 2).reshape(len(heads), Pb * S)[:, :L]
        vs[i, :, :L] = w.v_scale[phys][:, hidx].permute(1, 0, 2).reshape(len(heads), Pb * S)[:, :L]
    return Kq, ks, Vq, vs


def bits(t: torch.Tensor):
    """bf16 (or float16) tensor -> numpy uint16 bit patterns (host copy)."""
    import numpy as np
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def from_bits(a, device="cpu", dtype=torch.bfloat16) -> torch.Tensor:
    """numpy uint16 bit patterns -> bf16 (or float16) tensor."""
    import numpy as np
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16).copy()).view(dtype).to(device)


def algorithmic_bytes(spec: WorkloadSpec, seq_lens, topk_per_seq=None) -> dict:
    """Bytes the method must move per decode step: 2*d bf16 per page scanned
    (min and max rows) plus S*d bf16 of K and of V per selected page, per
    (sequence, KV head).  Returns the dense-attention bytes alongside."""
    lens = seq_lens.to("cpu", torch.int64)
    P = (lens + spec.S - 1) // spec.S
    if topk_per_seq is not None:
        Kb = torch.minimum(topk_per_seq.to("cpu", torch.int64), P)
    else:
        Kb = torch.clamp(P, max=spec.topk)
    tok = 2 * spec.d + 8 if spec.kv == "int8" else 2 * spec.d * 2   # K + V (+ two scales) per token
    meta = int(P.sum()) * spec.Hkv * 2 * spec.d * 2
    kv = int(Kb.sum()) * spec.Hkv * spec.S * tok
    dense = int((P * spec.S).sum()) * spec.Hkv * tok
    return {"meta": meta, "kv": kv, "total": meta + kv, "dense": dense}
