// Sparse single-query attention over the selected pages (Section 3.5 SparseAttn;
// steps 3-4 of Algorithm 1) with bf16 MFMA and an online softmax, split over
// workgroups (flash-decoding style partial softmax + combine).
//
// One wavefront processes whole pages.  Per 16-token tile it computes
//   St[token][head] = K_tile[token][:] . Q^T[:][head]        (v_mfma_f32_16x16x16_bf16)
//   Ot[chan ][head] += V_tile^T[chan][token] . P^T[token][head]
// The accumulator layout of the first product (lane -> head lane%16, tokens
// 4*(lane/16)..+3) is exactly the B-operand layout of the second, so the
// softmax weights never leave their lane; the head index stays lane%16 in both
// products, so the running max / sum / rescale factor are per-lane scalars.
// K tiles [S][D] and V tiles [D][S] (channel-major) let every lane fetch its
// operand with plain 8/16-byte loads; nothing is transposed on chip.
#pragma once
#include "ts_device.h"

namespace ts {

typedef uint32_t uint2v_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ short4_t as_short4(uint32_t a, uint32_t b) {
  uint2v_t w = {a, b};
  return __builtin_bit_cast(short4_t, w);
}

__device__ __forceinline__ float4_t mfma16(short4_t a, short4_t b, float4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0);
}

struct AttendParams {
  const uint16_t* q;           // [B][Hq][D]
  const uint16_t* k_pool;      // [n_phys][Hkv] tiles of [S][D], tile_stride apart
  const uint16_t* v_pool;      // [n_phys][Hkv] tiles of [D][S], tile_stride apart
  const int32_t* block_table;  // [B][Pmax]
  const int32_t* seq_lens;     // [B]
  float* out;                  // [B][Hq][D]
  float* partials;             // [B*Hkv][n_split][G][D+2]
  int Hq, Hkv, G, Pmax, Kmax, n_phys, n_split, chunk;
  int tile_stride;             // elements between consecutive (page, head) tiles
  float scale_log2;            // softmax_scale * log2(e)
};

template <int D, int S>
struct PageFrag {
  static constexpr int NT = S / 16;   // 16-token tiles per page
  static constexpr int KQ = D / 32;   // 16-byte K loads per lane per tile (D/4 channels)
  static constexpr int NCB = D / 16;  // 16-channel output blocks
  uint4 k[NT][KQ];
  uint2 v[NT][NCB];
};

// Token held by MFMA row r of tile t.  For S = 32 the rows are permuted so that
// the eight tokens a lane needs for the two P.V products are contiguous in the
// channel-major V tile.
template <int S>
__device__ __forceinline__ int tile_token(int t, int r) {
  return S == 16 ? r : 8 * (r >> 2) + 4 * t + (r & 3);
}

template <int D, int S>
__device__ __forceinline__ void zero_page(PageFrag<D, S>& f) {
#pragma unroll
  for (int t = 0; t < PageFrag<D, S>::NT; ++t) {
#pragma unroll
    for (int i = 0; i < PageFrag<D, S>::KQ; ++i) f.k[t][i] = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < PageFrag<D, S>::NCB; ++i) f.v[t][i] = make_uint2(0, 0);
  }
}

// `spread` is 1 for a real page and 0 for a placeholder fetch: with 0 every
// lane reads the first bytes of the tile, so the instruction touches one cache
// line instead of the whole tile (the data is never used).
template <int D, int S>
__device__ __forceinline__ void load_page(PageFrag<D, S>& f, const uint16_t* ktile,
                                          const uint16_t* vtile, int spread) {
  const int lane = lane_id(), r = (lane & 15) * spread, kb = (lane >> 4) * spread;
#pragma unroll
  for (int t = 0; t < PageFrag<D, S>::NT; ++t) {
    const uint16_t* krow = ktile + tile_token<S>(t, r) * D * spread + kb * (D / 4);
#pragma unroll
    for (int i = 0; i < PageFrag<D, S>::KQ; ++i)
      f.k[t][i] = *reinterpret_cast<const uint4*>(krow + i * 8 * spread);
  }
#pragma unroll
  for (int cb = 0; cb < PageFrag<D, S>::NCB; ++cb) {
    const uint16_t* vrow = vtile + (16 * cb * spread + r) * S;
    if (S == 16) {
      f.v[0][cb] = *reinterpret_cast<const uint2*>(vrow + 4 * kb);
    } else {
      const uint4 w = *reinterpret_cast<const uint4*>(vrow + 8 * kb);
      f.v[0][cb] = make_uint2(w.x, w.y);
      f.v[S == 16 ? 0 : 1][cb] = make_uint2(w.z, w.w);
    }
  }
}

// A token appended in the same launch: it belongs to page j (-1: none), slot
// `slot` of that page; its key / value rows (D bf16 each) are read from the
// caller's arrays and spliced into the page's operands in registers, so the
// attention does not depend on when the pool itself receives them.  Without a
// token the two pointers must still be readable (D bf16; the data is not used).
struct NewToken {
  int j, slot;
  const uint16_t* k_row;
  const uint16_t* v_row;
};

template <int D, int S>
struct TokenPatch {
  uint4 k[PageFrag<D, S>::KQ];       // this lane's D/4 channels of the key
  uint32_t v[PageFrag<D, S>::NCB];   // value of channel 16 * cb + lane % 16
  __device__ __forceinline__ void load(const NewToken& nt) {
    const int lane = lane_id(), r = lane & 15, kb = lane >> 4;
#pragma unroll
    for (int i = 0; i < PageFrag<D, S>::KQ; ++i)
      k[i] = *reinterpret_cast<const uint4*>(nt.k_row + kb * (D / 4) + i * 8);
#pragma unroll
    for (int cb = 0; cb < PageFrag<D, S>::NCB; ++cb) v[cb] = nt.v_row[16 * cb + r];
  }
  // Splice into a page fetched from the pool (registers only).
  __device__ __forceinline__ void apply(PageFrag<D, S>& f, int slot) const {
    const int lane = lane_id(), r = lane & 15, kb = lane >> 4;
#pragma unroll
    for (int t = 0; t < PageFrag<D, S>::NT; ++t) {
      if (tile_token<S>(t, r) == slot) {
#pragma unroll
        for (int i = 0; i < PageFrag<D, S>::KQ; ++i) f.k[t][i] = k[i];
      }
      // V words of tile t hold tokens tile_token<S>(t, 4 * kb) .. + 3
      const int e = slot - tile_token<S>(t, 4 * kb);
      if (e >= 0 && e < 4) {
#pragma unroll
        for (int cb = 0; cb < PageFrag<D, S>::NCB; ++cb) {
          const uint32_t keep = (e & 1) ? 0x0000ffffu : 0xffff0000u;
          const uint32_t put = (e & 1) ? (v[cb] << 16) : v[cb];
          if (e < 2) f.v[t][cb].x = (f.v[t][cb].x & keep) | put;
          else f.v[t][cb].y = (f.v[t][cb].y & keep) | put;
        }
      }
    }
  }
};

template <int D>
struct WaveAcc {
  float m, l;  // running max (log2 domain) and this lane's share of the running sum
  float4_t o[D / 16];
  __device__ __forceinline__ void init() {
    m = -1e30f;
    l = 0.f;
#pragma unroll
    for (int i = 0; i < D / 16; ++i) o[i] = float4_t{0.f, 0.f, 0.f, 0.f};
  }
};

// Query operand: lane (head = lane%16, kb = lane/16) holds q[head][kb*D/4 .. +D/4).
template <int D>
__device__ __forceinline__ void load_q_frag(short4_t (&qf)[D / 16], const uint16_t* q_group,
                                            int G) {
  const int lane = lane_id(), head = lane & 15, kb = lane >> 4;
#pragma unroll
  for (int i = 0; i < D / 32; ++i) {
    // heads past G re-read head G - 1 (no branch around the load) and are zeroed
    uint4 w = *reinterpret_cast<const uint4*>(q_group + (size_t)min(head, G - 1) * D + kb * (D / 4) + i * 8);
    if (head >= G) w = make_uint4(0, 0, 0, 0);
    qf[2 * i] = as_short4(w.x, w.y);
    qf[2 * i + 1] = as_short4(w.z, w.w);
  }
}

// One page: logits, online-softmax update, weighted value accumulation.
// `valid` = number of tokens the page holds (tokens >= valid are masked).
template <int D, int S>
__device__ __forceinline__ void attend_page(const PageFrag<D, S>& f, const short4_t (&qf)[D / 16],
                                            int valid, float scale_log2, WaveAcc<D>& a) {
  constexpr int NT = PageFrag<D, S>::NT, NCB = PageFrag<D, S>::NCB;
  const int kb = lane_id() >> 4;
  float4_t sc[NT];
  float mx = -INFINITY;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    sc[t] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < D / 32; ++i) {
      sc[t] = mfma16(as_short4(f.k[t][i].x, f.k[t][i].y), qf[2 * i], sc[t]);
      sc[t] = mfma16(as_short4(f.k[t][i].z, f.k[t][i].w), qf[2 * i + 1], sc[t]);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int tok = tile_token<S>(t, 4 * kb + v);
      const float x = tok < valid ? sc[t][v] * scale_log2 : -INFINITY;
      sc[t][v] = x;
      mx = fmaxf(mx, x);
    }
  }
  mx = rows_max_f32(mx);
  const float m_new = fmaxf(a.m, mx);
  const float alpha = __builtin_amdgcn_exp2f(a.m - m_new);
  a.m = m_new;
  a.l *= alpha;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) a.o[cb] *= alpha;
  const bool partial = valid < S;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    // softmax weights split into two bf16 terms (truncated high part + remainder)
    // so the P.V product keeps ~16 significant bits of each weight
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float pv = __builtin_amdgcn_exp2f(sc[t][v] - m_new);
      a.l += pv;
      hi[v] = __float_as_uint(pv) & 0xffff0000u;
      lo[v] = __float_as_uint(pv - __uint_as_float(hi[v]));
    }
    const short4_t ph = as_short4((hi[0] >> 16) | hi[1], (hi[2] >> 16) | hi[3]);
    const short4_t pl = as_short4((lo[0] >> 16) | (lo[1] & 0xffff0000u),
                                  (lo[2] >> 16) | (lo[3] & 0xffff0000u));
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      uint32_t v0 = f.v[t][cb].x, v1 = f.v[t][cb].y;
      if (partial) {  // slots past the sequence end may hold anything: zero them
        const int t0 = tile_token<S>(t, 4 * kb);
        if (t0 + 0 >= valid) v0 &= 0xffff0000u;
        if (t0 + 1 >= valid) v0 &= 0x0000ffffu;
        if (t0 + 2 >= valid) v1 &= 0xffff0000u;
        if (t0 + 3 >= valid) v1 &= 0x0000ffffu;
      }
      const short4_t vf = as_short4(v0, v1);
      a.o[cb] = mfma16(vf, ph, a.o[cb]);
      a.o[cb] = mfma16(vf, pl, a.o[cb]);
    }
  }
}

// The workgroup attends `count` selected pages of unit (b, h): entry i of its
// list is page sel_at(i), stored in physical page phys_at(page).  Wave w takes
// entries w, w + kWaves, ...  The four wave states are merged through LDS
// (lds: kWaves * G * (D + 2) floats).  With n_split == 1 the normalised result
// goes to `out`; otherwise the unnormalised partial (o[D], m, l per head) is
// handed to the combining workgroup through agent-scope stores.
// Ends with a barrier after which `lds` may be reused; on return (n_split > 1)
// the caller still has to wait for its stores and count its arrival.
// kBranchless: the ring is refilled without a branch around the loads (see
// below); with false the refill past the end of the list is skipped instead,
// which suits bandwidth-bound launches with thousands of units.
// kPatch: a token appended in the same launch may have to be spliced in (nt).
template <int D, int S, bool kBranchless, bool kPatch, typename SelAt, typename PhysAt>
__device__ __forceinline__ void attend_split(const AttendParams& p, int b, int h, int split,
                                             int count, int L, const NewToken& nt, SelAt sel_at,
                                             PhysAt phys_at, float* lds) {
  const int lane = lane_id(), wave = wave_id();
  const int head = lane & 15, kb = lane >> 4;
  const int G = p.G;
  L = uniform(L);
  count = uniform(count);

  short4_t qf[D / 16];
  load_q_frag<D>(qf, p.q + ((size_t)b * p.Hq + (size_t)h * G) * D, G);
  // The new token's page is the sequence's last, so in the ascending list it can
  // only be the very last entry: one wave of one workgroup ever needs the token.
  TokenPatch<D, S> patch;
  const bool splice = kPatch && nt.j >= 0 && count > 0 && wave == (count - 1) % kWaves &&
                      uniform(sel_at(count - 1)) == nt.j;
  if (splice) patch.load(nt);
  WaveAcc<D> acc;
  acc.init();

  for (int batch = wave; batch < count; batch += kWave * kWaves) {
    // lane x holds the ids of this wave's x-th page of the batch
    const int my_i = batch + lane * kWaves;
    int my_j = -1, my_phys = -1;
    if (my_i < count) {
      my_j = sel_at(my_i);
      if (my_j >= 0 && my_j < p.Pmax) my_phys = phys_at(my_j);
    }
    const int n = min(kWave, (count - batch + kWaves - 1) / kWaves);
    // A ring of NBUF page buffers: up to NBUF pages of this wave are in flight
    // (4 KiB - 8 KiB each) before the first is consumed.
    constexpr int NBUF = (D * S <= 1024) ? 4 : ((D == 64 && D * S <= 2048) ? 3 : 2);
    PageFrag<D, S> f[NBUF];
    int valid[NBUF], page[NBUF];
    // No branch around the loads (a load under a branch makes the compiler
    // wait for ALL outstanding loads wherever it needs one of them, so the ring
    // would drain before the first page is used): a slot past the end of the
    // list, or one whose page id is out of range, re-reads a page that is
    // certainly mapped (a single cache line of it) and counts zero valid tokens.
    auto issue = [&](PageFrag<D, S>& fr, int& jp, int x) -> int {
      const int xc = min(x, n - 1);
      const int j = __builtin_amdgcn_readlane(my_j, xc);
      jp = j;
      const int phys = __builtin_amdgcn_readlane(my_phys, xc);
      const bool good = x < n && phys >= 0 && phys < p.n_phys;
      const size_t tile = ((size_t)(good ? phys : 0) * p.Hkv + h) * (size_t)p.tile_stride;
      load_page<D, S>(fr, p.k_pool + tile, p.v_pool + tile, good ? 1 : 0);
      return good ? max(0, min(S, L - j * S)) : 0;
    };
#pragma unroll
    for (int i = 0; i < NBUF; ++i) valid[i] = issue(f[i], page[i], i);
    TS_MARK(17);
    for (int x0 = 0; x0 < n; x0 += NBUF) {
#pragma unroll
      for (int i = 0; i < NBUF; ++i) {
        if (x0 + i < n) {
          if (splice && page[i] == nt.j) patch.apply(f[i], nt.slot);
          attend_page<D, S>(f[i], qf, valid[i], p.scale_log2, acc);
        }
        if (kBranchless || x0 + i + NBUF < n) valid[i] = issue(f[i], page[i], x0 + i + NBUF);
      }
    }
  }

  TS_MARK(18);
  // merge the wave states
  const float l = rows_sum_f32(acc.l);
  constexpr int RS = D + 2;
  if (head < G) {
    float* row = lds + ((size_t)wave * G + head) * RS;
#pragma unroll
    for (int cb = 0; cb < D / 16; ++cb)
#pragma unroll
      for (int v = 0; v < 4; ++v) row[16 * cb + 4 * kb + v] = acc.o[cb][v];
    if (kb == 0) { row[D] = acc.m; row[D + 1] = l; }
  }
  __syncthreads();
  float* part = p.partials + (((size_t)b * p.Hkv + h) * p.n_split + split) * (size_t)G * RS;
  // one thread per (head, channel); the thread of channel 0 also hands on the
  // head's running max and sum
  for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
    const int g = idx / D, c = idx % D;
    float mw[kWaves], M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      mw[w] = lds[((size_t)w * G + g) * RS + D];
      M = fmaxf(M, mw[w]);
    }
    float Lsum = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float* row = lds + ((size_t)w * G + g) * RS;
      const float wgt = __builtin_amdgcn_exp2f(mw[w] - M);
      Lsum += row[D + 1] * wgt;
      O += row[c] * wgt;
    }
    if (p.n_split == 1) {
      p.out[((size_t)b * p.Hq + (size_t)h * G + g) * D + c] = Lsum > 0.f ? O / Lsum : 0.f;
    } else {
      store_agent(part + g * RS + c, O);
      if (c == 0) {
        store_agent(part + g * RS + D, M);
        store_agent(part + g * RS + D + 1, Lsum);
      }
    }
  }
  __syncthreads();
}

// Merge the n_split partials of unit (b, h) and write the normalised output.
// The caller has observed every producer's arrival; the partials are read with
// agent-scope loads.
template <int D>
__device__ __forceinline__ void combine_splits(const AttendParams& p, int b, int h) {
  constexpr int RS = D + 2;
  const int G = p.G;
  const float* part = p.partials + ((size_t)b * p.Hkv + h) * p.n_split * (size_t)G * RS;
  for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
    const int g = idx / D, c = idx % D;
    // online merge, 8 partials per round with all their loads in flight together
    float M = -1e30f, Lsum = 0.f, O = 0.f;
    for (int s0 = 0; s0 < p.n_split; s0 += 8) {
      float o[8], m[8], l[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const bool on = s0 + i < p.n_split;  // rows past the end re-read row 0, unused
        const float* row = part + ((size_t)(on ? s0 + i : 0) * G + g) * RS;
        const float ov = load_agent(row + c), mv = load_agent(row + D), lv = load_agent(row + D + 1);
        o[i] = on ? ov : 0.f;
        m[i] = on ? mv : -1e30f;
        l[i] = on ? lv : 0.f;
      }
      float Mn = M;
#pragma unroll
      for (int i = 0; i < 8; ++i) Mn = fmaxf(Mn, m[i]);
      const float sc = __builtin_amdgcn_exp2f(M - Mn);
      Lsum *= sc;
      O *= sc;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float wgt = __builtin_amdgcn_exp2f(m[i] - Mn);
        Lsum += l[i] * wgt;
        O += o[i] * wgt;
      }
      M = Mn;
    }
    p.out[((size_t)b * p.Hq + (size_t)h * G + g) * D + c] = Lsum > 0.f ? O / Lsum : 0.f;
  }
}

}  // namespace ts
