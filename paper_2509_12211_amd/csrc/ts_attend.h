// Sparse single-query attention over the selected pages (Section 3.5 SparseAttn;
// steps 3-4 of Algorithm 1) with 16-bit MFMA (bf16, or IEEE half for the FP16
// cache; the INT8 cache is expanded to bf16) and an online softmax, split over
// workgroups (flash-decoding style partial softmax + combine).
//
// One wavefront processes whole pages.  Per 16-token tile it computes
//   St[token][head] = K_tile[token][:] . Q^T[:][head]        (v_mfma_f32_16x16x16_bf16 / _f16)
//   Ot[chan ][head] += V_tile^T[chan][token] . P^T[token][head]
// The accumulator layout of the first product (lane -> head lane%16, tokens
// 4*(lane/16)..+3) is exactly the B-operand layout of the second, so the
// softmax weights never leave their lane; the head index stays lane%16 in both
// products, so the running max / sum / rescale factor are per-lane scalars.
// K tiles [S][D] and V tiles [D][S] (channel-major) let every lane fetch its
// operand with plain 8/16-byte loads; nothing is transposed on chip.
//
// Page sizes other than 16 and 32 map onto the same two fragment shapes: a
// wave works on fragments of F = 16 tokens (S <= 16) or F = 32 tokens
// (S >= 32).  With S < 16 a fragment is made of 16 / S consecutive entries of
// the selected list (each lane picks the tile of the page its MFMA row or its
// four value tokens belong to); with S = 64 a page is two fragments, its first
// and its second 32 tokens.
#pragma once
#include <type_traits>

#include "ts_device.h"

namespace ts {

typedef uint32_t uint2v_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ short4_t as_short4(uint32_t a, uint32_t b) {
  uint2v_t w = {a, b};
  return __builtin_bit_cast(short4_t, w);
}

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));

// 16x16x16 product of 16-bit operands (bf16, or IEEE half for the FP16 cache), fp32 accumulate.
template <bool kHalf = false>
__device__ __forceinline__ float4_t mfma16(short4_t a, short4_t b, float4_t c) {
  if constexpr (kHalf)
    return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4_t, a),
                                                 __builtin_bit_cast(half4_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0);
}

// Four softmax weights as two 16-bit operand sets whose sum carries ~16 (bf16) or
// ~21 (half) significant bits of each weight: a truncated high part and the remainder.
template <bool kHalf>
__device__ __forceinline__ void split_weights(const float (&pv)[4], short4_t& ph, short4_t& pl) {
  if constexpr (kHalf) {
    typedef __fp16 h2_t __attribute__((ext_vector_type(2)));
    const h2_t h01 = __builtin_amdgcn_cvt_pkrtz(pv[0], pv[1]);
    const h2_t h23 = __builtin_amdgcn_cvt_pkrtz(pv[2], pv[3]);
    const h2_t l01 = __builtin_amdgcn_cvt_pkrtz(pv[0] - (float)h01[0], pv[1] - (float)h01[1]);
    const h2_t l23 = __builtin_amdgcn_cvt_pkrtz(pv[2] - (float)h23[0], pv[3] - (float)h23[1]);
    ph = as_short4(__builtin_bit_cast(uint32_t, h01), __builtin_bit_cast(uint32_t, h23));
    pl = as_short4(__builtin_bit_cast(uint32_t, l01), __builtin_bit_cast(uint32_t, l23));
  } else {
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      hi[v] = __float_as_uint(pv[v]) & 0xffff0000u;
      lo[v] = __float_as_uint(pv[v] - __uint_as_float(hi[v]));
    }
    ph = as_short4((hi[0] >> 16) | hi[1], (hi[2] >> 16) | hi[3]);
    pl = as_short4((lo[0] >> 16) | (lo[1] & 0xffff0000u), (lo[2] >> 16) | (lo[3] & 0xffff0000u));
  }
}

struct AttendParams {
  const uint16_t* q;           // [B][Hq][D]
  const uint16_t* k_pool;      // [n_phys][Hkv] tiles of [S][D], tile_stride apart
  const uint16_t* v_pool;      // [n_phys][Hkv] tiles of [D][S], tile_stride apart
                               // (INT8 cache: the same shapes in int8, stride in bytes)
  const int32_t* block_table;  // [B][Pmax]
  const int32_t* seq_lens;     // [B]
  float* out;                  // [B][Hq][D] fp32, or bf16 when out_bf16 != 0
  float* partials;             // [B*Hkv][n_split][G][D+2]
  int Hq, Hkv, G, Pmax, Kmax, n_phys, n_split, chunk;
  int tile_stride;             // elements between consecutive (page, head) tiles
  float scale_log2;            // softmax_scale * log2(e)
  // (rarely used fields last: the kernels fetch their arguments front to back)
  int out_bf16;                // the final output is rounded to bf16 (nearest even)
  float* lse;                  // nullable [B][Hq]: log of the softmax denominator
  const float* k_scale;        // INT8 cache only: fp32 [n_phys][Hkv][S], one scale per token
  const float* v_scale;
};

// Element idx of the output, in the caller's format.
__device__ __forceinline__ void store_out(const AttendParams& p, size_t idx, float v) {
  if (p.out_bf16) reinterpret_cast<uint16_t*>(p.out)[idx] = f32_to_bf16_rn(v);
  else p.out[idx] = v;
}

template <int S>
struct PageGeom {
  static_assert(S == 4 || S == 8 || S == 16 || S == 32 || S == 64, "page size");
  static constexpr int F = S <= 16 ? 16 : 32;     // tokens per fragment
  static constexpr int NS = S < 16 ? 16 / S : 1;  // list entries (pages) per fragment
  static constexpr int NH = S > 32 ? S / 32 : 1;  // fragments per page
  static constexpr uint32_t kAll = F == 32 ? 0xffffffffu : 0xffffu;
  // fragments needed for `count` list entries
  __device__ __forceinline__ static int items(int count) {
    return S < 16 ? (count + NS - 1) / NS : count * NH;
  }
};

// A fragment of F tokens (F = 16 or 32) in MFMA operand order.
template <int D, int F>
struct PageFrag {
  static constexpr int NT = F / 16;   // 16-token tiles per fragment
  static constexpr int KQ = D / 32;   // 16-byte K loads per lane per tile (D/4 channels)
  static constexpr int NCB = D / 16;  // 16-channel output blocks
  uint4 k[NT][KQ];
  uint2 v[NT][NCB];
};

// Fragment token held by MFMA row r of tile t.  For F = 32 the rows are permuted
// so that the eight tokens a lane needs for the two P.V products are contiguous
// in the channel-major V tile.
template <int F>
__device__ __forceinline__ int tile_token(int t, int r) {
  return F == 16 ? r : 8 * (r >> 2) + 4 * t + (r & 3);
}

// Fetch one fragment of a page with S >= 16 tokens.  ktile / vtile: the page's
// K and V tiles; hoff: first token of the fragment inside the page (0, or 32
// for the second half of a 64-token page).  `spread` is 1 for a real fragment
// and 0 for a placeholder fetch: with 0 every lane reads the first bytes of the
// tile, so the instruction touches one cache line instead of the whole tile
// (the data is never used).
template <int D, int S>
__device__ __forceinline__ void load_page(PageFrag<D, PageGeom<S>::F>& f, const uint16_t* ktile,
                                          const uint16_t* vtile, int hoff, int spread) {
  constexpr int F = PageGeom<S>::F;
  static_assert(S >= 16, "whole-page fragments");
  const int lane = lane_id(), r = (lane & 15) * spread, kb = (lane >> 4) * spread;
  hoff *= spread;
#pragma unroll
  for (int t = 0; t < PageFrag<D, F>::NT; ++t) {
    const uint16_t* krow = ktile + (hoff + tile_token<F>(t, r)) * D * spread + kb * (D / 4);
#pragma unroll
    for (int i = 0; i < PageFrag<D, F>::KQ; ++i)
      f.k[t][i] = *reinterpret_cast<const uint4*>(krow + i * 8 * spread);
  }
#pragma unroll
  for (int cb = 0; cb < PageFrag<D, F>::NCB; ++cb) {
    const uint16_t* vrow = vtile + (16 * cb * spread + r) * S + hoff;
    if (F == 16) {
      f.v[0][cb] = load_stream8(vrow + 4 * kb);
    } else {
      const uint4 w = load_stream16(vrow + 8 * kb);
      f.v[0][cb] = make_uint2(w.x, w.y);
      f.v[F == 16 ? 0 : 1][cb] = make_uint2(w.z, w.w);
    }
  }
}

// Fetch one 16-token fragment made of 16 / S small pages: toff[s] is the
// element offset of the tile of the fragment's s-th page (the same offset in
// the K and in the V pool).  Fragment token x lives in page x / S, slot x % S.
// spread as above (0: every lane reads the first bytes of page 0's tiles).
template <int D, int S>
__device__ __forceinline__ void load_small_pages(PageFrag<D, 16>& f, const uint16_t* k_pool,
                                                 const uint16_t* v_pool,
                                                 const size_t (&toff)[PageGeom<S>::NS],
                                                 int spread) {
  constexpr int NS = PageGeom<S>::NS;
  static_assert(S < 16, "several pages per fragment");
  const int lane = lane_id(), r = (lane & 15) * spread, kb = (lane >> 4) * spread;
  // K: MFMA row r is fragment token r; V: this lane's four tokens are 4 * kb .. + 3
  const int sk = r / S, sv = (4 * kb) / S;
  size_t ok = toff[0], ov = toff[0];
#pragma unroll
  for (int s = 1; s < NS; ++s) {
    ok = sk == s ? toff[s] : ok;
    ov = sv == s ? toff[s] : ov;
  }
  const uint16_t* krow = k_pool + ok + (r % S) * D + kb * (D / 4);
#pragma unroll
  for (int i = 0; i < PageFrag<D, 16>::KQ; ++i)
    f.k[0][i] = *reinterpret_cast<const uint4*>(krow + i * 8 * spread);
  const uint16_t* vbase = v_pool + ov + (4 * kb) % S;
#pragma unroll
  for (int cb = 0; cb < PageFrag<D, 16>::NCB; ++cb)
    f.v[0][cb] = load_stream8(vbase + (16 * cb * spread + r) * S);
}

// ---------------------------------------------------------------------------
// INT8 cache: the same fragments fetched as int8 (half the bytes) together with
// the per-token scales, and expanded to 16-bit MFMA operands in registers; the
// token's scale multiplies the logit (K) and the softmax weight (V) afterwards.
//
// The operands are IEEE halves holding code + kI8Bias: in [1024, 2048) a half
// has a step of 1, so the half of 1024 + u (u = code + 128, the byte with its top
// bit flipped) is the bit pattern 0x6400 | u, and four codes become four operands
// with three byte-shuffling instructions and no conversion (against eight for
// converting each code to a float and packing pairs: the expansion is what bounds
// this path on large batches).  The products stay exact (11-bit x 11-bit
// significands in an fp32 accumulator); the bias is taken out again afterwards:
//   sum_c (code_c + B) q_c  =  sum_c code_c q_c + B sum_c q_c     (logits)
//   sum_t (code_t + B) p_t  =  sum_t code_t p_t + B sum_t p_t     (output)
// with sum_c q_c once per unit and sum_t p_t carried along with the softmax sum.
// The queries are converted from bf16 to half for this (exact for magnitudes
// from 2^-14 to 65504; smaller ones lose low bits to the subnormals, larger ones
// stop at 65504).
// ---------------------------------------------------------------------------
constexpr float kI8Bias = 1152.0f;   // 1024 + 128
template <int D, int F>
struct PageFrag8 {
  static constexpr int NT = F / 16;
  static constexpr int KW = D / 16;   // 32-bit words of this lane's D/4 key bytes
  static constexpr int NCB = D / 16;
  uint32_t k[NT][KW];
  uint32_t v[NT][NCB];   // this lane's four tokens of channel 16 * cb + lane % 16
  float4 ks[NT], vs[NT]; // scales of this lane's four tokens of tile t
};

// bytes b, b + 1 (b = 0 or 2) of x as two biased halves; x: four codes with their
// top bits flipped
__device__ __forceinline__ uint32_t i8_pair_to_half(uint32_t x, int b) {
  // v_perm_b32: result byte i = byte sel[i] of {0x64646464 (4..7), x (0..3)}
  return __builtin_amdgcn_perm(0x64646464u, x, b == 0 ? 0x04010400u : 0x04030402u);
}

template <int D, int F>
__device__ __forceinline__ void expand_frag(const PageFrag8<D, F>& r, PageFrag<D, F>& f) {
#pragma unroll
  for (int t = 0; t < PageFrag<D, F>::NT; ++t) {
#pragma unroll
    for (int i = 0; i < PageFrag<D, F>::KQ; ++i) {
      const uint32_t a = r.k[t][2 * i] ^ 0x80808080u, b = r.k[t][2 * i + 1] ^ 0x80808080u;
      f.k[t][i] = make_uint4(i8_pair_to_half(a, 0), i8_pair_to_half(a, 2), i8_pair_to_half(b, 0),
                             i8_pair_to_half(b, 2));
    }
#pragma unroll
    for (int cb = 0; cb < PageFrag<D, F>::NCB; ++cb) {
      const uint32_t a = r.v[t][cb] ^ 0x80808080u;
      f.v[t][cb] = make_uint2(i8_pair_to_half(a, 0), i8_pair_to_half(a, 2));
    }
  }
}

// One fragment of a page with S >= 16 tokens (see load_page).  scales: the
// page's S scales in k_scale / v_scale.
template <int D, int S>
__device__ __forceinline__ void load_page8(PageFrag8<D, PageGeom<S>::F>& f, const uint8_t* ktile,
                                           const uint8_t* vtile, const float* kscale,
                                           const float* vscale, int hoff, int spread) {
  constexpr int F = PageGeom<S>::F;
  static_assert(S >= 16, "whole-page fragments");
  const int lane = lane_id(), r = (lane & 15) * spread, kb = (lane >> 4) * spread;
  hoff *= spread;
#pragma unroll
  for (int t = 0; t < PageFrag8<D, F>::NT; ++t) {
    const uint8_t* krow = ktile + (hoff + tile_token<F>(t, r)) * D * spread + kb * (D / 4);
    if (D == 64) {
      const uint4 w = *reinterpret_cast<const uint4*>(krow);
      f.k[t][0] = w.x; f.k[t][1] = w.y; f.k[t][2] = w.z; f.k[t][3] = w.w;
    } else {
#pragma unroll
      for (int i = 0; i < D / 64; ++i) {
        const uint4 w = *reinterpret_cast<const uint4*>(krow + 16 * i * spread);
        f.k[t][4 * i] = w.x; f.k[t][4 * i + 1] = w.y; f.k[t][4 * i + 2] = w.z; f.k[t][4 * i + 3] = w.w;
      }
    }
    const int tok0 = hoff + tile_token<F>(t, 4 * kb);
    f.ks[t] = *reinterpret_cast<const float4*>(kscale + tok0);
    f.vs[t] = *reinterpret_cast<const float4*>(vscale + tok0);
  }
  if constexpr (F == 16 && S == 16) {
    // A channel's 16 tokens are 16 contiguous bytes: lane (r, kb) fetches the whole row of
    // channel 16 * (4 * q + kb) + r (a wave-wide load covers 1 KiB in one piece, a quarter
    // of the instructions of four-byte loads), and the four lanes r, r + 16, r + 32, r + 48
    // then trade words so that each ends up with its own four tokens of four channel
    // blocks: a 4 x 4 transpose over the wave's four rows of lanes, two row-swap steps.
    static_assert(PageFrag8<D, F>::NCB % 4 == 0, "channel blocks in fours");
#pragma unroll
    for (int q = 0; q < PageFrag8<D, F>::NCB / 4; ++q) {
      const uint4 w = load_stream16(vtile + ((64 * q * spread + 16 * kb + r) * S));
      // rows 2, 3 of (x, y) against rows 0, 1 of (z, w), then odd rows against even rows
      const uint2s_t xz = __builtin_amdgcn_permlane32_swap(w.x, w.z, false, false);
      const uint2s_t yw = __builtin_amdgcn_permlane32_swap(w.y, w.w, false, false);
      const uint2s_t a = __builtin_amdgcn_permlane16_swap(xz.x, yw.x, false, false);
      const uint2s_t b = __builtin_amdgcn_permlane16_swap(xz.y, yw.y, false, false);
      f.v[0][4 * q] = a.x;
      f.v[0][4 * q + 1] = a.y;
      f.v[0][4 * q + 2] = b.x;
      f.v[0][4 * q + 3] = b.y;
    }
  } else {
#pragma unroll
    for (int cb = 0; cb < PageFrag8<D, F>::NCB; ++cb) {
      const uint8_t* vrow = vtile + (16 * cb * spread + r) * S + hoff;
      if (F == 16) {
        f.v[0][cb] = load_stream4(vrow + 4 * kb);
      } else {
        const uint2 w = load_stream8(vrow + 8 * kb);
        f.v[0][cb] = w.x;
        f.v[F == 16 ? 0 : 1][cb] = w.y;
      }
    }
  }
}

// One 16-token fragment made of 16 / S small pages (see load_small_pages);
// soff[s]: offset of the s-th page's scales in k_scale / v_scale.
template <int D, int S>
__device__ __forceinline__ void load_small_pages8(PageFrag8<D, 16>& f, const uint8_t* k_pool,
                                                  const uint8_t* v_pool, const float* k_scale,
                                                  const float* v_scale,
                                                  const size_t (&toff)[PageGeom<S>::NS],
                                                  const size_t (&soff)[PageGeom<S>::NS],
                                                  int spread) {
  constexpr int NS = PageGeom<S>::NS;
  static_assert(S < 16, "several pages per fragment");
  const int lane = lane_id(), r = (lane & 15) * spread, kb = (lane >> 4) * spread;
  const int sk = r / S, sv = (4 * kb) / S;
  size_t ok = toff[0], ov = toff[0], os = soff[0];
#pragma unroll
  for (int s = 1; s < NS; ++s) {
    ok = sk == s ? toff[s] : ok;
    ov = sv == s ? toff[s] : ov;
    os = sv == s ? soff[s] : os;
  }
  const uint8_t* krow = k_pool + ok + (r % S) * D + kb * (D / 4);
#pragma unroll
  for (int i = 0; i < D / 64; ++i) {
    const uint4 w = *reinterpret_cast<const uint4*>(krow + 16 * i * spread);
    f.k[0][4 * i] = w.x; f.k[0][4 * i + 1] = w.y; f.k[0][4 * i + 2] = w.z; f.k[0][4 * i + 3] = w.w;
  }
  f.ks[0] = *reinterpret_cast<const float4*>(k_scale + os + (4 * kb) % S);
  f.vs[0] = *reinterpret_cast<const float4*>(v_scale + os + (4 * kb) % S);
  const uint8_t* vbase = v_pool + ov + (4 * kb) % S;
#pragma unroll
  for (int cb = 0; cb < PageFrag8<D, 16>::NCB; ++cb)
    f.v[0][cb] = load_stream4(vbase + (16 * cb * spread + r) * S);
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

template <int D, int F>
struct TokenPatch {
  uint4 k[PageFrag<D, F>::KQ];       // this lane's D/4 channels of the key
  uint32_t v[PageFrag<D, F>::NCB];   // value of channel 16 * cb + lane % 16
  __device__ __forceinline__ void load(const NewToken& nt) {
    const int lane = lane_id(), r = lane & 15, kb = lane >> 4;
#pragma unroll
    for (int i = 0; i < PageFrag<D, F>::KQ; ++i)
      k[i] = *reinterpret_cast<const uint4*>(nt.k_row + kb * (D / 4) + i * 8);
#pragma unroll
    for (int cb = 0; cb < PageFrag<D, F>::NCB; ++cb) v[cb] = nt.v_row[16 * cb + r];
  }
  // Splice into a fragment fetched from the pool (registers only); x: the
  // token's position inside the fragment.
  __device__ __forceinline__ void apply(PageFrag<D, F>& f, int x) const {
    const int lane = lane_id(), r = lane & 15, kb = lane >> 4;
#pragma unroll
    for (int t = 0; t < PageFrag<D, F>::NT; ++t) {
      if (tile_token<F>(t, r) == x) {
#pragma unroll
        for (int i = 0; i < PageFrag<D, F>::KQ; ++i) f.k[t][i] = k[i];
      }
      // V words of tile t hold tokens tile_token<F>(t, 4 * kb) .. + 3
      const int e = x - tile_token<F>(t, 4 * kb);
      if (e >= 0 && e < 4) {
#pragma unroll
        for (int cb = 0; cb < PageFrag<D, F>::NCB; ++cb) {
          const uint32_t keep = (e & 1) ? 0x0000ffffu : 0xffff0000u;
          const uint32_t put = (e & 1) ? (v[cb] << 16) : v[cb];
          if (e < 2) f.v[t][cb].x = (f.v[t][cb].x & keep) | put;
          else f.v[t][cb].y = (f.v[t][cb].y & keep) | put;
        }
      }
    }
  }
};

// The same for the INT8 cache: the rows are quantised here (scale = max |x| / 127
// over the row, code = x / scale rounded half to even), the codes spliced in as
// the biased halves the expanded fragments hold and the two scales put where the
// fragment keeps the token's.  To be called by a whole wave.
template <int D, int F>
struct TokenPatch8 : TokenPatch<D, F> {
  float ksc, vsc;
  __device__ __forceinline__ static uint32_t code_half(float x, float scale) {
    return 0x6400u | (static_cast<uint32_t>(i8_code(x, scale) + 128) & 0xffu);   // half of code + kI8Bias
  }
  __device__ __forceinline__ void load(const NewToken& nt) {
    TokenPatch<D, F>::load(nt);
    float ka = 0.f, va = 0.f;
#pragma unroll
    for (int i = 0; i < PageFrag<D, F>::KQ; ++i) ka = fmaxf(ka, chunk_amax_bf16(this->k[i]));
#pragma unroll
    for (int cb = 0; cb < PageFrag<D, F>::NCB; ++cb) va = fmaxf(va, fabsf(bf16_lo(this->v[cb])));
    // a lane holds a quarter of the key row (the quarters sit 16 lanes apart) and
    // every 16th channel of the value row (lane % 16 picks which)
    ka = fmaxf(ka, shfl_xor_f(ka, 16));
    ka = fmaxf(ka, shfl_xor_f(ka, 32));
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) va = fmaxf(va, shfl_xor_f(va, m));
    ksc = i8_row_scale(ka);
    vsc = i8_row_scale(va);
#pragma unroll
    for (int i = 0; i < PageFrag<D, F>::KQ; ++i) {
      const uint32_t w[4] = {this->k[i].x, this->k[i].y, this->k[i].z, this->k[i].w};
      uint32_t o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        o[e] = code_half(bf16_lo(w[e]), ksc) | (code_half(bf16_hi(w[e]), ksc) << 16);
      this->k[i] = make_uint4(o[0], o[1], o[2], o[3]);
    }
#pragma unroll
    for (int cb = 0; cb < PageFrag<D, F>::NCB; ++cb) this->v[cb] = code_half(bf16_lo(this->v[cb]), vsc);
  }
  // the token's scales, where the fragment holds them (x as in apply)
  __device__ __forceinline__ void apply_scales(float4 (&ks)[PageFrag<D, F>::NT],
                                               float4 (&vs)[PageFrag<D, F>::NT], int x) const {
    const int kb = lane_id() >> 4;
#pragma unroll
    for (int t = 0; t < PageFrag<D, F>::NT; ++t) {
      const int e = x - tile_token<F>(t, 4 * kb);
      if (e == 0) { ks[t].x = ksc; vs[t].x = vsc; }
      if (e == 1) { ks[t].y = ksc; vs[t].y = vsc; }
      if (e == 2) { ks[t].z = ksc; vs[t].z = vsc; }
      if (e == 3) { ks[t].w = ksc; vs[t].w = vsc; }
    }
  }
};

// Natural log of sum_t exp(scale * q.k_t) from the running maximum m (log2
// domain) and the sum l of exp2(logit - m); -inf when no token was attended.
__device__ __forceinline__ float log_sum_exp(float m, float l) {
  return l > 0.f ? (m + log2f(l)) * 0.6931471805599453f : -INFINITY;
}

template <int D>
struct WaveAcc {
  float m, l;  // running max (log2 domain) and this lane's share of the running sum
  float lp;    // INT8 cache: this lane's share of the sum of the weights that went into P.V
  float4_t o[D / 16];
  __device__ __forceinline__ void init() {
    m = -1e30f;
    l = 0.f;
    lp = 0.f;
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
    // MFMA columns past G re-read head G - 1 (no branch around the load) and compute
    // a redundant copy of it that nobody reads.  They are deliberately NOT zeroed:
    // overwriting the destination of a load in flight makes the wave wait for it,
    // two serial memory round trips at the start of every attention phase.
    const uint4 w = *reinterpret_cast<const uint4*>(q_group + (size_t)min(head, G - 1) * D + kb * (D / 4) + i * 8);
    qf[2 * i] = as_short4(w.x, w.y);
    qf[2 * i + 1] = as_short4(w.z, w.w);
  }
}

// One fragment: logits, online-softmax update, weighted value accumulation.
// Bit x of `vmask` says whether fragment token x exists (tokens past the end of
// the sequence, and the tokens of a missing page, are masked).
//
// kScaled (INT8 cache): the operands are biased halves (see kI8Bias; qf then holds
// halves too, qbias = kI8Bias * the sum of this lane's query row).  ks[t] / vs[t]
// hold the scales of this lane's four tokens of tile t; a logit is multiplied by
// its token's key scale, and a softmax weight by its token's value scale on its
// way into the P.V product (not in the running sum); the sum of those weights is
// kept in a.lp for the caller to take the bias out of the output.
template <int D, int F, bool kScaled = false, bool kHalf = false>
__device__ __forceinline__ void attend_page(const PageFrag<D, F>& f, const short4_t (&qf)[D / 16],
                                            uint32_t vmask, float scale_log2, WaveAcc<D>& a,
                                            const float4* ks = nullptr, const float4* vs = nullptr,
                                            float qbias = 0.f) {
  constexpr int NT = PageFrag<D, F>::NT, NCB = PageFrag<D, F>::NCB;
  constexpr bool kH = kHalf || kScaled;   // the MFMA's 16-bit operand type
  const int kb = lane_id() >> 4;
  float4_t sc[NT];
  float mx = -INFINITY;
  const bool partial = vmask != (F == 32 ? 0xffffffffu : 0xffffu);
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    sc[t] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < D / 32; ++i) {
      sc[t] = mfma16<kH>(as_short4(f.k[t][i].x, f.k[t][i].y), qf[2 * i], sc[t]);
      sc[t] = mfma16<kH>(as_short4(f.k[t][i].z, f.k[t][i].w), qf[2 * i + 1], sc[t]);
    }
    float kst[4] = {1.f, 1.f, 1.f, 1.f};
    if (kScaled) { kst[0] = ks[t].x; kst[1] = ks[t].y; kst[2] = ks[t].z; kst[3] = ks[t].w; }
#pragma unroll
    for (int v = 0; v < 4; ++v)
      sc[t][v] = (kScaled ? (sc[t][v] - qbias) * kst[v] : sc[t][v]) * scale_log2;
    if (partial) {   // (uniform) a fragment with all its tokens, the common case, masks nothing
      const uint32_t mine = vmask >> tile_token<F>(t, 4 * kb);   // this lane's four tokens
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (!((mine >> v) & 1u)) sc[t][v] = -INFINITY;
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) mx = fmaxf(mx, sc[t][v]);
  }
  mx = rows_max_f32(mx);
  const float m_new = fmaxf(a.m, mx);
  const float alpha = __builtin_amdgcn_exp2f(a.m - m_new);
  a.m = m_new;
  a.l *= alpha;
  if (kScaled) a.lp *= alpha;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) a.o[cb] *= alpha;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    // softmax weights split into two bf16 terms (truncated high part + remainder)
    // so the P.V product keeps ~16 significant bits of each weight
    const uint32_t mine = vmask >> tile_token<F>(t, 4 * kb);
    float vst[4] = {1.f, 1.f, 1.f, 1.f};
    if (kScaled) { vst[0] = vs[t].x; vst[1] = vs[t].y; vst[2] = vs[t].z; vst[3] = vs[t].w; }
    float pw[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      float pv = __builtin_amdgcn_exp2f(sc[t][v] - m_new);
      a.l += pv;
      // (a slot without a token may hold any scale: its weight is zero, keep it zero)
      if (kScaled) {
        pv = (mine >> v) & 1u ? pv * vst[v] : 0.f;
        a.lp += pv;
      }
      pw[v] = pv;
    }
    short4_t ph, pl;
    split_weights<kH>(pw, ph, pl);
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      uint32_t v0 = f.v[t][cb].x, v1 = f.v[t][cb].y;
      if (partial && !kScaled) {  // slots that hold no token may hold anything: zero them
        if (!(mine & 1u)) v0 &= 0xffff0000u;
        if (!(mine & 2u)) v0 &= 0x0000ffffu;
        if (!(mine & 4u)) v1 &= 0xffff0000u;
        if (!(mine & 8u)) v1 &= 0x0000ffffu;
      }
      const short4_t vf = as_short4(v0, v1);
      a.o[cb] = mfma16<kH>(vf, ph, a.o[cb]);
      a.o[cb] = mfma16<kH>(vf, pl, a.o[cb]);
    }
  }
}

// The query operand of the attention: the G rows as MFMA fragments (for the INT8 cache
// converted to halves, with the bias term of this lane's row).  The fused kernel fetches
// it while it waits for the other members' scores, long before the selection is through.
template <int D, bool kInt8>
struct QOperand {
  short4_t qf[D / 16];
  float qbias;   // INT8 cache: kI8Bias * sum over the channels of this lane's query row
  __device__ __forceinline__ void load(const uint16_t* rows, int G) {
    load_q_frag<D>(qf, rows, G);
    qbias = 0.f;
    if constexpr (kInt8) {
      typedef __fp16 h2_t __attribute__((ext_vector_type(2)));
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < D / 16; ++i) {
        const uint32_t w0 = (uint32_t)(uint16_t)qf[i][0] | ((uint32_t)(uint16_t)qf[i][1] << 16);
        const uint32_t w1 = (uint32_t)(uint16_t)qf[i][2] | ((uint32_t)(uint16_t)qf[i][3] << 16);
        const h2_t a = __builtin_amdgcn_cvt_pkrtz(bf16_lo(w0), bf16_hi(w0));
        const h2_t c = __builtin_amdgcn_cvt_pkrtz(bf16_lo(w1), bf16_hi(w1));
        part += ((float)a[0] + (float)a[1]) + ((float)c[0] + (float)c[1]);
        qf[i] = as_short4(__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, c));
      }
      // the row is spread over the four lanes head, head + 16, head + 32, head + 48
      qbias = kI8Bias * rows_sum_f32(part);
    }
  }
};

// Partials handed on as tagged words (attend_split with a tag): merges the first
// `n` partials of a unit into the running state (M, Lsum, O) of head g, channel c.
// The words are polled until all carry this launch's tag, so the data arrive with the
// flag, in one trip through the memory system, with no counter and no wait for store
// acknowledgements on the producers' side.  To be called by whole waves whose threads
// share the head g (D is a multiple of the wave size).  What a round of polls costs
// grows with the loads in it (measured: 24 agent-scope loads per thread take 1.7 us to
// come back, 8 take under 1), so a thread fetches its own channel of every partial,
// the head's max and sum are fetched once per wave (lane i: the max of partial i, lane
// 32 + i: its sum) and handed round in registers, and a round asks only for what the
// rounds before have not brought.
// `spins` counts the polls of this thread against spin_limit; returns false if
// the bounded wait expired (the state is then invalid).
// NB: partials polled together (all their loads in flight at once).
template <int D, int NB>
__device__ __forceinline__ bool merge_tagged(const uint64_t* part, int G, int g, int c, int n,
                                             uint32_t tag, int spin_limit, int& spins, float& M,
                                             float& Lsum, float& O) {
  static_assert(D % kWave == 0 && NB <= 16, "a wave works on one head; lanes i and 32 + i serve partial i");
  constexpr int RS = D + 2;
  const int lane = lane_id();
  bool ok = true;
  // (the empty asm keeps the address arithmetic below from being moved up in front of
  // the attention, where it would only hold registers)
  asm volatile("" : "+v"(c));
  const uint32_t off_o = (uint32_t)(g * RS + c);            // this thread's word of a partial
  const uint32_t stride = (uint32_t)(G * RS);               // words per partial
  for (int s0 = 0; s0 < n; s0 += NB) {
    const int nb = uniform(min(NB, n - s0));
    // the head's running max and sum of the batch's partials: lane i holds the max of
    // partial s0 + i, lane 32 + i its sum (one load for the wave instead of two per
    // partial and thread)
    const bool ml_role = (lane & 31) < nb;
    const uint64_t* base = part + (size_t)s0 * stride;      // (uniform)
    const uint32_t off_ml = (uint32_t)(ml_role ? (lane & 31) : 0) * stride + (uint32_t)(g * RS + D + (lane >> 5));
    uint64_t ml = 0, v[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) v[i] = 0;
    // bit i: partial s0 + i has not arrived yet; bit 31: this lane's max / sum word
    uint32_t pending = ((1u << nb) - 1u) | (ml_role ? 0x80000000u : 0u);
    for (;;) {
      // only what has not arrived yet is asked for again: a round's cost grows with the
      // loads in it, and the last rounds wait for one or two late members
#pragma unroll
      for (int i = 0; i < NB; ++i)
        if ((pending >> i) & 1u) v[i] = load_agent_u64(base + (size_t)i * stride + off_o);
      if (pending >> 31) ml = load_agent_u64(base + off_ml);
#pragma unroll
      for (int i = 0; i < NB; ++i)
        if ((uint32_t)(v[i] >> 32) == tag) pending &= ~(1u << i);
      if ((uint32_t)(ml >> 32) == tag) pending &= 0x7fffffffu;
      if (__ballot(pending != 0u) == 0ull) break;   // the wave leaves together
      if (++spins > spin_limit) { ok = false; break; }
      __builtin_amdgcn_s_sleep(1);
    }
    // merged in the order of the partials, whatever order they arrived in
    const uint32_t mlw = (uint32_t)ml;
    float Mn = M;
    if constexpr (NB <= 4) {
#pragma unroll
      for (int i = 0; i < NB; ++i)
        if (i < nb) Mn = fmaxf(Mn, __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)mlw, i)));
      const float sc = __builtin_amdgcn_exp2f(M - Mn);
      Lsum *= sc;
      O *= sc;
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        if (i < nb) {
          const float mi = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)mlw, i));
          const float li = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)mlw, 32 + i));
          const float wgt = __builtin_amdgcn_exp2f(mi - Mn);
          Lsum += li * wgt;
          O += __uint_as_float((uint32_t)v[i]) * wgt;
        }
      }
    } else {
      // a large batch: the weights are worked out side by side, lane i that of partial
      // s0 + i, and a thread then needs one broadcast and one multiply-add per partial
      const float mval = (lane < 32 && ml_role) ? __uint_as_float(mlw) : -INFINITY;
      Mn = fmaxf(M, wave_max_f32(mval));
      const float wgt = __builtin_amdgcn_exp2f(mval - Mn);   // 0 in the lanes without a partial
      // lane 32 + i needs the weight of lane i: the halves swapped and added (the upper
      // half holds zeros)
      const uint2s_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(wgt), __float_as_uint(wgt), false, false);
      const float wgt_both = __uint_as_float(r.x) + __uint_as_float(r.y);
      const float lnew = wave_sum_f32((lane >= 32 && ml_role) ? __uint_as_float(mlw) * wgt_both : 0.f);
      const float sc = __builtin_amdgcn_exp2f(M - Mn);
      Lsum = Lsum * sc + lnew;
      O *= sc;
#pragma unroll
      for (int i = 0; i < NB; ++i)
        if (i < nb)
          O += __uint_as_float((uint32_t)v[i]) *
               __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(wgt), i));
    }
    M = Mn;
  }
  return ok;
}

// The workgroup attends `count` selected pages of unit (b, h): entry i of its
// list is page sel_at(i), stored in physical page phys_at(page).  The list is
// cut into fragments (PageGeom<S>); wave w takes fragments w, w + kWaves, ...
// The waves' states are merged through LDS
// (lds: kWaves * G * (D + 2) floats).  With n_split == 1 the normalised result
// goes to `out`; otherwise the unnormalised partial (o[D], m, l per head) is
// handed to the combining workgroup through agent-scope stores.
// Ends with a barrier after which `lds` may be reused; on return (n_split > 1)
// the caller still has to wait for its stores and count its arrival.
// kLatency: the launch is bound by the latency of its single pass (every workgroup has
// one unit): the ring waits for each fragment by count (see below).
// kPatch: a token appended in the same launch may have to be spliced in (nt).
// kInt8: the cache holds int8 keys / values with per-token scales.
// kHalf: queries, keys and values are IEEE half instead of bf16.
// q_rows: see below.
// tag != 0 (n_split > 1): the partial is handed on as 8-byte words {value, tag}
// (see merge_tagged), so the caller neither waits for the stores nor counts an
// arrival; the partial area then holds uint64 [.][n_split][G][D + 2].  The LAST
// split keeps its own partial in registers, polls for the others (bounded by
// spin_limit polls per thread) and writes the unit's output; the function
// returns false if that wait expired.
template <int D, int S, bool kLatency, bool kPatch, bool kInt8, bool kHalf, bool kHaveQ = false,
          typename SelAt, typename PhysAt>
__device__ __forceinline__ bool attend_split(const AttendParams& p, int b, int h, int split,
                                             int count, int L, const NewToken& nt, SelAt sel_at,
                                             PhysAt phys_at, float* lds, uint32_t tag = 0u,
                                             const uint16_t* q_rows = nullptr, int spin_limit = 0,
                                             const QOperand<D, kInt8>* q_ready = nullptr) {
  using Geo = PageGeom<S>;
  constexpr int F = Geo::F, NS = Geo::NS, NH = Geo::NH;
  static_assert(!(kHalf && kInt8), "the INT8 cache goes with bf16 queries");
  using Frag = std::conditional_t<kInt8, PageFrag8<D, F>, PageFrag<D, F>>;
  const uint8_t* k_pool8 = reinterpret_cast<const uint8_t*>(p.k_pool);
  const uint8_t* v_pool8 = reinterpret_cast<const uint8_t*>(p.v_pool);
  const int lane = lane_id(), wave = wave_id();
  const int head = lane & 15, kb = lane >> 4;
  const int G = p.G;
  L = uniform(L);
  count = uniform(count);
  const int n_items = Geo::items(count);
  TS_MARK(26);

  // q_rows: the unit's G query rows where the caller already holds them (the fused
  // kernel: in LDS, staged by the scoring phase); nullptr: fetched from memory.
  // kHaveQ: the caller has the operand in registers already (q_ready).
  QOperand<D, kInt8> qop;
  if constexpr (kHaveQ) qop = *q_ready;
  else qop.load(q_rows ? q_rows : p.q + ((size_t)b * p.Hq + (size_t)h * G) * D, G);
  const short4_t (&qf)[D / 16] = qop.qf;
  const float qbias = qop.qbias;
  // The new token's page is the sequence's last, so in the ascending list it can
  // only be the very last entry: one wave of one workgroup ever needs the token.
  // splice_item: the fragment it falls into, splice_x: its position there.
  std::conditional_t<kInt8, TokenPatch8<D, F>, TokenPatch<D, F>> patch;
  int splice_item = -1, splice_x = 0;
  if (kPatch && nt.j >= 0 && count > 0 && uniform(sel_at(count - 1)) == nt.j) {
    if (S < 16) {
      splice_item = (count - 1) / NS;
      splice_x = ((count - 1) % NS) * S + nt.slot;
    } else {
      splice_item = (count - 1) * NH + nt.slot / F;
      splice_x = nt.slot % F;
    }
  }
  const bool splice = kPatch && splice_item >= 0 && wave == splice_item % kWaves;
  if (splice) patch.load(nt);
  WaveAcc<D> acc;
  acc.init();
  TS_MARK(27);

  for (int batch = wave; batch < n_items; batch += kWave * kWaves) {
    // lane x holds the page ids of this wave's x-th fragment of the batch
    const int my_item = batch + lane * kWaves;
    int my_j[NS], my_phys[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      my_j[s] = -1;
      my_phys[s] = -1;
      const int e = S < 16 ? my_item * NS + s : my_item / NH;
      if (my_item < n_items && e < count) {
        my_j[s] = sel_at(e);
        if (my_j[s] >= 0 && my_j[s] < p.Pmax) my_phys[s] = phys_at(my_j[s]);
      }
    }
    const int n = min(kWave, (n_items - batch + kWaves - 1) / kWaves);
    TS_MARK(28);
    // A ring of NBUF fragment buffers: up to NBUF fragments of this wave are in
    // flight (2 KiB - 8 KiB each) before the first is consumed.
    constexpr int NBUF = (D * F <= 1024) ? 4 : ((D == 64 && D * F <= 2048) ? 3 : 2);
    Frag f[NBUF];
    uint32_t vmask[NBUF];
    int item[NBUF];
    // issue(buffer, item, x): fetch this wave's x-th fragment of the batch.  x >= n, or an
    // entry whose page id is out of range, re-reads a page that is certainly mapped (a
    // single cache line of it) and has no valid token: no branch around the loads.
    auto issue = [&](Frag& fr, int& it, int x) -> uint32_t {
      const int xc = min(x, n - 1);
      it = batch + xc * kWaves;
      if constexpr (S >= 16) {
        const int j = __builtin_amdgcn_readlane(my_j[0], xc);
        const int phys = __builtin_amdgcn_readlane(my_phys[0], xc);
        const int hoff = NH > 1 ? (it % NH) * F : 0;
        const bool good = x < n && phys >= 0 && phys < p.n_phys;
        const size_t tile = ((size_t)(good ? phys : 0) * p.Hkv + h) * (size_t)p.tile_stride;
        if constexpr (kInt8) {
          const size_t so = ((size_t)(good ? phys : 0) * p.Hkv + h) * (size_t)S;
          load_page8<D, S>(fr, k_pool8 + tile, v_pool8 + tile, p.k_scale + so, p.v_scale + so, hoff,
                           good ? 1 : 0);
        } else {
          load_page<D, S>(fr, p.k_pool + tile, p.v_pool + tile, hoff, good ? 1 : 0);
        }
        const int valid = good ? max(0, min(F, L - j * S - hoff)) : 0;
        return valid >= 32 ? 0xffffffffu : (1u << valid) - 1u;
      } else {
        size_t toff[NS], soff[NS];
        uint32_t m = 0;
        bool any = false;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          const int j = __builtin_amdgcn_readlane(my_j[s], xc);
          const int phys = __builtin_amdgcn_readlane(my_phys[s], xc);
          const bool good = x < n && phys >= 0 && phys < p.n_phys;
          toff[s] = ((size_t)(good ? phys : 0) * p.Hkv + h) * (size_t)p.tile_stride;
          soff[s] = ((size_t)(good ? phys : 0) * p.Hkv + h) * (size_t)S;
          const int valid = good ? max(0, min(S, L - j * S)) : 0;
          m |= ((1u << valid) - 1u) << (s * S);
          any = any || good;
        }
        if constexpr (kInt8)
          load_small_pages8<D, S>(fr, k_pool8, v_pool8, p.k_scale, p.v_scale, toff, soff,
                                  any ? 1 : 0);
        else
          load_small_pages<D, S>(fr, p.k_pool, p.v_pool, toff, any ? 1 : 0);
        return m;
      }
    };
    auto consume = [&](int i) {
      if constexpr (kInt8) {
        PageFrag<D, F> fx;
        expand_frag<D, F>(f[i], fx);
        if constexpr (kPatch) {
          if (splice && item[i] == splice_item) {
            patch.apply(fx, splice_x);
            patch.apply_scales(f[i].ks, f[i].vs, splice_x);
          }
        }
        attend_page<D, F, true>(fx, qf, vmask[i], p.scale_log2, acc, f[i].ks, f[i].vs, qbias);
      } else {
        if (splice && item[i] == splice_item) patch.apply(f[i], splice_x);
        attend_page<D, F, false, kHalf>(f[i], qf, vmask[i], p.scale_log2, acc);
      }
    };
    if constexpr (kLatency) {
      // The ring.  A wait for a fragment can only count the loads sent out after it
      // ("all but the newest k have arrived") where that number is the same on every path
      // that leads to the wait; where paths with different numbers meet, the compiler falls
      // back to waiting for everything in flight, which exposes a full memory latency per
      // fragment.  So the code is laid out by how many buffers are in use:
      //   - n >= NBUF: all buffers filled with no test in between; whole rounds (every
      //     buffer consumed and refilled, no test) as long as a full ring lies ahead; one
      //     round that consumes every buffer and refills the first `live` of them; then
      //   - the last `live` < NBUF fragments (also the whole of a short list, fetched
      //     under a test each): these are waited for together.
      // No placeholder loads anywhere: a load with nothing to fetch would still queue
      // behind the compute unit's outstanding misses.
      int live;   // fragments in buffers 0 .. live - 1 once the rounds are through
      if (n >= NBUF) {
  #pragma unroll
        for (int i = 0; i < NBUF; ++i) vmask[i] = issue(f[i], item[i], i);
        TS_MARK(17);
        TS_MARK_WAVE(48);
        int x0 = 0;
        for (; x0 + 2 * NBUF <= n; x0 += NBUF) {
  #pragma unroll
          for (int i = 0; i < NBUF; ++i) {
            consume(i);
            vmask[i] = issue(f[i], item[i], x0 + i + NBUF);
          }
        }
        live = n - x0 - NBUF;
  #pragma unroll
        for (int i = 0; i < NBUF; ++i) {
          consume(i);
          if (i < live) vmask[i] = issue(f[i], item[i], x0 + i + NBUF);
        }
      } else {
        live = n;
  #pragma unroll
        for (int i = 0; i < NBUF - 1; ++i)
          if (i < live) vmask[i] = issue(f[i], item[i], i);
        TS_MARK(17);
        TS_MARK_WAVE(48);
      }
  #pragma unroll
      for (int i = 0; i < NBUF - 1; ++i)
        if (i < live) consume(i);
    } else {
      // Bandwidth-bound launches (thousands of units, other workgroups to hide a wave's
      // waits): every buffer is filled at once (a slot past the end re-reads one cache
      // line) and refilled under a test of its own, which makes the compiler wait for
      // everything in flight before each fragment.  Measured on the 64-sequence batch,
      // that is 2 % FASTER than the counted waits above: with fewer bytes of a wave in
      // flight, the lines of a key tile, which four instructions come back to, are still
      // in the L1 when the last of them arrives.
#pragma unroll
      for (int i = 0; i < NBUF; ++i) vmask[i] = issue(f[i], item[i], i);
      TS_MARK(17);
      TS_MARK_WAVE(48);
      for (int x0 = 0; x0 < n; x0 += NBUF) {
#pragma unroll
        for (int i = 0; i < NBUF; ++i) {
          if (x0 + i < n) consume(i);
          if (x0 + i + NBUF < n) vmask[i] = issue(f[i], item[i], x0 + i + NBUF);
        }
      }
    }
    // Every fragment has been consumed, so nothing is in flight here; saying so (a wait
    // that never waits) keeps the compiler from assuming, where the loop over the batches
    // closes, that a buffer may still be waiting for a refill: it then drained the memory
    // pipeline in front of each buffer's first fill, so that the ring's fragments were
    // fetched one after the other (-0.3 us on the 16-sequence configuration).
    if (kLatency) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), other counters untouched
  }

  TS_MARK(18);
  TS_MARK_WAVE(56);
  if constexpr (kInt8) {   // the bias of the value operands, out of the accumulator
    const float wsum = kI8Bias * rows_sum_f32(acc.lp);
#pragma unroll
    for (int cb = 0; cb < D / 16; ++cb)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc.o[cb][v] -= wsum;
  }
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
  TS_MARK(24);
  float* part = p.partials + (((size_t)b * p.Hkv + h) * p.n_split + split) * (size_t)G * RS;
  bool ok = true;
  int spins = 0;
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
      store_out(p, ((size_t)b * p.Hq + (size_t)h * G + g) * D + c, Lsum > 0.f ? O / Lsum : 0.f);
      if (c == 0 && p.lse) p.lse[(size_t)b * p.Hq + (size_t)h * G + g] = log_sum_exp(M, Lsum);
    } else if (tag != 0u) {
      uint64_t* unit64 = reinterpret_cast<uint64_t*>(p.partials) +
                         ((size_t)b * p.Hkv + h) * p.n_split * (size_t)G * RS;
      if (split == p.n_split - 1) {   // (uniform) the merging split: its own partial never leaves
        // (small clusters take the partials four at a time, large ones sixteen)
        const int others = p.n_split - 1;
        ok = (others <= 4 ? merge_tagged<D, 4>(unit64, G, g, c, others, tag, spin_limit, spins, M, Lsum, O)
                          : merge_tagged<D, 16>(unit64, G, g, c, others, tag, spin_limit, spins, M, Lsum, O)) && ok;
        store_out(p, ((size_t)b * p.Hq + (size_t)h * G + g) * D + c, Lsum > 0.f ? O / Lsum : 0.f);
        if (c == 0 && p.lse) p.lse[(size_t)b * p.Hq + (size_t)h * G + g] = log_sum_exp(M, Lsum);
      } else {
        uint64_t* part64 = unit64 + (size_t)split * G * RS;
        store_agent_tagged(part64 + g * RS + c, O, tag);
        if (c == 0) {
          store_agent_tagged(part64 + g * RS + D, M, tag);
          store_agent_tagged(part64 + g * RS + D + 1, Lsum, tag);
        }
      }
    } else {
      store_agent(part + g * RS + c, O);
      if (c == 0) {
        store_agent(part + g * RS + D, M);
        store_agent(part + g * RS + D + 1, Lsum);
      }
    }
  }
  TS_MARK(25);
  __syncthreads();
  return ok;
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
    store_out(p, ((size_t)b * p.Hq + (size_t)h * G + g) * D + c, Lsum > 0.f ? O / Lsum : 0.f);
    if (c == 0 && p.lse) p.lse[(size_t)b * p.Hq + (size_t)h * G + g] = log_sum_exp(M, Lsum);
  }
}

}  // namespace ts
