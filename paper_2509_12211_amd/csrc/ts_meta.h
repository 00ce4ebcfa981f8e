// Page metadata kernels: bulk rebuild (Eq. 1) and per-token incremental update.
#pragma once
#include "ts_device.h"

namespace ts {

struct MetaParams {
  const uint16_t* k_pool;
  uint16_t* k_pool_w;
  uint16_t* v_pool_w;
  const int32_t* block_table;
  int32_t* seq_lens;
  uint16_t* page_min;
  uint16_t* page_max;
  int B, Hkv, S, Pmax, n_phys, tile_stride;
};

// One wavefront summarises one (sequence, KV head, logical page): the S x D
// bf16 tile is contiguous, so the wave reads it as 16-byte chunks (lane ->
// token lane / (D/8), channels 8 * (lane % (D/8)) ..+7), takes the channel-wise
// min / max over its tokens, then folds the lanes that share a channel group.
template <int D>
__global__ __launch_bounds__(kThreads) void build_page_meta_kernel(MetaParams p) {
  constexpr int LPR = D / 8;        // lanes per token row
  constexpr int TPW = kWave / LPR;  // token rows per wave-wide load
  const int lane = lane_id();
  const int j = blockIdx.x * kWaves + wave_id();
  const int h = blockIdx.y, b = blockIdx.z;
  const int L = p.seq_lens[b];
  const int Pb = (L + p.S - 1) / p.S;
  if (j >= Pb || j >= p.Pmax) return;
  const int phys = p.block_table[(size_t)b * p.Pmax + j];
  if (phys < 0 || phys >= p.n_phys) return;
  const int valid = min(p.S, L - j * p.S);
  const uint16_t* tile = p.k_pool + ((size_t)phys * p.Hkv + h) * (size_t)p.tile_stride;
  const int cg = lane % LPR;
  float lo[8], hi[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { lo[i] = INFINITY; hi[i] = -INFINITY; }
  for (int t = lane / LPR; t < valid; t += TPW) {
    const uint4 w = *reinterpret_cast<const uint4*>(tile + (size_t)t * D + cg * 8);
    float f[8];
    unpack8(w, f);
#pragma unroll
    for (int i = 0; i < 8; ++i) { lo[i] = fminf(lo[i], f[i]); hi[i] = fmaxf(hi[i], f[i]); }
  }
#pragma unroll
  for (int m = LPR; m < kWave; m <<= 1) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      lo[i] = fminf(lo[i], shfl_xor_f(lo[i], m));
      hi[i] = fmaxf(hi[i], shfl_xor_f(hi[i], m));
    }
  }
  if (lane < LPR) {
    const size_t row = (((size_t)b * p.Hkv + h) * p.Pmax + j) * D + cg * 8;
    uint4 a, c;
    a.x = (__float_as_uint(lo[0]) >> 16) | (__float_as_uint(lo[1]) & 0xffff0000u);
    a.y = (__float_as_uint(lo[2]) >> 16) | (__float_as_uint(lo[3]) & 0xffff0000u);
    a.z = (__float_as_uint(lo[4]) >> 16) | (__float_as_uint(lo[5]) & 0xffff0000u);
    a.w = (__float_as_uint(lo[6]) >> 16) | (__float_as_uint(lo[7]) & 0xffff0000u);
    c.x = (__float_as_uint(hi[0]) >> 16) | (__float_as_uint(hi[1]) & 0xffff0000u);
    c.y = (__float_as_uint(hi[2]) >> 16) | (__float_as_uint(hi[3]) & 0xffff0000u);
    c.z = (__float_as_uint(hi[4]) >> 16) | (__float_as_uint(hi[5]) & 0xffff0000u);
    c.w = (__float_as_uint(hi[6]) >> 16) | (__float_as_uint(hi[7]) & 0xffff0000u);
    *reinterpret_cast<uint4*>(p.page_min + row) = a;
    *reinterpret_cast<uint4*>(p.page_max + row) = c;
  }
}

// Element-wise box update of eight packed bf16: lo = k where k < lo, hi = k
// where k > hi (strict, as the stand-alone append kernel does it).
__device__ __forceinline__ uint32_t widen_pair(uint32_t box, uint32_t k, bool is_min) {
  const float bl = bf16_lo(box), bh = bf16_hi(box), kl = bf16_lo(k), kh = bf16_hi(k);
  const bool tl = is_min ? kl < bl : kl > bl, th = is_min ? kh < bh : kh > bh;
  return ((tl ? k : box) & 0x0000ffffu) | ((th ? k : box) & 0xffff0000u);
}
__device__ __forceinline__ uint4 widen_box(const uint4& box, const uint4& k, bool is_min) {
  return make_uint4(widen_pair(box.x, k.x, is_min), widen_pair(box.y, k.y, is_min),
                    widen_pair(box.z, k.z, is_min), widen_pair(box.w, k.w, is_min));
}

// One workgroup per sequence.  A thread takes eight channels of one KV head at a
// time: it widens (or opens) the 16-byte chunk of the box of page seq_len / S
// and, when v_new is given, puts the token into its pool slot (one 16-byte store
// for the key; the value tile is channel-major, so eight 2-byte stores).  The
// kernel is a chain of dependent memory round trips, arranged to need only two:
// the token's values (which do not depend on the length) go out together with
// the length, then the block-table entry and the old box together.  All threads
// read seq_lens[b] before the barrier; thread 0 advances it after.
__global__ __launch_bounds__(kThreads) void append_token_meta_kernel(MetaParams p, int D,
                                                                      const uint16_t* k_new,
                                                                      const uint16_t* v_new,
                                                                      int advance) {
  const int b = blockIdx.x, n8 = p.Hkv * D / 8, cpr = D / 8;   // chunks, chunks per head row
  const uint4* k_src = reinterpret_cast<const uint4*>(k_new + (size_t)b * p.Hkv * D);
  const uint4* v_src = reinterpret_cast<const uint4*>((v_new ? v_new : k_new) + (size_t)b * p.Hkv * D);
  const int first = min((int)threadIdx.x, n8 - 1);
  const uint4 k0 = k_src[first], v0 = v_src[first];   // fetched ahead of the length
  const int L = p.seq_lens[b];
  const int sh = __builtin_ctz(p.S);  // page sizes are powers of two
  const int j = L >> sh, slot = L & (p.S - 1);
  const bool fits = j < p.Pmax;
  const int jc = fits ? j : 0;
  const int phys = p.block_table[(size_t)b * p.Pmax + jc];
  for (int i0 = threadIdx.x; i0 < n8; i0 += kThreads) {
    const int h = i0 / cpr, c8 = (i0 % cpr) * 8;
    const size_t m = (((size_t)b * p.Hkv + h) * p.Pmax + jc) * D + c8;
    const uint4 lo = *reinterpret_cast<const uint4*>(p.page_min + m);   // before phys is looked at
    const uint4 hi = *reinterpret_cast<const uint4*>(p.page_max + m);
    const uint4 kn = i0 == (int)threadIdx.x ? k0 : k_src[i0];
    const uint4 vn = i0 == (int)threadIdx.x ? v0 : v_src[i0];
    const bool ok = fits && (v_new == nullptr || (phys >= 0 && phys < p.n_phys));
    if (ok) {
      *reinterpret_cast<uint4*>(p.page_min + m) = slot == 0 ? kn : widen_box(lo, kn, true);
      *reinterpret_cast<uint4*>(p.page_max + m) = slot == 0 ? kn : widen_box(hi, kn, false);
      if (v_new != nullptr) {
        const size_t tile = ((size_t)phys * p.Hkv + h) * (size_t)p.tile_stride;
        *reinterpret_cast<uint4*>(p.k_pool_w + tile + (size_t)slot * D + c8) = kn;
        const uint32_t vw[4] = {vn.x, vn.y, vn.z, vn.w};
#pragma unroll
        for (int i = 0; i < 8; ++i)
          p.v_pool_w[tile + (size_t)(c8 + i) * p.S + slot] = (uint16_t)(vw[i >> 1] >> (16 * (i & 1)));
      }
    }
  }
  const bool ok = fits && (v_new == nullptr || (phys >= 0 && phys < p.n_phys));
  __syncthreads();
  if (ok && advance && threadIdx.x == 0) p.seq_lens[b] = L + 1;
}

}  // namespace ts
