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

// One workgroup per sequence: every (KV head, channel) of the new token widens
// (or opens) the box of page seq_len / S and, when v_new is given, lands in its
// pool slot.  The kernel is a chain of dependent memory round trips, so it is
// arranged to need only two: the token's values (which do not depend on the
// length) go out together with the length, then the block-table entry and the
// old box together.  All threads read seq_lens[b] before the barrier; thread 0
// advances it after.
__global__ __launch_bounds__(kThreads) void append_token_meta_kernel(MetaParams p, int D,
                                                                      const uint16_t* k_new,
                                                                      const uint16_t* v_new,
                                                                      int advance) {
  const int b = blockIdx.x, n = p.Hkv * D;
  const size_t row = (size_t)b * n;  // [Hkv][D] values of this sequence's token
  const int first = min((int)threadIdx.x, n - 1);
  uint16_t kn = k_new[row + first];
  uint16_t vn = v_new ? v_new[row + first] : (uint16_t)0;
  const int L = p.seq_lens[b];
  const int sh = __builtin_ctz(p.S);  // page sizes are powers of two
  const int j = L >> sh, slot = L & (p.S - 1);
  const bool fits = j < p.Pmax;
  const int jc = fits ? j : 0;
  const int phys = p.block_table[(size_t)b * p.Pmax + jc];
  bool ok = fits;
  for (int idx = threadIdx.x; idx < n; idx += kThreads) {
    if (idx != (int)threadIdx.x) {
      kn = k_new[row + idx];
      vn = v_new ? v_new[row + idx] : (uint16_t)0;
    }
    const int h = idx / D, c = idx % D;
    const size_t m = (((size_t)b * p.Hkv + h) * p.Pmax + jc) * D + c;
    const uint16_t lo = p.page_min[m], hi = p.page_max[m];  // fetched before phys is looked at
    ok = fits && (v_new == nullptr || (phys >= 0 && phys < p.n_phys));
    if (ok) {
      const float x = bf16_to_f32(kn);
      if (slot == 0 || x < bf16_to_f32(lo)) p.page_min[m] = kn;
      if (slot == 0 || x > bf16_to_f32(hi)) p.page_max[m] = kn;
      if (v_new != nullptr) {
        const size_t tile = ((size_t)phys * p.Hkv + h) * (size_t)p.tile_stride;
        p.k_pool_w[tile + (size_t)slot * D + c] = kn;
        p.v_pool_w[tile + (size_t)c * p.S + slot] = vn;
      }
    }
  }
  ok = fits && (v_new == nullptr || (phys >= 0 && phys < p.n_phys));
  __syncthreads();
  if (ok && advance && threadIdx.x == 0) p.seq_lens[b] = L + 1;
}

}  // namespace ts
