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
  float* k_scale;   // INT8 cache only: fp32 [n_phys][Hkv][S]
  float* v_scale;
};

// A wavefront summarises kWave / (D/8) logical pages of one (sequence, KV head) at
// a time: a page's D/8 consecutive lanes each own eight channels (one 16-byte
// chunk of a token row) and walk down the page's tokens, so a lane takes the
// channel-wise min / max over the tokens in its own registers and nothing is
// folded across lanes.  A wave-wide load reads one token row of every page of
// the group (128 or 256 contiguous bytes each); up to NT = 16 of them are in
// flight per wave before the first is used (16 KiB), behind ONE dependent
// look-up of the sequence length and the block-table entries, so the kernel
// streams the pool at memory speed instead of paying that chain per page.
// NT: token rows fetched together, min(page_size, 16); longer pages take several
// rounds.  Slots past the sequence's last token are read (they lie inside the
// page's tile) and ignored.  The rows are fetched with streaming loads (each
// instruction takes whole lines that nobody reads again): -9 % on the 128 MiB pool.
template <int D, bool kHalf, int NT>
__global__ __launch_bounds__(kThreads) void build_page_meta_kernel(MetaParams p) {
  constexpr int LPR = D / 8;        // lanes per page (one per 16-byte chunk of a token row)
  constexpr int PPW = kWave / LPR;  // pages per wave
  const int lane = lane_id(), cg = lane % LPR;
  const int j = (blockIdx.y * kWaves + wave_id()) * PPW + lane / LPR;
  const int h = blockIdx.x, b = blockIdx.z;
  const int L = p.seq_lens[b];
  const int Pb = min((L + p.S - 1) / p.S, p.Pmax);
  if (uniform((blockIdx.y * kWaves + wave_id()) * PPW) >= Pb) return;   // the whole group is past the end
  const bool page_on = j < Pb;
  const int phys = p.block_table[(size_t)b * p.Pmax + min(j, Pb - 1)];
  const bool on = page_on && phys >= 0 && phys < p.n_phys;
  const int valid = min(p.S, L - j * p.S);   // tokens the page holds (only looked at when `on`)
  const uint16_t* tile =
      p.k_pool + ((size_t)(on ? phys : 0) * p.Hkv + h) * (size_t)p.tile_stride + cg * 8;
  float lo[8], hi[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { lo[i] = INFINITY; hi[i] = -INFINITY; }
  for (int t0 = 0; t0 < p.S; t0 += NT) {
    uint4 w[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) w[t] = load_stream16(tile + (size_t)(t0 + t) * D);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      float f[8];
      unpack8e<kHalf>(w[t], f);
      const bool tok = t0 + t < valid;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        lo[i] = fminf(lo[i], tok ? f[i] : INFINITY);
        hi[i] = fmaxf(hi[i], tok ? f[i] : -INFINITY);
      }
    }
  }
  if (on) {
    const size_t row = (((size_t)b * p.Hkv + h) * p.Pmax + j) * D + cg * 8;
    // back to 16-bit elements: the values are elements of the cache, so this is exact
    // (bf16: the upper half of the fp32 pattern)
    auto pack = [](float x, float y) -> uint32_t {
      if (kHalf) return (uint32_t)f32_to_half(x) | ((uint32_t)f32_to_half(y) << 16);
      return (__float_as_uint(x) >> 16) | (__float_as_uint(y) & 0xffff0000u);
    };
    const uint4 a = make_uint4(pack(lo[0], lo[1]), pack(lo[2], lo[3]), pack(lo[4], lo[5]),
                               pack(lo[6], lo[7]));
    const uint4 c = make_uint4(pack(hi[0], hi[1]), pack(hi[2], hi[3]), pack(hi[4], hi[5]),
                               pack(hi[6], hi[7]));
    *reinterpret_cast<uint4*>(p.page_min + row) = a;
    *reinterpret_cast<uint4*>(p.page_max + row) = c;
  }
}

// Element-wise box update of eight packed bf16: lo = k where k < lo, hi = k
// where k > hi (strict, as the stand-alone append kernel does it).
template <bool kHalf = false>
__device__ __forceinline__ uint32_t widen_pair(uint32_t box, uint32_t k, bool is_min) {
  const float bl = elem_lo<kHalf>(box), bh = elem_hi<kHalf>(box), kl = elem_lo<kHalf>(k),
              kh = elem_hi<kHalf>(k);
  const bool tl = is_min ? kl < bl : kl > bl, th = is_min ? kh < bh : kh > bh;
  return ((tl ? k : box) & 0x0000ffffu) | ((th ? k : box) & 0xffff0000u);
}
template <bool kHalf = false>
__device__ __forceinline__ uint4 widen_box(const uint4& box, const uint4& k, bool is_min) {
  return make_uint4(widen_pair<kHalf>(box.x, k.x, is_min), widen_pair<kHalf>(box.y, k.y, is_min),
                    widen_pair<kHalf>(box.z, k.z, is_min), widen_pair<kHalf>(box.w, k.w, is_min));
}

// One workgroup per sequence.  A thread takes eight channels of one KV head at a
// time: it widens (or opens) the 16-byte chunk of the box of page seq_len / S
// and, when v_new is given, puts the token into its pool slot (one 16-byte store
// for the key; the value tile is channel-major, so eight 2-byte stores).  The
// kernel is a chain of dependent memory round trips, arranged to need only two:
// the token's values (which do not depend on the length) go out together with
// the length, then the block-table entry and the old box together.  All threads
// read seq_lens[b] before the barrier; thread 0 advances it after.
// kHalf: the cache holds IEEE half (the comparison is the only thing that differs).
template <bool kHalf>
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
      *reinterpret_cast<uint4*>(p.page_min + m) = slot == 0 ? kn : widen_box<kHalf>(lo, kn, true);
      *reinterpret_cast<uint4*>(p.page_max + m) = slot == 0 ? kn : widen_box<kHalf>(hi, kn, false);
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

// ---------------------------------------------------------------------------
// INT8 cache.  The key of a token is code * scale (one fp32 scale per token and
// KV head) as a real number; a page's box has to contain those numbers for
// Eq. 2 to remain an upper bound, so the minimum is rounded DOWN to bf16 and
// the maximum UP.  int8 x fp32 is exact in fp64.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint16_t bf16_directed(double x, bool up) {
  float f = static_cast<float>(x);   // nearest; then moved to the right side of x
  uint32_t b = __float_as_uint(f);
  if (up ? static_cast<double>(f) < x : static_cast<double>(f) > x) {
    const bool away = up ? !(b >> 31) : (b >> 31) != 0;   // a step away from zero
    if ((b & 0x7fffffffu) == 0u) b = up ? 0x00000001u : 0x80000001u;
    else b = away ? b + 1u : b - 1u;
  }
  uint16_t hi = static_cast<uint16_t>(b >> 16);
  if ((b & 0xffffu) != 0u) {
    // dropping the low bits moves towards zero: down for positive values, up for negative
    const bool negative = (b >> 31) != 0;
    if (negative ? !up : up) hi = static_cast<uint16_t>(hi + 1);
  }
  return hi;
}

// The eight codes of a chunk as bytes in channel order.
__device__ __forceinline__ uint2 i8_chunk_codes(const uint4& c, float scale) {
  const uint32_t w[4] = {c.x, c.y, c.z, c.w};
  uint32_t o[2] = {0u, 0u};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t lo = static_cast<uint32_t>(i8_code(bf16_lo(w[i]), scale)) & 0xffu;
    const uint32_t hi = static_cast<uint32_t>(i8_code(bf16_hi(w[i]), scale)) & 0xffu;
    o[i >> 1] |= (lo | (hi << 8)) << (16 * (i & 1));
  }
  return make_uint2(o[0], o[1]);
}
// The dequantised values of a chunk rounded outwards to bf16: lo <= code * scale <= hi.
__device__ __forceinline__ void i8_chunk_box(const uint4& c, float scale, uint4& lo, uint4& hi) {
  const uint32_t w[4] = {c.x, c.y, c.z, c.w};
  uint32_t l[4], h[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const double a = static_cast<double>(i8_code(bf16_lo(w[i]), scale)) * static_cast<double>(scale);
    const double b = static_cast<double>(i8_code(bf16_hi(w[i]), scale)) * static_cast<double>(scale);
    l[i] = bf16_directed(a, false) | (static_cast<uint32_t>(bf16_directed(b, false)) << 16);
    h[i] = bf16_directed(a, true) | (static_cast<uint32_t>(bf16_directed(b, true)) << 16);
  }
  lo = make_uint4(l[0], l[1], l[2], l[3]);
  hi = make_uint4(h[0], h[1], h[2], h[3]);
}

// One thread per (page, channel): kThreads / D pages per workgroup.  Set-up
// work (a page is summarised once; appends keep it current), kept plain.
template <int D>
__global__ __launch_bounds__(kThreads) void build_page_meta_i8_kernel(MetaParams p) {
  constexpr int PPB = kThreads / D;
  const int c = threadIdx.x % D;
  const int j = blockIdx.x * PPB + threadIdx.x / D;
  const int h = blockIdx.y, b = blockIdx.z;
  const int L = p.seq_lens[b];
  const int Pb = (L + p.S - 1) / p.S;
  if (j >= Pb || j >= p.Pmax) return;
  const int phys = p.block_table[(size_t)b * p.Pmax + j];
  if (phys < 0 || phys >= p.n_phys) return;
  const int valid = min(p.S, L - j * p.S);
  const int8_t* tile = reinterpret_cast<const int8_t*>(p.k_pool) +
                       ((size_t)phys * p.Hkv + h) * (size_t)p.tile_stride;
  const float* sc = p.k_scale + ((size_t)phys * p.Hkv + h) * (size_t)p.S;
  double lo = INFINITY, hi = -INFINITY;
  for (int t = 0; t < valid; ++t) {
    const double k = static_cast<double>(tile[(size_t)t * D + c]) * static_cast<double>(sc[t]);
    lo = fmin(lo, k);
    hi = fmax(hi, k);
  }
  const size_t row = (((size_t)b * p.Hkv + h) * p.Pmax + j) * D + c;
  p.page_min[row] = bf16_directed(lo, false);
  p.page_max[row] = bf16_directed(hi, true);
}

// Append to the INT8 cache: one workgroup per sequence, a wave per KV head at a
// time.  The bf16 key and value are quantised (scale = max |x| / 127, 1 for a
// zero vector; code = x / scale rounded half to even, in fp32 with correctly
// rounded division), stored with their scales when v_new is given, and the
// page's box is opened / widened with the dequantised key rounded outwards.
static __global__ __launch_bounds__(kThreads) void append_token_i8_kernel(MetaParams p, int D,
                                                                   const uint16_t* k_new,
                                                                   const uint16_t* v_new,
                                                                   int advance) {
  const int b = blockIdx.x, lane = lane_id();
  const int L = p.seq_lens[b];
  const int sh = __builtin_ctz(p.S);
  const int j = L >> sh, slot = L & (p.S - 1);
  const bool fits = j < p.Pmax;
  const int phys = p.block_table[(size_t)b * p.Pmax + (fits ? j : 0)];
  const bool ok = fits && (v_new == nullptr || (phys >= 0 && phys < p.n_phys));
  if (ok) {
    for (int h = wave_id(); h < p.Hkv; h += kWaves) {
      const uint16_t* kr = k_new + ((size_t)b * p.Hkv + h) * D;
      const uint16_t* vr = (v_new ? v_new : k_new) + ((size_t)b * p.Hkv + h) * D;
      float kv[2], vv[2], ka = 0.f, va = 0.f;   // channels lane, lane + 64
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int c = lane + 64 * i;
        kv[i] = c < D ? bf16_to_f32(kr[c]) : 0.f;
        vv[i] = c < D ? bf16_to_f32(vr[c]) : 0.f;
        ka = fmaxf(ka, fabsf(kv[i]));
        va = fmaxf(va, fabsf(vv[i]));
      }
#pragma unroll
      for (int m = 1; m < kWave; m <<= 1) {
        ka = fmaxf(ka, shfl_xor_f(ka, m));
        va = fmaxf(va, shfl_xor_f(va, m));
      }
      const float ksc = i8_row_scale(ka), vsc = i8_row_scale(va);
      const size_t tile = ((size_t)phys * p.Hkv + h) * (size_t)p.tile_stride;
      int8_t* k8 = reinterpret_cast<int8_t*>(p.k_pool_w);
      int8_t* v8 = reinterpret_cast<int8_t*>(p.v_pool_w);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int c = lane + 64 * i;
        if (c < D) {
          const int kq = i8_code(kv[i], ksc), vq = i8_code(vv[i], vsc);
          if (v_new != nullptr) {
            k8[tile + (size_t)slot * D + c] = static_cast<int8_t>(kq);
            v8[tile + (size_t)c * p.S + slot] = static_cast<int8_t>(vq);
          }
          const double kd = static_cast<double>(kq) * static_cast<double>(ksc);
          const uint16_t lo = bf16_directed(kd, false), hi = bf16_directed(kd, true);
          const size_t m = (((size_t)b * p.Hkv + h) * p.Pmax + j) * D + c;
          if (slot == 0) {
            p.page_min[m] = lo;
            p.page_max[m] = hi;
          } else {
            if (bf16_to_f32(lo) < bf16_to_f32(p.page_min[m])) p.page_min[m] = lo;
            if (bf16_to_f32(hi) > bf16_to_f32(p.page_max[m])) p.page_max[m] = hi;
          }
        }
      }
      if (v_new != nullptr && lane == 0) {
        const size_t so = ((size_t)phys * p.Hkv + h) * (size_t)p.S + slot;
        p.k_scale[so] = ksc;
        p.v_scale[so] = vsc;
      }
    }
  }
  __syncthreads();   // every thread has read seq_lens[b]
  if (ok && advance && threadIdx.x == 0) p.seq_lens[b] = L + 1;
}

}  // namespace ts
