// Device-side helpers shared by the gfx950 kernels: bf16 unpacking, wave64
// cross-lane primitives, agent-scope synchronisation words.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ts {

constexpr int kWave = 64;
constexpr int kThreads = 512;            // every kernel here runs 8 wavefronts per workgroup
constexpr int kWaves = kThreads / kWave;

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// A 32-bit word holds two bf16: the low half is element 0.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t x) {
  return __uint_as_float(static_cast<uint32_t>(x) << 16);
}

// fp32 -> bf16, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16_rn(float f) {
  const uint32_t b = __float_as_uint(f);
  if ((b & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((b >> 16) | 0x0040u);
  return (uint16_t)((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
}
// The same for IEEE half (the FP16 cache format).
__device__ __forceinline__ float half_to_f32(uint16_t x) {
  return static_cast<float>(__builtin_bit_cast(_Float16, x));
}
__device__ __forceinline__ uint16_t f32_to_half(float f) {   // exact for values that are halves
  return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f));
}
// 16-bit element -> fp32 in either format
template <bool kHalf>
__device__ __forceinline__ float elem_to_f32(uint16_t x) {
  return kHalf ? half_to_f32(x) : bf16_to_f32(x);
}
template <bool kHalf>
__device__ __forceinline__ float elem_lo(uint32_t w) {
  return kHalf ? half_to_f32(static_cast<uint16_t>(w)) : bf16_lo(w);
}
template <bool kHalf>
__device__ __forceinline__ float elem_hi(uint32_t w) {
  return kHalf ? half_to_f32(static_cast<uint16_t>(w >> 16)) : bf16_hi(w);
}
template <bool kHalf>
__device__ __forceinline__ void unpack8e(const uint4& w, float (&f)[8]) {
  f[0] = elem_lo<kHalf>(w.x); f[1] = elem_hi<kHalf>(w.x);
  f[2] = elem_lo<kHalf>(w.y); f[3] = elem_hi<kHalf>(w.y);
  f[4] = elem_lo<kHalf>(w.z); f[5] = elem_hi<kHalf>(w.z);
  f[6] = elem_lo<kHalf>(w.w); f[7] = elem_hi<kHalf>(w.w);
}
__device__ __forceinline__ void unpack8(const uint4& w, float (&f)[8]) {
  f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x);
  f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
  f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z);
  f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
}

// INT8 cache: quantisation of one token's key or value row.  scale = max |x| / 127
// (1 for a zero row), code = x / scale rounded half to even and clamped to
// +-127, in fp32 with correctly rounded division.
__device__ __forceinline__ float i8_row_scale(float amax) {
  return amax > 0.f ? __fdiv_rn(amax, 127.0f) : 1.0f;
}
__device__ __forceinline__ int i8_code(float x, float scale) {
  // (through the integer: a code that rounded to -0.0f is 0, as the stored byte is)
  return static_cast<int>(fminf(fmaxf(rintf(__fdiv_rn(x, scale)), -127.f), 127.f));
}
// Largest magnitude among the eight bf16 values of a 16-byte chunk.
__device__ __forceinline__ float chunk_amax_bf16(const uint4& c) {
  const uint32_t w[4] = {c.x, c.y, c.z, c.w};
  float a = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) a = fmaxf(a, fmaxf(fabsf(bf16_lo(w[i])), fabsf(bf16_hi(w[i]))));
  return a;
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Values that are the same in every lane of a wavefront must be KNOWN to be so
// by the compiler wherever they steer a branch around a barrier: a value read
// from LDS or global memory counts as divergent, and a barrier reached through
// control flow the compiler regards as divergent may be executed lane-subset by
// lane-subset.  uniform() pins such a value into a scalar register.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int wave_id() { return uniform(threadIdx.x >> 6); }

// Number of set bits of `mask` below this lane.
__device__ __forceinline__ int popc_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0));
}

__device__ __forceinline__ float shfl_xor_f(float v, int m) { return __shfl_xor(v, m, kWave); }

// Wave64 scans / reductions on the DPP data path (a few cycles per step; the
// ds_bpermute route of __shfl_* costs an LDS round trip per step).  Lanes whose
// DPP source does not exist, or whose row is masked off, receive `identity`.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ int dpp_move(int identity, int src) {
  return __builtin_amdgcn_update_dpp(identity, src, CTRL, ROW_MASK, 0xf, false);
}
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143;

__device__ __forceinline__ int wave_inclusive_sum(int v) {
  v += dpp_move<kDppRowShr1>(0, v);
  v += dpp_move<kDppRowShr2>(0, v);
  v += dpp_move<kDppRowShr4>(0, v);
  v += dpp_move<kDppRowShr8>(0, v);
  v += dpp_move<kDppRowBcast15, 0xa>(0, v);
  v += dpp_move<kDppRowBcast31, 0xc>(0, v);
  return v;
}
// Sum over each aligned group of N (8 or 16) lanes, delivered to every lane of
// the group: butterfly on quad permutes, then the half-row / row mirrors.
// (the controls used here name a source for every lane, so the destination needs no
// initial value: one instruction per half)
template <int CTRL>
__device__ __forceinline__ double dpp_move_f64(double v) {
  const int lo = __builtin_amdgcn_mov_dpp(__double2loint(v), CTRL, 0xf, 0xf, true);
  const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(v), CTRL, 0xf, 0xf, true);
  return __hiloint2double(hi, lo);
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E;          // quad_perm [1,0,3,2], [2,3,0,1]
constexpr int kDppHalfMirror = 0x141, kDppMirror = 0x140;  // lane i <-> 7 - i of 8, 15 - i of 16

// Four values per lane, each to be summed over the aligned group of N (8 or 16) lanes the
// lane belongs to: returns, in lanes 2u and 2u + 1 of the group's first eight lanes, the
// sum of v[u].  A butterfly in which every stage halves what a lane still carries (the
// partner takes over the other half): 4 additions (N = 8) instead of the 12 of four
// separate sums.
template <int N>
__device__ __forceinline__ double group_sum4_f64(const double (&v)[4], int lane_in_group) {
  static_assert(N == 8 || N == 16, "group of 8 or 16 lanes");
  double s[4] = {v[0], v[1], v[2], v[3]};
  if (N == 16) {
#pragma unroll
    for (int u = 0; u < 4; ++u) s[u] += dpp_move_f64<kDppMirror>(s[u]);
  }
  // lanes 0-3 of each eight go on with v[0], v[1], lanes 4-7 with v[2], v[3]
  const bool upper = (lane_in_group & 4) != 0;
  double k0 = upper ? s[2] : s[0], k1 = upper ? s[3] : s[1];
  k0 += dpp_move_f64<kDppHalfMirror>(upper ? s[0] : s[2]);
  k1 += dpp_move_f64<kDppHalfMirror>(upper ? s[1] : s[3]);
  // of those, lanes with bit 1 clear go on with the first, the others with the second
  const bool second = (lane_in_group & 2) != 0;
  double k = second ? k1 : k0;
  k += dpp_move_f64<kDppXor2>(second ? k0 : k1);
  k += dpp_move_f64<kDppXor1>(k);
  return k;
}

// Combine a value over the four lanes {l, l^16, l^32, l^48} (the four rows of a
// wave) with the gfx950 row-swap instructions.
typedef unsigned uint2s_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float rows_max_f32(float v) {
  uint2s_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  const float m = fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(m), __float_as_uint(m), false, false);
  return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float rows_sum_f32(float v) {
  uint2s_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  const float m = __uint_as_float(r.x) + __uint_as_float(r.y);
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(m), __float_as_uint(m), false, false);
  return __uint_as_float(r.x) + __uint_as_float(r.y);
}

// Reductions over the wave; the result is returned as a scalar (lane 63 of the scan).
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
  int x = (int)v;
  const int id = -1;  // 0xffffffff
  x = (int)min((uint32_t)x, (uint32_t)dpp_move<kDppRowShr1>(id, x));
  x = (int)min((uint32_t)x, (uint32_t)dpp_move<kDppRowShr2>(id, x));
  x = (int)min((uint32_t)x, (uint32_t)dpp_move<kDppRowShr4>(id, x));
  x = (int)min((uint32_t)x, (uint32_t)dpp_move<kDppRowShr8>(id, x));
  x = (int)min((uint32_t)x, (uint32_t)dpp_move<kDppRowBcast15, 0xa>(id, x));
  x = (int)min((uint32_t)x, (uint32_t)dpp_move<kDppRowBcast31, 0xc>(id, x));
  return (uint32_t)__builtin_amdgcn_readlane(x, 63);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  int x = (int)v;
  x = (int)max((uint32_t)x, (uint32_t)dpp_move<kDppRowShr1>(0, x));
  x = (int)max((uint32_t)x, (uint32_t)dpp_move<kDppRowShr2>(0, x));
  x = (int)max((uint32_t)x, (uint32_t)dpp_move<kDppRowShr4>(0, x));
  x = (int)max((uint32_t)x, (uint32_t)dpp_move<kDppRowShr8>(0, x));
  x = (int)max((uint32_t)x, (uint32_t)dpp_move<kDppRowBcast15, 0xa>(0, x));
  x = (int)max((uint32_t)x, (uint32_t)dpp_move<kDppRowBcast31, 0xc>(0, x));
  return (uint32_t)__builtin_amdgcn_readlane(x, 63);
}

__device__ __forceinline__ float wave_max_f32(float v) {
  const int id = (int)0xff800000u;  // -inf
  int x = (int)__float_as_uint(v);
  auto mx = [](int a, int b) { return (int)__float_as_uint(fmaxf(__uint_as_float((uint32_t)a), __uint_as_float((uint32_t)b))); };
  x = mx(x, dpp_move<kDppRowShr1>(id, x));
  x = mx(x, dpp_move<kDppRowShr2>(id, x));
  x = mx(x, dpp_move<kDppRowShr4>(id, x));
  x = mx(x, dpp_move<kDppRowShr8>(id, x));
  x = mx(x, dpp_move<kDppRowBcast15, 0xa>(id, x));
  x = mx(x, dpp_move<kDppRowBcast31, 0xc>(id, x));
  return __uint_as_float((uint32_t)__builtin_amdgcn_readlane(x, 63));
}
__device__ __forceinline__ float wave_sum_f32(float v) {
  int x = (int)__float_as_uint(v);
  auto ad = [](int a, int b) { return (int)__float_as_uint(__uint_as_float((uint32_t)a) + __uint_as_float((uint32_t)b)); };
  x = ad(x, dpp_move<kDppRowShr1>(0, x));
  x = ad(x, dpp_move<kDppRowShr2>(0, x));
  x = ad(x, dpp_move<kDppRowShr4>(0, x));
  x = ad(x, dpp_move<kDppRowShr8>(0, x));
  x = ad(x, dpp_move<kDppRowBcast15, 0xa>(0, x));
  x = ad(x, dpp_move<kDppRowBcast31, 0xc>(0, x));
  return __uint_as_float((uint32_t)__builtin_amdgcn_readlane(x, 63));
}

// x / d for 0 <= x < 2^16 and 1 <= d < 2^16 by one multiply, with a constant the host
// works out: magic = floor(2^32 / d) + 1 (exact as long as x * d < 2^32); 0 stands for
// d == 1.  The kernels' first instructions run ahead of their first loads, and a
// division by a run-time value costs some thirty of them.
struct FastDiv {
  uint32_t d, magic;
};
inline FastDiv make_fast_div(int d) {
  FastDiv f;
  f.d = (uint32_t)(d < 1 ? 1 : d);
  f.magic = f.d == 1 ? 0u : 0xffffffffu / f.d + 1u;
  return f;
}
__device__ __forceinline__ int fast_div(int x, const FastDiv& f) {
  return f.magic ? (int)__umulhi((uint32_t)x, f.magic) : x;
}
__device__ __forceinline__ int fast_mod(int x, const FastDiv& f) {
  return x - fast_div(x, f) * (int)f.d;
}

// Streaming loads (the `nt` bit): for lines that ONE instruction of one wave consumes whole
// and nobody reads again (metadata rows, value tiles), so that they do not take a place in
// the compute unit's L1.  Measured on the fused decode: -0.8 to -1.1 us per launch on the
// 16-sequence and 8-sequence configurations, -0.5 us on the long-context one.  A line that
// a second instruction comes back to (a key tile: each row is fetched in halves by two
// instructions) must NOT be loaded this way: the first touch drops it and the second one
// fetches it again (+0.3 us where a wave has one page).
typedef uint32_t stream_u4 __attribute__((ext_vector_type(4)));
typedef uint32_t stream_u2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  const stream_u4 v = __builtin_nontemporal_load(reinterpret_cast<const stream_u4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 load_stream8(const void* p) {
  const stream_u2 v = __builtin_nontemporal_load(reinterpret_cast<const stream_u2*>(p));
  return make_uint2(v.x, v.y);
}
__device__ __forceinline__ uint32_t load_stream4(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p));
}

// Agent-scope (whole GPU, all XCDs) synchronisation words.
__device__ __forceinline__ int atomic_add_agent(int* p, int v) {
  return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int atomic_load_agent(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void atomic_store_agent(int* p, int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Data handed from one workgroup to another inside a kernel travels through
// agent-scope stores and loads (write-through / cache-bypassing accesses of
// just those words) instead of cache-wide release/acquire fences: on this part
// an agent-scope fence writes back or invalidates a whole L2 and serialises
// across workgroups (measured ~0.5 us each, ~100 us for a thousand workgroups).
// Protocol: producer: store_agent(...) x n; stores_complete(); __syncthreads();
// one thread bumps a counter.  Consumer: observes the counter; __syncthreads();
// load_agent(...).
__device__ __forceinline__ void store_agent(float* p, float v) {
  __hip_atomic_store(reinterpret_cast<int*>(p), __float_as_int(v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_agent(const float* p) {
  return __int_as_float(__hip_atomic_load(reinterpret_cast<const int*>(p), __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_AGENT));
}
// A value handed over together with the tag that says which launch wrote it:
// one aligned 8-byte store, so a reader sees both or neither.  The reader polls
// the word itself until the tag is the current one; no counter, no wait for
// the store's acknowledgement, one trip through the memory system in all.
__device__ __forceinline__ void store_agent_tagged(uint64_t* p, float v, uint32_t tag) {
  __hip_atomic_store(p, ((uint64_t)tag << 32) | (uint64_t)__float_as_uint(v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t load_agent_u64(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// All of this wave's outstanding memory operations have been acknowledged.
__device__ __forceinline__ void stores_complete() { __builtin_amdgcn_s_waitcnt(0); }

// Bounded wait until *p >= target.  Returns 1 on success, 0 if the limit expired.
__device__ __forceinline__ int wait_at_least(const int* p, int target, int limit) {
  for (int spin = 0; spin < limit; ++spin) {
    if (atomic_load_agent(p) >= target) return 1;
    __builtin_amdgcn_s_sleep(1);
  }
  return 0;
}


// Phase timestamps for tuning builds (-DTS_PROFILE): thread 0 of every
// workgroup records the constant-rate 100 MHz clock at numbered points.  The
// buffer address is parked in LDS once (TS_MARK_INIT at kernel entry) so that a
// mark costs an LDS read and a store, and waits for no memory load in flight.
// Compiled out of the product library (build.py builds the tuning library,
// libtinyserve_prof.so, on request).  The buffer pointer is a device variable of
// each translation unit: ts_debug_set_profile_buffer sets all of them.
#ifdef TS_PROFILE
static __device__ unsigned long long* g_profile_buf = nullptr;   // [workgroup][64]
__device__ __forceinline__ unsigned long long** profile_slot() {
  __shared__ unsigned long long* slot;
  return &slot;
}
#define TS_MARK_INIT()                                                                  \
  do {                                                                                  \
    if (threadIdx.x == 0) *ts::profile_slot() = ts::g_profile_buf;                      \
  } while (0)
#ifndef TS_PROFILE_MASK
#define TS_PROFILE_MASK 0xffffffffu   // which of the numbered marks are compiled in
#endif
#define TS_MARK(i)                                                                      \
  do {                                                                                  \
    if (((TS_PROFILE_MASK >> (i)) & 1u) && threadIdx.x == 0) {                          \
      unsigned long long* ts_pb = *ts::profile_slot();                                  \
      if (ts_pb) ts_pb[(size_t)blockIdx.x * 64 + (i)] = wall_clock64();                 \
    }                                                                                   \
  } while (0)
// the same by the first lane of EVERY wave: slot base + wave (base = 32, 40, 48, 56)
#define TS_MARK_WAVE(base)                                                              \
  do {                                                                                  \
    if ((threadIdx.x & 63) == 0) {                                                      \
      unsigned long long* ts_pb = *ts::profile_slot();                                  \
      if (ts_pb) ts_pb[(size_t)blockIdx.x * 64 + (base) + (threadIdx.x >> 6)] = wall_clock64(); \
    }                                                                                   \
  } while (0)
#else
#define TS_MARK_INIT() do { } while (0)
#define TS_MARK(i) do { } while (0)
#define TS_MARK_WAVE(base) do { } while (0)
#endif

}  // namespace ts
