// Device-side helpers shared by the gfx950 kernels: bf16 unpacking, wave64
// cross-lane primitives, agent-scope synchronisation words.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ts {

constexpr int kWave = 64;
constexpr int kThreads = 256;            // every kernel here runs 4 wavefronts per workgroup
constexpr int kWaves = kThreads / kWave;

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// A 32-bit word holds two bf16: the low half is element 0.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t x) {
  return __uint_as_float(static_cast<uint32_t>(x) << 16);
}

__device__ __forceinline__ void unpack8(const uint4& w, float (&f)[8]) {
  f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x);
  f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
  f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z);
  f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
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

}  // namespace ts
