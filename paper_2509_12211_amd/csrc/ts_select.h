// Top-K page selection (Section 3.5; step 2 of Algorithm 1) by one workgroup,
// entirely in LDS: a radix select over an order-preserving integer image of the
// fp32 scores, then an ordered compaction that emits the kept page ids in
// ascending order and resolves equal scores in favour of the lower page id.
//
// The radix digits are taken from (key - min key): the scores of one unit span
// a narrow range, so the raw high bits are identical for every page (one LDS
// bin would take every atomic); after subtracting the minimum, the top 11
// significant bits of the range spread the pages over 2048 bins, and one pass
// usually leaves only a handful of candidates in the cut-off bin.
#pragma once
#include "ts_device.h"

namespace ts {

// Larger float <=> larger key.  -0 is folded onto +0 so the two rank equal.
__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t b = __float_as_uint(f);
  if (b == 0x80000000u) b = 0u;
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr int kRadixBits = 11;
constexpr int kRadixBins = 1 << kRadixBits;

struct SelectLds {
  uint32_t* keys;  // [>= Pb]      keys of pages 0..Pb-1 (filled by the caller)
  uint32_t* hist;  // [kRadixBins]
  int* red;        // [32]         small reductions / broadcasts
};
constexpr size_t select_lds_bytes(int Pmax) {
  return (size_t)Pmax * 4 + kRadixBins * 4 + 32 * 4;
}
__device__ __forceinline__ SelectLds carve_select(unsigned char* smem, int Pmax) {
  SelectLds L;
  L.keys = reinterpret_cast<uint32_t*>(smem);
  L.hist = L.keys + Pmax;
  L.red = reinterpret_cast<int*>(L.hist + kRadixBins);
  return L;
}

// Inclusive scan of one int per thread over the workgroup (thread order).
// red: 4 ints of LDS scratch.  Contains two barriers.
__device__ __forceinline__ int block_inclusive_scan(int v, int* red) {
  const int lane = lane_id(), wave = wave_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int up = __shfl_up(v, d, kWave);
    if (lane >= d) v += up;
  }
  __syncthreads();  // red free
  if (lane == kWave - 1) red[wave] = v;
  __syncthreads();
  int off = 0;
  for (int w = 0; w < wave; ++w) off += uniform(red[w]);
  return v + off;
}

// Keeps the Kb largest of keys[0..Pb) (ties: lower index first) and calls
// emit(rank, page) for every kept page, rank = its position in ascending page
// order.  All kThreads threads must call; Pb, Kb workgroup-uniform.
template <typename Emit>
__device__ __forceinline__ void select_topk_lds(const SelectLds& L, int Pb, int Kb, Emit emit) {
  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  Pb = uniform(Pb);
  Kb = uniform(Kb);
  if (Kb <= 0) return;
  if (Kb >= Pb) {  // everything is kept
    for (int j = tid; j < Pb; j += kThreads) emit(j, j);
    return;
  }
  // range of the keys
  uint32_t kmin = 0xffffffffu, kmax = 0u;
  for (int j = tid; j < Pb; j += kThreads) {
    const uint32_t k = L.keys[j];
    kmin = min(kmin, k);
    kmax = max(kmax, k);
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, m, kWave));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, m, kWave));
  }
  if (lane == 0) { L.red[8 + wave] = (int)kmin; L.red[12 + wave] = (int)kmax; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    kmin = min(kmin, (uint32_t)L.red[8 + w]);
    kmax = max(kmax, (uint32_t)L.red[12 + w]);
  }
  kmin = (uint32_t)uniform((int)kmin);
  kmax = (uint32_t)uniform((int)kmax);

  // Candidates: normalised keys nk = key - kmin with nk in [base, base + 2^bits).
  // Everything above that interval is already known to be kept; `need` more are
  // wanted from inside it.
  uint32_t base = 0u;
  int bits = 32 - __clz((int)(kmax - kmin));  // 0 when all keys are equal
  int need = Kb;
  while (bits > 0) {
    const int s = max(bits - kRadixBits, 0);
    for (int i = tid; i < kRadixBins; i += kThreads) L.hist[i] = 0u;
    __syncthreads();
    for (int j = tid; j < Pb; j += kThreads) {
      const uint32_t nk = L.keys[j] - kmin;
      if (nk >= base) {
        const uint32_t d = nk - base;
        if (bits >= 32 || (d >> bits) == 0u) atomicAdd(&L.hist[d >> s], 1u);
      }
    }
    __syncthreads();
    // thread t owns bins 2047-8t .. 2040-8t (descending), so a scan in thread
    // order accumulates from the top bin down
    constexpr int BPT = kRadixBins / kThreads;
    int c[BPT], tot = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) { c[i] = (int)L.hist[kRadixBins - 1 - (tid * BPT + i)]; tot += c[i]; }
    const int incl = block_inclusive_scan(tot, L.red);
    int run = incl - tot;
    if (run < need && need <= incl) {  // exactly one thread: the cut-off bin is one of its own
#pragma unroll
      for (int i = 0; i < BPT; ++i) {
        if (run < need && need <= run + c[i]) {
          L.red[4] = kRadixBins - 1 - (tid * BPT + i);
          L.red[5] = run;
          L.red[6] = c[i];
        }
        run += c[i];
      }
    }
    __syncthreads();
    const int bsel = uniform(L.red[4]), above = uniform(L.red[5]), cnt = uniform(L.red[6]);
    base += (uint32_t)bsel << s;
    need -= above;
    bits = s;
    if (cnt == need) break;  // the whole cut-off bin is kept
  }
  // Kept: nk >= base + 2^bits, plus the first `need` (in page order) of the
  // pages with nk in [base, base + 2^bits).  (bits == 0: one exact value.)
  auto classify = [&](int j, bool& g, bool& e) {
    const uint32_t nk = L.keys[j] - kmin;
    const bool in = nk >= base;
    const uint32_t d = nk - base;
    const bool inside = bits >= 32 || (d >> bits) == 0u;
    g = in && !inside;
    e = in && inside;
  };
  // Ordered compaction.  Each wave owns a contiguous run of pages; count per
  // run, then emit with running offsets.
  const int seg = (((Pb + kWaves - 1) / kWaves) + kWave - 1) & ~(kWave - 1);
  const int s0 = wave * seg, s1 = min(Pb, s0 + seg);
  int cg = 0, ce = 0;
  for (int j0 = s0; j0 < s1; j0 += kWave) {
    const int j = j0 + lane;
    bool g = false, e = false;
    if (j < s1) classify(j, g, e);
    cg += __popcll(__ballot(g));
    ce += __popcll(__ballot(e));
  }
  __syncthreads();  // red[4..6] no longer read
  if (lane == 0) { L.red[16 + wave] = cg; L.red[20 + wave] = ce; }
  __syncthreads();
  int goff = 0, eoff = 0;
  for (int w = 0; w < wave; ++w) { goff += uniform(L.red[16 + w]); eoff += uniform(L.red[20 + w]); }
  for (int j0 = s0; j0 < s1; j0 += kWave) {
    const int j = j0 + lane;
    bool g = false, e = false;
    if (j < s1) classify(j, g, e);
    const uint64_t gm = __ballot(g), em = __ballot(e);
    const int gb = goff + popc_below(gm), eb = eoff + popc_below(em);
    if (g) emit(gb + min(eb, need), j);
    else if (e && eb < need) emit(gb + eb, j);
    goff += __popcll(gm);
    eoff += __popcll(em);
  }
}

}  // namespace ts
