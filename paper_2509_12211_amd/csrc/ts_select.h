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
// keys padded to a multiple of 4 words: hist is accessed 16 bytes at a time
constexpr size_t select_lds_bytes(int Pmax) {
  return (size_t)((Pmax + 3) / 4 * 4) * 4 + kRadixBins * 4 + 32 * 4;
}
__device__ __forceinline__ SelectLds carve_select(unsigned char* smem, int Pmax) {
  SelectLds L;
  L.keys = reinterpret_cast<uint32_t*>(smem);
  L.hist = L.keys + (Pmax + 3) / 4 * 4;
  L.red = reinterpret_cast<int*>(L.hist + kRadixBins);
  return L;
}

// Keeps the Kb largest of keys[0..Pb) (ties: lower index first) and calls
// emit(rank, page) for every kept page, rank = its position in ascending page
// order.  All kThreads threads must call; Pb, Kb workgroup-uniform.
//
// hist is stored top bin first (slot k holds bin 2047 - k), so that a thread
// reads its 8 consecutive bins with two 16-byte LDS loads and a scan in thread
// order accumulates from the top bin down.
template <typename Emit>
__device__ __forceinline__ void select_topk_lds(const SelectLds& L, int Pb, int Kb, Emit emit) {
  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  constexpr int BPT = kRadixBins / kThreads;  // 8 bins per thread
  Pb = uniform(Pb);
  Kb = uniform(Kb);
  if (Kb <= 0) return;
  if (Kb >= Pb) {  // everything is kept
    for (int j = tid; j < Pb; j += kThreads) emit(j, j);
    return;
  }
  // range of the keys (and the bins cleared for the first pass)
  uint32_t kmin = 0xffffffffu, kmax = 0u;
  for (int j0 = tid; j0 < Pb; j0 += kThreads * 4) {
    uint32_t k[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) k[i] = j0 + i * kThreads < Pb ? L.keys[j0 + i * kThreads] : 0u;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (j0 + i * kThreads < Pb) { kmin = min(kmin, k[i]); kmax = max(kmax, k[i]); }
  }
  kmin = wave_min_u32(kmin);
  kmax = wave_max_u32(kmax);
  if (lane == 0) { L.red[8 + wave] = (int)kmin; L.red[12 + wave] = (int)kmax; }
  reinterpret_cast<uint4*>(L.hist)[tid * 2] = make_uint4(0, 0, 0, 0);
  reinterpret_cast<uint4*>(L.hist)[tid * 2 + 1] = make_uint4(0, 0, 0, 0);
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    kmin = min(kmin, (uint32_t)L.red[8 + w]);
    kmax = max(kmax, (uint32_t)L.red[12 + w]);
  }
  kmin = (uint32_t)uniform((int)kmin);
  kmax = (uint32_t)uniform((int)kmax);
  TS_MARK(10);

  // Candidates: normalised keys nk = key - kmin with nk in [base, base + 2^bits).
  // Everything above that interval is already known to be kept; `need` more are
  // wanted from inside it.
  uint32_t base = 0u;
  int bits = 32 - __clz((int)(kmax - kmin));  // 0 when all keys are equal
  int need = Kb;
  bool first = true;
  while (bits > 0) {
    const int s = max(bits - kRadixBits, 0);
    if (!first) {
      reinterpret_cast<uint4*>(L.hist)[tid * 2] = make_uint4(0, 0, 0, 0);
      reinterpret_cast<uint4*>(L.hist)[tid * 2 + 1] = make_uint4(0, 0, 0, 0);
      __syncthreads();
    }
    first = false;
    for (int j0 = tid; j0 < Pb; j0 += kThreads * 4) {
      uint32_t k[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) k[i] = j0 + i * kThreads < Pb ? L.keys[j0 + i * kThreads] : 0u;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t nk = k[i] - kmin;
        const uint32_t d = nk - base;
        const bool in = j0 + i * kThreads < Pb && nk >= base && (bits >= 32 || (d >> bits) == 0u);
        if (in) atomicAdd(&L.hist[kRadixBins - 1 - (d >> s)], 1u);
      }
    }
    __syncthreads();
    TS_MARK(11);
    // thread t owns slots 8t..8t+7 = bins 2047-8t .. 2040-8t
    const uint4 h0 = reinterpret_cast<const uint4*>(L.hist)[tid * 2];
    const uint4 h1 = reinterpret_cast<const uint4*>(L.hist)[tid * 2 + 1];
    const int c[BPT] = {(int)h0.x, (int)h0.y, (int)h0.z, (int)h0.w,
                        (int)h1.x, (int)h1.y, (int)h1.z, (int)h1.w};
    int tot = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) tot += c[i];
    int incl = wave_inclusive_sum(tot);
    if (lane == kWave - 1) L.red[wave] = incl;
    __syncthreads();
    for (int w = 0; w < wave; ++w) incl += uniform(L.red[w]);
    TS_MARK(12);
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
  TS_MARK(13);
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
  TS_MARK(14);
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
