// Top-K page selection (Section 3.5; step 2 of Algorithm 1) by one workgroup:
// MSB-first radix select on an order-preserving integer image of the fp32
// score, then an ordered compaction that emits the kept page ids ascending and
// resolves equal scores in favour of the lower page id.
#pragma once
#include "ts_device.h"

namespace ts {

// Larger float <=> larger key.  -0 is folded onto +0 so the two rank equal.
__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t b = __float_as_uint(f);
  if (b == 0x80000000u) b = 0u;
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

struct SelectScratch {
  uint32_t* keys;   // [>= Pb] LDS
  uint32_t* hist;   // [256]   LDS
  int* misc;        // [16]    LDS
};

// srow: the unit's fp32 scores (global), Pb valid pages, keep Kb of them.
// sel_row (global, Kmax entries) receives ascending ids then -1 padding.
// Must be called by all kThreads threads of the workgroup.
__device__ __forceinline__ void select_topk_unit(const float* srow, int Pb, int Kb, int Kmax,
                                                 int32_t* sel_row, const SelectScratch& sc) {
  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  Pb = uniform(Pb);  // workgroup-uniform by contract; they steer branches around barriers
  Kb = uniform(Kb);
  for (int i = max(Kb, 0) + tid; i < Kmax; i += kThreads) sel_row[i] = -1;
  if (Kb <= 0) return;
  if (Kb >= Pb) {  // everything is kept
    for (int i = tid; i < Pb; i += kThreads) sel_row[i] = i;
    return;
  }
  for (int j = tid; j < Pb; j += kThreads) sc.keys[j] = score_key(srow[j]);

  // Radix select: after each 8-bit digit, `prefix` (under `mask`) identifies the
  // bucket holding the Kb-th largest key and `need` how many keys of that bucket
  // are still wanted.
  uint32_t prefix = 0u, mask = 0u;
  int need = Kb;
  bool whole_bucket = false;
  for (int shift = 24; shift >= 0; shift -= 8) {
    sc.hist[tid] = 0u;  // kThreads == 256 bins
    __syncthreads();
    for (int j = tid; j < Pb; j += kThreads) {
      const uint32_t k = sc.keys[j];
      if ((k & mask) == prefix) atomicAdd(&sc.hist[(k >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (wave == 0) {
      // lane l owns bins 255-4l .. 252-4l; an inclusive scan over lanes then
      // counts keys in this lane's bins and all higher ones.
      const int b0 = 255 - 4 * lane;
      const int c0 = sc.hist[b0], c1 = sc.hist[b0 - 1], c2 = sc.hist[b0 - 2], c3 = sc.hist[b0 - 3];
      const int tot = c0 + c1 + c2 + c3;
      int incl = tot;
#pragma unroll
      for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
      }
      const int excl = incl - tot;
      if (excl < need && need <= incl) {  // exactly one lane
        int bsel, above, cnt;
        if (need <= excl + c0) { bsel = b0; above = excl; cnt = c0; }
        else if (need <= excl + c0 + c1) { bsel = b0 - 1; above = excl + c0; cnt = c1; }
        else if (need <= excl + c0 + c1 + c2) { bsel = b0 - 2; above = excl + c0 + c1; cnt = c2; }
        else { bsel = b0 - 3; above = excl + c0 + c1 + c2; cnt = c3; }
        sc.misc[0] = bsel;
        sc.misc[1] = above;
        sc.misc[2] = cnt;
      }
    }
    __syncthreads();
    // broadcast through scalar registers: these steer the loop around barriers
    const int bsel = uniform(sc.misc[0]), above = uniform(sc.misc[1]), cnt = uniform(sc.misc[2]);
    prefix |= static_cast<uint32_t>(bsel) << shift;
    mask |= 255u << shift;
    need -= above;
    if (cnt == need) { whole_bucket = true; break; }  // every key of the bucket is kept
  }
  // Kept: keys above the bucket, plus the first `take_eq` keys (in page order)
  // inside it.  With all 32 bits resolved the bucket is one exact value.
  const int take_eq = whole_bucket ? 0x7fffffff : need;

  // Ordered compaction.  Each wave owns a contiguous run of pages; first count
  // per run, then write with running offsets.
  const int seg = (((Pb + kWaves - 1) / kWaves) + kWave - 1) & ~(kWave - 1);
  const int s0 = wave * seg, s1 = min(Pb, s0 + seg);
  int cg = 0, ce = 0;
  for (int j0 = s0; j0 < s1; j0 += kWave) {
    const int j = j0 + lane;
    const uint32_t k = j < s1 ? (sc.keys[j] & mask) : 0u;
    const bool g = j < s1 && k > prefix, e = j < s1 && k == prefix;
    cg += __popcll(__ballot(g));
    ce += __popcll(__ballot(e));
  }
  __syncthreads();  // misc[0..2] no longer read by anyone
  if (lane == 0) { sc.misc[4 + wave] = cg; sc.misc[8 + wave] = ce; }
  __syncthreads();
  int goff = 0, eoff = 0;
  for (int w = 0; w < wave; ++w) { goff += uniform(sc.misc[4 + w]); eoff += uniform(sc.misc[8 + w]); }
  for (int j0 = s0; j0 < s1; j0 += kWave) {
    const int j = j0 + lane;
    const uint32_t k = j < s1 ? (sc.keys[j] & mask) : 0u;
    const bool g = j < s1 && k > prefix, e = j < s1 && k == prefix;
    const uint64_t gm = __ballot(g), em = __ballot(e);
    const int gb = goff + popc_below(gm), eb = eoff + popc_below(em);
    if (g) sel_row[gb + min(eb, take_eq)] = j;
    else if (e && eb < take_eq) sel_row[gb + eb] = j;
    goff += __popcll(gm);
    eoff += __popcll(em);
  }
}

}  // namespace ts
