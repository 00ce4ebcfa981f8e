// Top-K page selection (Section 3.5; step 2 of Algorithm 1) by one workgroup,
// entirely in LDS: a two-stage bin select over the scores, then an ordered
// compaction that emits the kept page ids in ascending order and resolves
// equal scores in favour of the lower page id.
//
// A lone wave issues roughly one instruction every 6-8 cycles, so with two
// waves per SIMD this step is bound by its instruction count, not by LDS
// bandwidth: the keys are passed over as few times as possible (range while
// loading, one histogram pass, one compaction pass), every LDS read of a pass
// is issued before the first is used, and nothing goes through ds_bpermute.
#pragma once
#include "../../include/tinyserve.h"
#include "ts_device.h"

namespace ts {

// Larger float <=> larger key.  -0 is folded onto +0 so the two rank equal.
__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t b = __float_as_uint(f);
  if (b == 0x80000000u) b = 0u;
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_score(uint32_t k) {
  return (k & 0x80000000u) ? __uint_as_float(k & 0x7fffffffu) : __uint_as_float(~k);
}

// Pages kept whatever their score (an option outside the paper: the first pages
// of a sequence as attention sinks, its last pages as the newest tokens).  The
// selection gives them the key kForcedKey, above every score's key, so they rank
// ahead of all other pages and among themselves by page id.  Callers fill the
// keys from the scores as if there were no such pages; select_topk_lds
// overwrites the few keys concerned, so a selection without them pays one
// scalar branch.
constexpr uint32_t kForcedKey = 0xffffffffu;
struct ForcedPages {
  int first;       // pages [0, first) are kept
  int last_begin;  // pages [last_begin, Pb) are kept; first <= last_begin <= Pb
  int count;       // first + Pb - last_begin
  __device__ __forceinline__ static ForcedPages make(int keep_first, int keep_last, int Pb) {
    ForcedPages f;
    f.first = min(max(keep_first, 0), Pb);
    f.last_begin = max(f.first, Pb - max(keep_last, 0));
    f.count = f.first + Pb - f.last_begin;
    return f;
  }
};

constexpr int kRadixBits = 11;
constexpr int kRadixBins = 1 << kRadixBits;
static_assert(TS_MAX_PAGES_PER_SEQ / kThreads <= 64, "a thread's chunk must fit a 64-bit mask");

// Keys live in LDS thread-chunked: thread t owns pages t*C .. t*C+C-1 (C =
// ceil(Pb / kThreads)), stored at t*stride + i with an odd stride, so that both
// "every thread reads its i-th key" and "consecutive lanes write consecutive
// pages" are free of bank conflicts.
struct KeyLayout {
  int C, stride;
  uint32_t magic;  // ceil(2^32 / C): j / C == umulhi(j, magic) for j < 2^20
  __device__ __forceinline__ static KeyLayout make(int Pb) {
    KeyLayout k;
    k.C = max(1, (Pb + kThreads - 1) / kThreads);
    k.stride = k.C | 1;
    // (= ceil(2^32 / C) for every C >= 2, with a 32-bit division)
    k.magic = k.C == 1 ? 0u : 0xffffffffu / (uint32_t)k.C + 1u;
    return k;
  }
  __device__ __forceinline__ int at(int j) const {
    const int t = C == 1 ? j : (int)__umulhi((uint32_t)j, magic);
    return t * stride + (j - t * C);
  }
};

struct SelectLds {
  uint32_t* keys;  // [select_key_words(Pmax)]  filled by the caller through KeyLayout::at
  uint32_t* hist;  // [kRadixBins]  bin counts, see bin_slot_index
  int* red;        // [64]   [0..7] wave sums, [16..31] key range of the waves, [40] candidate count
  uint32_t* cand;  // [2 * kMaxCandidates]  (key, page) of the pages in the cut-off bin
};
constexpr int kMaxCandidates = 32;
constexpr size_t select_key_words(int Pmax) {
  // kThreads chunks of (C | 1) words, C = ceil(Pmax / kThreads), padded to 16 bytes
  return (size_t)((kThreads * ((((Pmax + kThreads - 1) / kThreads)) | 1) + 3) / 4 * 4);
}
constexpr size_t select_lds_bytes(int Pmax) {
  return select_key_words(Pmax) * 4 + kRadixBins * 4 + 64 * 4 + 2 * kMaxCandidates * 4;
}
__device__ __forceinline__ SelectLds carve_select(unsigned char* smem, int Pmax) {
  SelectLds L;
  L.keys = reinterpret_cast<uint32_t*>(smem);
  L.hist = L.keys + select_key_words(Pmax);
  L.red = reinterpret_cast<int*>(L.hist + kRadixBins);
  L.cand = reinterpret_cast<uint32_t*>(L.red + 64);
  return L;
}

// Bins are counted top bin first: slot k holds bin kRadixBins - 1 - k, so a scan
// in slot order accumulates from the highest scores down.  Lane l of a wave
// scans slots 32 l .. 32 l + 31; they are laid out so that the lanes' 16-byte
// reads of a round fall on consecutive addresses.
__device__ __forceinline__ int bin_slot_index(int k) {
  // k = l * 32 + j  ->  (j >> 2) * 256 + l * 4 + (j & 3): three bit fields moved
  const uint32_t u = (uint32_t)k;
  return (int)((u & 3u) | ((u >> 5) << 2) | (((u >> 2) & 7u) << 8));
}
static_assert(kRadixBins == 64 * 32, "slot layout written for 64 lanes x 32 slots");

// Clears the bins and the candidate count; all threads, a barrier before the
// first count.
__device__ __forceinline__ void select_clear(const SelectLds& L) {
  reinterpret_cast<uint4*>(L.hist)[threadIdx.x] = make_uint4(0, 0, 0, 0);
  static_assert(kRadixBins == 4 * kThreads, "one 16-byte store per thread clears the bins");
  if (threadIdx.x == 0) L.red[40] = 0;
}
// First half of the selection, to be called by all threads BEFORE the barrier
// that makes the keys visible: clears the bins and deposits each wave's share
// of the key range.  tmin / tmax: this thread's share of the min / max over ALL
// keys (any partition over the threads; 0xffffffff / 0 if it saw none).
__device__ __forceinline__ void select_begin(const SelectLds& L, uint32_t tmin, uint32_t tmax) {
  select_clear(L);
  const uint32_t a = wave_min_u32(tmin), b = wave_max_u32(tmax);
  if (lane_id() == 0) {
    L.red[16 + wave_id()] = (int)a;
    L.red[24 + wave_id()] = (int)b;
  }
}

// Stage 1 of the selection spreads the pages over the kRadixBins bins linearly in
// score: bin = floor((s - lo) * scale), clamped to the bins.  ANY lo and scale >= 0
// give a monotone map (bins respect the order of the keys), which is all the
// selection needs to be exact; they only decide how evenly the pages spread.
// With lo = s_min and scale = 2047 / (s_max - s_min) the scores of a unit spread
// evenly whatever their sign or exponent range.  kForcedKey decodes to a quiet
// NaN, which fminf drops in favour of 2047 (IEEE minNum, v_min_f32 in the
// kernels' IEEE mode): the always-kept pages land in slot 0, the slot of the
// highest scores, with no test of their own (the parity tests with such pages
// cover it).
struct BinMap {
  float lo, scale;
  // slot of a key; 0 = highest scores (see bin_slot_index).  kClampBelow: scores
  // below lo occur (only with an estimated range).
  template <bool kClampBelow>
  __device__ __forceinline__ int slot(uint32_t k) const {
    float x = fminf((key_score(k) - lo) * scale, 2047.0f);
    if (kClampBelow) x = fmaxf(x, 0.f);
    return kRadixBins - 1 - (int)x;
  }
  // the exact range [kmin, kmax] of the keys (all equal: everything in one bin)
  __device__ __forceinline__ static BinMap exact(uint32_t kmin, uint32_t kmax) {
    BinMap m;
    m.lo = key_score(kmin);
    m.scale = kmax > kmin ? 2047.0f / (key_score(kmax) - m.lo) : 0.f;
    return m;
  }
  // A range estimated from a SAMPLE of the keys: [kmin, kmax] of the sample
  // widened by a quarter of its width on either side; keys outside fall into the
  // end bins.  No sample, or a single value: everything goes to one bin, and the
  // selection's exact passes sort it out.
  __device__ __forceinline__ static BinMap widened(uint32_t kmin, uint32_t kmax) {
    BinMap m;
    const float a = key_score(kmin), b = key_score(kmax), w = b - a;
    const bool usable = kmax > kmin && w > 0.f && w < 1e37f;
    m.lo = usable ? a - 0.25f * w : 0.f;
    m.scale = usable ? 2047.0f / (1.5f * w) : 0.f;
    return m;
  }
};

// The key range the waves deposited with select_begin (a barrier in between).
__device__ __forceinline__ void select_deposited_range(const SelectLds& L, uint32_t& kmin,
                                                       uint32_t& kmax) {
  kmin = 0xffffffffu;
  kmax = 0u;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    kmin = min(kmin, (uint32_t)L.red[16 + w]);
    kmax = max(kmax, (uint32_t)L.red[24 + w]);
  }
  kmin = (uint32_t)uniform((int)kmin);
  kmax = (uint32_t)uniform((int)kmax);
}

// Second half: keeps the Kb largest of the Pb keys in L.keys (ties: lower page
// first) and calls emit(rank, page) for every kept page, rank = its position in
// ascending page order.  All kThreads threads must call; Pb, Kb
// workgroup-uniform; select_begin and a barrier must precede the call.
//
// Stage 1 spreads the pages over the 2048 bins LINEARLY in score,
// bin = floor((s - s_min) * 2047 / (s_max - s_min)): a monotone map, so bins
// respect the order of the keys, and one that spreads the scores of a unit
// evenly whatever their sign or exponent range (the raw float bit patterns
// would put a whole binade, or everything on one side of zero, into a handful
// of bins).  Every wave then finds the cut-off bin for itself (no exchange
// between waves, no barrier).  If that bin has to be split, its few pages are
// listed in LDS and every wave ranks them directly; the list and the per-wave
// counts of the pages above the bin share ONE barrier, behind which a page's place
// in the ascending list follows without a further exchange.  Only a cut-off bin
// with more than kMaxCandidates pages (heavy ties) goes through exact radix passes
// on the integer keys and a separate compaction instead.
//
// fp: the always-kept pages (their keys become kForcedKey: linear_slot puts them
// into the top bin, everything after that works on the integer keys).
//
// kCounted = true: the caller has already done stage 1's counting while it filled
// in the keys (into bins cleared by select_begin a barrier earlier), with the bin
// map `counted` and BinMap::slot<true>, and has given the always-kept pages the
// key kForcedKey itself.  The map may come from an estimate of the range: if the
// cut then falls into an end bin crowded with the keys outside the estimate,
// stage 2b's exact passes resolve it like any other crowded bin.
template <bool kCounted = false, typename Emit>
__device__ __forceinline__ void select_topk_lds(const SelectLds& L, const KeyLayout& kl, int Pb,
                                                int Kb, const ForcedPages& fp, Emit emit,
                                                const BinMap counted = BinMap{0.f, 0.f}) {
  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  static_assert(kWaves <= 8, "red[] layout holds 8 wave slots");
  constexpr int kBatch = 8;  // LDS reads issued together
  Pb = uniform(Pb);
  Kb = uniform(Kb);
  if (Kb <= 0) return;
  if (Kb >= Pb) {  // everything is kept
    for (int j = tid; j < Pb; j += kThreads) emit(j, j);
    return;
  }
  if (fp.count >= Kb) {  // the always-kept pages fill the budget: the Kb lowest ids of them
    for (int r = tid; r < Kb; r += kThreads) emit(r, r < fp.first ? r : fp.last_begin + (r - fp.first));
    return;
  }
  const bool any_forced = !kCounted && uniform(fp.count) != 0;
  if (any_forced) {   // (uniform) the keys of the always-kept pages, over what the caller wrote
    for (int j = tid; j < fp.first; j += kThreads) L.keys[kl.at(j)] = kForcedKey;
    for (int j = fp.last_begin + tid; j < Pb; j += kThreads) L.keys[kl.at(j)] = kForcedKey;
    __syncthreads();
  }
  const int C = kl.C;
  const int my_first = tid * C;                       // first page of this thread's chunk
  const int my_n = max(0, min(C, Pb - my_first));     // pages in it
  const uint32_t* my_keys = L.keys + tid * kl.stride;

  auto clear_bins = [&] {
    reinterpret_cast<uint4*>(L.hist)[tid] = make_uint4(0, 0, 0, 0);
  };
  // Block-wide min / max from per-thread partials; one barrier.
  auto block_range = [&](uint32_t& lo, uint32_t& hi) {
    uint32_t a = wave_min_u32(lo), b = wave_max_u32(hi);
    __syncthreads();  // earlier readers of the slots are done
    if (lane == 0) { L.red[16 + wave] = (int)a; L.red[24 + wave] = (int)b; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      a = min(a, (uint32_t)L.red[16 + w]);
      b = max(b, (uint32_t)L.red[24 + w]);
    }
    lo = (uint32_t)uniform((int)a);
    hi = (uint32_t)uniform((int)b);
  };
  // fn(key, i) for each of this thread's keys, kBatch LDS reads in flight at a time
  // A wave all of whose lanes hold a whole batch runs it without per-key tests
  // (all but the wave at the end of the page range do).
  auto for_my_keys = [&](auto fn) {
    int i0 = 0;
    for (; i0 + kBatch <= C && __ballot(my_n < i0 + kBatch) == 0ull; i0 += kBatch) {
      uint32_t k[kBatch];
#pragma unroll
      for (int i = 0; i < kBatch; ++i) k[i] = my_keys[i0 + i];
#pragma unroll
      for (int i = 0; i < kBatch; ++i) fn(k[i], i0 + i);
    }
    for (; i0 < C; i0 += kBatch) {
      uint32_t k[kBatch];
      // (the first test is uniform: a chunk shorter than a batch skips the rest of it)
#pragma unroll
      for (int i = 0; i < kBatch; ++i) k[i] = (i0 + i < C && i0 + i < my_n) ? my_keys[i0 + i] : 0u;
#pragma unroll
      for (int i = 0; i < kBatch; ++i)
        if (i0 + i < C && i0 + i < my_n) fn(k[i], i0 + i);
    }
  };
  // Top-down scan of the bins by ONE wave (every wave does it for itself): the
  // slot in which the `need`-th largest counted key falls, the keys above it,
  // the keys in it.  The counts must be visible (barrier) before the call.
  auto find_cut = [&](int need, int& slot, int& above, int& cnt) {
    int tot = 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const uint4 h = reinterpret_cast<const uint4*>(L.hist)[r * 64 + lane];
      tot += (int)(h.x + h.y + h.z + h.w);
    }
    const int incl = wave_inclusive_sum(tot), excl = incl - tot;
    const uint64_t m = __ballot(excl < need && need <= incl);
    const int cl = m ? __builtin_ctzll(m) : kWave - 1;  // lane holding the cut-off slot
    const int base = __builtin_amdgcn_readlane(excl, cl);
    // second level: the 32 slots of that lane, one per lane
    const int v = lane < 32 ? (int)L.hist[bin_slot_index(32 * cl + lane)] : 0;
    const int incl2 = wave_inclusive_sum(v), excl2 = incl2 - v;
    const uint64_t m2 = __ballot(lane < 32 && base + excl2 < need && need <= base + incl2);
    const int j = m2 ? __builtin_ctzll(m2) : 31;
    slot = 32 * cl + j;
    above = base + __builtin_amdgcn_readlane(excl2, j);
    cnt = __builtin_amdgcn_readlane(v, j);
  };

  // ---- stage 1: linear bins over [s_min, s_max] ------------------------------
  // (counted by the caller: the keys' range is not known here, and need not be)
  uint32_t kmin = 0u, kmax = 0xffffffffu;
  if (!kCounted) select_deposited_range(L, kmin, kmax);
  TS_MARK(10);
  const BinMap bins = kCounted ? counted : BinMap::exact(kmin, kmax);
  auto linear_slot = [&](uint32_t k) { return bins.template slot<kCounted>(k); };
  int need = Kb, cut_slot = 0;
  uint32_t clo = kmin, chi = kmax, base = 0u;  // stage 2b: the keys still undecided are
  int bits = 0;                                // those k with k - clo in [base, base + 2^bits)
  if (kmax > kmin) {
    if (!kCounted) {
      for_my_keys([&](uint32_t k, int) { atomicAdd(&L.hist[bin_slot_index(linear_slot(k))], 1u); });
      __syncthreads();
    }
    TS_MARK(11);
    int above, cnt;
    find_cut(need, cut_slot, above, cnt);
    TS_MARK(12);
    need -= above;
    if (cnt == need || cnt <= kMaxCandidates) {
      // ---- stage 2a, the usual case: the cut-off bin is kept whole, or holds few enough
      // pages to list them.  ONE pass over the keys and ONE barrier: every thread marks
      // the pages of its chunk that are kept for certain (above the cut-off bin), lists
      // those in the bin, and the per-wave counts of the certain ones go out with the
      // list.  Behind the barrier every wave ranks the listed pages by itself; a page's
      // place in the ascending list is then the certain pages before it (a prefix over
      // the threads) plus the listed pages kept before it (counted off the list).
      const bool whole = uniform(cnt == need ? 1 : 0) != 0;
      uint64_t sbits = 0, cbits = 0;   // chunk masks (C <= 64): kept for certain / in the cut-off bin
      for_my_keys([&](uint32_t k, int i) {
        const int s = linear_slot(k);
        const bool in_cut = s == cut_slot;
        sbits |= (uint64_t)((s < cut_slot || (whole && in_cut)) ? 1 : 0) << i;
        if (!whole && in_cut) {
          cbits |= 1ull << i;
          const int at = atomicAdd(&L.red[40], 1);
          L.cand[2 * at] = k;
          L.cand[2 * at + 1] = (uint32_t)(my_first + i);
        }
      });
      const int cs = __popcll(sbits);
      int incl = wave_inclusive_sum(cs);
      if (lane == kWave - 1) L.red[wave] = incl;   // slots 0..7 are used by nothing else
      __syncthreads();
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const int t = uniform(L.red[w]);
        if (w < wave) incl += t;
      }
      TS_MARK(13);
      int rank = incl - cs;   // certain pages before this thread's chunk
      uint64_t gbits = sbits;
      if (!whole) {
        // a listed page as one 64-bit number that sorts the way the selection does
        // (higher key first, then lower page): key in the upper half, ~page in the lower
        const uint32_t ck = lane < cnt ? L.cand[2 * lane] : 0u;
        const int cp = lane < cnt ? (int)L.cand[2 * lane + 1] : 0x7fffffff;
        const uint64_t mine = ((uint64_t)ck << 32) | (uint32_t)~cp;
        int before = 0;  // listed pages that come before the one in this lane
        for (int t = 0; t < cnt; ++t) {
          const uint64_t other = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)ck, t) << 32) |
                                 (uint32_t)~__builtin_amdgcn_readlane(cp, t);
          before += other > mine ? 1 : 0;
        }
        const bool kept = lane < cnt && before < need;   // the listed page in this lane is kept
        const uint64_t mt = __ballot(lane < cnt && before == need - 1);
        const int tl = mt ? __builtin_ctzll(mt) : 0;
        const uint32_t key_t = (uint32_t)__builtin_amdgcn_readlane((int)ck, tl);
        const int page_t = __builtin_amdgcn_readlane(cp, tl);
        // my own listed pages: kept iff at or before the threshold
        for (uint64_t todo = cbits; todo != 0; todo &= todo - 1) {
          const int i = __builtin_ctzll(todo);
          const uint32_t k = my_keys[i];
          const int page = my_first + i;
          if (k > key_t || (k == key_t && page <= page_t)) gbits |= 1ull << i;
        }
        // listed pages kept in the chunks before mine: those of the waves before mine (the
        // owner of page p is thread p / C; one ballot over the list), and those of the
        // lanes before mine in my own wave, which are these lanes' own (a scan)
        const int owner_wave = (C == 1 ? cp : (int)__umulhi((uint32_t)cp, kl.magic)) >> 6;
        const int own = __popcll(gbits & ~sbits);
        rank += __popcll(__ballot(kept && owner_wave < wave)) + (wave_inclusive_sum(own) - own);
      }
      TS_MARK(14);
      for (uint64_t todo = gbits; todo != 0; todo &= todo - 1) emit(rank++, my_first + __builtin_ctzll(todo));
      return;
    } else {
      // ---- stage 2b: exact radix passes on the keys of the cut-off bin ----------
      __syncthreads();  // every wave has read the stage-1 counts
      clear_bins();
      clo = 0xffffffffu;
      chi = 0u;
      for_my_keys([&](uint32_t k, int) {
        if (linear_slot(k) == cut_slot) { clo = min(clo, k); chi = max(chi, k); }
      });
      block_range(clo, chi);
      bits = 32 - __clz((int)(chi - clo));  // 0: all of the bin's keys are equal
      while (bits > 0) {
        const int s = max(bits - kRadixBits, 0);
        for_my_keys([&](uint32_t k, int) {
          const uint32_t nk = k - clo, d = nk - base;
          if (k >= clo && k <= chi && nk >= base && (bits >= 32 || (d >> bits) == 0u))
            atomicAdd(&L.hist[bin_slot_index(kRadixBins - 1 - (int)(d >> s))], 1u);
        });
        __syncthreads();
        int ssel, above2, cnt2;
        find_cut(need, ssel, above2, cnt2);
        base += (uint32_t)(kRadixBins - 1 - ssel) << s;
        need -= above2;
        bits = s;
        if (cnt2 == need || bits == 0) break;
        __syncthreads();  // every wave has read the counts
        clear_bins();
        __syncthreads();
      }
    }
  }
  TS_MARK(13);
  // Heavy ties (or all scores equal).  Kept for certain (g): above the cut; kept while the
  // quota `need` lasts, in page order (e): keys k with k - clo in [base, base + 2^bits),
  // one exact value when bits == 0.
  if (!(kmax > kmin)) need = Kb - fp.count;  // all scores equal: the always-kept pages, then the lowest ids
  // Ordered compaction in one pass: every thread classifies its own chunk of
  // consecutive pages (bit masks in registers), a workgroup scan of the packed
  // counts gives its starting offsets, and it emits its kept pages in order.
  uint64_t gbits = 0, ebits = 0;  // chunk masks (C <= 64)
  for_my_keys([&](uint32_t k, int i) {
    const uint32_t nk = k - clo, d = nk - base;
    const bool inside = bits >= 32 || (d >> bits) == 0u;
    const bool in = k >= clo && k <= chi && nk >= base;
    gbits |= (uint64_t)((k > chi || (in && !inside)) ? 1 : 0) << i;
    ebits |= (uint64_t)((in && inside) ? 1 : 0) << i;
  });
  const int cg = __popcll(gbits), ce = __popcll(ebits);
  const int packed = cg | (ce << 16);  // both sums stay below 2^15
  int incl = wave_inclusive_sum(packed);
  if (lane == kWave - 1) L.red[wave] = incl;   // slots 0..7 are used by nothing else
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const int t = uniform(L.red[w]);
    if (w < wave) incl += t;
  }
  TS_MARK(14);
  const int excl = incl - packed;
  const int goff = excl & 0xffff, eoff = excl >> 16;
  // only the marked pages are visited (few threads hold any when K << P)
  for (uint64_t todo = gbits | ebits; todo != 0; todo &= todo - 1) {
    const int i = __builtin_ctzll(todo);
    const uint64_t below = (1ull << i) - 1;
    const int gb = goff + __popcll(gbits & below), eb = eoff + __popcll(ebits & below);
    if ((gbits >> i) & 1) emit(gb + min(eb, need), my_first + i);
    else if (eb < need) emit(gb + eb, my_first + i);
  }
}

}  // namespace ts
