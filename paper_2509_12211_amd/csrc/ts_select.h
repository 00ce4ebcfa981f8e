// Top-K page selection (Section 3.5; step 2 of Algorithm 1) by one workgroup,
// entirely in LDS: a two-stage bin select over the scores, then an ordered
// compaction that emits the kept page ids in ascending order and resolves
// equal scores in favour of the lower page id.
//
// A lone wave issues roughly one instruction every 6-8 cycles, so with four
// waves per workgroup this step is bound by its instruction count, not by LDS
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
    k.magic = k.C == 1 ? 0u : (uint32_t)((0x100000000ull + k.C - 1) / k.C);
    return k;
  }
  __device__ __forceinline__ int at(int j) const {
    const int t = C == 1 ? j : (int)__umulhi((uint32_t)j, magic);
    return t * stride + (j - t * C);
  }
};

struct SelectLds {
  uint32_t* keys;  // [select_key_words(Pmax)]  filled by the caller through KeyLayout::at
  uint32_t* hist;  // [kRadixBins]
  int* red;        // [64]   [0..7] wave sums, [8..10] cut, [16..31] / [32..47] key ranges
};
constexpr size_t select_key_words(int Pmax) {
  // kThreads chunks of (C | 1) words, C = ceil(Pmax / kThreads), padded to 16 bytes
  return (size_t)((kThreads * ((((Pmax + kThreads - 1) / kThreads)) | 1) + 3) / 4 * 4);
}
constexpr size_t select_lds_bytes(int Pmax) {
  return select_key_words(Pmax) * 4 + kRadixBins * 4 + 64 * 4;
}
__device__ __forceinline__ SelectLds carve_select(unsigned char* smem, int Pmax) {
  SelectLds L;
  L.keys = reinterpret_cast<uint32_t*>(smem);
  L.hist = L.keys + select_key_words(Pmax);
  L.red = reinterpret_cast<int*>(L.hist + kRadixBins);
  return L;
}

// Keeps the Kb largest of the Pb keys in L.keys (ties: lower page first) and
// calls emit(rank, page) for every kept page, rank = its position in ascending
// page order.  tmin / tmax: this thread's share of the min / max over ALL keys
// (any partition over the threads; 0xffffffff / 0 if it saw none).  All
// kThreads threads must call; Pb, Kb workgroup-uniform; the keys must be
// visible (barrier) before the call.
//
// Stage 1 spreads the pages over the 2048 bins LINEARLY in score,
// bin = floor((s - s_min) * 2047 / (s_max - s_min)): a monotone map, so bins
// respect the order of the keys, and one that spreads the scores of a unit
// evenly whatever their sign or exponent range (the raw float bit patterns
// would put a whole binade, or everything on one side of zero, into a handful
// of bins).  If the cut-off bin has to be split, stage 2 runs exact radix
// passes on the integer keys of that bin's pages only, normalised by their own
// minimum.
//
// hist is stored top bin first (slot k holds bin 2047 - k), so that a thread
// reads its consecutive bins with 16-byte LDS loads and a scan in thread
// order accumulates from the top bin down.
template <typename Emit>
__device__ __forceinline__ void select_topk_lds(const SelectLds& L, const KeyLayout& kl, int Pb,
                                                int Kb, uint32_t tmin, uint32_t tmax, Emit emit) {
  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  constexpr int BPT = kRadixBins / kThreads;  // bins per thread
  static_assert(BPT == 4 || BPT == 8, "bin scan written for 4 or 8 bins per thread");
  static_assert(kWaves <= 8, "red[] layout holds 8 wave slots");
  constexpr int kBatch = 8;  // LDS reads issued together
  Pb = uniform(Pb);
  Kb = uniform(Kb);
  if (Kb <= 0) return;
  if (Kb >= Pb) {  // everything is kept
    for (int j = tid; j < Pb; j += kThreads) emit(j, j);
    return;
  }
  const int C = kl.C;
  const int my_first = tid * C;                       // first page of this thread's chunk
  const int my_n = max(0, min(C, Pb - my_first));     // pages in it
  const uint32_t* my_keys = L.keys + tid * kl.stride;

  auto clear_bins = [&] {
#pragma unroll
    for (int i = 0; i < BPT / 4; ++i)
      reinterpret_cast<uint4*>(L.hist)[tid * (BPT / 4) + i] = make_uint4(0, 0, 0, 0);
  };
  // Block-wide min / max from per-thread partials; one barrier.
  auto block_range = [&](uint32_t& lo, uint32_t& hi, int slot) {
    uint32_t a = wave_min_u32(lo), b = wave_max_u32(hi);
    if (lane == 0) { L.red[slot + wave] = (int)a; L.red[slot + kWaves + wave] = (int)b; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      a = min(a, (uint32_t)L.red[slot + w]);
      b = max(b, (uint32_t)L.red[slot + kWaves + w]);
    }
    lo = (uint32_t)uniform((int)a);
    hi = (uint32_t)uniform((int)b);
  };
  // fn(key, i) for each of this thread's keys, kBatch LDS reads in flight at a time
  auto for_my_keys = [&](auto fn) {
    for (int i0 = 0; i0 < my_n; i0 += kBatch) {
      uint32_t k[kBatch];
#pragma unroll
      for (int i = 0; i < kBatch; ++i) k[i] = i0 + i < my_n ? my_keys[i0 + i] : 0u;
#pragma unroll
      for (int i = 0; i < kBatch; ++i)
        if (i0 + i < my_n) fn(k[i], i0 + i);
    }
  };
  // Top-down scan of the bins: finds the bin in which the `need`-th largest
  // counted key falls.  Two barriers.  Returns bin, keys above it, keys in it.
  auto find_cut = [&](int need, int& bin, int& above, int& cnt) {
    int c[BPT];
#pragma unroll
    for (int i = 0; i < BPT / 4; ++i) {
      const uint4 h = reinterpret_cast<const uint4*>(L.hist)[tid * (BPT / 4) + i];
      c[4 * i] = (int)h.x; c[4 * i + 1] = (int)h.y; c[4 * i + 2] = (int)h.z; c[4 * i + 3] = (int)h.w;
    }
    int tot = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) tot += c[i];
    int incl = wave_inclusive_sum(tot);
    if (lane == kWave - 1) L.red[wave] = incl;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const int t = uniform(L.red[w]);
      if (w < wave) incl += t;
    }
    int run = incl - tot;
    if (run < need && need <= incl) {  // exactly one thread: the cut-off bin is one of its own
#pragma unroll
      for (int i = 0; i < BPT; ++i) {
        if (run < need && need <= run + c[i]) {
          L.red[8] = kRadixBins - 1 - (tid * BPT + i);
          L.red[9] = run;
          L.red[10] = c[i];
        }
        run += c[i];
      }
    }
    __syncthreads();
    bin = uniform(L.red[8]);
    above = uniform(L.red[9]);
    cnt = uniform(L.red[10]);
  };

  // ---- stage 1: linear bins over [s_min, s_max] ------------------------------
  uint32_t kmin = tmin, kmax = tmax;
  clear_bins();
  block_range(kmin, kmax, 16);
  TS_MARK(10);
  const float smin = key_score(kmin);
  const float scale = kmax > kmin ? 2047.0f / (key_score(kmax) - smin) : 0.f;
  auto linear_bin = [&](uint32_t k) {
    return (int)fminf((key_score(k) - smin) * scale, 2047.0f);
  };
  int need = Kb, cut_bin = 0;
  bool by_bin = false;        // true: the cut-off bin is kept whole
  uint32_t clo = kmin, chi = kmax, base = 0u;
  int bits = 0;
  if (kmax > kmin) {
    for_my_keys([&](uint32_t k, int) { atomicAdd(&L.hist[kRadixBins - 1 - linear_bin(k)], 1u); });
    __syncthreads();
    TS_MARK(11);
    int above, cnt;
    find_cut(need, cut_bin, above, cnt);
    TS_MARK(12);
    need -= above;
    by_bin = cnt == need;
    if (!by_bin) {
      // ---- stage 2: exact radix passes on the keys of the cut-off bin ------------
      clear_bins();
      clo = 0xffffffffu;
      chi = 0u;
      for_my_keys([&](uint32_t k, int) {
        if (linear_bin(k) == cut_bin) { clo = min(clo, k); chi = max(chi, k); }
      });
      block_range(clo, chi, 32);
      bits = 32 - __clz((int)(chi - clo));  // 0: all of the bin's keys are equal
      while (bits > 0) {
        const int s = max(bits - kRadixBits, 0);
        for_my_keys([&](uint32_t k, int) {
          const uint32_t nk = k - clo, d = nk - base;
          if (k >= clo && k <= chi && nk >= base && (bits >= 32 || (d >> bits) == 0u))
            atomicAdd(&L.hist[kRadixBins - 1 - (d >> s)], 1u);
        });
        __syncthreads();
        int bsel, above2, cnt2;
        find_cut(need, bsel, above2, cnt2);
        base += (uint32_t)bsel << s;
        need -= above2;
        bits = s;
        if (cnt2 == need || bits == 0) break;
        clear_bins();
        __syncthreads();
      }
    }
  }
  TS_MARK(13);
  // Kept: everything above the cut, plus the first `need` (in page order) of
  // the pages at the cut (by_bin: the whole cut-off bin, and need == its size;
  // otherwise keys k with k - clo in [base, base + 2^bits), one exact value
  // when bits == 0).
  auto classify = [&](uint32_t k, bool& g, bool& e) {
    if (by_bin) {
      const int b = linear_bin(k);
      g = b > cut_bin;
      e = b == cut_bin;
    } else {
      const uint32_t nk = k - clo, d = nk - base;
      const bool inside = bits >= 32 || (d >> bits) == 0u;
      const bool in = k >= clo && k <= chi && nk >= base;
      g = k > chi || (in && !inside);
      e = in && inside;
    }
  };
  // Ordered compaction in one pass: every thread classifies its own chunk of
  // consecutive pages (bit masks in registers), a workgroup scan of the packed
  // counts gives its starting offsets, and it emits its kept pages in order.
  uint64_t gbits = 0, ebits = 0;  // chunk masks (C <= 64)
  for_my_keys([&](uint32_t k, int i) {
    bool g, e;
    classify(k, g, e);
    gbits |= (uint64_t)g << i;
    ebits |= (uint64_t)e << i;
  });
  const int cg = __popcll(gbits), ce = __popcll(ebits);
  const int packed = cg | (ce << 16);  // both sums stay below 2^15
  int incl = wave_inclusive_sum(packed);
  __syncthreads();  // red[0..10] no longer read
  if (lane == kWave - 1) L.red[wave] = incl;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const int t = uniform(L.red[w]);
    if (w < wave) incl += t;
  }
  TS_MARK(14);
  const int excl = incl - packed;
  int goff = excl & 0xffff, eoff = excl >> 16;
  for (int i = 0; i < my_n; ++i) {
    const bool g = (gbits >> i) & 1, e = (ebits >> i) & 1;
    if (g) emit(goff + min(eoff, need), my_first + i);
    else if (e && eoff < need) emit(goff + eoff, my_first + i);
    goff += g;
    eoff += e;
  }
}

}  // namespace ts
