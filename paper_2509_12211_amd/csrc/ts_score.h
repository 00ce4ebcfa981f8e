// Page scoring (Eq. 2): the directional bounding-box bound, group-summed.
#pragma once
#include "ts_device.h"

namespace ts {

// For a group of G query heads sharing one KV head,
//   sum_g sum_c max(q_gc * m_c, q_gc * M_c) = sum_c (Qp_c * M_c + Qn_c * m_c)
// with Qp_c = sum_g max(q_gc, 0) and Qn_c = sum_g min(q_gc, 0): a term takes
// M when q >= 0 and m otherwise (the sign test of Eq. 2), so the per-head sum
// factorises.  Two FMAs per channel per page, whatever G is.
//
// The sum is accumulated in fp64 and rounded to fp32 once at the end: with
// temporally correlated keys the terms are large and of mixed sign, the bound
// itself can be 1e3-1e4 times smaller than their magnitudes, and an fp32
// running sum then misses the 1e-5 relative tolerance on the score.  Qp, Qn
// (sums of <= 16 bf16 values) and the bf16 x fp64 products are exact in fp64.
//
// Lane layout: a metadata row (D bf16) is read as D/8 chunks of 16 bytes, so
// one wave-wide 16-byte load covers 64 / (D/8) consecutive pages; each lane
// keeps Qp / Qn for its 8 channels.
template <int D, bool kHalf = false>
struct ScoreLanes {
  static constexpr int LPR = D / 8;         // lanes per metadata row
  static constexpr int PPW = kWave / LPR;   // pages per wave-wide load
  static constexpr int U = 4;               // wave-wide loads of min (and of max) in flight
  static constexpr int PPI = PPW * U;       // pages one wave covers per iteration
  double qp[8], qn[8];

  // Qp / Qn of the unit, computed once per workgroup through LDS: the G query
  // rows arrive with a single round of 16-byte loads (a per-lane loop over the
  // heads would pay one memory round trip per head), threads 0..D-1 reduce one
  // channel each over the heads, and every lane picks up its 8 channels.
  // Split in two so the caller can issue other loads between the query load
  // and its first use (loads return in issue order: what is needed first is
  // issued first).  stage: LDS scratch of query_stage_bytes(G) bytes.
  static constexpr size_t query_stage_bytes(int G) { return (size_t)G * D * 2 + 2 * D * 8; }
  static constexpr int kQueryLoads = 16 * D / 8 / kThreads > 0 ? 16 * D / 8 / kThreads : 1;

  struct QueryRegs { uint4 w[kQueryLoads]; };

  // Every thread loads and every thread stages what it loaded (thread i takes
  // chunk i, threads past the last chunk take the last one again; duplicates carry
  // identical data): a
  // load under a branch makes the compiler wait for ALL outstanding loads
  // wherever it needs one of them, instead of counting, and a load whose only
  // use sits under a branch is moved down into that branch.
  __device__ __forceinline__ static void issue_query(QueryRegs& r, const uint16_t* q_group, int G) {
    const int n16 = G * D / 8;
#pragma unroll
    for (int k = 0; k < kQueryLoads; ++k)
      r.w[k] = reinterpret_cast<const uint4*>(q_group)[min((int)threadIdx.x + k * kThreads, n16 - 1)];
  }

  // Two barriers.
  __device__ __forceinline__ void finish_query(const QueryRegs& r, int G, unsigned char* stage) {
    uint4* raw = reinterpret_cast<uint4*>(stage);
    double* red = reinterpret_cast<double*>(stage + (size_t)G * D * 2);   // [2][D]
    const int n16 = G * D / 8;
#pragma unroll
    for (int k = 0; k < kQueryLoads; ++k) {
      raw[min((int)threadIdx.x + k * kThreads, n16 - 1)] = r.w[k];
    }
    TS_MARK(20);
    __syncthreads();
    TS_MARK(21);
    if (threadIdx.x < D) {
      const uint16_t* col = reinterpret_cast<const uint16_t*>(stage) + threadIdx.x;
      double p = 0.0, n = 0.0;
      for (int g = 0; g < G; ++g) {
        const float f = elem_to_f32<kHalf>(col[g * D]);
        p += static_cast<double>(fmaxf(f, 0.f));
        n += static_cast<double>(fminf(f, 0.f));
      }
      red[threadIdx.x] = p;
      red[D + threadIdx.x] = n;
    }
    __syncthreads();
    const int cg = lane_id() % LPR;
#pragma unroll
    for (int i = 0; i < 8; ++i) { qp[i] = red[cg * 8 + i]; qn[i] = red[D + cg * 8 + i]; }
  }

  // Two chains of eight (the max terms, the min terms) instead of one of sixteen: with
  // four rows a wave has eight independent chains to interleave.
  __device__ __forceinline__ double row_partial(const uint4& mn, const uint4& mx) const {
    float lo[8], hi[8];
    unpack8e<kHalf>(mn, lo);
    unpack8e<kHalf>(mx, hi);
    double sp = 0.0, sn = 0.0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      sp = fma(qp[i], static_cast<double>(hi[i]), sp);
      sn = fma(qn[i], static_cast<double>(lo[i]), sn);
    }
    return sp + sn;
  }
};

// The metadata rows one wave has in flight: U wave-wide loads of min and of max,
// each covering PPW consecutive pages, the u-th starting at page base + u * rstep
// (rstep = PPW: the pages [base, base + PPI); larger when the groups of PPW pages
// are dealt out in turn to several workgroups).  Rows up to Pmax are always
// readable (whatever they hold), so the loads do not wait for the sequence length.
template <int D, bool kHalf = false>
struct MetaTile {
  static constexpr int U = ScoreLanes<D, kHalf>::U;
  uint4 mn[U], mx[U];

  // Plimit >= 1.  Pages at or past Plimit read row Plimit - 1 instead (no branch
  // around the loads); reduce() never reports them.
  __device__ __forceinline__ void load(const uint16_t* pmin_u, const uint16_t* pmax_u, int base,
                                       int Plimit, int rstep) {
    constexpr int LPR = ScoreLanes<D, kHalf>::LPR;
    const int lane = lane_id(), cg = lane % LPR, prow = lane / LPR;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int pg = min(base + u * rstep + prow, Plimit - 1);
      mn[u] = load_stream16(pmin_u + (size_t)pg * D + cg * 8);
      mx[u] = load_stream16(pmax_u + (size_t)pg * D + cg * 8);
    }
  }

  // sink(page, score) is called once per page < Pmax by one lane (a lane takes at most
  // one page of the tile); pages >= Pb get -inf.  patch(min_row, max_row, page) may first
  // amend the row chunks this lane holds (a token appended in the same launch).
  template <typename Patch, typename Sink>
  __device__ __forceinline__ void reduce(const ScoreLanes<D, kHalf>& ql, int base, int Pb, int Pmax,
                                         int rstep, Patch patch, Sink sink) {
    constexpr int LPR = ScoreLanes<D, kHalf>::LPR;
    static_assert(U == 4, "group_sum4_f64 folds four rows");
    const int lane = lane_id(), cg = lane % LPR, prow = lane / LPR;
    double part[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      patch(mn[u], mx[u], base + u * rstep + prow);
      part[u] = ql.row_partial(mn[u], mx[u]);
    }
    const double s = group_sum4_f64<LPR>(part, cg);
    // lanes 0, 2, 4, 6 of a page's lanes hold the sums of rows 0, 1, 2, 3
    const int pg = base + (cg >> 1) * rstep + prow;
    if ((cg & 1) == 0 && cg < 8 && pg < Pmax) sink(pg, pg < Pb ? static_cast<float>(s) : -INFINITY);
  }
};

// Scoring one (sequence, KV head) is split in two so that a kernel can put the
// first loads of a unit as early as it likes (before unrelated set-up work):
// scan_issue sends out the query rows and the wave's first metadata tile,
// scan_finish does everything else.  A wave's iterations are it = first_iter,
// first_iter + iter_stride, ..., each covering U groups of PPW consecutive pages
// (PPI pages in all).  With gs == 1 these are the pages [it * PPI, (it + 1) * PPI);
// in general the sequence's groups of PPW pages are dealt out in turn to gs
// parties, and the caller, party goff, gets the groups (it * U + u) * gs + goff:
// its share is then spread as evenly as can be over the whole sequence.
template <int D, bool kHalf = false>
struct ScanRegs {
  typename ScoreLanes<D, kHalf>::QueryRegs q;
  MetaTile<D, kHalf> tile;
};

template <int D, bool kHalf>
__device__ __forceinline__ void scan_issue_query(ScanRegs<D, kHalf>& r, const uint16_t* q_group, int G) {
  ScoreLanes<D, kHalf>::issue_query(r.q, q_group, G);
}
template <int D, bool kHalf>
__device__ __forceinline__ void scan_issue_tile(ScanRegs<D, kHalf>& r, const uint16_t* pmin_u,
                                                const uint16_t* pmax_u, int Pmax, int first_iter,
                                                int gs = 1, int goff = 0) {
  constexpr int PPW = ScoreLanes<D, kHalf>::PPW, PPI = ScoreLanes<D, kHalf>::PPI;
  r.tile.load(pmin_u, pmax_u, first_iter * PPI * gs + goff * PPW, Pmax, PPW * gs);
}

// `after_query` runs once the query is in registers and returns Pb.  Must be
// called by the whole workgroup (the query goes through LDS, q_stage, with
// barriers).
//
// fill_to_pmax: the sink also wants the -inf of the pages from Pb to Pmax (a
// caller that writes scores out for others to read); otherwise the scan stops at
// the sequence's last page.
//
// kBranchless: the next tile is fetched without a branch around the loads even
// when there is none (the clamped loads then cost a cache line or two), so the
// compiler can count outstanding loads and overlap the fetch with the reduction
// of the current tile.  That is what a latency-bound launch wants; a launch with
// thousands of units is bound by bandwidth and overlaps across workgroups, and
// there the plain branch is a little cheaper.  (Putting the branch around the
// fetch AND the reduction it overlaps with, two copies of the reduction, so that
// no load is issued where there is no next tile, measured 0.7 us slower on the
// 16-sequence configuration.)
template <int D, bool kBranchless, bool kHalf, typename AfterQuery, typename Patch, typename Sink>
__device__ __forceinline__ void scan_finish(ScanRegs<D, kHalf>& r, const uint16_t* pmin_u,
                                            const uint16_t* pmax_u, int G, int Pmax, int first_iter,
                                            int iter_stride, unsigned char* q_stage,
                                            AfterQuery after_query, Patch patch, Sink sink,
                                            int gs = 1, int goff = 0, bool fill_to_pmax = true) {
  constexpr int PPW = ScoreLanes<D, kHalf>::PPW, PPI = ScoreLanes<D, kHalf>::PPI;
  const int rstep = PPW * gs;
  TS_MARK(19);
  ScoreLanes<D, kHalf> ql;
  ql.finish_query(r.q, G, q_stage);
  TS_MARK(16);
  const int Pb = after_query();
  const int limit = uniform(fill_to_pmax ? Pmax : Pb);
  // only the first tile is fetched blind; later ones stop at the sequence's
  // last page (pages >= Pb still get their -inf through the sink)
  int base = first_iter * PPI * gs + goff * PPW;   // first page of the tile's first group
  if (kBranchless) {
    // The first tile is reduced whether or not it holds a page below the limit (the sink
    // sees no page at or past the limit).  With a path around the loop the tile's loads
    // would still be in flight where the two paths meet, and the compiler, which cannot
    // count across such a join, would wait there for EVERY outstanding memory operation:
    // the write-through stores of the scores included, a trip to memory and back in front
    // of the barrier that follows (measured, with the arrival count below: 0.3-0.5 us).
    do {
      const int next = base + iter_stride * PPI * gs;
      MetaTile<D, kHalf> cur = r.tile;
      r.tile.load(pmin_u, pmax_u, next, max(Pb, 1), rstep);
      cur.reduce(ql, base, Pb, min(Pmax, limit), rstep, patch, sink);
      base = next;
    } while (base < limit);
  } else {
    while (base < limit) {
      const int next = base + iter_stride * PPI * gs;
      MetaTile<D, kHalf> cur = r.tile;
      if (next < Pb) r.tile.load(pmin_u, pmax_u, next, Pb, rstep);
      cur.reduce(ql, base, Pb, Pmax, rstep, patch, sink);
      base = next;
    }
  }
}

// Both halves back to back.  Loads go out in the order their data is needed:
// the query rows, then whatever `issue_extra` loads, then the first metadata
// tile; only then is anything waited for.
template <int D, bool kHalf, typename IssueExtra, typename AfterQuery, typename Sink>
__device__ __forceinline__ void score_pages_waves(const uint16_t* pmin_u, const uint16_t* pmax_u,
                                                  const uint16_t* q_group, int G, int Pmax,
                                                  int first_iter, int iter_stride,
                                                  unsigned char* q_stage, IssueExtra issue_extra,
                                                  AfterQuery after_query, Sink sink) {
  ScanRegs<D, kHalf> r;
  scan_issue_query<D, kHalf>(r, q_group, G);
  issue_extra();
  scan_issue_tile<D, kHalf>(r, pmin_u, pmax_u, Pmax, first_iter);
  scan_finish<D, true, kHalf>(r, pmin_u, pmax_u, G, Pmax, first_iter, iter_stride, q_stage, after_query,
                       [](uint4&, uint4&, int) {}, sink);
}

}  // namespace ts
