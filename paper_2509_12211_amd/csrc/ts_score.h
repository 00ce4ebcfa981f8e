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
template <int D>
struct ScoreLanes {
  static constexpr int LPR = D / 8;         // lanes per metadata row
  static constexpr int PPW = kWave / LPR;   // pages per wave-wide load
  static constexpr int U = 4;               // wave-wide loads of min (and of max) in flight
  static constexpr int PPI = PPW * U;       // pages one wave covers per iteration
  double qp[8], qn[8];

  __device__ __forceinline__ void load_query(const uint16_t* q_group, int G) {
    const int cg = lane_id() % LPR;
#pragma unroll
    for (int i = 0; i < 8; ++i) { qp[i] = 0.0; qn[i] = 0.0; }
    for (int g = 0; g < G; ++g) {
      const uint4 w = *reinterpret_cast<const uint4*>(q_group + (size_t)g * D + cg * 8);
      float f[8];
      unpack8(w, f);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        qp[i] += static_cast<double>(fmaxf(f[i], 0.f));
        qn[i] += static_cast<double>(fminf(f[i], 0.f));
      }
    }
  }

  __device__ __forceinline__ double row_partial(const uint4& mn, const uint4& mx) const {
    float lo[8], hi[8];
    unpack8(mn, lo);
    unpack8(mx, hi);
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
      s = fma(qp[i], static_cast<double>(hi[i]), fma(qn[i], static_cast<double>(lo[i]), s));
    return s;
  }
};

// The metadata rows one wave has in flight: U wave-wide loads of min and of max
// covering pages [base, base + PPI).  Rows up to Pmax are always readable
// (whatever they hold), so the loads do not wait for the sequence length.
template <int D>
struct MetaTile {
  static constexpr int U = ScoreLanes<D>::U;
  uint4 mn[U], mx[U];

  __device__ __forceinline__ void load(const uint16_t* pmin_u, const uint16_t* pmax_u, int base,
                                       int Pmax) {
    constexpr int LPR = ScoreLanes<D>::LPR, PPW = ScoreLanes<D>::PPW;
    const int lane = lane_id(), cg = lane % LPR, prow = lane / LPR;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int pg = base + u * PPW + prow;
      if (pg < Pmax) {
        mn[u] = *reinterpret_cast<const uint4*>(pmin_u + (size_t)pg * D + cg * 8);
        mx[u] = *reinterpret_cast<const uint4*>(pmax_u + (size_t)pg * D + cg * 8);
      } else {
        mn[u] = make_uint4(0, 0, 0, 0);
        mx[u] = make_uint4(0, 0, 0, 0);
      }
    }
  }

  // sink(page, score) is called once per page < Pmax by one lane; pages >= Pb
  // get -inf.
  template <typename Sink>
  __device__ __forceinline__ void reduce(const ScoreLanes<D>& ql, int base, int Pb, int Pmax,
                                         Sink sink) const {
    constexpr int LPR = ScoreLanes<D>::LPR, PPW = ScoreLanes<D>::PPW;
    const int lane = lane_id(), cg = lane % LPR, prow = lane / LPR;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int pg = base + u * PPW + prow;
      double s = ql.row_partial(mn[u], mx[u]);
#pragma unroll
      for (int m = 1; m < LPR; m <<= 1) s += __shfl_xor(s, m, kWave);
      if (cg == 0 && pg < Pmax) sink(pg, pg < Pb ? static_cast<float>(s) : -INFINITY);
    }
  }
};

// Scores the pages of one (sequence, KV head) that fall to this wave: wave
// iterations it = first_iter, first_iter + iter_stride, ... each cover
// ScoreLanes<D>::PPI consecutive pages.  The first metadata loads are issued
// before the query is read.  Pb is passed as a callable so its (scalar) load
// need not be waited for before the metadata loads go out.
template <int D, typename PbFn, typename Sink>
__device__ __forceinline__ void score_pages_waves(const uint16_t* pmin_u, const uint16_t* pmax_u,
                                                  const uint16_t* q_group, int G, int Pmax,
                                                  int first_iter, int iter_stride, PbFn pb_fn,
                                                  Sink sink) {
  constexpr int PPI = ScoreLanes<D>::PPI;
  MetaTile<D> tile;
  int base = first_iter * PPI;
  if (base < Pmax) tile.load(pmin_u, pmax_u, base, Pmax);
  ScoreLanes<D> ql;
  ql.load_query(q_group, G);
  const int Pb = pb_fn();
  while (base < Pmax) {
    const int next = base + iter_stride * PPI;
    MetaTile<D> cur = tile;
    if (next < Pmax) tile.load(pmin_u, pmax_u, next, Pmax);
    cur.reduce(ql, base, Pb, Pmax, sink);
    base = next;
  }
}

}  // namespace ts
