// The kernels that depend on the cache format (attention over the selected
// pages, and Algorithm 1 in one launch) and their host-side launch logic.  Each
// format and head_dim is compiled in a file of its own (fmt_*.hip instantiate
// launch_fused_format / launch_attention_format / append_capacity_format for
// one pair each, so that they build in parallel); tinyserve.hip holds the entry
// points and everything that does not depend on the format.
#pragma once
#include "../../include/tinyserve.h"

#include <hip/hip_runtime.h>

#include <map>
#include <mutex>
#include <tuple>
#include <utility>

#include "ts_attend.h"
#include "ts_device.h"
#include "ts_meta.h"
#include "ts_score.h"
#include "ts_select.h"

namespace ts {


// ---------------------------------------------------------------------------
// Work decomposition shared by host and device
// ---------------------------------------------------------------------------
// A unit is one (sequence, KV head).  A unit is worked on by a cluster of g
// workgroups: each scores 1/g of the unit's pages and attends 1/g of its
// selected pages.  g is chosen so that units * g is about one workgroup (eight
// waves) per compute unit; with thousands of units g = 1 and nothing is exchanged
// between workgroups at all.
constexpr int kCtrlWords = 64;   // control words at the head of the workspace
constexpr int kCtrlTicket = 0;   // next unit (fused kernel, g == 1, more units than workgroups)
constexpr int kCtrlExit = 1;     // workgroups that have finished taking tickets
constexpr int kCtrlError = 2;    // sticky: a bounded wait expired
constexpr int kCtrlEpoch = 16;   // launches of the fused kernel with clusters so far (own 64-byte line)
constexpr int kCtrlArrive = 32;  // workgroups of the current launch that have read the epoch (own line)
constexpr int kSpinLimit = 1 << 20;  // polls (a few hundred ns each) before a wait gives up
constexpr int kTargetWorkgroups = 256;
constexpr int kMaxCluster = 64;
// Per-unit counters are bumped by every member of a cluster at about the same
// time.  Each gets a 256-byte slot of its own while the batch is small: sixteen
// units' counters packed into one 64-byte line made every workgroup of the
// launch hammer the same line (measured: 6 us of waiting with 16 x 16
// workgroups).  Only clusters (g > 1, at most a few hundred units) use the
// counters, so large batches keep them packed.
constexpr int kCounterPadUnits = 512;
constexpr int kCounterPadStride = 64;   // int32 words

struct Plan {
  int units;          // B * Hkv
  int g;              // workgroups per unit (= attention splits = score slices)
  int chunk;          // selected pages per workgroup
  size_t off_unit;    // int32 [2][units * cstride]: [1] = arrival counters of the staged attention ([0] unused)
  int cstride;        // words between the counters of consecutive units
  size_t off_scores;  // {fp32 score, uint32 launch tag} [units][Pmax]
  size_t off_part;    // [units][g][G][d+2]: {fp32, launch tag} words (fused) or fp32 (staged attention)
  size_t total;
  size_t lds_fused;   // dynamic LDS of the fused kernel
};

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct FusedParams {
  AttendParams at;
  const uint16_t* page_min;
  const uint16_t* page_max;
  uint64_t* scores;     // [units][Pmax] exchange buffer (workspace): score | launch tag << 32
  float* scores_out;    // nullable, caller's
  int32_t* sel_out;     // nullable [units][Kmax]
  int32_t* sel_count;   // nullable [B]
  const int32_t* topk_per_seq;
  int32_t* ctrl;        // control words
  // One token per sequence appended by the same launch (k_new == nullptr: none).
  // (the pool, the metadata and the lengths are then written through the
  // pointers above: the caller's buffers are writable, the const is this
  // library's view of them in the calls that only read)
  const uint16_t* k_new;   // [B][Hkv][D]
  const uint16_t* v_new;
  int topk, S, units, g, cstride, B;
  int keep_first, keep_last;   // pages kept whatever their score (0, 0: the paper's selection)
  int spin_limit;              // polls before a cross-workgroup wait gives up
  int xcds;                    // > 1: clusters laid out one per XCD over that many XCDs (see cluster_of)
  int n_arrive;                // workgroups of the launch that work on a unit
  FastDiv div_g, div_xcds, div_hkv;   // divisions by g, xcds and the number of KV heads
};

// Which cluster a workgroup belongs to, and as which member.  The hardware deals
// consecutive workgroup ids out to the XCDs in turn (on a part with eight of them,
// ids congruent modulo 8 share a die; the first id of a launch goes wherever the
// previous launch left off; ts_debug_xcc_ids lets a test look), and each XCD has an
// L2 of its own.
// With xcds > 1 the g members of a cluster are the workgroups
// id = xcd + xcds * (k * g + member): all on one XCD.  Nothing depends on it for
// correctness (everything the members hand each other goes through agent-scope
// accesses whichever die they run on); measured, it is worth 0.5 us on a single
// short sequence and nothing either way on the 16- and 4-sequence batches, whose
// exchanges wait for the slowest member rather than for the hand-off itself.  The
// host asks for it only when the grid is a multiple of xcds * g workgroups;
// clusters beyond the last unit then have nothing to do.  Otherwise the members
// are consecutive ids.
struct ClusterSlot { int cluster, member; };
__device__ __forceinline__ ClusterSlot cluster_of(int wg, const FastDiv& g, const FastDiv& xcds,
                                                  bool by_xcd) {
  ClusterSlot c;
  if (by_xcd) {
    const int slot = fast_div(wg, xcds), xcd = wg - slot * (int)xcds.d;
    c.cluster = fast_div(slot, g);
    c.member = slot - c.cluster * (int)g.d;
    c.cluster = c.cluster * (int)xcds.d + xcd;
  } else {
    c.cluster = fast_div(wg, g);
    c.member = wg - c.cluster * (int)g.d;
  }
  return c;
}

__device__ __forceinline__ int pages_of(int len, int S) { return (len + S - 1) / S; }

// grid (g, units).  The last workgroup of a unit to deposit its partial merges
// them (unit_done counts arrivals and is left at zero again).
template <int D, int S, bool kInt8, bool kHalf>
__global__ __launch_bounds__(kThreads) void sparse_attention_kernel(AttendParams p,
                                                                    const int32_t* sel,
                                                                    const int32_t* sel_count,
                                                                    int32_t* unit_done,
                                                                    int cstride) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_last;
  const int u = blockIdx.y, b = u / p.Hkv, h = u % p.Hkv, split = blockIdx.x;
  // sel == nullptr: the dense baseline, every page of the sequence in order
  const int all = sel ? 0 : min((p.seq_lens[b] + S - 1) / S, p.Kmax);
  const int Kb = uniform(sel ? max(0, min(sel_count[b], p.Kmax)) : all);
  const int c0 = min(split * p.chunk, Kb), count = min(c0 + p.chunk, Kb) - c0;
  const int32_t* sel_row = sel ? sel + (size_t)u * p.Kmax + c0 : nullptr;
  const int32_t* bt_row = p.block_table + (size_t)b * p.Pmax;
  const NewToken none{-1, 0, p.q, p.q};
  attend_split<D, S, true, false, kInt8, kHalf>(
      p, b, h, split, count, p.seq_lens[b], none,
      [&](int i) { return sel_row ? sel_row[i] : c0 + i; },
      [&](int j) { return bt_row[j]; }, reinterpret_cast<float*>(smem));
  if (p.n_split == 1) return;
  stores_complete();
  __syncthreads();
  if (threadIdx.x == 0) s_last = atomic_add_agent(&unit_done[u * cstride], 1) == p.n_split - 1;
  __syncthreads();
  if (!uniform(s_last)) return;
  combine_splits<D>(p, b, h);
  if (threadIdx.x == 0) atomic_store_agent(&unit_done[u * cstride], 0);
}

// ---------------------------------------------------------------------------
// Fused kernel (Algorithm 1 in one launch).
//
// Workgroup w belongs to cluster w / g as member w % g; a cluster takes units
// cluster, cluster + n_clusters, ...  For each unit a member
//   1. scores every g-th group of the unit's pages (metadata loads are issued
//      before anything else; the unit's block-table row is copied to LDS
//      meanwhile),
//   2. g > 1: publishes each score as a word tagged with the launch tag and
//      polls (bounded) the unit's score row until every word carries the tag,
//      counting the scores into the selection's bins as they come in;
//      g == 1: the scores never leave LDS,
//   3. runs the top-K selection itself (every member computes the same list),
//   4. attends its own 1/g of the selected pages,
//   5. g > 1: hands its partial softmax state on as words tagged with the launch
//      tag; the cluster's last member polls for all g partials (data and flag
//      arrive together) and merges them.
// Members only ever wait for members of their own cluster, all of which are
// resident: the host launches at most as many workgroups as fit on the device
// at once.  Every wait is bounded and raises the workspace's error word.
//
// Every thread-0-only block sits between two barriers and every value that
// steers a branch around a barrier is pinned uniform.
// ---------------------------------------------------------------------------
//
// kLoop = false is the build for launches in which every cluster has exactly one
// unit (units * g workgroups all resident: every latency-bound shape).  Without
// the loop around the body the compiler has nothing to hoist: with it, every
// unit-independent value of the whole body (several hundred instructions, most
// of them spilled at once) is computed ahead of the first unit, that is ahead of
// the first load.
//
// kApp = true is the build that first appends one token per sequence
// (ts_append_and_decode); the plain build carries none of its registers.  With
// the INT8 cache the token's bf16 rows are quantised in the launch, by the few
// waves that need the codes (the one that scores the token's page, the one that
// writes the pool, the one that attends the page).
//
// The host launches at most one workgroup (eight waves) per compute unit, that is
// two waves per SIMD: saying so lets the compiler schedule for latency with the
// registers of that occupancy instead of saving registers for waves that never
// come (measured: 0.5 us of 26 on the 16-sequence configuration).
//
// kCluster says whether a unit is shared by several workgroups (p.g > 1): the
// build for one workgroup per unit carries nothing of the exchange, the build
// for clusters nothing of the selection's stand-alone first stages.
template <int D, int S, bool kLoop, bool kApp, bool kInt8, bool kHalf, bool kCluster>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void
query_aware_decode_kernel(FusedParams p) {
  static_assert(!(kLoop && kApp), "the append is folded only into the loop-free build");
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_flag;
  TS_MARK_INIT();
  TS_MARK(22);
  const AttendParams& at = p.at;
  // Everything the unit's first loads are addressed with is asked for here, ahead of the
  // first branch: the compiler fetches a kernel argument in the block that first uses it,
  // and arguments first used behind the tests below came in a second and a third trip to
  // memory, each waited for, before the first load could go out.
  asm volatile("" ::"s"(p.ctrl), "s"(p.page_min), "s"(p.page_max), "s"(p.topk_per_seq), "s"(p.k_new),
               "s"(p.v_new), "s"(p.topk), "s"(p.units), "s"(p.g), "s"(p.xcds), "s"(p.div_hkv.d),
               "s"(p.div_hkv.magic), "s"(p.div_g.d), "s"(p.div_g.magic), "s"(p.div_xcds.d),
               "s"(p.div_xcds.magic), "s"(at.q), "s"(at.block_table), "s"(at.seq_lens), "s"(at.Hq),
               "s"(at.Hkv), "s"(at.G), "s"(at.Pmax), "s"(at.chunk), "s"(at.lse), "s"(at.k_scale),
               "s"(at.v_scale));
  const int g = kCluster ? p.g : 1, G = at.G, Pmax = at.Pmax;
  const ClusterSlot where = kCluster ? cluster_of(blockIdx.x, p.div_g, p.div_xcds, p.xcds > 1)
                                     : ClusterSlot{(int)blockIdx.x, 0};
  const int member = kCluster ? where.member : 0;
  const int n_clusters = kCluster ? fast_div(gridDim.x, p.div_g) : (int)gridDim.x;
  // (a launch laid out by XCD is padded to whole rounds of the XCDs: clusters past
  // the last unit leave before any barrier, see below, and are not counted in)
  const bool padding = kCluster && !kLoop && where.cluster >= p.units;
  const SelectLds sl = carve_select(smem, Pmax);
  const size_t sel_bytes = select_lds_bytes(Pmax);
  const size_t att_bytes = (size_t)kWaves * G * (D + 2) * 4;
  int32_t* bt_lds = reinterpret_cast<int32_t*>(smem + (sel_bytes > att_bytes ? sel_bytes : att_bytes));
  int32_t* my_sel = bt_lds + Pmax;  // [chunk]
  unsigned char* q_stage = reinterpret_cast<unsigned char*>(bt_lds) +
                           ((size_t)Pmax * 4 + (size_t)at.chunk * 4 + 15) / 16 * 16;
  constexpr bool exchange = kCluster;
  // With one workgroup per unit and more units than workgroups (long ragged
  // batches) the units are handed out from a counter as workgroups become
  // free: a unit then takes tens of microseconds, so the counter is not
  // contended, and the spread of sequence lengths no longer decides the finish
  // time.  Nothing ever waits on a ticket holder.
  const bool dynamic = kLoop && !exchange && p.units > (int)gridDim.x;
  int u = padding ? 0 : where.cluster;
  if (dynamic) {
    if (threadIdx.x == 0) s_flag = atomic_add_agent(&p.ctrl[kCtrlTicket], 1);
    __syncthreads();
    u = uniform(s_flag);
    __syncthreads();
  }

  // The first loads of a unit (sequence length, K, query rows, block-table row,
  // first metadata tile) are sent out ahead of everything else: for the first
  // unit right here, before the set-up work that follows, for later units at the
  // end of the unit before.  What they fetch is only looked at inside the loop.
  // Which pages a member scores: the sequence's groups of PPW consecutive pages
  // (one wave-wide load each) are dealt out to the cluster's members in turn.
  // The selection bins the scores over a range it estimates from the member's
  // own share (see the exchange below), so that share has to be a fair sample
  // of the sequence; dealing out whole tiles of PPI pages reads 0.3 us faster on
  // the 16-sequence configuration, but where the scores vary smoothly along the
  // sequence the few pages that matter then lie in tiles most members never see.
  constexpr int kBtRegs = 8;  // block-table entries per thread fetched through registers
  int L_raw, K_raw, epoch_raw, bt_regs[kBtRegs];
  ScanRegs<D, kHalf> scan;
  // Append mode: the new token's key / value rows of this unit, as the 16-byte
  // chunk (channels 8 * (lane % (D/8)) .. + 7) every lane needs for the box update
  // and the pool write (bf16 also for the INT8 cache, which quantises them).
  constexpr bool app = kApp;
  constexpr int LPR = ScoreLanes<D, kHalf>::LPR;
  uint4 kn16 = make_uint4(0, 0, 0, 0), vn16 = make_uint4(0, 0, 0, 0);
  auto issue_unit = [&](int uu) {
    const int b = fast_div(uu, p.div_hkv), h = uu - b * at.Hkv;
    epoch_raw = p.ctrl[kCtrlEpoch];
    L_raw = at.seq_lens[b];
    K_raw = p.topk_per_seq ? p.topk_per_seq[b] : p.topk;
    scan_issue_query<D, kHalf>(scan, at.q + ((size_t)b * at.Hq + (size_t)h * G) * D, G);
    if (app) {  // behind the query (needed first), ahead of the metadata (needed with it)
      const size_t row = ((size_t)b * at.Hkv + h) * D + (lane_id() % LPR) * 8;
      kn16 = *reinterpret_cast<const uint4*>(p.k_new + row);
      vn16 = *reinterpret_cast<const uint4*>(p.v_new + row);
    }
    const int32_t* bt_row = at.block_table + (size_t)b * Pmax;
#pragma unroll
    for (int k = 0; k < kBtRegs; ++k)   // no branch around the loads
      bt_regs[k] = bt_row[min((int)threadIdx.x + k * kThreads, Pmax - 1)];
    scan_issue_tile<D, kHalf>(scan, p.page_min + (size_t)uu * Pmax * D, p.page_max + (size_t)uu * Pmax * D,
                       Pmax, wave_id(), g, member);
  };
  if (kLoop ? u < p.units : true) issue_unit(u);   // the host launches no idle cluster
  // (a padding workgroup leaves only here, behind the loads of unit 0, whose results it
  // drops: with an exit ahead of them the kernel's arguments would be fetched in two
  // dependent trips, the second one behind the test)
  if (padding) return;
  TS_MARK(23);

  // Launch tag of the score exchange.  The epoch word is read by every
  // workgroup before it counts itself in; the launch's first workgroup advances it
  // for the next launch on its way out, once the count says that every workgroup
  // has read it.
  uint32_t tag = 0;
  bool counted = false;
  while (kLoop ? u < p.units : true) {
    TS_MARK(0);
    const int b = fast_div(u, p.div_hkv), h = u - b * at.Hkv;
    const int32_t* bt_row = at.block_table + (size_t)b * Pmax;
    uint64_t* srow = p.scores + (size_t)u * Pmax;
    float* srow_out = p.scores_out ? p.scores_out + (size_t)u * Pmax : nullptr;

    // 1. score my share of the pages; the unit's block-table row is parked in LDS
    KeyLayout kl;
    int L_unit = 0, j_new = -1, slot_new = 0;  // length after the append; the new token's page / slot
    int pb_scan = 0;                         // the unit's page count, known once the scan runs
    int K_unit = 0;                          // the sequence's page budget (read with the length)
    uint32_t tmin = 0xffffffffu, tmax = 0u;  // this thread's share of the key range
    scan_finish<D, !kLoop, kHalf>(
        scan, p.page_min + (size_t)u * Pmax * D, p.page_max + (size_t)u * Pmax * D, G, Pmax,
        wave_id(), kWaves, q_stage,
        [&] {
#pragma unroll
          for (int k = 0; k < kBtRegs; ++k) {
            const int j = threadIdx.x + k * kThreads;
            if (j < Pmax) bt_lds[j] = bt_regs[k];
          }
          for (int j = threadIdx.x + kBtRegs * kThreads; j < Pmax; j += kThreads)
            bt_lds[j] = bt_row[j];
          // (the empty asm pins the first use of the two values to this point:
          // using them earlier would put a memory round trip in front of the scan)
          asm volatile("" : "+v"(L_raw), "+v"(K_raw), "+v"(epoch_raw));
          // the tag is fixed by the first unit: the epoch word may already have
          // been advanced (by the launch's first workgroup, once it is through
          // with its own units) when a later unit's loads go out
          // (0 is never a tag: it marks words nobody has written since
          // ts_workspace_init, so the count skips it when it wraps)
          if (tag == 0u) tag = max((uint32_t)uniform(epoch_raw) + 1u, 1u);
          L_unit = uniform(L_raw);
          K_unit = uniform(K_raw);
          if (app && L_unit / S < Pmax) {  // a sequence with no room left is not extended
            j_new = L_unit / S;
            slot_new = L_unit % S;
            L_unit += 1;
          }
          pb_scan = uniform(min(pages_of(L_unit, S), Pmax));
          kl = KeyLayout::make(pb_scan);
          return pb_scan;
        },
        [&](uint4& mn, uint4& mx, int pg) {
          // the wave that scores the new token's page first widens (or opens)
          // its box, in registers and in memory (the outer test is uniform over
          // the wave: all the others jump over the block instead of executing
          // it with every lane masked off)
          if constexpr (kInt8) {
            // INT8 cache: the box takes the dequantised key rounded outwards; the
            // whole wave works out the row's scale (the LPR lanes of a row each
            // hold one chunk of it), the page's lanes do the rest
            if (kApp && __ballot(pg == j_new) != 0ull) {
              float amax = chunk_amax_bf16(kn16);
#pragma unroll
              for (int m = 1; m < LPR; m <<= 1) amax = fmaxf(amax, shfl_xor_f(amax, m));
              if (pg == j_new) {
                uint4 lo, hi;
                i8_chunk_box(kn16, i8_row_scale(amax), lo, hi);
                mn = slot_new == 0 ? lo : widen_box<false>(mn, lo, true);
                mx = slot_new == 0 ? hi : widen_box<false>(mx, hi, false);
                const size_t row = ((size_t)u * Pmax + pg) * D + (lane_id() % LPR) * 8;
                *reinterpret_cast<uint4*>(const_cast<uint16_t*>(p.page_min) + row) = mn;
                *reinterpret_cast<uint4*>(const_cast<uint16_t*>(p.page_max) + row) = mx;
              }
            }
          } else if (__ballot(pg == j_new) != 0ull && pg == j_new) {
            mn = slot_new == 0 ? kn16 : widen_box<kHalf>(mn, kn16, true);
            mx = slot_new == 0 ? kn16 : widen_box<kHalf>(mx, kn16, false);
            const size_t row = ((size_t)u * Pmax + pg) * D + (lane_id() % LPR) * 8;
            *reinterpret_cast<uint4*>(const_cast<uint16_t*>(p.page_min) + row) = mn;
            *reinterpret_cast<uint4*>(const_cast<uint16_t*>(p.page_max) + row) = mx;
          }
        },
        [&](int pg, float s) {
          if (exchange) store_agent_tagged(srow + pg, s, tag);
          if (pg < pb_scan) {   // (with an exchange: the range of my own share of the scores)
            const uint32_t k = score_key(s);
            if (!exchange) sl.keys[kl.at(pg)] = k;
            tmin = min(tmin, k);
            tmax = max(tmax, k);
          }
          if (srow_out) srow_out[pg] = s;
        },
        g, member, srow_out != nullptr);
    TS_MARK_WAVE(32);
    const int L = uniform(L_unit);
    const int Pb = uniform(min(pages_of(L, S), Pmax));
    const int Kb = uniform(max(0, min(min(K_unit, Pb), at.Kmax)));

    // count this workgroup in (once): it has read the epoch and, in append mode,
    // the sequence length.  The count's value is not asked for: an atomic that
    // returns one would hold this wave, and with it the barrier below, for a trip
    // to memory and back.
    if (!kLoop || exchange) {
      if (!counted && threadIdx.x == 0 && (exchange || app))
        (void)atomic_add_agent(&p.ctrl[kCtrlArrive], 1);
      counted = true;
    }

    // (the attention's query operand, out of the rows the scoring staged in LDS: fetched
    // here, where the waves are about to wait for the other members anyway)
    QOperand<D, kInt8> qop;
    qop.load(reinterpret_cast<const uint16_t*>(q_stage), G);   // the raw rows head the staging area
    // 2. exchange the scores inside the cluster
    TS_MARK(1);
    // The new token lands in its pool slot (one member's first lanes; the
    // block-table row is complete in LDS once the barrier above is passed).
    // Nothing in this launch reads it from there: the attention splices it in
    // from the caller's arrays.  It is done now rather than at the end (stores
    // issued last would hold up the completion of the kernel), by the first
    // lanes of the last wave (the first wave carries the workgroup's atomics).
    auto store_new_token = [&] {
      const int t = (int)threadIdx.x - (kThreads - kWave);
      if constexpr (kInt8) {
        if (j_new >= 0 && member == 0 && wave_id() == kWaves - 1) {   // (uniform) the whole last wave
          float ka = chunk_amax_bf16(kn16), va = chunk_amax_bf16(vn16);
#pragma unroll
          for (int m = 1; m < LPR; m <<= 1) {
            ka = fmaxf(ka, shfl_xor_f(ka, m));
            va = fmaxf(va, shfl_xor_f(va, m));
          }
          const int phys = bt_lds[j_new];
          if (t < LPR && phys >= 0 && phys < at.n_phys) {
            const float ksc = i8_row_scale(ka), vsc = i8_row_scale(va);
            const size_t tile = ((size_t)phys * at.Hkv + h) * (size_t)at.tile_stride;
            uint8_t* k8 = reinterpret_cast<uint8_t*>(const_cast<uint16_t*>(at.k_pool));
            uint8_t* v8 = reinterpret_cast<uint8_t*>(const_cast<uint16_t*>(at.v_pool));
            *reinterpret_cast<uint2*>(k8 + tile + (size_t)slot_new * D + t * 8) = i8_chunk_codes(kn16, ksc);
            const uint2 vc = i8_chunk_codes(vn16, vsc);
#pragma unroll
            for (int i = 0; i < 8; ++i)
              v8[tile + (size_t)(t * 8 + i) * S + slot_new] =
                  (uint8_t)((i < 4 ? vc.x : vc.y) >> (8 * (i & 3)));
            if (t == 0) {
              const size_t so = ((size_t)phys * at.Hkv + h) * (size_t)S + slot_new;
              const_cast<float*>(at.k_scale)[so] = ksc;
              const_cast<float*>(at.v_scale)[so] = vsc;
            }
          }
        }
        return;
      }
      if (j_new >= 0 && member == 0 && t >= 0 && t < LPR) {
        const int phys = bt_lds[j_new];
        if (phys >= 0 && phys < at.n_phys) {
          const size_t tile = ((size_t)phys * at.Hkv + h) * (size_t)at.tile_stride;
          uint16_t* k_pool_w = const_cast<uint16_t*>(at.k_pool);
          uint16_t* v_pool_w = const_cast<uint16_t*>(at.v_pool);
          *reinterpret_cast<uint4*>(k_pool_w + tile + (size_t)slot_new * D + t * 8) = kn16;
          const uint32_t vw[4] = {vn16.x, vn16.y, vn16.z, vn16.w};
#pragma unroll
          for (int i = 0; i < 8; ++i)
            v_pool_w[tile + (size_t)(t * 8 + i) * S + slot_new] =
                (uint16_t)(vw[i >> 1] >> (16 * (i & 1)));
        }
      }
    };

    const ForcedPages forced = ForcedPages::make(p.keep_first, p.keep_last, Pb);
    BinMap bins{0.f, 0.f};
    if (exchange) {
      // The selection's first stage (counting the pages into score bins) is done
      // here, key by key as the scores come in, instead of in a pass of its own
      // after them.  The bins need a score range before the first score of the
      // other members is looked at: the range of this workgroup's own share
      // (every g-th group of pages: a fair sample), widened; any monotone map
      // keeps the selection exact.  Each member bins in its own way and all
      // arrive at the same pages.
      select_begin(sl, tmin, tmax);
      __syncthreads();
      if (kApp) store_new_token();   // (the block-table row is complete behind this barrier)
      {
        uint32_t lo_key, hi_key;
        select_deposited_range(sl, lo_key, hi_key);
        bins = BinMap::widened(lo_key, hi_key);
      }
      // every thread polls its own entries of the row until all carry this
      // launch's tag (all loads of a round in flight together; bounded)
      bool expired = false;
      int spins = 0;
      auto poll = [&](auto np_tag) {
        constexpr int NP = decltype(np_tag)::value;
        for (int j0 = threadIdx.x; j0 < Pb; j0 += kThreads * NP) {
          uint64_t v[NP];
          for (;;) {
            bool all = true;
#pragma unroll
            for (int i = 0; i < NP; ++i) {
              v[i] = load_agent_u64(srow + min(j0 + i * kThreads, Pb - 1));  // no branch around the load
              all = all && (uint32_t)(v[i] >> 32) == tag;
            }
            if (all) break;
            if (++spins > p.spin_limit) { expired = true; break; }
            __builtin_amdgcn_s_sleep(1);
          }
#pragma unroll
          for (int i = 0; i < NP; ++i) {
            const int j = j0 + i * kThreads;
            if (j < Pb) {
              const bool always = j < forced.first || j >= forced.last_begin;
              const uint32_t k = always ? kForcedKey : score_key(__uint_as_float((uint32_t)v[i]));
              sl.keys[kl.at(j)] = k;
              atomicAdd(&sl.hist[bin_slot_index(bins.slot<true>(k))], 1u);
            }
          }
        }
      };
      const int per_thread = uniform((Pb + kThreads - 1) / kThreads);
      if (per_thread <= 1) poll(std::integral_constant<int, 1>{});
      else if (per_thread <= 2) poll(std::integral_constant<int, 2>{});
      else if (per_thread <= 4) poll(std::integral_constant<int, 4>{});
      else poll(std::integral_constant<int, 8>{});
      if (expired) atomic_store_agent(&p.ctrl[kCtrlError], 1);
      TS_MARK(3);
      TS_MARK_WAVE(40);
    } else {
      select_begin(sl, tmin, tmax);
    }
    __syncthreads();
    TS_MARK(4);
    if (kApp && !exchange) store_new_token();

    // 3. select; keep my own chunk of the ascending list
    const int c0 = min(member * at.chunk, Kb), count = min(c0 + at.chunk, Kb) - c0;
    int32_t* sel_row = (p.sel_out && member == 0) ? p.sel_out + (size_t)u * at.Kmax : nullptr;
    if (sel_row)
      for (int i = Kb + threadIdx.x; i < at.Kmax; i += kThreads) sel_row[i] = -1;
    if (p.sel_count && member == 0 && h == 0 && threadIdx.x == 0) p.sel_count[b] = Kb;
    auto keep_page = [&](int rank, int page) {
      if (rank >= c0 && rank < c0 + count) my_sel[rank - c0] = page;
      if (sel_row) sel_row[rank] = page;
    };
    if (exchange) select_topk_lds<true>(sl, kl, Pb, Kb, forced, keep_page, bins);
    else select_topk_lds<false>(sl, kl, Pb, Kb, forced, keep_page);
    __syncthreads();
    TS_MARK(5);
    // 4. attend my chunk (the wave-merge area reuses the select scratch)
    const size_t new_row = ((size_t)b * at.Hkv + h) * D;
    const NewToken nt{j_new, slot_new, app ? p.k_new + new_row : at.q, app ? p.v_new + new_row : at.q};
    // 5. (inside the same call) the cluster's partials are handed on as tagged
    // words; the cluster's last member (its chunk of the list is the one that
    // can be short) keeps its own in registers, polls for the others and writes
    // the output.  Nobody else waits for anything.
    const bool merged = attend_split<D, S, !kLoop, kApp, kInt8, kHalf, true>(
        at, b, h, member, count, L, nt, [&](int i) { return my_sel[i]; },
        [&](int j) { return bt_lds[j]; }, reinterpret_cast<float*>(smem), exchange ? tag : 0u,
        nullptr, p.spin_limit, &qop);
    TS_MARK(6);
    if (!merged) atomic_store_agent(&p.ctrl[kCtrlError], 1);
    if (!kLoop) break;
    if (dynamic) {
      __syncthreads();
      if (threadIdx.x == 0) s_flag = atomic_add_agent(&p.ctrl[kCtrlTicket], 1);
      __syncthreads();
      u = uniform(s_flag);
      __syncthreads();
    } else {
      u += n_clusters;
    }
    if (u >= p.units) break;
    issue_unit(u);
  }
  // The launch's first workgroup, at the end of its own work, closes the books: once
  // the count shows that every workgroup has read the epoch word and, with one unit per
  // workgroup, its sequence length (all of them did so microseconds ago), its first
  // wave re-arms the count, advances the epoch and (append mode) the lengths.
  if ((!kLoop || exchange) && (exchange || app) && blockIdx.x == 0 && wave_id() == 0) {
    if (!wait_at_least(&p.ctrl[kCtrlArrive], p.n_arrive, p.spin_limit))
      atomic_store_agent(&p.ctrl[kCtrlError], 1);
    if (lane_id() == 0) {
      atomic_store_agent(&p.ctrl[kCtrlArrive], 0);
      if (exchange) atomic_store_agent(&p.ctrl[kCtrlEpoch], (int)tag);
    }
    if (app) {
      int32_t* seq_lens_w = const_cast<int32_t*>(at.seq_lens);
      for (int i = lane_id(); i < p.B; i += kWave) {
        const int len = seq_lens_w[i];
        if (len / S < Pmax) seq_lens_w[i] = len + 1;
      }
    }
  }
  if (dynamic) {  // the last workgroup out re-arms the counters for the next launch
    __syncthreads();
    if (threadIdx.x == 0 && atomic_add_agent(&p.ctrl[kCtrlExit], 1) == (int)gridDim.x - 1) {
      atomic_store_agent(&p.ctrl[kCtrlTicket], 0);
      atomic_store_agent(&p.ctrl[kCtrlExit], 0);
    }
  }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
static int launch_status() { return hipGetLastError() == hipSuccess ? TS_OK : TS_ERR_LAUNCH; }

static int num_compute_units() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    cus = n;
  }
  return cus;
}

// XCDs (dies with an L2 of their own) the device deals workgroups out to: eight
// on the full part (32 compute units each), one in the single-die partition modes.
constexpr int kCusPerXcd = 32;
static int num_xcds() {
  const int cus = num_compute_units();
  return cus >= 2 * kCusPerXcd && cus % kCusPerXcd == 0 ? cus / kCusPerXcd : 1;
}

template <typename KernelT>
static int allow_lds(KernelT kernel, size_t bytes) {
  if (bytes <= 64 * 1024) return TS_OK;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)bytes) == hipSuccess
             ? TS_OK
             : TS_ERR_LAUNCH;
}

// Workgroups of `kernel` that can be resident on the whole device at once.  The
// runtime's answer is remembered per (device, kernel, LDS size): the query costs more
// host time than the launch itself.
template <typename KernelT>
static int resident_capacity(KernelT kernel, size_t lds) {
  static std::mutex mu;
  static std::map<std::tuple<int, const void*, size_t>, int> known;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  const std::tuple<int, const void*, size_t> key(dev, reinterpret_cast<const void*>(kernel), lds);
  std::lock_guard<std::mutex> lock(mu);
  auto it = known.find(key);
  if (it != known.end()) return it->second;
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kThreads, lds) != hipSuccess)
    return 0;
  const int cap = per_cu * num_compute_units();
  if (cap > 0) known[key] = cap;
  return cap;
}

// CALL(DD, S) for the layout's page_size (check_layout has admitted it).
#define TS_DISPATCH_PAGE(DD, S, CALL) \
  switch (S) {                        \
    case 4: CALL(DD, 4); break;       \
    case 8: CALL(DD, 8); break;       \
    case 16: CALL(DD, 16); break;     \
    case 32: CALL(DD, 32); break;     \
    default: CALL(DD, 64); break;     \
  }

// One unit per cluster and everything resident: the loop-free build, which
// also exists with the append folded in.  Otherwise (thousands of
// units, bound by bandwidth) the looping build; an append then runs as a launch
// of its own in front of it: the looping build has no registers to spare for
// it, and against hundreds of microseconds the extra launch does not count.
// max_resident: workgroups the launch may count on being resident together.
// kCluster: pl.g > 1.
template <int D, int S, int kFmt, bool kCluster>
static int launch_fused_shape(const ts_layout* layout, FusedParams& p, const Plan& pl,
                              const void* k_new, const void* v_new, int max_resident,
                              void* stream) {
  hipStream_t s = (hipStream_t)stream;
  constexpr bool kInt8 = kFmt == TS_KV_INT8, kHalf = kFmt == TS_KV_FP16;
  auto loop_kernel = query_aware_decode_kernel<D, S, true, false, kInt8, kHalf, kCluster>;
  auto one_kernel = query_aware_decode_kernel<D, S, false, false, kInt8, kHalf, kCluster>;
  auto app_kernel = query_aware_decode_kernel<D, S, false, true, kInt8, kHalf, kCluster>;
  int st;
  if ((st = allow_lds(loop_kernel, pl.lds_fused)) != TS_OK ||
      (st = allow_lds(one_kernel, pl.lds_fused)) != TS_OK ||
      (st = allow_lds(app_kernel, pl.lds_fused)) != TS_OK)
    return st;
  const bool fold_append = k_new != nullptr;
  int cap1 = resident_capacity(fold_append ? app_kernel : one_kernel, pl.lds_fused);
  if (cap1 > max_resident) cap1 = max_resident;
  const bool one_unit_each = pl.units * pl.g <= cap1;
  if (k_new && !(one_unit_each && fold_append)) {
    if ((st = ts_append_token_meta(layout, k_new, v_new, 1, stream)) != TS_OK) return st;
    p.k_new = p.v_new = nullptr;
  }
  const int xcds = num_xcds();
  p.xcds = 0;
  p.n_arrive = 0;
  if (one_unit_each) {
    unsigned grid = (unsigned)(pl.units * pl.g);
    p.n_arrive = (int)grid;
    // clusters one per XCD: the grid is padded to whole rounds of the XCDs if the
    // padded launch is still resident at once
    const unsigned padded = (unsigned)((pl.units + xcds - 1) / xcds * xcds * pl.g);
    if (kCluster && xcds > 1 && (int)padded <= cap1) {
      grid = padded;
      p.xcds = xcds;
      p.div_xcds = make_fast_div(xcds);
    }
    if (p.k_new)
      app_kernel<<<grid, kThreads, pl.lds_fused, s>>>(p);
    else
      one_kernel<<<grid, kThreads, pl.lds_fused, s>>>(p);
    return TS_OK;
  }
  int cap = resident_capacity(loop_kernel, pl.lds_fused);
  if (cap > max_resident) cap = max_resident;
  int clusters = cap / pl.g;
  if (clusters < 1) return TS_ERR_DEVICE;   // a cluster must be co-resident
  if (clusters > pl.units) clusters = pl.units;
  if (kCluster && xcds > 1 && clusters >= xcds) {
    clusters = clusters / xcds * xcds;
    p.xcds = xcds;
    p.div_xcds = make_fast_div(xcds);
  }
  p.n_arrive = clusters * pl.g;
  loop_kernel<<<(unsigned)(clusters * pl.g), kThreads, pl.lds_fused, s>>>(p);
  return TS_OK;
}

// The fused launch for the layout's page_size in one cache format and head_dim.
template <int kFmt, int kD>
int launch_fused_format(const ts_layout* layout, FusedParams& p, const Plan& pl, const void* k_new,
                        const void* v_new, int max_resident, void* stream) {
  int st = TS_ERR_UNSUPPORTED;
#define TS_LAUNCH_FUSED(DD, SS)                                                                     \
  st = pl.g > 1 ? launch_fused_shape<DD, SS, kFmt, true>(layout, p, pl, k_new, v_new, max_resident, \
                                                         stream)                                    \
                : launch_fused_shape<DD, SS, kFmt, false>(layout, p, pl, k_new, v_new,              \
                                                          max_resident, stream)
  TS_DISPATCH_PAGE(kD, layout->page_size, TS_LAUNCH_FUSED)
#undef TS_LAUNCH_FUSED
  return st;
}

// The staged attention kernel (grid (g, units)); sel == nullptr: every page.
template <int kFmt, int kD>
int launch_attention_format(const ts_layout* layout, const AttendParams& a, const Plan& pl,
                            const int32_t* sel, const int32_t* sel_count, int32_t* unit_done,
                            void* stream) {
  constexpr bool kInt8 = kFmt == TS_KV_INT8, kHalf = kFmt == TS_KV_FP16;
  const size_t lds = (size_t)kWaves * a.G * (layout->head_dim + 2) * 4;
  dim3 grid(pl.g, pl.units);
  hipStream_t s = (hipStream_t)stream;
#define TS_LAUNCH_ATTENTION(DD, SS)              \
  sparse_attention_kernel<DD, SS, kInt8, kHalf> \
      <<<grid, kThreads, lds, s>>>(a, sel, sel_count, unit_done, pl.cstride)
  TS_DISPATCH_PAGE(kD, layout->page_size, TS_LAUNCH_ATTENTION)
#undef TS_LAUNCH_ATTENTION
  return launch_status();
}

// Workgroups of the loop-free build with the append folded in that can be
// resident at once.
template <int kFmt, int kD>
int append_capacity_format(const ts_layout* layout, const Plan& pl) {
  constexpr bool kInt8 = kFmt == TS_KV_INT8, kHalf = kFmt == TS_KV_FP16;
  int cap = 0;
#define TS_CAPACITY(DD, SS)                                                                        \
  cap = pl.g > 1 ? resident_capacity(query_aware_decode_kernel<DD, SS, false, true, kInt8, kHalf, true>, \
                                     pl.lds_fused)                                                 \
                 : resident_capacity(query_aware_decode_kernel<DD, SS, false, true, kInt8, kHalf, false>, \
                                     pl.lds_fused)
  TS_DISPATCH_PAGE(kD, layout->page_size, TS_CAPACITY)
#undef TS_CAPACITY
  return cap;
}

#ifdef TS_PROFILE
// The timestamp buffer of the translation unit that holds this format's kernels.
template <int kFmt, int kD>
int set_profile_buffer_format(void* buf) {
  return hipMemcpyToSymbol(HIP_SYMBOL(g_profile_buf), &buf, sizeof(buf)) == hipSuccess ? TS_OK
                                                                                        : TS_ERR_LAUNCH;
}
#define TS_FORMAT_PROFILE(LINKAGE, FMT, DD) LINKAGE template int set_profile_buffer_format<FMT, DD>(void*);
#else
#define TS_FORMAT_PROFILE(LINKAGE, FMT, DD)
#endif

// Instantiated once per format and head_dim, each in its own file.
#define TS_FORMAT_FUNCTIONS(LINKAGE, FMT, DD)                                                      \
  TS_FORMAT_PROFILE(LINKAGE, FMT, DD)                                                              \
  LINKAGE template int launch_fused_format<FMT, DD>(const ts_layout*, FusedParams&, const Plan&,   \
                                                    const void*, const void*, int, void*);         \
  LINKAGE template int launch_attention_format<FMT, DD>(const ts_layout*, const AttendParams&,     \
                                                        const Plan&, const int32_t*,               \
                                                        const int32_t*, int32_t*, void*);          \
  LINKAGE template int append_capacity_format<FMT, DD>(const ts_layout*, const Plan&);

// CALL(FMT, DD) for the layout's cache format and head_dim (check_layout has admitted them).
#define TS_DISPATCH_FORMAT(layout, CALL)                            \
  do {                                                              \
    const bool d64 = (layout)->head_dim == 64;                      \
    switch ((layout)->kv_format) {                                  \
      case TS_KV_INT8:                                              \
        if (d64) { CALL(TS_KV_INT8, 64); } else { CALL(TS_KV_INT8, 128); } \
        break;                                                      \
      case TS_KV_FP16:                                              \
        if (d64) { CALL(TS_KV_FP16, 64); } else { CALL(TS_KV_FP16, 128); } \
        break;                                                      \
      default:                                                      \
        if (d64) { CALL(TS_KV_BF16, 64); } else { CALL(TS_KV_BF16, 128); } \
    }                                                               \
  } while (0)

}  // namespace ts
