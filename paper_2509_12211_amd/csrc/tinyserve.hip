// C-ABI entry points (include/tinyserve.h) and the kernels behind them.
// gfx950 only.  Device code is in ts_*.h; this file holds the __global__
// wrappers, the work decomposition, and the host-side validation / launches.
#include "ts_fused.h"

#include <atomic>
#include <mutex>

namespace ts {

// every cache format and head_dim is compiled in a file of its own (fmt_<format>_d<head_dim>.hip)
TS_FORMAT_FUNCTIONS(extern, TS_KV_BF16, 64)
TS_FORMAT_FUNCTIONS(extern, TS_KV_BF16, 128)
TS_FORMAT_FUNCTIONS(extern, TS_KV_FP16, 64)
TS_FORMAT_FUNCTIONS(extern, TS_KV_FP16, 128)
TS_FORMAT_FUNCTIONS(extern, TS_KV_INT8, 64)
TS_FORMAT_FUNCTIONS(extern, TS_KV_INT8, 128)

// Launch-shape overrides for tuning sweeps (ts_set_tuning): process-wide, read once
// per call; a layout's own cluster_size takes precedence.
static std::atomic<int> g_tune_splits{0}, g_tune_wg_per_cu{0};

// target_workgroups: about how many workgroups a launch should have.  The
// query-aware path is latency-bound and wants one per compute unit; the dense
// baseline streams the whole cache and wants several.
constexpr int kDenseTargetWorkgroups = 1024;

static Plan make_plan(const ts_layout* L, int max_topk, int target_workgroups = kTargetWorkgroups) {
  Plan pl;
  const int G = L->num_q_heads / L->num_kv_heads;
  const int Pmax = L->max_pages_per_seq;
  pl.units = L->num_seqs * L->num_kv_heads;
  // The query-aware path: as many workgroups per unit as keep the WHOLE launch
  // resident (the members of a cluster wait for each other, and clusters that do
  // not fit take the units in turns: 160 units in clusters of two take 53 us, one
  // workgroup each 33 us).  The dense baseline's workgroups wait for nobody, so
  // it rounds up.
  int g = target_workgroups == kTargetWorkgroups
              ? target_workgroups / pl.units
              : (target_workgroups + pl.units - 1) / pl.units;
  if (g < 1) g = 1;
  const int cap = (max_topk + 3) / 4;  // at least one page per wave
  if (g > cap) g = cap;
  if (g > kMaxCluster) g = kMaxCluster;
  // (Even the shortest configurations measured, 256 pages with 32 kept, are
  // faster spread over a cluster than on one workgroup: 12.5 against 14.0 us.)
  if (target_workgroups == kTargetWorkgroups) {
    const int tuned = g_tune_splits.load(std::memory_order_relaxed);
    const int forced = L->cluster_size > 0 ? L->cluster_size : tuned;
    if (forced > 0) g = forced < kMaxCluster ? forced : kMaxCluster;
  }
  if (g > max_topk) g = max_topk;
  if (g < 1) g = 1;
  pl.chunk = (max_topk + g - 1) / g;
  // pages smaller than an MFMA tile are attended four / two at a time: whole
  // groups per workgroup
  if (L->page_size < 16) pl.chunk = (pl.chunk + 3) / 4 * 4;
  pl.g = (max_topk + pl.chunk - 1) / pl.chunk;
  size_t off = kCtrlWords * sizeof(int32_t);
  pl.off_unit = off;
  pl.cstride = pl.units <= kCounterPadUnits ? kCounterPadStride : 1;
  off = align_up(off + 2 * (size_t)pl.units * pl.cstride * sizeof(int32_t), 256);
  // (one workgroup per unit exchanges nothing: its scores never leave LDS and its
  // result goes straight to the output)
  pl.off_scores = off;
  if (pl.g > 1) off = align_up(off + (size_t)pl.units * Pmax * sizeof(uint64_t), 256);
  pl.off_part = off;
  if (pl.g > 1)
    off = align_up(off + (size_t)pl.units * pl.g * G * (L->head_dim + 2) * sizeof(uint64_t), 256);
  pl.total = off;
  // fused kernel LDS: select scratch (keys, bins), the unit's block-table row,
  // this workgroup's selected pages; the wave-merge area aliases the keys
  const size_t lds_sel = select_lds_bytes(Pmax);
  const size_t lds_att = (size_t)kWaves * G * (L->head_dim + 2) * 4;
  // ... and, in an area of its own, the query staging: a wave that is done
  // scoring starts the selection (which clears the bins) while another may not
  // have picked up its query sums yet, so the two must not share memory
  const size_t lds_query = (size_t)G * L->head_dim * 2 + 2 * (size_t)L->head_dim * 8;
  pl.lds_fused = (lds_sel > lds_att ? lds_sel : lds_att) +
                 align_up((size_t)Pmax * 4 + (size_t)pl.chunk * 4, 16) + lds_query;
  return pl;
}

// ---------------------------------------------------------------------------
// Staged kernels
// ---------------------------------------------------------------------------
// grid (gx, units): workgroup x scores every gx-th group of pages of its unit.
template <int D, bool kHalf>
__global__ __launch_bounds__(kThreads) void score_pages_kernel(const uint16_t* q,
                                                               const uint16_t* page_min,
                                                               const uint16_t* page_max,
                                                               const int32_t* seq_lens, float* scores,
                                                               int Hq, int Hkv, int S, int Pmax) {
  __shared__ __align__(16) unsigned char q_stage[ScoreLanes<D, kHalf>::query_stage_bytes(16)];
  const int u = blockIdx.y, b = u / Hkv, h = u % Hkv, G = Hq / Hkv;
  float* srow = scores + (size_t)u * Pmax;
  score_pages_waves<D, kHalf>(
      page_min + (size_t)u * Pmax * D, page_max + (size_t)u * Pmax * D,
      q + ((size_t)b * Hq + (size_t)h * G) * D, G, Pmax, blockIdx.x * kWaves + wave_id(),
      gridDim.x * kWaves, q_stage, [] {}, [&] { return min(pages_of(seq_lens[b], S), Pmax); },
      [&](int pg, float s) { srow[pg] = s; });
}

__global__ __launch_bounds__(kThreads) void select_topk_kernel(const float* scores,
                                                               const int32_t* seq_lens, int topk,
                                                               const int32_t* topk_per_seq,
                                                               int32_t* sel, int32_t* sel_count,
                                                               int Hkv, int S, int Pmax, int Kmax,
                                                               int keep_first, int keep_last) {
  extern __shared__ __align__(16) unsigned char smem[];
  TS_MARK_INIT();
  TS_MARK(0);
  const int u = blockIdx.x, b = u / Hkv, h = u % Hkv;
  const int Pb = uniform(min(pages_of(seq_lens[b], S), Pmax));
  const int K = topk_per_seq ? topk_per_seq[b] : topk;
  const int Kb = uniform(max(0, min(min(K, Pb), Kmax)));
  if (h == 0 && threadIdx.x == 0) sel_count[b] = Kb;
  const SelectLds L = carve_select(smem, Pmax);
  const float* srow = scores + (size_t)u * Pmax;
  int32_t* row = sel + (size_t)u * Kmax;
  for (int i = Kb + threadIdx.x; i < Kmax; i += kThreads) row[i] = -1;
  // eight loads per thread in flight per round (a plain loop would pay one
  // memory round trip per iteration); the key range is gathered on the way
  const KeyLayout kl = KeyLayout::make(Pb);
  const ForcedPages fp = ForcedPages::make(keep_first, keep_last, Pb);
  uint32_t tmin = 0xffffffffu, tmax = 0u;
  for (int j0 = threadIdx.x; j0 < Pb; j0 += kThreads * 8) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = srow[min(j0 + i * kThreads, Pb - 1)];  // no branch around the load
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int j = j0 + i * kThreads;
      if (j < Pb) {
        const uint32_t k = score_key(v[i]);
        L.keys[kl.at(j)] = k;
        tmin = min(tmin, k);
        tmax = max(tmax, k);
      }
    }
  }
  select_begin(L, tmin, tmax);
  __syncthreads();
  TS_MARK(1);
  select_topk_lds(L, kl, Pb, Kb, fp, [&](int rank, int page) { row[rank] = page; });
  TS_MARK(5);
}

// Which XCD each workgroup of a launch runs on (the XCC_ID hardware register).
__global__ __launch_bounds__(kThreads) void xcc_ids_kernel(int32_t* out) {
  uint32_t id;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID, 0, 4)" : "=s"(id));
  if (threadIdx.x == 0) out[blockIdx.x] = (int32_t)id;
}

__global__ void fill_zero_kernel(int32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x)
    p[i] = 0;
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
static int check_layout(const ts_layout* L) {
  if (!L) return TS_ERR_NULL;
  if (L->num_seqs <= 0 || L->num_q_heads <= 0 || L->num_kv_heads <= 0 || L->head_dim <= 0 ||
      L->page_size <= 0 || L->max_pages_per_seq <= 0 || L->num_phys_pages <= 0)
    return TS_ERR_SHAPE;
  if (L->num_q_heads % L->num_kv_heads != 0) return TS_ERR_SHAPE;
  if (L->kv_tile_stride != 0 &&
      (L->kv_tile_stride < L->head_dim * L->page_size || L->kv_tile_stride % 8 != 0))
    return TS_ERR_SHAPE;
  if (L->head_dim != 64 && L->head_dim != 128) return TS_ERR_UNSUPPORTED;
  if (L->page_size != 4 && L->page_size != 8 && L->page_size != 16 && L->page_size != 32 &&
      L->page_size != 64)
    return TS_ERR_UNSUPPORTED;
  if (L->num_q_heads / L->num_kv_heads > 16) return TS_ERR_UNSUPPORTED;
  if (L->max_pages_per_seq > TS_MAX_PAGES_PER_SEQ) return TS_ERR_UNSUPPORTED;
  if ((long long)L->num_seqs * L->num_kv_heads > 65535) return TS_ERR_UNSUPPORTED;
  if (L->keep_first_pages < 0 || L->keep_last_pages < 0) return TS_ERR_SHAPE;
  if (L->cluster_size < 0 || L->wait_limit < 0) return TS_ERR_SHAPE;
  if (L->out_format != TS_OUT_F32 && L->out_format != TS_OUT_BF16) return TS_ERR_UNSUPPORTED;
  if (L->kv_format != TS_KV_BF16 && L->kv_format != TS_KV_INT8 && L->kv_format != TS_KV_FP16)
    return TS_ERR_UNSUPPORTED;
  if (L->kv_format == TS_KV_INT8 && L->kv_tile_stride % 16 != 0) return TS_ERR_SHAPE;
  return TS_OK;
}

// The pool pointers every call that attends (or appends into the pool) needs:
// K and V tiles, the block table, the lengths and, for the INT8 cache, the two
// per-token scale arrays the kernels dereference.
static int check_pool(const ts_layout* L) {
  if (!L->k_pool || !L->v_pool || !L->block_table || !L->seq_lens) return TS_ERR_NULL;
  if (L->kv_format == TS_KV_INT8 && (!L->k_scale || !L->v_scale)) return TS_ERR_NULL;
  return TS_OK;
}

static int tile_stride_of(const ts_layout* L) {
  return L->kv_tile_stride ? L->kv_tile_stride : L->head_dim * L->page_size;
}

static MetaParams meta_params(const ts_layout* L) {
  MetaParams p;
  p.k_pool = static_cast<const uint16_t*>(L->k_pool);
  p.k_pool_w = static_cast<uint16_t*>(L->k_pool);
  p.v_pool_w = static_cast<uint16_t*>(L->v_pool);
  p.block_table = L->block_table;
  p.seq_lens = L->seq_lens;
  p.page_min = static_cast<uint16_t*>(L->page_min);
  p.page_max = static_cast<uint16_t*>(L->page_max);
  p.B = L->num_seqs;
  p.Hkv = L->num_kv_heads;
  p.S = L->page_size;
  p.Pmax = L->max_pages_per_seq;
  p.n_phys = L->num_phys_pages;
  p.tile_stride = tile_stride_of(L);
  p.k_scale = L->k_scale;
  p.v_scale = L->v_scale;
  return p;
}

static AttendParams attend_params(const ts_layout* L, const Plan& pl, const void* q, void* out,
                                  unsigned char* ws, int max_topk, float softmax_scale) {
  AttendParams a;
  a.q = static_cast<const uint16_t*>(q);
  a.k_pool = static_cast<const uint16_t*>(L->k_pool);
  a.v_pool = static_cast<const uint16_t*>(L->v_pool);
  a.k_scale = L->k_scale;
  a.v_scale = L->v_scale;
  a.block_table = L->block_table;
  a.seq_lens = L->seq_lens;
  a.out = static_cast<float*>(out);
  a.lse = nullptr;
  a.partials = reinterpret_cast<float*>(ws + pl.off_part);
  a.Hq = L->num_q_heads;
  a.Hkv = L->num_kv_heads;
  a.G = L->num_q_heads / L->num_kv_heads;
  a.Pmax = L->max_pages_per_seq;
  a.Kmax = max_topk;
  a.n_phys = L->num_phys_pages;
  a.tile_stride = tile_stride_of(L);
  a.n_split = pl.g;
  a.chunk = pl.chunk;
  a.scale_log2 = softmax_scale * 1.4426950408889634f;
  a.out_bf16 = L->out_format == TS_OUT_BF16 ? 1 : 0;
  return a;
}

}  // namespace ts

using namespace ts;

static int launch_fused(const ts_layout* layout, const void* k_new, const void* v_new,
                        const void* q, int32_t topk, const int32_t* topk_per_seq,
                        int32_t max_topk, float softmax_scale, void* out, float* scores_out,
                        int32_t* sel_out, int32_t* sel_count_out, void* workspace,
                        size_t workspace_bytes, void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!q || !out || !workspace || !layout->page_min || !layout->page_max) return TS_ERR_NULL;
  if ((st = check_pool(layout)) != TS_OK) return st;
  if (max_topk < 1 || (!topk_per_seq && (topk < 1 || max_topk < topk))) return TS_ERR_SHAPE;
  Plan pl = make_plan(layout, max_topk);
  if (workspace_bytes < pl.total) return TS_ERR_WORKSPACE;
  const int cus = num_compute_units();
  if (cus <= 0) return TS_ERR_DEVICE;
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  FusedParams p;
  p.at = attend_params(layout, pl, q, out, ws, max_topk, softmax_scale);
  p.page_min = static_cast<const uint16_t*>(layout->page_min);
  p.page_max = static_cast<const uint16_t*>(layout->page_max);
  p.scores = reinterpret_cast<uint64_t*>(ws + pl.off_scores);
  p.scores_out = scores_out;
  p.sel_out = sel_out;
  p.sel_count = sel_count_out;
  p.topk_per_seq = topk_per_seq;
  p.ctrl = reinterpret_cast<int32_t*>(ws);
  p.cstride = pl.cstride;
  p.k_new = static_cast<const uint16_t*>(k_new);
  p.v_new = static_cast<const uint16_t*>(v_new);
  p.B = layout->num_seqs;
  p.topk = topk;
  p.keep_first = layout->keep_first_pages;
  p.keep_last = layout->keep_last_pages;
  p.S = layout->page_size;
  p.units = pl.units;
  p.g = pl.g;
  p.div_g = make_fast_div(pl.g);
  p.div_hkv = make_fast_div(layout->num_kv_heads);
  p.div_xcds = make_fast_div(1);
  p.spin_limit = layout->wait_limit > 0 ? layout->wait_limit : kSpinLimit;
  const int tuned_per_cu = g_tune_wg_per_cu.load(std::memory_order_relaxed);
  const int per_cu = tuned_per_cu > 0 ? tuned_per_cu : 1;
#define TS_CALL(FMT, DD) \
  st = launch_fused_format<FMT, DD>(layout, p, pl, k_new, v_new, cus * per_cu, stream)
  TS_DISPATCH_FORMAT(layout, TS_CALL);
#undef TS_CALL
  if (st != TS_OK) return st;
  return launch_status();
}


extern "C" {

int ts_version(void) { return 4; }

#ifdef TS_PROFILE
// buf: device, uint64 [workgroups of the largest launch][64] (NULL: stop recording).
int ts_debug_set_profile_buffer(void* buf) {
  int st = hipMemcpyToSymbol(HIP_SYMBOL(g_profile_buf), &buf, sizeof(buf)) == hipSuccess
               ? TS_OK
               : TS_ERR_LAUNCH;
#define TS_SET(FMT, DD) \
  if (st == TS_OK) st = set_profile_buffer_format<FMT, DD>(buf)
  TS_SET(TS_KV_BF16, 64); TS_SET(TS_KV_BF16, 128); TS_SET(TS_KV_FP16, 64);
  TS_SET(TS_KV_FP16, 128); TS_SET(TS_KV_INT8, 64); TS_SET(TS_KV_INT8, 128);
#undef TS_SET
  return st;
}
#endif

const char* ts_strerror(int status) {
  switch (status) {
    case TS_OK: return "ok";
    case TS_ERR_NULL: return "required pointer is NULL";
    case TS_ERR_SHAPE: return "invalid shape or count";
    case TS_ERR_UNSUPPORTED: return "head_dim / page_size / group size / page count not supported";
    case TS_ERR_WORKSPACE: return "workspace too small";
    case TS_ERR_LAUNCH: return "HIP launch failed";
    case TS_ERR_DEVICE: return "no usable HIP device";
    default: return "unknown status";
  }
}

int ts_set_tuning(int32_t reserved, int32_t num_splits, int32_t workgroups_per_cu) {
  if (reserved != 0 || num_splits < 0 || workgroups_per_cu < 0) return TS_ERR_SHAPE;
  g_tune_splits.store(num_splits, std::memory_order_relaxed);
  g_tune_wg_per_cu.store(workgroups_per_cu, std::memory_order_relaxed);
  return TS_OK;
}

size_t ts_workspace_bytes(const ts_layout* layout, int32_t max_topk) {
  if (check_layout(layout) != TS_OK || max_topk < 1) return 0;
  return make_plan(layout, max_topk).total;
}

int ts_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace) return TS_ERR_NULL;
  if (workspace_bytes < kCtrlWords * sizeof(int32_t)) return TS_ERR_WORKSPACE;
  // Everything is zeroed: the control words and counters must start at zero,
  // and no word of the exchange areas may carry a launch tag from an earlier
  // life of the memory (tags start at 1 and only grow).
  const size_t n = workspace_bytes / sizeof(int32_t);
  const unsigned blocks = (unsigned)((n + 256 * 64 - 1) / (256 * 64));
  fill_zero_kernel<<<dim3(blocks), dim3(256), 0, (hipStream_t)stream>>>(
      static_cast<int32_t*>(workspace), n);
  return launch_status();
}

int ts_debug_xcc_ids(int32_t* ids, int32_t num_workgroups, void* stream) {
  if (!ids) return TS_ERR_NULL;
  if (num_workgroups < 1 || num_workgroups > 65535) return TS_ERR_SHAPE;
  xcc_ids_kernel<<<(unsigned)num_workgroups, kThreads, 0, (hipStream_t)stream>>>(ids);
  return launch_status();
}

int ts_workspace_status(const void* workspace, int32_t* status_host) {
  if (!workspace || !status_host) return TS_ERR_NULL;
  if (hipMemcpy(status_host, static_cast<const int32_t*>(workspace) + kCtrlError, sizeof(int32_t),
                hipMemcpyDeviceToHost) != hipSuccess)
    return TS_ERR_LAUNCH;
  return TS_OK;
}

int ts_build_page_meta(const ts_layout* layout, void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!layout->k_pool || !layout->block_table || !layout->seq_lens || !layout->page_min ||
      !layout->page_max)
    return TS_ERR_NULL;
  MetaParams p = meta_params(layout);
  if (p.B > 65535) return TS_ERR_UNSUPPORTED;
  if (layout->kv_format == TS_KV_INT8) {
    if (!layout->k_scale) return TS_ERR_NULL;
    const int ppb = kThreads / layout->head_dim;   // pages per workgroup
    dim3 grid8((p.Pmax + ppb - 1) / ppb, p.Hkv, p.B);
    if (layout->head_dim == 64)
      build_page_meta_i8_kernel<64><<<grid8, kThreads, 0, (hipStream_t)stream>>>(p);
    else
      build_page_meta_i8_kernel<128><<<grid8, kThreads, 0, (hipStream_t)stream>>>(p);
    return launch_status();
  }
  const int pages_per_wg = kWaves * (kWave / (layout->head_dim / 8));
  // (the KV head is the fastest grid index: a physical page's tiles of all heads are
  // contiguous in the pool, and workgroups dispatched together then read neighbouring
  // memory: -3 % on the 16-head batch)
  if ((p.Pmax + pages_per_wg - 1) / pages_per_wg > 65535) return TS_ERR_UNSUPPORTED;
  dim3 grid(p.Hkv, (p.Pmax + pages_per_wg - 1) / pages_per_wg, p.B);
  const bool half = layout->kv_format == TS_KV_FP16;
  hipStream_t s = (hipStream_t)stream;
#define TS_LAUNCH_BUILD(DD, HH)                                                                 \
  do {                                                                                          \
    if (p.S == 4) build_page_meta_kernel<DD, HH, 4><<<grid, kThreads, 0, s>>>(p);               \
    else if (p.S == 8) build_page_meta_kernel<DD, HH, 8><<<grid, kThreads, 0, s>>>(p);          \
    else build_page_meta_kernel<DD, HH, 16><<<grid, kThreads, 0, s>>>(p);                       \
  } while (0)
  if (layout->head_dim == 64 && !half) TS_LAUNCH_BUILD(64, false);
  else if (layout->head_dim == 64) TS_LAUNCH_BUILD(64, true);
  else if (!half) TS_LAUNCH_BUILD(128, false);
  else TS_LAUNCH_BUILD(128, true);
#undef TS_LAUNCH_BUILD
  return launch_status();
}

int ts_append_token_meta(const ts_layout* layout, const void* k_new, const void* v_new,
                         int advance_seq_lens, void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!k_new || !layout->seq_lens || !layout->page_min || !layout->page_max) return TS_ERR_NULL;
  if (v_new && (!layout->k_pool || !layout->v_pool || !layout->block_table)) return TS_ERR_NULL;
  MetaParams p = meta_params(layout);
  if (layout->kv_format == TS_KV_INT8) {
    if (v_new && (!layout->k_scale || !layout->v_scale)) return TS_ERR_NULL;
    append_token_i8_kernel<<<p.B, kThreads, 0, (hipStream_t)stream>>>(
        p, layout->head_dim, static_cast<const uint16_t*>(k_new),
        static_cast<const uint16_t*>(v_new), advance_seq_lens);
    return launch_status();
  }
  if (layout->kv_format == TS_KV_FP16)
    append_token_meta_kernel<true><<<p.B, kThreads, 0, (hipStream_t)stream>>>(
        p, layout->head_dim, static_cast<const uint16_t*>(k_new),
        static_cast<const uint16_t*>(v_new), advance_seq_lens);
  else
    append_token_meta_kernel<false><<<p.B, kThreads, 0, (hipStream_t)stream>>>(
        p, layout->head_dim, static_cast<const uint16_t*>(k_new),
        static_cast<const uint16_t*>(v_new), advance_seq_lens);
  return launch_status();
}

int ts_score_pages(const ts_layout* layout, const void* q, float* scores, void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!q || !scores || !layout->seq_lens || !layout->page_min || !layout->page_max)
    return TS_ERR_NULL;
  const int units = layout->num_seqs * layout->num_kv_heads;
  const int Pmax = layout->max_pages_per_seq;
  const int ppi_wg = (layout->head_dim == 64 ? 32 : 16) * kWaves;  // pages per workgroup pass
  int gx = (2 * kTargetWorkgroups + units - 1) / units;
  const int most = (Pmax + ppi_wg - 1) / ppi_wg;
  if (gx > most) gx = most;
  if (gx < 1) gx = 1;
  dim3 grid(gx, units);
  const uint16_t* pmin = static_cast<const uint16_t*>(layout->page_min);
  const uint16_t* pmax = static_cast<const uint16_t*>(layout->page_max);
  const bool half = layout->kv_format == TS_KV_FP16;
#define TS_LAUNCH_SCORE(DD, HH)                                                                   \
  score_pages_kernel<DD, HH><<<grid, kThreads, 0, (hipStream_t)stream>>>(                          \
      static_cast<const uint16_t*>(q), pmin, pmax, layout->seq_lens, scores, layout->num_q_heads, \
      layout->num_kv_heads, layout->page_size, Pmax)
  if (layout->head_dim == 64 && !half) TS_LAUNCH_SCORE(64, false);
  else if (layout->head_dim == 64) TS_LAUNCH_SCORE(64, true);
  else if (!half) TS_LAUNCH_SCORE(128, false);
  else TS_LAUNCH_SCORE(128, true);
#undef TS_LAUNCH_SCORE
  return launch_status();
}

int ts_select_topk_pages(const ts_layout* layout, const float* scores, int32_t topk,
                         const int32_t* topk_per_seq, int32_t max_topk, int32_t* sel,
                         int32_t* sel_count, void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!scores || !sel || !sel_count || !layout->seq_lens) return TS_ERR_NULL;
  if (max_topk < 1 || (!topk_per_seq && (topk < 1 || max_topk < topk))) return TS_ERR_SHAPE;
  const int units = layout->num_seqs * layout->num_kv_heads;
  const size_t lds = select_lds_bytes(layout->max_pages_per_seq);
  if ((st = allow_lds(select_topk_kernel, lds)) != TS_OK) return st;
  select_topk_kernel<<<units, kThreads, lds, (hipStream_t)stream>>>(
      scores, layout->seq_lens, topk, topk_per_seq, sel, sel_count, layout->num_kv_heads,
      layout->page_size, layout->max_pages_per_seq, max_topk, layout->keep_first_pages,
      layout->keep_last_pages);
  return launch_status();
}

static int launch_attention(const ts_layout* layout, const Plan& pl, const void* q,
                            const int32_t* sel, const int32_t* sel_count, int32_t max_topk,
                            float softmax_scale, void* out, float* lse_out, void* workspace,
                            void* stream) {
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  AttendParams a = attend_params(layout, pl, q, out, ws, max_topk, softmax_scale);
  a.lse = lse_out;
  int32_t* unit_done = reinterpret_cast<int32_t*>(ws + pl.off_unit) + (size_t)pl.units * pl.cstride;
  int st = TS_ERR_UNSUPPORTED;
#define TS_CALL(FMT, DD) \
  st = launch_attention_format<FMT, DD>(layout, a, pl, sel, sel_count, unit_done, stream)
  TS_DISPATCH_FORMAT(layout, TS_CALL);
#undef TS_CALL
  return st;
}

int ts_sparse_decode_attention(const ts_layout* layout, const void* q, const int32_t* sel,
                               const int32_t* sel_count, int32_t max_topk, float softmax_scale,
                               void* out, float* lse_out, void* workspace,
                               size_t workspace_bytes, void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!q || !sel || !sel_count || !out || !workspace) return TS_ERR_NULL;
  if ((st = check_pool(layout)) != TS_OK) return st;
  if (max_topk < 1) return TS_ERR_SHAPE;
  const Plan pl = make_plan(layout, max_topk);
  if (workspace_bytes < pl.total) return TS_ERR_WORKSPACE;
  return launch_attention(layout, pl, q, sel, sel_count, max_topk, softmax_scale, out, lse_out,
                          workspace, stream);
}

size_t ts_dense_workspace_bytes(const ts_layout* layout) {
  if (check_layout(layout) != TS_OK) return 0;
  return make_plan(layout, layout->max_pages_per_seq, kDenseTargetWorkgroups).total;
}

int ts_dense_decode_attention(const ts_layout* layout, const void* q, float softmax_scale, void* out,
                              float* lse_out, void* workspace, size_t workspace_bytes,
                              void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!q || !out || !workspace) return TS_ERR_NULL;
  if ((st = check_pool(layout)) != TS_OK) return st;
  const Plan pl = make_plan(layout, layout->max_pages_per_seq, kDenseTargetWorkgroups);
  if (workspace_bytes < pl.total) return TS_ERR_WORKSPACE;
  return launch_attention(layout, pl, q, nullptr, nullptr, layout->max_pages_per_seq, softmax_scale,
                          out, lse_out, workspace, stream);
}

int ts_append_and_decode_launches(const ts_layout* layout, int32_t max_topk) {
  const int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (max_topk < 1) return TS_ERR_SHAPE;
  const Plan pl = make_plan(layout, max_topk);
  const int cus = num_compute_units();
  if (cus <= 0) return TS_ERR_DEVICE;
  const int tuned_per_cu = g_tune_wg_per_cu.load(std::memory_order_relaxed);
  const int per_cu = tuned_per_cu > 0 ? tuned_per_cu : 1;
  int cap1 = 0;
#define TS_CALL(FMT, DD) cap1 = append_capacity_format<FMT, DD>(layout, pl)
  TS_DISPATCH_FORMAT(layout, TS_CALL);
#undef TS_CALL
  if (cap1 <= 0) return TS_ERR_DEVICE;
  if (cap1 > cus * per_cu) cap1 = cus * per_cu;
  return pl.units * pl.g <= cap1 ? 1 : 2;
}

int ts_query_aware_decode(const ts_layout* layout, const void* q, int32_t topk,
                          const int32_t* topk_per_seq, int32_t max_topk, float softmax_scale,
                          void* out, float* scores_out, int32_t* sel_out,
                          int32_t* sel_count_out, void* workspace, size_t workspace_bytes,
                          void* stream) {
  return launch_fused(layout, nullptr, nullptr, q, topk, topk_per_seq, max_topk, softmax_scale, out,
                      scores_out, sel_out, sel_count_out, workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------------------
// The workspace of ts_query_aware_decode_static: device memory of the library
// itself.  In host code the array's name only stands for the symbol: its address
// on a given device comes from hipGetSymbolAddress with that device current, is
// asked for once per device, and is what every launch is given.  A __device__
// array starts out zeroed, which is the state ts_workspace_init would leave; from
// then on the launches keep it consistent themselves (launch tags only grow,
// whatever layout the bytes were last used for: every exchange word is an aligned
// 8-byte {value, tag} pair and the control words always sit at the front).
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[TS_STATIC_WORKSPACE_BYTES];
constexpr int kMaxDevices = 64;
static void* g_scratch_of_device[kMaxDevices];
static std::mutex g_scratch_mutex;

static int static_scratch(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TS_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_of_device[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr)
      return TS_ERR_DEVICE;
    g_scratch_of_device[dev] = p;
  }
  *ptr = g_scratch_of_device[dev];
  return TS_OK;
}

int ts_query_aware_decode_static(const ts_layout* layout, const void* q, int32_t topk,
                                 const int32_t* topk_per_seq, int32_t max_topk,
                                 float softmax_scale, void* out, float* scores_out,
                                 int32_t* sel_out, int32_t* sel_count_out, void* stream) {
  const int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (max_topk < 1) return TS_ERR_SHAPE;
  if (make_plan(layout, max_topk).total > (size_t)TS_STATIC_WORKSPACE_BYTES) return TS_ERR_WORKSPACE;
  void* ws = nullptr;
  const int sw = static_scratch(&ws);
  if (sw != TS_OK) return sw;
  return launch_fused(layout, nullptr, nullptr, q, topk, topk_per_seq, max_topk, softmax_scale, out,
                      scores_out, sel_out, sel_count_out, ws, (size_t)TS_STATIC_WORKSPACE_BYTES,
                      stream);
}

int ts_append_and_decode(const ts_layout* layout, const void* k_new, const void* v_new,
                         const void* q, int32_t topk, const int32_t* topk_per_seq,
                         int32_t max_topk, float softmax_scale, void* out, float* scores_out,
                         int32_t* sel_out, int32_t* sel_count_out, void* workspace,
                         size_t workspace_bytes, void* stream) {
  const int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!k_new || !v_new) return TS_ERR_NULL;
  return launch_fused(layout, k_new, v_new, q, topk, topk_per_seq, max_topk, softmax_scale, out,
                      scores_out, sel_out, sel_count_out, workspace, workspace_bytes, stream);
}

}  // extern "C"
