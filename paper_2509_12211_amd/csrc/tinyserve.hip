// C-ABI entry points (include/tinyserve.h) and the kernels behind them.
// gfx950 only.  Device code is in ts_*.h; this file holds the __global__
// wrappers, the work decomposition, and the host-side validation / launches.
#include "../../include/tinyserve.h"

#include <hip/hip_runtime.h>

#include "ts_attend.h"
#include "ts_device.h"
#include "ts_meta.h"
#include "ts_score.h"
#include "ts_select.h"

namespace ts {

// ---------------------------------------------------------------------------
// Work decomposition shared by host and device
// ---------------------------------------------------------------------------
constexpr int kCtrlWords = 64;   // control words at the head of the workspace
constexpr int kCtrlTicket = 0;   // next work item of the fused kernel
constexpr int kCtrlExit = 1;     // workgroups that have left the fused kernel
constexpr int kCtrlError = 2;    // sticky: a bounded wait expired
constexpr int kSpinLimit = 1 << 20;   // polls (>= ~1 us each) before a wait gives up

struct Plan {
  int units;           // B * Hkv
  int scan_pages;      // pages per scan work item
  int scan_items;      // scan work items per unit
  int n_split;         // attention work items per unit
  int chunk;           // selected pages per attention work item
  size_t off_unit;     // int32 [3][units]: scan_done, sel_ready, attend_done
  size_t off_scores;   // fp32 [units][Pmax]
  size_t off_sel;      // int32 [units][Kmax]
  size_t off_part;     // fp32 [units][n_split][G][d+2]
  size_t total;
  size_t lds_bytes;    // dynamic LDS of the select / attend / fused kernels
};

static int g_tune_scan_pages = 0, g_tune_splits = 0, g_tune_wg_per_cu = 0;

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static Plan make_plan(const ts_layout* L, int max_topk) {
  Plan pl;
  const int G = L->num_q_heads / L->num_kv_heads;
  const int Pmax = L->max_pages_per_seq;
  pl.units = L->num_seqs * L->num_kv_heads;
  // scan items: 128 pages (32-64 KiB of metadata) each, coarser when there are
  // already thousands of items
  int sp = 128;
  while ((long long)pl.units * ((Pmax + sp - 1) / sp) > 4096 && sp < 4096) sp *= 2;
  if (g_tune_scan_pages > 0) sp = (g_tune_scan_pages + 31) / 32 * 32;
  pl.scan_pages = sp;
  pl.scan_items = (Pmax + sp - 1) / sp;
  // attention items: aim at ~4 per compute unit (256 CUs), at least 4 pages each
  int ns = (1024 + pl.units - 1) / pl.units;
  const int cap = (max_topk + 3) / 4;
  if (ns > cap) ns = cap;
  if (ns > 64) ns = 64;
  if (g_tune_splits > 0) ns = g_tune_splits;
  if (ns > max_topk) ns = max_topk;
  if (ns < 1) ns = 1;
  pl.chunk = (max_topk + ns - 1) / ns;
  pl.n_split = (max_topk + pl.chunk - 1) / pl.chunk;
  size_t off = kCtrlWords * sizeof(int32_t);
  pl.off_unit = off;
  off = align_up(off + 3 * (size_t)pl.units * sizeof(int32_t), 256);
  pl.off_scores = off;
  off = align_up(off + (size_t)pl.units * Pmax * sizeof(float), 256);
  pl.off_sel = off;
  off = align_up(off + (size_t)pl.units * max_topk * sizeof(int32_t), 256);
  pl.off_part = off;
  off = align_up(off + (size_t)pl.units * pl.n_split * G * (L->head_dim + 2) * sizeof(float), 256);
  pl.total = off;
  const size_t lds_sel = (size_t)Pmax * 4 + 256 * 4 + 16 * 4;
  const size_t lds_att = (size_t)kWaves * G * (L->head_dim + 2) * 4;
  pl.lds_bytes = lds_sel > lds_att ? lds_sel : lds_att;
  return pl;
}

struct FusedParams {
  AttendParams at;
  const uint16_t* page_min;
  const uint16_t* page_max;
  float* scores;        // [units][Pmax]  (workspace or caller's)
  int32_t* sel;         // [units][Kmax]
  int32_t* sel_count;   // nullable [B]
  const int32_t* topk_per_seq;
  int32_t* ctrl;        // control words
  int32_t* scan_done;   // [units]
  int32_t* sel_ready;   // [units]
  int32_t* attend_done; // [units]
  int topk, S, units, scan_pages, scan_items;
};

__device__ __forceinline__ int pages_of(int len, int S) { return (len + S - 1) / S; }

__device__ __forceinline__ SelectScratch carve_select(unsigned char* smem, int Pmax) {
  SelectScratch sc;
  sc.keys = reinterpret_cast<uint32_t*>(smem);
  sc.hist = sc.keys + Pmax;
  sc.misc = reinterpret_cast<int*>(sc.hist + 256);
  return sc;
}

// ---------------------------------------------------------------------------
// Staged kernels
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kThreads) void score_pages_kernel(const uint16_t* q,
                                                               const uint16_t* page_min,
                                                               const uint16_t* page_max,
                                                               const int32_t* seq_lens, float* scores,
                                                               int Hq, int Hkv, int S, int Pmax,
                                                               int scan_pages) {
  const int u = blockIdx.y, b = u / Hkv, h = u % Hkv, G = Hq / Hkv;
  const int Pb = min(pages_of(seq_lens[b], S), Pmax);
  ScoreLanes<D> ql;
  ql.load_query(q + ((size_t)b * Hq + (size_t)h * G) * D, G);
  const int p0 = blockIdx.x * scan_pages, p1 = min(p0 + scan_pages, Pmax);
  score_pages_slice<D>(ql, page_min + (size_t)u * Pmax * D, page_max + (size_t)u * Pmax * D, Pb, p0,
                       p1, scores + (size_t)u * Pmax);
}

__global__ __launch_bounds__(kThreads) void select_topk_kernel(const float* scores,
                                                               const int32_t* seq_lens, int topk,
                                                               const int32_t* topk_per_seq,
                                                               int32_t* sel, int32_t* sel_count,
                                                               int Hkv, int S, int Pmax, int Kmax) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int u = blockIdx.x, b = u / Hkv, h = u % Hkv;
  const int Pb = min(pages_of(seq_lens[b], S), Pmax);
  const int K = topk_per_seq ? topk_per_seq[b] : topk;
  const int Kb = max(0, min(min(K, Pb), Kmax));
  if (h == 0 && threadIdx.x == 0) sel_count[b] = Kb;
  select_topk_unit(scores + (size_t)u * Pmax, Pb, Kb, Kmax, sel + (size_t)u * Kmax,
                   carve_select(smem, Pmax));
}

// grid (n_split, units).  The last workgroup of a unit to deposit its partial
// merges them (unit_done counts arrivals and is left at zero again).
template <int D, int S>
__global__ __launch_bounds__(kThreads) void sparse_attention_kernel(AttendParams p,
                                                                    const int32_t* sel,
                                                                    const int32_t* sel_count,
                                                                    int32_t* unit_done) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_last;
  const int u = blockIdx.y, b = u / p.Hkv, h = u % p.Hkv;
  const int Kb = max(0, min(sel_count[b], p.Kmax));
  attend_split<D, S>(p, b, h, blockIdx.x, sel + (size_t)u * p.Kmax, Kb,
                     reinterpret_cast<float*>(smem));
  if (p.n_split == 1) return;
  fence_release_agent();
  __syncthreads();
  if (threadIdx.x == 0) s_last = atomic_add_agent(&unit_done[u], 1) == p.n_split - 1;
  __syncthreads();
  if (!uniform(s_last)) return;
  fence_acquire_agent();
  combine_splits<D>(p, b, h);
  if (threadIdx.x == 0) atomic_store_agent(&unit_done[u], 0);
}

// ---------------------------------------------------------------------------
// Fused kernel: one launch, persistent workgroups pulling work items in ticket
// order.  Items [0, units*scan_items) score a slice of one unit's pages; items
// after that attend one split of one unit's selected pages.  The workgroup
// that completes a unit's last slice runs the selection for that unit and
// publishes it; attention items wait (bounded) for that publication.  Because
// tickets are handed out in increasing order, every item an attention item can
// wait for is already held by a running workgroup that itself never waits, so
// the waits end whatever the number of resident workgroups.
// ---------------------------------------------------------------------------
template <int D, int S>
__global__ __launch_bounds__(kThreads) void query_aware_decode_kernel(FusedParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_ticket, s_flag;
  const AttendParams& at = p.at;
  const int scan_total = p.units * p.scan_items;
  const int total = scan_total + p.units * at.n_split;
  const int G = at.G;

  // Every thread-0-only block below sits between two barriers, and every value
  // that steers a branch is pinned uniform: the compiler must never be able to
  // merge two thread-0 regions across the loop back-edge, which would let the
  // other lanes run ahead to the next barrier.
  if (threadIdx.x == 0) s_ticket = atomic_add_agent(&p.ctrl[kCtrlTicket], 1);
  __syncthreads();
  int t = uniform(s_ticket);
  while (t < total) {
    int done_unit = -1;  // unit whose last attention item this workgroup finished
    if (t < scan_total) {
      const int u = t / p.scan_items, it = t % p.scan_items;
      const int b = u / at.Hkv, h = u % at.Hkv;
      const int Pb = uniform(min(pages_of(at.seq_lens[b], p.S), at.Pmax));
      ScoreLanes<D> ql;
      ql.load_query(at.q + ((size_t)b * at.Hq + (size_t)h * G) * D, G);
      const int p0 = it * p.scan_pages, p1 = min(p0 + p.scan_pages, at.Pmax);
      float* srow = p.scores + (size_t)u * at.Pmax;
      score_pages_slice<D>(ql, p.page_min + (size_t)u * at.Pmax * D,
                           p.page_max + (size_t)u * at.Pmax * D, Pb, p0, p1, srow);
      fence_release_agent();
      __syncthreads();
      if (threadIdx.x == 0) s_flag = atomic_add_agent(&p.scan_done[u], 1) == p.scan_items - 1;
      __syncthreads();
      if (uniform(s_flag)) {  // this workgroup completed the unit's scores: select
        fence_acquire_agent();
        const int K = p.topk_per_seq ? p.topk_per_seq[b] : p.topk;
        const int Kb = uniform(max(0, min(min(K, Pb), at.Kmax)));
        select_topk_unit(srow, Pb, Kb, at.Kmax, p.sel + (size_t)u * at.Kmax,
                         carve_select(smem, at.Pmax));
        fence_release_agent();
        __syncthreads();
        if (threadIdx.x == 0) {
          if (p.sel_count && h == 0) p.sel_count[b] = Kb;
          atomic_store_agent(&p.sel_ready[u], 1);
        }
      }
    } else {
      const int a = t - scan_total;
      const int u = a / at.n_split, split = a % at.n_split;
      const int b = u / at.Hkv, h = u % at.Hkv;
      if (threadIdx.x == 0) {
        int ok = 0;
        for (int spin = 0; spin < kSpinLimit; ++spin) {
          if (atomic_load_agent(&p.sel_ready[u]) != 0) { ok = 1; break; }
          __builtin_amdgcn_s_sleep(2);
        }
        if (!ok) atomic_store_agent(&p.ctrl[kCtrlError], 1);
        s_flag = ok;
      }
      __syncthreads();
      const int ok = uniform(s_flag);
      fence_acquire_agent();
      const int Pb = uniform(min(pages_of(at.seq_lens[b], p.S), at.Pmax));
      const int K = p.topk_per_seq ? p.topk_per_seq[b] : p.topk;
      const int Kb = uniform(ok ? max(0, min(min(K, Pb), at.Kmax)) : 0);
      attend_split<D, S>(at, b, h, split, p.sel + (size_t)u * at.Kmax, Kb,
                         reinterpret_cast<float*>(smem));  // ends with a barrier
      int last = 1;
      if (at.n_split > 1) {
        fence_release_agent();
        __syncthreads();
        if (threadIdx.x == 0) s_flag = atomic_add_agent(&p.attend_done[u], 1) == at.n_split - 1;
        __syncthreads();
        last = uniform(s_flag);
        if (last) {
          fence_acquire_agent();
          combine_splits<D>(at, b, h);
        }
      }
      if (last) done_unit = u;
    }
    __syncthreads();  // the item is finished; s_ticket / s_flag are free again
    if (threadIdx.x == 0) {
      if (done_unit >= 0) {  // every item of this unit has passed its waits: re-arm it
        atomic_store_agent(&p.scan_done[done_unit], 0);
        atomic_store_agent(&p.sel_ready[done_unit], 0);
        atomic_store_agent(&p.attend_done[done_unit], 0);
      }
      s_ticket = atomic_add_agent(&p.ctrl[kCtrlTicket], 1);
    }
    __syncthreads();
    t = uniform(s_ticket);
  }
  // the last workgroup to leave re-arms the ticket counter for the next launch
  if (threadIdx.x == 0) {
    if (atomic_add_agent(&p.ctrl[kCtrlExit], 1) == (int)gridDim.x - 1) {
      atomic_store_agent(&p.ctrl[kCtrlTicket], 0);
      atomic_store_agent(&p.ctrl[kCtrlExit], 0);
    }
  }
}

__global__ void fill_zero_kernel(int32_t* p, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
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
  if (L->head_dim != 64 && L->head_dim != 128) return TS_ERR_UNSUPPORTED;
  if (L->page_size != 16 && L->page_size != 32) return TS_ERR_UNSUPPORTED;
  if (L->num_q_heads / L->num_kv_heads > 16) return TS_ERR_UNSUPPORTED;
  if (L->max_pages_per_seq > TS_MAX_PAGES_PER_SEQ) return TS_ERR_UNSUPPORTED;
  if ((long long)L->num_seqs * L->num_kv_heads > 65535) return TS_ERR_UNSUPPORTED;
  return TS_OK;
}

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

template <typename KernelT>
static int allow_lds(KernelT kernel, size_t bytes) {
  if (bytes <= 64 * 1024) return TS_OK;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)bytes) == hipSuccess
             ? TS_OK
             : TS_ERR_LAUNCH;
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
  return p;
}

static AttendParams attend_params(const ts_layout* L, const Plan& pl, const void* q, float* out,
                                  unsigned char* ws, int max_topk, float softmax_scale) {
  AttendParams a;
  a.q = static_cast<const uint16_t*>(q);
  a.k_pool = static_cast<const uint16_t*>(L->k_pool);
  a.v_pool = static_cast<const uint16_t*>(L->v_pool);
  a.block_table = L->block_table;
  a.seq_lens = L->seq_lens;
  a.out = out;
  a.partials = reinterpret_cast<float*>(ws + pl.off_part);
  a.Hq = L->num_q_heads;
  a.Hkv = L->num_kv_heads;
  a.G = L->num_q_heads / L->num_kv_heads;
  a.Pmax = L->max_pages_per_seq;
  a.Kmax = max_topk;
  a.n_phys = L->num_phys_pages;
  a.n_split = pl.n_split;
  a.chunk = pl.chunk;
  a.scale_log2 = softmax_scale * 1.4426950408889634f;
  return a;
}

}  // namespace ts

using namespace ts;

extern "C" {

int ts_version(void) { return 1; }

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

int ts_set_tuning(int32_t scan_pages_per_task, int32_t num_splits, int32_t workgroups_per_cu) {
  if (scan_pages_per_task < 0 || num_splits < 0 || workgroups_per_cu < 0) return TS_ERR_SHAPE;
  g_tune_scan_pages = scan_pages_per_task;
  g_tune_splits = num_splits;
  g_tune_wg_per_cu = workgroups_per_cu;
  return TS_OK;
}

size_t ts_workspace_bytes(const ts_layout* layout, int32_t max_topk) {
  if (check_layout(layout) != TS_OK || max_topk < 1) return 0;
  return make_plan(layout, max_topk).total;
}

int ts_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace) return TS_ERR_NULL;
  if (workspace_bytes < kCtrlWords * sizeof(int32_t)) return TS_ERR_WORKSPACE;
  // control words + per-unit counters live at the head; zeroing the first
  // min(bytes, 1 MiB) covers them for every supported unit count (<= 65535)
  size_t n = workspace_bytes / sizeof(int32_t);
  const size_t cap = (kCtrlWords + 3 * 65536) ;
  if (n > cap) n = cap;
  fill_zero_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
      static_cast<int32_t*>(workspace), n);
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
  dim3 grid((p.Pmax + kWaves - 1) / kWaves, p.Hkv, p.B);
  if (p.B > 65535) return TS_ERR_UNSUPPORTED;
  if (layout->head_dim == 64)
    build_page_meta_kernel<64><<<grid, kThreads, 0, (hipStream_t)stream>>>(p);
  else
    build_page_meta_kernel<128><<<grid, kThreads, 0, (hipStream_t)stream>>>(p);
  return launch_status();
}

int ts_append_token_meta(const ts_layout* layout, const void* k_new, const void* v_new,
                         int advance_seq_lens, void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!k_new || !layout->seq_lens || !layout->page_min || !layout->page_max) return TS_ERR_NULL;
  if (v_new && (!layout->k_pool || !layout->v_pool || !layout->block_table)) return TS_ERR_NULL;
  MetaParams p = meta_params(layout);
  append_token_meta_kernel<<<p.B, kThreads, 0, (hipStream_t)stream>>>(
      p, layout->head_dim, static_cast<const uint16_t*>(k_new),
      static_cast<const uint16_t*>(v_new), advance_seq_lens);
  return launch_status();
}

int ts_score_pages(const ts_layout* layout, const void* q, float* scores, void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!q || !scores || !layout->seq_lens || !layout->page_min || !layout->page_max)
    return TS_ERR_NULL;
  Plan pl = make_plan(layout, 1);
  dim3 grid(pl.scan_items, pl.units);
  const uint16_t* pmin = static_cast<const uint16_t*>(layout->page_min);
  const uint16_t* pmax = static_cast<const uint16_t*>(layout->page_max);
  if (layout->head_dim == 64)
    score_pages_kernel<64><<<grid, kThreads, 0, (hipStream_t)stream>>>(
        static_cast<const uint16_t*>(q), pmin, pmax, layout->seq_lens, scores, layout->num_q_heads,
        layout->num_kv_heads, layout->page_size, layout->max_pages_per_seq, pl.scan_pages);
  else
    score_pages_kernel<128><<<grid, kThreads, 0, (hipStream_t)stream>>>(
        static_cast<const uint16_t*>(q), pmin, pmax, layout->seq_lens, scores, layout->num_q_heads,
        layout->num_kv_heads, layout->page_size, layout->max_pages_per_seq, pl.scan_pages);
  return launch_status();
}

int ts_select_topk_pages(const ts_layout* layout, const float* scores, int32_t topk,
                         const int32_t* topk_per_seq, int32_t max_topk, int32_t* sel,
                         int32_t* sel_count, void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!scores || !sel || !sel_count || !layout->seq_lens) return TS_ERR_NULL;
  if (max_topk < 1 || (!topk_per_seq && (topk < 1 || max_topk < topk))) return TS_ERR_SHAPE;
  Plan pl = make_plan(layout, max_topk);
  const size_t lds = (size_t)layout->max_pages_per_seq * 4 + 256 * 4 + 16 * 4;
  if ((st = allow_lds(select_topk_kernel, lds)) != TS_OK) return st;
  select_topk_kernel<<<pl.units, kThreads, lds, (hipStream_t)stream>>>(
      scores, layout->seq_lens, topk, topk_per_seq, sel, sel_count, layout->num_kv_heads,
      layout->page_size, layout->max_pages_per_seq, max_topk);
  return launch_status();
}

int ts_sparse_decode_attention(const ts_layout* layout, const void* q, const int32_t* sel,
                               const int32_t* sel_count, int32_t max_topk, float softmax_scale,
                               float* out, void* workspace, size_t workspace_bytes,
                               void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!q || !sel || !sel_count || !out || !workspace || !layout->k_pool || !layout->v_pool ||
      !layout->block_table || !layout->seq_lens)
    return TS_ERR_NULL;
  if (max_topk < 1) return TS_ERR_SHAPE;
  Plan pl = make_plan(layout, max_topk);
  if (workspace_bytes < pl.total) return TS_ERR_WORKSPACE;
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  AttendParams a = attend_params(layout, pl, q, out, ws, max_topk, softmax_scale);
  int32_t* unit_done = reinterpret_cast<int32_t*>(ws + pl.off_unit) + 2 * (size_t)pl.units;
  const size_t lds = (size_t)kWaves * a.G * (layout->head_dim + 2) * 4;
  dim3 grid(pl.n_split, pl.units);
  hipStream_t s = (hipStream_t)stream;
  const int D = layout->head_dim, S = layout->page_size;
  if (D == 64 && S == 16)
    sparse_attention_kernel<64, 16><<<grid, kThreads, lds, s>>>(a, sel, sel_count, unit_done);
  else if (D == 64 && S == 32)
    sparse_attention_kernel<64, 32><<<grid, kThreads, lds, s>>>(a, sel, sel_count, unit_done);
  else if (D == 128 && S == 16)
    sparse_attention_kernel<128, 16><<<grid, kThreads, lds, s>>>(a, sel, sel_count, unit_done);
  else
    sparse_attention_kernel<128, 32><<<grid, kThreads, lds, s>>>(a, sel, sel_count, unit_done);
  return launch_status();
}

int ts_query_aware_decode(const ts_layout* layout, const void* q, int32_t topk,
                          const int32_t* topk_per_seq, int32_t max_topk, float softmax_scale,
                          float* out, float* scores_out, int32_t* sel_out,
                          int32_t* sel_count_out, void* workspace, size_t workspace_bytes,
                          void* stream) {
  int st = check_layout(layout);
  if (st != TS_OK) return st;
  if (!q || !out || !workspace || !layout->k_pool || !layout->v_pool || !layout->block_table ||
      !layout->seq_lens || !layout->page_min || !layout->page_max)
    return TS_ERR_NULL;
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
  p.scores = scores_out ? scores_out : reinterpret_cast<float*>(ws + pl.off_scores);
  p.sel = sel_out ? sel_out : reinterpret_cast<int32_t*>(ws + pl.off_sel);
  p.sel_count = sel_count_out;
  p.topk_per_seq = topk_per_seq;
  p.ctrl = reinterpret_cast<int32_t*>(ws);
  p.scan_done = reinterpret_cast<int32_t*>(ws + pl.off_unit);
  p.sel_ready = p.scan_done + pl.units;
  p.attend_done = p.sel_ready + pl.units;
  p.topk = topk;
  p.S = layout->page_size;
  p.units = pl.units;
  p.scan_pages = pl.scan_pages;
  p.scan_items = pl.scan_items;
  const long long items = (long long)pl.units * (pl.scan_items + pl.n_split);
  const int per_cu = g_tune_wg_per_cu > 0 ? g_tune_wg_per_cu : 4;
  long long grid = (long long)cus * per_cu;
  if (grid > items) grid = items;
  hipStream_t s = (hipStream_t)stream;
  const int D = layout->head_dim, S = layout->page_size;
#define TS_LAUNCH_FUSED(DD, SS)                                                        \
  do {                                                                                 \
    if ((st = allow_lds(query_aware_decode_kernel<DD, SS>, pl.lds_bytes)) != TS_OK)    \
      return st;                                                                       \
    query_aware_decode_kernel<DD, SS><<<(unsigned)grid, kThreads, pl.lds_bytes, s>>>(p); \
  } while (0)
  if (D == 64 && S == 16) TS_LAUNCH_FUSED(64, 16);
  else if (D == 64 && S == 32) TS_LAUNCH_FUSED(64, 32);
  else if (D == 128 && S == 16) TS_LAUNCH_FUSED(128, 16);
  else TS_LAUNCH_FUSED(128, 32);
#undef TS_LAUNCH_FUSED
  return launch_status();
}

}  // extern "C"
