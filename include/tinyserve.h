/*
 * tinyserve.h -- C ABI of the MI355X (gfx950) query-aware decode-attention library.
 *
 * The operations are the decode-time hot path of TinyServe:
 *   - every KV page carries bounding-box metadata, the channel-wise min and max
 *     of its keys (Section 3.4; Eq. 1, phi(K_j) = (m_j, M_j));
 *   - a query scores every page with the directional bounding-box estimator
 *     r(q, phi_j) = sum_i q_i * (q_i >= 0 ? M_ji : m_ji)
 *                 = sum_i max(q_i * m_ji, q_i * M_ji)                    (Eq. 2);
 *   - the K highest-scoring pages are selected (Section 3.5, S_t = TopK_j r);
 *   - single-query softmax attention runs over the tokens of the selected
 *     pages only (Section 3.5, SparseAttn; Algorithm 1, steps 3-4).
 * Algorithm 1 fuses the last three into one kernel; ts_query_aware_decode is
 * that fused, single-launch form.  The paper is silent on heads: here a unit of
 * work is one (sequence, KV head); with grouped-query attention the page score
 * of a KV head is the sum of r over the G = Hq / Hkv query heads sharing it.
 *
 * Conventions
 *   - All pointers are DEVICE pointers unless marked "host".  The caller owns
 *     every buffer; the library allocates nothing and keeps no state between
 *     calls except what lives in the caller's workspace.
 *   - bf16 tensors are raw 16-bit patterns.  `stream` is a hipStream_t cast to
 *     void* (NULL = the default stream).  Calls enqueue work and return; they
 *     never synchronise.
 *   - Every function returns TS_OK or a negative ts_status.  Validation is done
 *     on the host from the struct fields and scalar arguments only; device-side
 *     contents (seq_lens, block_table, sel) are trusted: seq_lens[b] must lie in
 *     [0, max_pages_per_seq * page_size], block_table entries of pages that
 *     hold tokens must lie in [0, num_phys_pages).
 *   - P_b = ceil(seq_lens[b] / page_size) is the number of pages of sequence b
 *     (Section 3.5, P = ceil(t / S)).  A partly filled last page is summarised,
 *     scored and attended over the tokens it holds; pool slots past seq_lens[b]
 *     may hold anything (NaN included) and never influence a result.
 *
 * Supported shapes: head_dim in {64, 128}; page_size in {4, 8, 16, 32, 64};
 * 1 <= G = Hq / Hkv <= 16; max_pages_per_seq <= TS_MAX_PAGES_PER_SEQ.
 */
#ifndef TINYSERVE_H_
#define TINYSERVE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TS_MAX_PAGES_PER_SEQ 16384

enum { TS_OUT_F32 = 0, TS_OUT_BF16 = 1 };
enum { TS_KV_BF16 = 0, TS_KV_INT8 = 1, TS_KV_FP16 = 2 };

typedef enum ts_status {
  TS_OK = 0,
  TS_ERR_NULL = -1,        /* a required pointer is NULL (with the INT8 cache: k_scale / v_scale
                              in every call that reads or writes the pool)                  */
  TS_ERR_SHAPE = -2,       /* non-positive dimension, Hq % Hkv != 0, topk < 1, max_topk < topk,
                              0 < kv_tile_stride < S*d or not a multiple of 8, a negative
                              keep_*_pages count, cluster_size or wait_limit, a non-zero
                              reserved argument */
  TS_ERR_UNSUPPORTED = -3, /* head_dim / page_size / group size / page count outside the built set */
  TS_ERR_WORKSPACE = -4,   /* workspace_bytes smaller than ts_workspace_bytes()             */
  TS_ERR_LAUNCH = -5,      /* the HIP runtime reported an error when enqueueing             */
  TS_ERR_DEVICE = -6       /* no usable HIP device                                          */
} ts_status;

/* Paged KV cache of one attention layer plus its page metadata.
 *   k_pool      bf16 [num_phys_pages][Hkv][S][d]   a (page, head) K tile is S*d contiguous
 *   v_pool      bf16 [num_phys_pages][Hkv][d][S]   V tile stored channel-major (transposed),
 *                                                  so the token axis is contiguous
 *   The tile of (physical page p, head h) starts kv_tile_stride elements after
 *   the tile of (p, h-1) in both pools; 0 means S*d (two dense pools).  The
 *   layout this library is tuned for interleaves the two: one allocation
 *   [num_phys_pages][Hkv][2][S*d], k_pool = base, v_pool = base + S*d,
 *   kv_tile_stride = 2*S*d, so the K and V tiles of a page form one contiguous
 *   4-8 KiB block (random 4 KiB reads reach ~40 % more HBM bandwidth than
 *   random 2 KiB reads on this part).
 *   block_table int32 [B][P_max]                   logical page -> physical page
 *   seq_lens    int32 [B]                          tokens currently cached per sequence
 *   page_min,
 *   page_max    bf16 [B][Hkv][P_max][d]            metadata in LOGICAL page order, so the
 *                                                  scoring pass is one contiguous stream
 */
typedef struct ts_layout {
  int32_t num_seqs;          /* B                                   */
  int32_t num_q_heads;       /* Hq                                  */
  int32_t num_kv_heads;      /* Hkv, Hq % Hkv == 0                  */
  int32_t head_dim;          /* d                                   */
  int32_t page_size;         /* S                                   */
  int32_t max_pages_per_seq; /* P_max: row stride of block_table, page_min, page_max, scores */
  int32_t num_phys_pages;    /* pool capacity                       */
  int32_t kv_tile_stride;    /* elements between consecutive (page, head) tiles; 0 = S*d */
  void* k_pool;
  void* v_pool;
  const int32_t* block_table;
  int32_t* seq_lens;
  void* page_min;
  void* page_max;
  /* Selection option outside the paper (which selects by score alone; leave both 0
   * for that): the first keep_first_pages pages of every sequence (attention
   * sinks) and its last keep_last_pages pages (the newest tokens) are selected
   * whatever their score.  They count towards K; if they alone exceed it, the
   * lowest page ids among them are kept. */
  int32_t keep_first_pages;
  int32_t keep_last_pages;
  /* Format of the attention output `out` of every call: TS_OUT_F32 (0, the
   * default) fp32 [B][Hq][d]; TS_OUT_BF16: the same values rounded to bf16
   * (nearest even), `out` then points to 16-bit elements. */
  int32_t out_format;
  /* Format of the KV pool: TS_KV_BF16 (0, the default) as described above;
   * TS_KV_FP16: every 16-bit tensor of the interface (k_pool, v_pool, page_min,
   * page_max, q, k_new, v_new) holds IEEE half instead of bf16 (the paper's
   * experiments run in FP16), nothing else changes; or
   * TS_KV_INT8 (Section 3.1 names INT8 KV support and gives no format; this one
   * is this library's):
   *   k_pool int8 [num_phys_pages][Hkv][S][d], v_pool int8 [num_phys_pages][Hkv][d][S]
   *   (kv_tile_stride counts bytes and must be a multiple of 16),
   *   k_scale, v_scale fp32 [num_phys_pages][Hkv][S]: one positive scale per token
   *   and KV head; the key of a token is code * scale as a real number.
   * Queries, appended tokens and metadata stay bf16.  ts_build_page_meta rounds a
   * page's minimum down and its maximum up to bf16, so the box contains the
   * dequantised keys and Eq. 2 remains an upper bound.  ts_append_token_meta
   * quantises the bf16 token: scale = max_c |x_c| / 127 (1 for a zero vector),
   * code = x_c / scale rounded half to even, all in fp32; with v_new == NULL only
   * the box is widened, by the key so quantised.  ts_append_and_decode does the
   * same quantisation inside its launch.  The attention over an INT8 cache
   * multiplies in IEEE half: the bf16 queries are converted (exactly, for
   * magnitudes from 2^-14 to 65504; smaller ones lose low bits, larger ones are
   * taken as 65504), the int8 codes are exact. */
  int32_t kv_format;
  /* How the fused calls (ts_query_aware_decode, ts_append_and_decode) spread one
   * (sequence, KV head) over workgroups.  0 (the default): automatic, about one
   * workgroup per compute unit in all; with few units a unit is then shared by a
   * cluster of workgroups that wait for each other inside the launch, which needs
   * the whole launch resident at once, i.e. a device that runs nothing else at the
   * same time.  1: one workgroup per unit; no workgroup ever waits for another, so
   * the launch is safe beside kernels of other streams (slower for small batches).
   * A serving engine that overlaps other work with the decode step on the same
   * device should set 1; one that runs the step alone should leave 0.  n > 1: that
   * many workgroups per unit (for sweeps).  Changes ts_workspace_bytes. */
  int32_t cluster_size;
  /* Polls after which a workgroup of a cluster stops waiting for its partners
   * (0 = the default, about a second; see ts_query_aware_decode).  Tests of the
   * expiry path set a tiny value. */
  int32_t wait_limit;
  float* k_scale;
  float* v_scale;
} ts_layout;

/* Section 3.4 / Eq. 1.  Rebuilds page_min / page_max of every page j < P_b of
 * every (sequence, KV head) from k_pool.  Rows of pages j >= P_b are not
 * written.  min / max of bf16 values are exact. */
int ts_build_page_meta(const ts_layout* layout, void* stream);

/* Section 3.4 ("metadata ... is maintained").  Appends one token per sequence
 * at position p = seq_lens[b]: page j = p / S; if p % S == 0 the page is
 * opened (m = M = k_new) else its box is widened.  k_new, v_new: bf16
 * [B][Hkv][d].  If v_new != NULL the token's key and value are also stored
 * into the pool slot (block_table[b][j], h, p % S); if v_new == NULL only the
 * metadata is updated (the caller has stored K/V itself).  With
 * advance_seq_lens != 0 the kernel increments seq_lens[b] after use.  A
 * sequence whose page j would be >= P_max is left unchanged. */
int ts_append_token_meta(const ts_layout* layout, const void* k_new, const void* v_new,
                         int advance_seq_lens, void* stream);

/* Eq. 2, step 1 of Algorithm 1.  q: bf16 [B][Hq][d].  scores: fp32
 * [B][Hkv][P_max]; entry (b, h, j) is the group-summed bound for j < P_b and
 * -inf for j >= P_b.  Accumulated in fp64, rounded to fp32 once. */
int ts_score_pages(const ts_layout* layout, const void* q, float* scores, void* stream);

/* Section 3.5 (S_t = TopK_j r, |S_t| = K), step 2 of Algorithm 1.  For each
 * (b, h) keeps the K_b = min(K, P_b, max_topk) pages with the largest score,
 * equal scores resolved in favour of the lower page id; K = topk_per_seq[b] if
 * that pointer is non-NULL, else topk.  sel: int32 [B][Hkv][max_topk], page
 * ids ascending, padded with -1.  sel_count: int32 [B] = K_b.  The comparison
 * is on the fp32 values as given (-0 ranks equal to +0; NaN is undefined).
 * layout->keep_first_pages / keep_last_pages (see ts_layout) are honoured here
 * and in the fused calls. */
int ts_select_topk_pages(const ts_layout* layout, const float* scores, int32_t topk,
                         const int32_t* topk_per_seq, int32_t max_topk, int32_t* sel,
                         int32_t* sel_count, void* stream);

/* Section 3.5 SparseAttn; steps 3-4 of Algorithm 1.  For every query head:
 * logits softmax_scale * q.k over the valid tokens of the pages listed in sel
 * (first sel_count[b] entries of each row), softmax over exactly those tokens,
 * weighted sum of their values.  The paper writes softmax(q.k) with no factor:
 * softmax_scale = 1 is its literal form, 1/sqrt(d) the usual one.
 * out: fp32 [B][Hq][d] (bf16 with layout->out_format = TS_OUT_BF16); a (b, head)
 * with no token gets zeros.  bf16 inputs,
 * fp32 accumulation.  lse_out (optional, NULL = not reported): fp32 [B][Hq],
 * the natural logarithm of the softmax denominator, log sum_t exp(softmax_scale
 * * q.k_t) over the attended tokens (-inf with no token); the share of the
 * dense softmax mass that a selection captures is exp(lse_sparse - lse_dense).
 * workspace: ts_workspace_bytes(layout, max_topk) bytes, initialised once with
 * ts_workspace_init. */
int ts_sparse_decode_attention(const ts_layout* layout, const void* q, const int32_t* sel,
                               const int32_t* sel_count, int32_t max_topk, float softmax_scale,
                               void* out, float* lse_out, void* workspace,
                               size_t workspace_bytes, void* stream);

/* Algorithm 1 as ONE kernel launch: score -> select -> gather -> attend.
 * Arguments as in the three staged calls.  scores_out (fp32 [B][Hkv][P_max]),
 * sel_out (int32 [B][Hkv][max_topk]) and sel_count_out (int32 [B]) are
 * optional (NULL = not reported).
 * With few (sequence, KV head) units the kernel spreads each over several
 * workgroups that exchange data while running, and sizes its grid so that all
 * of them are resident at once on an otherwise idle device.  If other kernels
 * occupy compute units at the same time, a workgroup may wait for a partner
 * that cannot start; every such wait is bounded (about a second), after which
 * the launch finishes with invalid results and ts_workspace_status reports
 * non-zero.  It never hangs. */
int ts_query_aware_decode(const ts_layout* layout, const void* q, int32_t topk,
                          const int32_t* topk_per_seq, int32_t max_topk, float softmax_scale,
                          void* out, float* scores_out, int32_t* sel_out,
                          int32_t* sel_count_out, void* workspace, size_t workspace_bytes,
                          void* stream);

/* ts_query_aware_decode for callers that cannot allocate device memory at all, not
 * even a workspace: code under HIP graph capture that has no buffer of its own to
 * hand over, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results, minus the workspace: the kernels use a fixed region of
 * TS_STATIC_WORKSPACE_BYTES of device memory that belongs to the library (every
 * GPU the library runs on holds its own copy until the process ends) and needs no
 * ts_workspace_init.  The call allocates nothing and frees nothing.  Layouts whose
 * ts_workspace_bytes exceeds the region are rejected with TS_ERR_WORKSPACE
 * (batches of up to 256 (sequence, KV head) units fit with room to spare up to
 * about 4000 pages a sequence; larger batches run one workgroup per unit and
 * need a few KiB).  All calls on one GPU share the region: calls that overlap in
 * time on the same GPU (two streams) race; order them.  A bounded wait that
 * expired cannot be read back here (there is no workspace to ask):
 * callers that share the device with other kernels use ts_layout.cluster_size = 1,
 * with which nothing waits.  The first call on a device looks the region's
 * address up (no allocation, but not a stream operation: make that first call
 * outside a graph capture). */
#define TS_STATIC_WORKSPACE_BYTES (4 << 20)
int ts_query_aware_decode_static(const ts_layout* layout, const void* q, int32_t topk,
                                 const int32_t* topk_per_seq, int32_t max_topk,
                                 float softmax_scale, void* out, float* scores_out,
                                 int32_t* sel_out, int32_t* sel_count_out, void* stream);

/* Section 3.4 + Algorithm 1: one decode step of a layer in ONE launch.  With
 * valid block-table entries it leaves exactly the state and results of
 * ts_append_token_meta(layout, k_new, v_new, 1, stream) followed by
 * ts_query_aware_decode(...) with the same remaining arguments: the new
 * token of every sequence (k_new, v_new: bf16 [B][Hkv][d], both required) is
 * stored in its pool slot, widens (or opens) the box of its page, takes part in
 * the scoring, selection and attention of this same call, and seq_lens[b] is
 * advanced by one before the call completes.  A sequence whose new page would
 * be >= P_max is left unchanged.  The block-table entry of the page that
 * receives the token must be valid: the two-call form leaves a sequence with an
 * out-of-range entry untouched, whereas the single launch decides from the
 * length alone, so it still widens the box and advances seq_lens[b] and only
 * skips the pool write.  It is a single launch whenever all
 * (sequence, KV head) units are worked on at once (up to one per compute unit);
 * for larger batches, which are bound by bandwidth, the append is enqueued as a
 * kernel of its own in front of the decode on the same stream. */
int ts_append_and_decode(const ts_layout* layout, const void* k_new, const void* v_new,
                         const void* q, int32_t topk, const int32_t* topk_per_seq,
                         int32_t max_topk, float softmax_scale, void* out, float* scores_out,
                         int32_t* sel_out, int32_t* sel_count_out, void* workspace,
                         size_t workspace_bytes, void* stream);

/* Host-only (needs the device to be present): 1 if ts_append_and_decode runs
 * this layout as a single launch, 2 if it enqueues the append as a kernel of
 * its own first; a negative ts_status on error. */
int ts_append_and_decode_launches(const ts_layout* layout, int32_t max_topk);

/* Host-only: bytes of workspace the three calls above need for this layout and
 * max_topk (0 on invalid arguments).  Reads only the scalar fields. */
size_t ts_workspace_bytes(const ts_layout* layout, int32_t max_topk);

/* The comparison the paper measures against (the FullCache rows of its latency
 * tables; Section 3.5 opens with this Attn(q_t, K, V) over the whole cache):
 * single-query softmax attention over EVERY cached token of every sequence,
 * through the same block table and pool layout, fp32 out [B][Hq][d]; lse_out
 * as in ts_sparse_decode_attention (optional).  Needs a workspace of its own
 * size, ts_dense_workspace_bytes(layout) (host-only, 0 on an invalid layout),
 * initialised with ts_workspace_init. */
size_t ts_dense_workspace_bytes(const ts_layout* layout);
int ts_dense_decode_attention(const ts_layout* layout, const void* q, float softmax_scale, void* out,
                              float* lse_out, void* workspace, size_t workspace_bytes,
                              void* stream);

/* Zeroes the whole workspace.  Required once after allocation (and after a
 * launch that was aborted); every call leaves the workspace ready for the
 * next, so repeated calls need no re-initialisation.  Calls sharing one
 * workspace must be ordered on one stream. */
int ts_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/* Blocking: copies the workspace's sticky error word to *status_host (host
 * pointer).  0 = no error; non-zero = a bounded wait inside the fused kernel
 * expired (results of that launch are invalid). */
int ts_workspace_status(const void* workspace, int32_t* status_host);

/* Launch-shape overrides for tuning sweeps; 0 restores the built-in choice.
 * A debugging aid, not part of the serving interface (use ts_layout.cluster_size,
 * which takes precedence over num_splits): the values are process-wide atomics
 * read once per call.
 *   reserved             must be 0 (TS_ERR_SHAPE otherwise)
 *   num_splits           workgroups sharing one (b, h): each scores 1/n of its pages and
 *                        attends 1/n of its selected pages
 *   workgroups_per_cu    resident workgroups per compute unit the fused kernel may count on
 *                        (capped by the occupancy the runtime reports; the kernels are
 *                        built for one per compute unit)
 * Process-wide; affects ts_workspace_bytes too, so set it before sizing. */
int ts_set_tuning(int32_t reserved, int32_t num_splits, int32_t workgroups_per_cu);

/* For tests and tuning: launches num_workgroups workgroups of the size the fused
 * kernel uses and stores into ids[w] (device, int32 [num_workgroups]) the number
 * of the XCD (die with an L2 of its own) workgroup w ran on.  The fused kernel
 * lays the workgroups of one cluster out so that they share a die under the
 * dispatch order this reports on MI355X (consecutive workgroups go to the eight
 * dies in turn, starting where the previous launch left off, so workgroups whose
 * numbers are congruent modulo 8 share a die); results never depend on it. */
int ts_debug_xcc_ids(int32_t* ids, int32_t num_workgroups, void* stream);

const char* ts_strerror(int status);
int ts_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TINYSERVE_H_ */
