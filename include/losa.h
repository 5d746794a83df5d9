/* losa.h — C ABI of the LoSA prefix-attention hot path for AMD MI355X (gfx950).
 *
 * One denoising step of a block-wise diffusion LM, per layer (paper: Methodology;
 * Fig. MethodOverview steps i-iii):
 *   (i)   locality score per block token and the active set A      -> losa_select_active
 *   (ii)  QUEST page bounds, per-query top pages, union per KV head -> losa_page_bounds, losa_score_pages
 *   (iii) prefix attention of the active queries over the union; stable tokens keep
 *         their cached (o_p, L_p)                                   -> losa_sparse_attn
 *   the three chained, with the dense initialisation at step 0     -> losa_step
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless marked host.  The caller owns every
 *     buffer (inputs, outputs, page metadata, workspace); the library allocates no
 *     device memory and keeps no caller pointer after a call returns, except the
 *     workspace handed to losa_create, which it uses until losa_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work; they never synchronise.  Counts (active tokens, union sizes)
 *     stay on the device.
 *   - Element type T of h, q, K, V and the page metadata is bfloat16 (LOSA_BF16) or
 *     float (LOSA_F32), fixed at losa_create.  Accumulation is float.  The cached
 *     prefix statistics o_p and lse_p are float in both modes.
 *   - Shapes use the paper's symbols: B block size, d head dim, g page size,
 *     Hq / Hkv query / KV heads, G = Hq/Hkv, H hidden size, P_b pages of sequence b.
 *     Arrays are row-major with the last index fastest.
 *   - Return value: LOSA_OK, or an error found by host-side validation before anything
 *     was enqueued (LOSA_ERR_INVALID_ARG: a value that makes no sense or a missing pointer;
 *     LOSA_ERR_UNSUPPORTED: a configuration the kernels are not built for - head_dim other
 *     than 64 / 128, page_size other than 16 / 32, block_size above 256, more than 16384
 *     pages per sequence, hidden_size not a multiple of 8; LOSA_ERR_WORKSPACE), or
 *     LOSA_ERR_HIP if a launch was rejected.  losa_last_error gives the text.  Nothing
 *     throws or aborts.  Device-side indices (page ids, token ids) outside their range
 *     are skipped by the kernels, never dereferenced.
 *   - Calls on one losa_ctx share its workspace: issue them on one stream, or
 *     serialise them.
 */
#ifndef LOSA_H
#define LOSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct losa_ctx losa_ctx; /* opaque, host memory */

typedef enum {
  LOSA_OK = 0,
  LOSA_ERR_INVALID_ARG = 1,
  LOSA_ERR_UNSUPPORTED = 2,
  LOSA_ERR_WORKSPACE = 3,
  LOSA_ERR_HIP = 4
} losa_status;

typedef enum { LOSA_BF16 = 0, LOSA_F32 = 1 } losa_dtype;

/* How the active set is chosen from the locality scores (Methodology, Locality Pruning):
 * TOPK: the `param` tokens with the largest score (the paper's rule; it uses 5 of 16);
 * FRACTION: top n with n = max(1, floor(param*B + 0.5));  THRESHOLD: score > param;
 * MASS: tokens in descending score order until their running sum reaches param (in [0,1])
 * times the block's total score (the 50 % line of the paper's locality heat maps is
 * param = 0.5); nothing is selected when the total is zero or param is zero.
 * Ties: larger score first, then smaller token index. */
typedef enum {
  LOSA_SEL_TOPK = 0,
  LOSA_SEL_FRACTION = 1,
  LOSA_SEL_THRESHOLD = 2,
  LOSA_SEL_MASS = 3
} losa_select_mode;

typedef struct {
  int32_t max_batch;         /* sequences per call, >= 1 */
  int32_t num_q_heads;       /* Hq */
  int32_t num_kv_heads;      /* Hkv, divides Hq */
  int32_t head_dim;          /* d: 64 or 128 */
  int32_t hidden_size;       /* H: row length of the tensor the detector compares; multiple of 8 */
  int32_t page_size;         /* g: 16 or 32 */
  int32_t block_size;        /* B: 1..256 */
  int32_t max_pages_per_seq; /* upper bound on P_b, 1..16384 */
  int32_t max_topk_pages;    /* upper bound on the per-query page budget K = k/g */
  int32_t dtype;             /* losa_dtype */
  float sm_scale;            /* score scale; 0 means 1/sqrt(d) */
} losa_config;

/* Ragged paged prefix KV cache of one layer (K_p, V_p of the paper, fixed across the
 * denoising steps of a block).  A page-head tile of keys is token-major, a tile of
 * values is channel-major (V is stored transposed inside each page), which is the
 * operand order the matrix cores consume without a shuffle. */
typedef struct {
  const void* k_pages;         /* T [num_pages, Hkv, g, d] */
  const void* v_pages;         /* T [num_pages, Hkv, d, g] */
  void* meta;                  /* T [num_pages, Hkv, 2, d]: row 0 elementwise min key, row 1 max key.
                                  Written by losa_page_bounds, read by losa_score_pages / losa_step. */
  const int32_t* page_indptr;  /* [batch+1] offsets into page_indices; sequence b lists indptr[b+1]-indptr[b]
                                  pages, of which the first P_b = ceil(L_b / g) hold tokens and are used
                                  (pages reserved ahead of the tokens may be listed: they are ignored) */
  const int32_t* page_indices; /* logical page p of sequence b -> physical page id */
  const int32_t* seq_lens;     /* [batch] prefix tokens L_b; the last page may be partly filled;
                                  slots past L_b may hold anything (NaN included) */
  int32_t batch;               /* host: 1..max_batch */
  int32_t num_pages;           /* host: pages in the pool (ids >= num_pages are skipped) */
  int32_t max_seq_pages;       /* host: an upper bound on the pages any sequence of this call uses, if the
                                  caller knows one (grids are sized by it), else 0 (= max_pages_per_seq).
                                  Pages of a sequence beyond the bound are left out of every step. */
} losa_kv;

/* Bytes of device workspace losa_create needs for this configuration (0 if it is invalid). */
size_t losa_workspace_bytes(const losa_config* cfg);

/* Validates cfg, takes `workspace` (device, 256-byte aligned, >= losa_workspace_bytes) and
 * returns a context in *out.  Enqueues nothing. */
losa_status losa_create(const losa_config* cfg, void* workspace, size_t workspace_bytes, losa_ctx** out);
losa_status losa_destroy(losa_ctx* ctx);
/* Text of the last error on this context (host string owned by the context);
 * with ctx == NULL, the text of the last failure on this thread of a call that takes no
 * context (losa_create, losa_select_active_static). */
const char* losa_last_error(const losa_ctx* ctx);

/* (i) Locality score and active set (eq. mse_locality; Locality Pruning).
 * delta[r] = mean_c (h_cur[r,c] - h_prev[r,c])^2 for each of the batch*B rows.
 *   h_cur, h_prev : T [batch*B, H]
 *   delta         : float [batch*B]
 *   mask          : uint8 [batch*B], 1 = active
 *   active_idx    : int32 [batch*B]; for sequence b, entries [b*B, b*B+count) are the active
 *                   token ids (0..B-1) ascending, the rest -1
 *   active_count  : int32 [batch] */
losa_status losa_select_active(losa_ctx* ctx, void* stream, int32_t batch,
                               const void* h_cur, const void* h_prev,
                               losa_select_mode mode, float param,
                               float* delta, uint8_t* mask, int32_t* active_idx, int32_t* active_count);

/* The same operation for callers that cannot allocate device memory or carry a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It
 * takes no context and allocates nothing, on the host or on the device: the per-sequence
 * ticket counters its kernel needs live in a device array inside the library (16 KiB, one
 * copy on every GPU the library runs on, held until the process ends).
 *   dtype       : losa_dtype of h_cur / h_prev
 *   batch       : 1..4096 (the counters the array holds); block_size : 1..1024;
 *                 hidden_size : a multiple of 8.  Larger values: LOSA_ERR_UNSUPPORTED.
 *   other arguments and results: exactly as losa_select_active.
 * Runs on the GPU that is current when it is called.  The first call on a GPU looks up the
 * array's device address (no allocation; make that call outside a graph capture).  All calls
 * on one GPU share the array, which keeps what the last call left (zeros after a completed
 * launch; cleared again at the start of every call): calls that overlap on one GPU - two
 * streams, two threads - race; serialise them.  Errors: text via losa_last_error(NULL). */
losa_status losa_select_active_static(void* stream, int32_t dtype, int32_t batch, int32_t block_size,
                                      int32_t hidden_size, const void* h_cur, const void* h_prev,
                                      losa_select_mode mode, float param,
                                      float* delta, uint8_t* mask, int32_t* active_idx, int32_t* active_count);

/* (ii-a) QUEST page metadata (Preliminaries, Sparse Attention Algorithms): elementwise
 * min and max key over the valid tokens of each page, for logical pages
 * [first_logical_page, first_logical_page + num_logical_pages) of every sequence
 * (num_logical_pages < 0: to the end).  Run once when pages are appended, not per step:
 * the prefix is fixed across the denoising steps of a block.  Writes kv->meta. */
losa_status losa_page_bounds(losa_ctx* ctx, void* stream, const losa_kv* kv,
                             int32_t first_logical_page, int32_t num_logical_pages);

/* (ii-b) Page scores, per-query top pages and their union (QUEST upper bound; eq. quest_union).
 * For every active token i, query head h (KV head j = h / G) and logical page p:
 *   s = sum_c max(q_c * min_{p,j,c}, q_c * max_{p,j,c});
 * the min(topk_pages, P_b) pages with the largest s are picked (ties: smaller page), and
 * the union over the active queries of a KV head is emitted ascending.
 *   q          : T [batch*B, Hq, d]
 *   active_idx, active_count : as written by losa_select_active
 *   topk_out   : nullable int32 [batch, B, Hq, topk_pages]; slot a of sequence b (its a-th
 *                active token) gets the picked pages ascending, padded with -1
 *   sel_pages  : int32 [batch, Hkv, cap] logical pages, ascending
 *   sel_count  : int32 [batch, Hkv]
 *   cap        : >= min(max P_b, B*G*topk_pages)  (the union's worst case) */
losa_status losa_score_pages(losa_ctx* ctx, void* stream, const losa_kv* kv, const void* q,
                             const int32_t* active_idx, const int32_t* active_count,
                             int32_t topk_pages, int32_t* topk_out,
                             int32_t* sel_pages, int32_t* sel_count, int32_t cap);

/* Variant of (ii-b) with ONE page set per (sequence, KV head) shared by all of its active
 * queries.  Not in the paper: it is the other reading of "a page budget per KV head".  Every
 * page is scored by the largest bound any active query of the head gives it (the scores are the
 * ones defined above), and the min(topk_pages, P_b) best pages are kept (ties: smaller page),
 * so the attention that follows reads exactly that many pages per head, where the per-query
 * budget reads between topk_pages and |A|*G*topk_pages.  Feed the result to losa_sparse_attn.
 *   sel_pages  : int32 [batch, Hkv, cap] logical pages, ascending
 *   sel_count  : int32 [batch, Hkv]   (0 for a sequence without active tokens)
 *   cap        : >= min(max P_b, topk_pages) */
losa_status losa_score_pages_shared(losa_ctx* ctx, void* stream, const losa_kv* kv, const void* q,
                                    const int32_t* active_idx, const int32_t* active_count,
                                    int32_t topk_pages, int32_t* sel_pages, int32_t* sel_count, int32_t cap);

/* (iii) Prefix attention of the active queries over the selected pages (Attention
 * Decomposition With Online Softmax; eq. update_rule).  For each active token i and head h:
 *   s_t = sm_scale * q . k_t over the valid tokens t of the pages of its KV head's list,
 *   lse_p[i,h] = ln sum_t exp(s_t),   o_p[i,h,:] = sum_t exp(s_t - lse_p) v_t.
 * Rows of tokens that are not active are not touched (eq. reuse_rule).
 *   active_idx, active_count : both NULL = every token of the block is active
 *   sel_pages, sel_count     : both NULL = every page (dense prefix attention)
 *   o_p   : float [batch*B, Hq, d]  in/out
 *   lse_p : float [batch*B, Hq]     in/out (natural log)
 * A sequence with no selected token gives o_p = 0, lse_p = -inf for its active rows.
 * Accuracy against exact attention of the given inputs: bfloat16 mode max-abs 2e-2 for values of
 * ordinary activation size (products accumulate in float; probabilities enter the value product
 * with 16 significant bits for up to 64 query rows per KV head, with 11 beyond that - see
 * LOSA_TUNE_HALF_PRECISION_VALUES, which also bounds |v| by 65504 there); float mode 1e-4. */
losa_status losa_sparse_attn(losa_ctx* ctx, void* stream, const losa_kv* kv, const void* q,
                             const int32_t* active_idx, const int32_t* active_count,
                             const int32_t* sel_pages, const int32_t* sel_count, int32_t cap,
                             void* o_p, float* lse_p);

/* One denoising step: step_index 0 = dense initialisation (all tokens, all pages; h_* unused
 * and may be NULL); otherwise (i) -> (ii-b) -> (iii) chained on `stream` with the
 * intermediate lists kept in the workspace.  The caller swaps h_cur / h_prev afterwards.
 *   mask      : nullable uint8 [batch*B]  (diagnostic: the active mask; untouched at step 0)
 *   sel_count : nullable int32 [batch, Hkv] (diagnostic: union sizes in pages; untouched at step 0) */
losa_status losa_step(losa_ctx* ctx, void* stream, const losa_kv* kv, int32_t step_index,
                      const void* h_cur, const void* h_prev, const void* q,
                      losa_select_mode mode, float param, int32_t topk_pages,
                      void* o_p, float* lse_p, uint8_t* mask, int32_t* sel_count);

/* (iv)+(v) Dense in-block attention and the final merge (Computation of the Suffix Tokens and
 * Final Output; eq. full_attn): for every token i of the block and query head h,
 *   s_b = sm_scale * q_{i,h} . k_b[t] over the B tokens t of the block (bidirectional),
 *   L_b = ln sum_t exp(s_b),  o_b = sum_t exp(s_b - L_b) v_b[t],
 *   out[i,h,:] = (e^{L_p} o_p + e^{L_b} o_b) / (e^{L_p} + e^{L_b})     with (o_p, L_p) as left by losa_step.
 *   q          : T [batch*B, Hq, d]
 *   k_b, v_b   : T [batch*B, Hkv, d]  keys / values of the block's own tokens (token-major, not paged)
 *   o_p, lse_p : float, inputs
 *   out        : float [batch*B, Hq, d]
 *   o_b, lse_b : nullable float [batch*B, Hq, d] / [batch*B, Hq]: the block statistics on their own */
losa_status losa_block_merge(losa_ctx* ctx, void* stream, int32_t batch, const void* q, const void* k_b,
                             const void* v_b, const float* o_p, const float* lse_p, float* out, float* o_b,
                             float* lse_b);

/* Tuning switches of a context: how the launches are shaped, never what they compute: every
 * decision (active set, picked pages, unions) is the same for every setting, and so is every
 * output bit except under the last two switches, which change the rounding order of the attention
 * over more than 64 query rows per KV head (outputs stay inside the bounds stated for losa_sparse_attn).
 * Each has a default chosen by measurement on MI355X; tests
 * use them to drive the code paths a workload of their size would not reach.  A value takes
 * effect with the next call on the context.
 *   LOSA_TUNE_ATTN_WORKGROUPS   : attention workgroups aimed at per launch (default 256: one per
 *                                 compute unit); 1..1024
 *   LOSA_TUNE_SELECT_ROUND      : selection workgroups counted as one round of the machine; a grid
 *                                 beyond it gives each workgroup up to four query rows (0: default)
 *   LOSA_TUNE_SCORE_ROUND       : the same for the scoring kernel (64-page tiles per workgroup); >= 1
 *   LOSA_TUNE_RANK_IN_SCORES    : 1 (default): inside losa_step the scoring kernel ranks the locality
 *                                 scores itself; 0: the locality kernel does, as in losa_select_active
 *   LOSA_TUNE_UNION_IN_ATTENTION: 1 (default): (sequence, KV head) pairs with up to 64 active query rows
 *                                 have the union of their picked pages built in the attention kernel;
 *                                 0: in the selection kernel, as in losa_score_pages
 *   LOSA_TUNE_SHARED_TILES      : 1 (default): above 64 query rows per KV head eight wavefronts share
 *                                 each key/value tile through LDS; 0: four independent wavefronts
 *   LOSA_TUNE_HALF_PRECISION_VALUES: 1 (default): in that shared-tile form the value product runs in
 *                                 half precision: probabilities rounded once to 11 significant bits
 *                                 (output error up to 2^-10 of the largest |v| a row attends to, in
 *                                 practice a tenth of that), values converted bfloat16 -> half, which
 *                                 is exact up to |v| = 65504 and saturates there; 0: probabilities as
 *                                 a bfloat16 pair (2^-16) and values in bfloat16's own range, at about
 *                                 a fifth more time.  Steps with up to 64 rows always take the pair. */
typedef enum {
  LOSA_TUNE_ATTN_WORKGROUPS = 0,
  LOSA_TUNE_SELECT_ROUND = 1,
  LOSA_TUNE_SCORE_ROUND = 2,
  LOSA_TUNE_RANK_IN_SCORES = 3,
  LOSA_TUNE_UNION_IN_ATTENTION = 4,
  LOSA_TUNE_SHARED_TILES = 5,
  LOSA_TUNE_HALF_PRECISION_VALUES = 6
} losa_tuning;
losa_status losa_set_tuning(losa_ctx* ctx, losa_tuning knob, int64_t value);

/* Measurement hooks (the paper's latency breakdown names four components: criticality
 * estimation, locality pruning, cache management, attention computation; cache management
 * costs nothing here because reuse is "do not write").  While enabled, every launch made
 * through this context is bracketed by HIP events on its stream.
 *   losa_profile_enable : enable != 0 creates the events (host objects), 0 releases them.
 *   losa_profile_read   : waits for the recorded events, adds up the elapsed milliseconds and
 *                         the launch count per stage into the two host arrays of
 *                         LOSA_NUM_STAGES entries, and clears the record. */
typedef enum {
  LOSA_STAGE_LOCALITY = 0, /* locality score + ranking kernels        ("locality pruning") */
  LOSA_STAGE_SCORE = 1,    /* page scoring kernel                      ("criticality estimation") */
  LOSA_STAGE_TOPK = 2,     /* top-k + union kernels                    ("criticality estimation") */
  LOSA_STAGE_ATTN = 3,     /* split-K attention kernel                 ("attention computation") */
  LOSA_STAGE_MERGE = 4,    /* split-K merge kernel                     ("attention computation") */
  LOSA_STAGE_BOUNDS = 5,   /* page min/max kernel (once per block) */
  LOSA_STAGE_BLOCK = 6,    /* in-block attention + final merge kernel */
  LOSA_NUM_STAGES = 7
} losa_stage;
losa_status losa_profile_enable(losa_ctx* ctx, int32_t enable);
losa_status losa_profile_read(losa_ctx* ctx, double* stage_ms, int64_t* stage_launches);
/* A plain device-to-device copy kernel of `bytes` bytes (a multiple of 16, both pointers
 * 16-byte aligned), enqueued on `stream`: the known-size reference that hardware byte
 * counters (FETCH_SIZE / WRITE_SIZE) are scaled by when the kernels above are profiled. */
losa_status losa_calibration_copy(void* dst, const void* src, size_t bytes, void* stream);

/* A read-only stream kernel, enqueued on `stream`: 256 workgroups of four wavefronts read `num_tiles`
 * tiles of `tile_bytes` bytes (a multiple of 16, at most 1 MiB) at pool + tile_ids[t] * tile_bytes, four
 * tiles in flight per wavefront, and write nothing (`sink`, 4 KiB of device memory, 16-byte aligned, is
 * only a formal destination).  The caller guarantees that every id addresses a tile inside the pool.  It
 * gives the read rate this GPU reaches on tiles of the page size, in order or scattered, which is
 * what the attention kernel's achieved bandwidth is set against beside the 8 TB/s peak. */
losa_status losa_calibration_read(const void* pool, size_t tile_bytes, const int32_t* tile_ids, int32_t num_tiles,
                                  void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LOSA_H */
