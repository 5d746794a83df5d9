// C ABI of liblosa.so: context, host-side validation, workspace carving and the launch
// sequences.  No device memory is allocated here; every call only enqueues kernels.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "losa_internal.h"

using namespace losa;

namespace losa {
__global__ void zero_ints_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}
hipError_t launch_zero_ints(hipStream_t st, int32_t* p, int n) {
  if (n <= 0) return hipSuccess;
  zero_ints_kernel<<<(n + 255) / 256, 256, 0, st>>>(p, n);
  return hipGetLastError();
}
__global__ __launch_bounds__(256) void calibration_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                               size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}
// Read-only stream over tiles of `tile16` 16-byte pieces picked by `ids` (tile t goes to wavefront
// t mod the number of wavefronts; four tiles in flight per wavefront).  Nothing is written: the sum
// of what was read is stored only if it has a value it never has.
__global__ __launch_bounds__(256) void calibration_read_kernel(const uint4* __restrict__ pool, int tile16,
                                                               const int32_t* __restrict__ ids, int ntiles,
                                                               uint4* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const int nwaves = gridDim.x * 4, w = blockIdx.x * 4 + (threadIdx.x >> 6);
  uint4 acc = make_uint4(0u, 0u, 0u, 0u);
  for (int t0 = w; t0 < ntiles; t0 += 4 * nwaves) {
    const uint4* src[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) src[k] = pool + (size_t)ids[min(t0 + k * nwaves, ntiles - 1)] * tile16;
    for (int i = lane; i < tile16; i += 64) {
      uint4 v[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {   // streaming loads, as the attention kernel reads its tiles
        typedef uint32_t cr_u32x4 __attribute__((ext_vector_type(4)));
        const cr_u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const cr_u32x4*>(src[k] + i));
        v[k] = make_uint4(x[0], x[1], x[2], x[3]);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const bool live = t0 + k * nwaves < ntiles;   // (the repeat of the last tile is read but not counted)
        acc.x ^= live ? v[k].x : 0u;
        acc.y ^= live ? v[k].y : 0u;
        acc.z ^= v[k].z;
        acc.w ^= v[k].w;
      }
    }
  }
  if (acc.x == 0x9E3779B9u && acc.y == 0x7F4A7C15u && acc.z == 0xF39CC060u && acc.w == 0x5CEDC834u) sink[threadIdx.x] = acc;
}
}  // namespace losa

struct losa_ctx {
  losa_config cfg;
  Shape sh;
  // workspace carve (device pointers)
  float* delta;
  uint8_t* mask;
  int32_t* active_idx;
  int32_t* active_count;
  float* scores;
  uint32_t* rowmaps;
  int32_t* tickets;
  int32_t* seq_tickets;   // [max_batch], kept at zero between launches
  bool seq_tickets_clean = false;
  int32_t* sel_pages;
  int32_t* sel_count;
  Partials part;
  long part_rows;           // capacity of the partial buffers in (work item, row) pairs
  long target_workgroups;   // attention workgroups aimed at per launch
  long select_round;        // selection workgroups per round (0: from the kernel's occupancy)
  long score_round;         // scoring workgroups the machine takes in one round
  bool rank_in_scores;      // losa_step lets the scoring kernel rank the locality scores
  bool union_in_attention;  // sparse steps of up to 64 rows: the attention kernel builds the union
  bool shared_tiles;        // more than 64 rows: 8 wavefronts share each tile through LDS (else 4 independent ones)
  bool half_values;         // ... and their value product runs in half precision (else P as a bfloat16 pair)
  AttnPrepared prep;
  char err[256];
  // measurement hooks
  bool profiling = false;
  std::vector<hipEvent_t> events;   // pool, used in pairs
  std::vector<int> rec_stage;       // stage of pair i
  size_t rec_used = 0;              // pairs recorded since the last read
};

namespace {

constexpr long kTargetItems = 1024;       // most split-K work items a sparse step may be given
constexpr long kTargetWorkgroups = 256;   // attention workgroups aimed at per launch: one per CU
constexpr int kSparseRows = 64;           // query rows per KV head up to which the split-pages work shape is used

thread_local char g_create_err[256] = "";

losa_status fail(losa_ctx* ctx, losa_status st, const char* fmt, ...) {
  char* dst = ctx ? ctx->err : g_create_err;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, 256, fmt, ap);
  va_end(ap);
  return st;
}

}  // namespace

namespace losa {
losa_status set_thread_error(losa_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_create_err, sizeof g_create_err, fmt, ap);
  va_end(ap);
  return st;
}
}  // namespace losa

namespace {

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// LOSA_OK, or what is wrong with the configuration: LOSA_ERR_INVALID_ARG for values that make
// no sense, LOSA_ERR_UNSUPPORTED for sensible ones outside what the kernels are built for.
losa_status config_problem(const losa_config* c, char* why, size_t n) {
#define BAD(cond, code, msg)      \
  if (cond) {                     \
    snprintf(why, n, "%s", msg);  \
    return code;                  \
  }
  const losa_status inv = LOSA_ERR_INVALID_ARG, uns = LOSA_ERR_UNSUPPORTED;
  BAD(!c, inv, "config is NULL");
  BAD(c->max_batch < 1, inv, "max_batch must be >= 1");
  BAD(c->num_q_heads < 1 || c->num_kv_heads < 1, inv, "head counts must be >= 1");
  BAD(c->num_q_heads % c->num_kv_heads != 0, inv, "num_q_heads must be a multiple of num_kv_heads");
  BAD(c->head_dim < 1 || c->page_size < 1 || c->block_size < 1 || c->hidden_size < 1 || c->max_pages_per_seq < 1, inv,
      "head_dim, page_size, block_size, hidden_size and max_pages_per_seq must be >= 1");
  BAD(c->max_topk_pages < 1, inv, "max_topk_pages must be >= 1");
  BAD(c->dtype != LOSA_BF16 && c->dtype != LOSA_F32, inv, "dtype must be LOSA_BF16 or LOSA_F32");
  BAD(!(c->sm_scale >= 0.f) || isinf(c->sm_scale), inv, "sm_scale must be finite and >= 0");
  BAD(c->head_dim != 64 && c->head_dim != 128, uns, "head_dim must be 64 or 128");
  BAD(c->page_size != 16 && c->page_size != 32, uns, "page_size must be 16 or 32");
  BAD(c->block_size > 256, uns, "block_size must be in 1..256");
  BAD(c->hidden_size % 8 != 0, uns, "hidden_size must be a multiple of 8");
  BAD(c->max_pages_per_seq > kMaxSelectPages, uns, "max_pages_per_seq must be in 1..16384");
  BAD((long)c->block_size * (c->num_q_heads / c->num_kv_heads) > 4096, uns, "block_size * group size must be <= 4096");
#undef BAD
  return LOSA_OK;
}

struct Carve {
  size_t off = 0;
  size_t take(size_t bytes) {
    const size_t at = off;
    off = align256(off + bytes);
    return at;
  }
};

struct Layout {
  size_t delta, mask, active_idx, active_count, scores, rowmaps, tickets, sel_pages, sel_count, po, pm, pl;
  size_t entries, q_act, ucount, mrows, seq_tickets, total;
  long part_rows;   // capacity of the split-K partial buffers, in (work item, query row) pairs
};

Layout make_layout(const losa_config* c) {
  Layout L;
  Carve cv;
  const size_t rows = (size_t)c->max_batch * c->block_size;
  const size_t G = c->num_q_heads / c->num_kv_heads;
  const size_t rows_max = (size_t)c->block_size * G;
  const size_t heads = (size_t)c->max_batch * c->num_kv_heads;
  const size_t words = ((size_t)c->max_pages_per_seq + 31) / 32;
  // Split-K partials: a sparse step has at most kSparseRows query rows per KV head and may use up to
  // kTargetItems work items; a launch with more rows (the dense initialisation, large active sets)
  // aims at kTargetWorkgroups work items (or one per head if there are more heads than that).
  {
    const long few = kTargetItems * (long)(rows_max < (size_t)kSparseRows ? rows_max : (size_t)kSparseRows);
    const long many = ((long)heads > kTargetWorkgroups ? (long)heads : kTargetWorkgroups) * (long)rows_max;
    L.part_rows = few > many ? few : many;
  }
  L.delta = cv.take(rows * 4);
  L.mask = cv.take(rows);
  L.active_idx = cv.take(rows * 4);
  L.active_count = cv.take((size_t)c->max_batch * 4);
  L.scores = cv.take(heads * rows_max * c->max_pages_per_seq * 4);
  L.rowmaps = cv.take(heads * (rows_max > (size_t)kUnionRows ? rows_max : (size_t)kUnionRows) * words * 4);   // row-major [rows_max] or word-major [kUnionRows] per word
  L.tickets = cv.take(heads * 4);
  L.sel_pages = cv.take(heads * c->max_pages_per_seq * 4);
  L.sel_count = cv.take(heads * 4);
  L.po = cv.take((size_t)L.part_rows * c->head_dim * 4);
  L.pm = cv.take((size_t)L.part_rows * 4);
  L.pl = cv.take((size_t)L.part_rows * 4);
  L.entries = cv.take(heads * c->max_pages_per_seq * 4);
  L.q_act = cv.take(heads * rows_max * c->head_dim * 2);
  L.ucount = cv.take(heads * 4);
  L.mrows = cv.take(heads * 4);
  L.seq_tickets = cv.take((size_t)c->max_batch * 4);
  L.total = cv.off;
  return L;
}

hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

constexpr size_t kMaxProfilePairs = 16384;

// Brackets the launches made in its scope with a pair of events when profiling is on.
struct StageTimer {
  losa_ctx* ctx;
  hipStream_t st;
  size_t pair = (size_t)-1;
  bool bound = false;   // the pair was handed to a launch that binds it to its dispatch
  StageTimer(losa_ctx* c, hipStream_t s, int stage, bool bind_to_dispatch = false)
      : ctx(c), st(s), bound(bind_to_dispatch) {
    if (!ctx->profiling || ctx->rec_used >= kMaxProfilePairs) return;
    pair = ctx->rec_used++;
    ctx->rec_stage[pair] = stage;
    if (!bound) (void)hipEventRecord(ctx->events[2 * pair], st);
  }
  hipEvent_t start() const { return pair != (size_t)-1 ? ctx->events[2 * pair] : nullptr; }
  hipEvent_t stop() const { return pair != (size_t)-1 ? ctx->events[2 * pair + 1] : nullptr; }
  ~StageTimer() {
    if (pair != (size_t)-1 && !bound) (void)hipEventRecord(ctx->events[2 * pair + 1], st);
  }
};

losa_status check_kv(losa_ctx* ctx, const losa_kv* kv, bool need_meta, int* max_seq_pages) {
  if (!kv) return fail(ctx, LOSA_ERR_INVALID_ARG, "kv is NULL");
  if (kv->batch < 1 || kv->batch > ctx->cfg.max_batch)
    return fail(ctx, LOSA_ERR_INVALID_ARG, "kv.batch %d outside 1..max_batch (%d)", kv->batch, ctx->cfg.max_batch);
  if (!kv->k_pages || !kv->v_pages || !kv->page_indptr || !kv->page_indices || !kv->seq_lens)
    return fail(ctx, LOSA_ERR_INVALID_ARG, "kv has a NULL device pointer");
  if (need_meta && !kv->meta) return fail(ctx, LOSA_ERR_INVALID_ARG, "kv.meta is NULL");
  if (kv->num_pages < 1 || kv->num_pages > (1 << kEntryShift))
    return fail(ctx, LOSA_ERR_INVALID_ARG, "kv.num_pages must be in 1..2^26");
  if (kv->max_seq_pages < 0 || kv->max_seq_pages > ctx->cfg.max_pages_per_seq)
    return fail(ctx, LOSA_ERR_INVALID_ARG, "kv.max_seq_pages %d outside 0..max_pages_per_seq (%d)", kv->max_seq_pages,
                ctx->cfg.max_pages_per_seq);
  *max_seq_pages = kv->max_seq_pages > 0 ? kv->max_seq_pages : ctx->cfg.max_pages_per_seq;
  return LOSA_OK;
}

KvView view_of(const losa_kv* kv, int max_seq_pages) {
  KvView v;
  v.k_pages = kv->k_pages;
  v.v_pages = kv->v_pages;
  v.meta = kv->meta;
  v.page_indptr = kv->page_indptr;
  v.page_indices = kv->page_indices;
  v.seq_lens = kv->seq_lens;
  v.num_pages = kv->num_pages;
  v.seq_page_limit = max_seq_pages;
  return v;
}

losa_status hip_fail(losa_ctx* ctx, const char* what, hipError_t e) {
  return fail(ctx, LOSA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// Number of equal shares a (sequence, KV head) page list of at most `upper` pages is split into,
// when every work item holds `part_stride` rows of partials.
int pick_nchunk(const losa_ctx* ctx, int batch, int upper, int row_groups, int part_stride) {
  const long heads = (long)batch * ctx->sh.Hkv;
  const long tiles = (upper + (32 / ctx->sh.g) - 1) / (32 / ctx->sh.g);
  long want = ctx->target_workgroups / (heads * row_groups);
  const long fit = ctx->part_rows / (heads * part_stride);
  if (want > fit) want = fit;
  if (want > tiles) want = tiles;
  if (want < 1) want = 1;
  return (int)want;
}

// |A| for the top-n modes (TOPK, FRACTION); the caller has validated param.
int select_count(const losa_ctx* ctx, int mode, float param) {
  const int B = ctx->sh.B;
  if (mode == LOSA_SEL_TOPK) return param >= (float)B ? B : (int)param;
  int n = (int)floorf(param * (float)B + 0.5f);
  return n < 1 ? 1 : (n > B ? B : n);
}

// Checks (mode, param) and turns them into what the kernels take: a count n or a threshold tau.
losa_status parse_select(losa_ctx* ctx, int mode, float param, int* n, float* tau) {
  *n = 0;
  *tau = 0.f;
  if (mode == LOSA_SEL_TOPK) {
    if (!(param >= 0.f)) return fail(ctx, LOSA_ERR_INVALID_ARG, "top-k parameter must be >= 0");
    *n = select_count(ctx, mode, param);
  } else if (mode == LOSA_SEL_FRACTION) {
    if (!(param >= 0.f && param <= 1.f)) return fail(ctx, LOSA_ERR_INVALID_ARG, "fraction must be in [0,1]");
    *n = select_count(ctx, mode, param);
  } else if (mode == LOSA_SEL_THRESHOLD) {
    if (isnan(param)) return fail(ctx, LOSA_ERR_INVALID_ARG, "threshold is NaN");
    *tau = param;
  } else if (mode == LOSA_SEL_MASS) {
    if (!(param >= 0.f && param <= 1.f)) return fail(ctx, LOSA_ERR_INVALID_ARG, "mass fraction must be in [0,1]");
    *tau = param;
  } else {
    return fail(ctx, LOSA_ERR_INVALID_ARG, "unknown select mode %d", mode);
  }
  return LOSA_OK;
}

losa_status select_active_impl(losa_ctx* ctx, hipStream_t st, int batch, const void* h_cur, const void* h_prev,
                               int mode, float param, float* delta, uint8_t* mask, int32_t* active_idx,
                               int32_t* active_count) {
  const int B = ctx->sh.B;
  int n = 0;
  float tau = 0.f;
  const losa_status ps = parse_select(ctx, mode, param, &n, &tau);
  if (ps != LOSA_OK) return ps;
  StageTimer timer(ctx, st, LOSA_STAGE_LOCALITY);
  hipError_t e;
  if (!ctx->seq_tickets_clean) {   // first use: the ticket counters must start at zero; the kernel leaves them so
    e = launch_zero_ints(st, ctx->seq_tickets, ctx->cfg.max_batch);
    if (e != hipSuccess) return hip_fail(ctx, "ticket clear launch", e);
    ctx->seq_tickets_clean = true;
  }
  e = launch_locality_select(st, ctx->cfg.dtype, h_cur, h_prev, batch, B, ctx->sh.H, mode, n, tau, delta, mask,
                             active_idx, active_count, ctx->seq_tickets);
  if (e != hipSuccess) return hip_fail(ctx, "locality_select launch", e);
  return LOSA_OK;
}

losa_status score_pages_impl(losa_ctx* ctx, hipStream_t st, const KvView& kv, int batch, int max_seq_pages,
                             const void* q, const int32_t* active_idx, const int32_t* active_count, int topk,
                             int32_t* topk_out, int32_t* sel_pages, int32_t* sel_count, int cap, bool prepare_attn,
                             int rows_upper, const InKernelRanking* ranking = nullptr, bool bitmaps_only = false) {
  const AttnPrepared* prep = prepare_attn ? &ctx->prep : nullptr;
  hipError_t e;
  {
    StageTimer timer(ctx, st, LOSA_STAGE_SCORE);
    e = launch_page_scores(st, ctx->cfg.dtype, kv, ctx->sh, batch, max_seq_pages, q, active_idx, active_count,
                           ctx->scores, ctx->tickets, sel_count, prep, ranking, ctx->score_round);
  }
  if (e != hipSuccess) return hip_fail(ctx, "page_scores launch", e);
  StageTimer timer(ctx, st, LOSA_STAGE_TOPK);
  e = launch_select_pages(st, kv, ctx->sh, batch, max_seq_pages, q, active_idx, active_count, ctx->scores, topk,
                          topk_out, sel_pages, sel_count, cap, ctx->rowmaps, ctx->tickets, prep, rows_upper,
                          ctx->select_round, bitmaps_only);
  if (e != hipSuccess) return hip_fail(ctx, "select_pages launch", e);
  return LOSA_OK;
}

losa_status sparse_attn_impl(losa_ctx* ctx, hipStream_t st, const KvView& kv, int batch, int max_seq_pages,
                             const void* q, const int32_t* active_idx, const int32_t* active_count,
                             const int32_t* sel_pages, const int32_t* sel_count, int cap, int rows_upper,
                             bool prepared, float* o_p, float* lse_p, const UnionInKernel* uni = nullptr) {
  const int upper = sel_pages ? (cap < max_seq_pages ? cap : max_seq_pages) : max_seq_pages;
  const bool mfma = ctx->cfg.dtype == LOSA_BF16;
  if (!active_idx) rows_upper = ctx->sh.rows_max;   // every token is active: the count is known
  const bool hinted = rows_upper >= 1 && rows_upper <= ctx->sh.rows_max;
  if (!hinted) rows_upper = ctx->sh.rows_max;
  // Row count known only on the device (threshold / cumulative-mass selection): both work shapes
  // of the matrix-core kernel are launched, each serving the (sequence, head) pairs whose count
  // falls in its range, so that a small active set still gets the shape built for it.  Needs
  // the two shapes to agree on the number of chunks, which they do up to 256 rows.
  const bool both_shapes = mfma && !hinted && ctx->sh.rows_max > 64 && ctx->sh.rows_max <= 256;
  // matrix-core kernel: up to 64 rows ride in one workgroup; more rows -> groups of 4 x 64 rows
  const int row_groups = mfma ? (rows_upper <= 64 ? 1 : (ctx->sh.rows_max + 255) / 256) : (ctx->sh.rows_max + 31) / 32;
  // rows of partials per work item: what the host knows the row count cannot exceed
  Partials part = ctx->part;
  part.rows = hinted ? (rows_upper + 15) / 16 * 16 : ctx->sh.rows_max;
  if (part.rows > ctx->sh.rows_max) part.rows = ctx->sh.rows_max;
  const int nchunk = pick_nchunk(ctx, batch, upper, mfma ? row_groups : 1, part.rows);
  hipError_t e;
  if (mfma && !prepared) {
    StageTimer timer(ctx, st, LOSA_STAGE_TOPK);
    e = launch_attn_prepare(st, kv, ctx->sh, batch, q, active_idx, active_count, sel_pages, sel_count, cap, ctx->prep);
    if (e != hipSuccess) return hip_fail(ctx, "attn_prepare launch", e);
  }
  {
    StageTimer timer(ctx, st, LOSA_STAGE_ATTN, /*bind_to_dispatch=*/mfma && !both_shapes);
    const int many_rows = !ctx->shared_tiles ? kManyRowsIndependent
                                             : (ctx->half_values ? kManyRowsSharedHalf : kManyRowsSharedPair);
    if (both_shapes) {
      e = launch_attn_mfma(st, kv, ctx->sh, batch, ctx->prep, nchunk, 64, part, nullptr, nullptr, 0, 64, uni,
                           many_rows);
      if (e == hipSuccess)
        e = launch_attn_mfma(st, kv, ctx->sh, batch, ctx->prep, nchunk, ctx->sh.rows_max, part, nullptr, nullptr,
                             64, 0x7fffffff, nullptr, many_rows);
    } else if (mfma)
      e = launch_attn_mfma(st, kv, ctx->sh, batch, ctx->prep, nchunk, rows_upper, part, timer.start(),
                           timer.stop(), 0, 0x7fffffff, uni, many_rows);
    else
      e = launch_attn_generic(st, ctx->cfg.dtype, kv, ctx->sh, batch, q, active_idx, active_count, sel_pages,
                              sel_count, cap, nchunk, part);
  }
  if (e != hipSuccess) return hip_fail(ctx, "attention launch", e);
  StageTimer timer(ctx, st, LOSA_STAGE_MERGE);
  e = launch_attn_merge(st, kv, ctx->sh, batch, active_idx, active_count, sel_count, cap, nchunk,
                        mfma ? &ctx->prep : nullptr, part, o_p, lse_p, hinted ? rows_upper : 0);
  if (e != hipSuccess) return hip_fail(ctx, "attn_merge launch", e);
  return LOSA_OK;
}

}  // namespace

extern "C" {

size_t losa_workspace_bytes(const losa_config* cfg) {
  char why[128];
  if (config_problem(cfg, why, sizeof why) != LOSA_OK) return 0;
  return make_layout(cfg).total;
}

losa_status losa_create(const losa_config* cfg, void* workspace, size_t workspace_bytes, losa_ctx** out) {
  if (!out) return fail(nullptr, LOSA_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  char why[128];
  const losa_status cs = config_problem(cfg, why, sizeof why);
  if (cs != LOSA_OK) return fail(nullptr, cs, "%s", why);
  const Layout L = make_layout(cfg);
  if (!workspace) return fail(nullptr, LOSA_ERR_WORKSPACE, "workspace is NULL");
  if (((uintptr_t)workspace & 255u) != 0) return fail(nullptr, LOSA_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (workspace_bytes < L.total)
    return fail(nullptr, LOSA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, L.total);
  losa_ctx* ctx = new (std::nothrow) losa_ctx();
  if (!ctx) return fail(nullptr, LOSA_ERR_INVALID_ARG, "out of host memory");
  ctx->cfg = *cfg;
  Shape& sh = ctx->sh;
  sh.Hq = cfg->num_q_heads;
  sh.Hkv = cfg->num_kv_heads;
  sh.G = sh.Hq / sh.Hkv;
  sh.d = cfg->head_dim;
  sh.H = cfg->hidden_size;
  sh.g = cfg->page_size;
  sh.B = cfg->block_size;
  sh.max_pages = cfg->max_pages_per_seq;
  sh.rows_max = sh.B * sh.G;
  sh.sm_scale = cfg->sm_scale > 0.f ? cfg->sm_scale : 1.0f / sqrtf((float)sh.d);
  char* base = static_cast<char*>(workspace);
  ctx->delta = (float*)(base + L.delta);
  ctx->mask = (uint8_t*)(base + L.mask);
  ctx->active_idx = (int32_t*)(base + L.active_idx);
  ctx->active_count = (int32_t*)(base + L.active_count);
  ctx->scores = (float*)(base + L.scores);
  ctx->rowmaps = (uint32_t*)(base + L.rowmaps);
  ctx->tickets = (int32_t*)(base + L.tickets);
  ctx->sel_pages = (int32_t*)(base + L.sel_pages);
  ctx->sel_count = (int32_t*)(base + L.sel_count);
  ctx->part.o = (float*)(base + L.po);
  ctx->part.m = (float*)(base + L.pm);
  ctx->part.l = (float*)(base + L.pl);
  ctx->part.rows = sh.rows_max;
  ctx->part_rows = L.part_rows;
  ctx->target_workgroups = kTargetWorkgroups;
  ctx->rank_in_scores = true;
  ctx->select_round = 0;
  ctx->score_round = 5L * 256;   // about five scoring workgroups per CU are resident at once
  ctx->union_in_attention = true;
  ctx->shared_tiles = true;
  ctx->half_values = true;
  ctx->prep.entries = (int32_t*)(base + L.entries);
  ctx->prep.q_act = (uint16_t*)(base + L.q_act);
  ctx->prep.ucount = (int32_t*)(base + L.ucount);
  ctx->prep.mrows = (int32_t*)(base + L.mrows);
  ctx->seq_tickets = (int32_t*)(base + L.seq_tickets);
  ctx->err[0] = 0;
  *out = ctx;
  return LOSA_OK;
}

losa_status losa_destroy(losa_ctx* ctx) {
  if (ctx) losa_profile_enable(ctx, 0);
  delete ctx;
  return LOSA_OK;
}

losa_status losa_set_tuning(losa_ctx* ctx, losa_tuning knob, int64_t value) {
  if (!ctx) return LOSA_ERR_INVALID_ARG;
  switch (knob) {
    case LOSA_TUNE_ATTN_WORKGROUPS:
      if (value < 1 || value > kTargetItems)
        return fail(ctx, LOSA_ERR_INVALID_ARG, "attention workgroups must be in 1..%ld", kTargetItems);
      ctx->target_workgroups = (long)value;
      return LOSA_OK;
    case LOSA_TUNE_SELECT_ROUND:
      if (value < 0) return fail(ctx, LOSA_ERR_INVALID_ARG, "selection round must be >= 0");
      ctx->select_round = (long)value;
      return LOSA_OK;
    case LOSA_TUNE_SCORE_ROUND:
      if (value < 1) return fail(ctx, LOSA_ERR_INVALID_ARG, "scoring round must be >= 1");
      ctx->score_round = (long)value;
      return LOSA_OK;
    case LOSA_TUNE_RANK_IN_SCORES: ctx->rank_in_scores = value != 0; return LOSA_OK;
    case LOSA_TUNE_UNION_IN_ATTENTION: ctx->union_in_attention = value != 0; return LOSA_OK;
    case LOSA_TUNE_SHARED_TILES: ctx->shared_tiles = value != 0; return LOSA_OK;
    case LOSA_TUNE_HALF_PRECISION_VALUES: ctx->half_values = value != 0; return LOSA_OK;
  }
  return fail(ctx, LOSA_ERR_INVALID_ARG, "unknown tuning switch %d", (int)knob);
}

losa_status losa_profile_enable(losa_ctx* ctx, int32_t enable) {
  if (!ctx) return LOSA_ERR_INVALID_ARG;
  if (enable && ctx->events.empty()) {
    ctx->events.resize(2 * kMaxProfilePairs, nullptr);
    ctx->rec_stage.assign(kMaxProfilePairs, 0);
    for (size_t i = 0; i < ctx->events.size(); ++i) {
      hipError_t e = hipEventCreate(&ctx->events[i]);
      if (e != hipSuccess) {
        for (size_t k = 0; k < i; ++k) (void)hipEventDestroy(ctx->events[k]);
        ctx->events.clear();
        return hip_fail(ctx, "hipEventCreate", e);
      }
    }
  }
  if (!enable && !ctx->events.empty()) {
    for (hipEvent_t ev : ctx->events) (void)hipEventDestroy(ev);
    ctx->events.clear();
  }
  ctx->profiling = enable != 0;
  ctx->rec_used = 0;
  return LOSA_OK;
}

losa_status losa_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || (bytes & 15) != 0 || (((uintptr_t)dst | (uintptr_t)src) & 15) != 0) return LOSA_ERR_INVALID_ARG;
  if (bytes == 0) return LOSA_OK;
  calibration_copy_kernel<<<2048, 256, 0, as_stream(stream)>>>((uint4*)dst, (const uint4*)src, bytes / 16);
  return hipGetLastError() == hipSuccess ? LOSA_OK : LOSA_ERR_HIP;
}

losa_status losa_calibration_read(const void* pool, size_t tile_bytes, const int32_t* tile_ids, int32_t num_tiles,
                                  void* sink, void* stream) {
  if (!pool || !tile_ids || !sink || tile_bytes == 0 || (tile_bytes & 15) != 0 || tile_bytes > (1u << 20) ||
      (((uintptr_t)pool | (uintptr_t)sink) & 15) != 0 || num_tiles < 0)
    return LOSA_ERR_INVALID_ARG;
  if (num_tiles == 0) return LOSA_OK;
  calibration_read_kernel<<<256, 256, 0, as_stream(stream)>>>((const uint4*)pool, (int)(tile_bytes / 16), tile_ids,
                                                              num_tiles, (uint4*)sink);
  return hipGetLastError() == hipSuccess ? LOSA_OK : LOSA_ERR_HIP;
}

losa_status losa_profile_read(losa_ctx* ctx, double* stage_ms, int64_t* stage_launches) {
  if (!ctx || !stage_ms || !stage_launches) return LOSA_ERR_INVALID_ARG;
  for (int s = 0; s < LOSA_NUM_STAGES; ++s) {
    stage_ms[s] = 0.0;
    stage_launches[s] = 0;
  }
  for (size_t i = 0; i < ctx->rec_used; ++i) {
    hipError_t e = hipEventSynchronize(ctx->events[2 * i + 1]);
    if (e != hipSuccess) return hip_fail(ctx, "hipEventSynchronize", e);
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, ctx->events[2 * i], ctx->events[2 * i + 1]);
    if (e != hipSuccess) return hip_fail(ctx, "hipEventElapsedTime", e);
    stage_ms[ctx->rec_stage[i]] += ms;
    stage_launches[ctx->rec_stage[i]] += 1;
  }
  ctx->rec_used = 0;
  return LOSA_OK;
}

const char* losa_last_error(const losa_ctx* ctx) { return ctx ? ctx->err : g_create_err; }

losa_status losa_select_active(losa_ctx* ctx, void* stream, int32_t batch, const void* h_cur, const void* h_prev,
                               losa_select_mode mode, float param, float* delta, uint8_t* mask, int32_t* active_idx,
                               int32_t* active_count) {
  if (!ctx) return LOSA_ERR_INVALID_ARG;
  if (batch < 1 || batch > ctx->cfg.max_batch)
    return fail(ctx, LOSA_ERR_INVALID_ARG, "batch %d outside 1..max_batch (%d)", batch, ctx->cfg.max_batch);
  if (!h_cur || !h_prev || !delta || !mask || !active_idx || !active_count)
    return fail(ctx, LOSA_ERR_INVALID_ARG, "losa_select_active: NULL pointer");
  return select_active_impl(ctx, as_stream(stream), batch, h_cur, h_prev, (int)mode, param, delta, mask, active_idx,
                            active_count);
}

losa_status losa_page_bounds(losa_ctx* ctx, void* stream, const losa_kv* kv, int32_t first_logical_page,
                             int32_t num_logical_pages) {
  if (!ctx) return LOSA_ERR_INVALID_ARG;
  int msp;
  losa_status s = check_kv(ctx, kv, true, &msp);
  if (s != LOSA_OK) return s;
  if (first_logical_page < 0) return fail(ctx, LOSA_ERR_INVALID_ARG, "first_logical_page is negative");
  int n = msp - first_logical_page;
  if (num_logical_pages >= 0 && num_logical_pages < n) n = num_logical_pages;
  if (n <= 0) return LOSA_OK;
  StageTimer timer(ctx, as_stream(stream), LOSA_STAGE_BOUNDS);
  hipError_t e = launch_page_bounds(as_stream(stream), ctx->cfg.dtype, view_of(kv, msp), ctx->sh, kv->batch,
                                    first_logical_page, n);
  if (e != hipSuccess) return hip_fail(ctx, "page_bounds launch", e);
  return LOSA_OK;
}

losa_status losa_score_pages(losa_ctx* ctx, void* stream, const losa_kv* kv, const void* q, const int32_t* active_idx,
                             const int32_t* active_count, int32_t topk_pages, int32_t* topk_out, int32_t* sel_pages,
                             int32_t* sel_count, int32_t cap) {
  if (!ctx) return LOSA_ERR_INVALID_ARG;
  int msp;
  losa_status s = check_kv(ctx, kv, true, &msp);
  if (s != LOSA_OK) return s;
  if (!q || !active_idx || !active_count || !sel_pages || !sel_count)
    return fail(ctx, LOSA_ERR_INVALID_ARG, "losa_score_pages: NULL pointer");
  if (topk_pages < 1 || topk_pages > ctx->cfg.max_topk_pages)
    return fail(ctx, LOSA_ERR_INVALID_ARG, "topk_pages %d outside 1..max_topk_pages (%d)", topk_pages,
                ctx->cfg.max_topk_pages);
  const long worst = (long)ctx->sh.rows_max * topk_pages;
  const long need = worst < msp ? worst : msp;
  if (cap < need) return fail(ctx, LOSA_ERR_INVALID_ARG, "cap %d is below the union's worst case %ld", cap, need);
  return score_pages_impl(ctx, as_stream(stream), view_of(kv, msp), kv->batch, msp, q, active_idx, active_count,
                          topk_pages, topk_out, sel_pages, sel_count, cap, /*prepare_attn=*/false, /*rows_upper=*/0);
}

losa_status losa_score_pages_shared(losa_ctx* ctx, void* stream, const losa_kv* kv, const void* q,
                                    const int32_t* active_idx, const int32_t* active_count, int32_t topk_pages,
                                    int32_t* sel_pages, int32_t* sel_count, int32_t cap) {
  if (!ctx) return LOSA_ERR_INVALID_ARG;
  int msp;
  losa_status s = check_kv(ctx, kv, true, &msp);
  if (s != LOSA_OK) return s;
  if (!q || !active_idx || !active_count || !sel_pages || !sel_count)
    return fail(ctx, LOSA_ERR_INVALID_ARG, "losa_score_pages_shared: NULL pointer");
  if (topk_pages < 1 || topk_pages > ctx->cfg.max_topk_pages)
    return fail(ctx, LOSA_ERR_INVALID_ARG, "topk_pages %d outside 1..max_topk_pages (%d)", topk_pages,
                ctx->cfg.max_topk_pages);
  const int need = topk_pages < msp ? topk_pages : msp;
  if (cap < need) return fail(ctx, LOSA_ERR_INVALID_ARG, "cap %d is below min(pages, topk_pages) = %d", cap, need);
  hipStream_t st = as_stream(stream);
  const KvView view = view_of(kv, msp);
  hipError_t e;
  {
    StageTimer timer(ctx, st, LOSA_STAGE_SCORE);
    e = launch_page_scores(st, ctx->cfg.dtype, view, ctx->sh, kv->batch, msp, q, active_idx, active_count, ctx->scores,
                           ctx->tickets, sel_count, nullptr, nullptr, ctx->score_round);
  }
  if (e != hipSuccess) return hip_fail(ctx, "page_scores launch", e);
  StageTimer timer(ctx, st, LOSA_STAGE_TOPK);
  e = launch_shared_select(st, view, ctx->sh, kv->batch, msp, active_count, ctx->scores, topk_pages, sel_pages,
                           sel_count, cap);
  if (e != hipSuccess) return hip_fail(ctx, "shared_select launch", e);
  return LOSA_OK;
}

losa_status losa_sparse_attn(losa_ctx* ctx, void* stream, const losa_kv* kv, const void* q, const int32_t* active_idx,
                             const int32_t* active_count, const int32_t* sel_pages, const int32_t* sel_count,
                             int32_t cap, void* o_p, float* lse_p) {
  if (!ctx) return LOSA_ERR_INVALID_ARG;
  int msp;
  losa_status s = check_kv(ctx, kv, false, &msp);
  if (s != LOSA_OK) return s;
  if (!q || !o_p || !lse_p) return fail(ctx, LOSA_ERR_INVALID_ARG, "losa_sparse_attn: NULL pointer");
  if ((active_idx == nullptr) != (active_count == nullptr))
    return fail(ctx, LOSA_ERR_INVALID_ARG, "active_idx and active_count must both be given or both be NULL");
  if ((sel_pages == nullptr) != (sel_count == nullptr))
    return fail(ctx, LOSA_ERR_INVALID_ARG, "sel_pages and sel_count must both be given or both be NULL");
  if (sel_pages && cap < 1) return fail(ctx, LOSA_ERR_INVALID_ARG, "cap must be >= 1");
  return sparse_attn_impl(ctx, as_stream(stream), view_of(kv, msp), kv->batch, msp, q, active_idx, active_count, sel_pages,
                          sel_count, cap, /*rows_upper=*/0, /*prepared=*/false, (float*)o_p, lse_p);
}

losa_status losa_block_merge(losa_ctx* ctx, void* stream, int32_t batch, const void* q, const void* k_b,
                             const void* v_b, const float* o_p, const float* lse_p, float* out, float* o_b,
                             float* lse_b) {
  if (!ctx) return LOSA_ERR_INVALID_ARG;
  if (batch < 1 || batch > ctx->cfg.max_batch)
    return fail(ctx, LOSA_ERR_INVALID_ARG, "batch %d outside 1..max_batch (%d)", batch, ctx->cfg.max_batch);
  if (!q || !k_b || !v_b || !o_p || !lse_p || !out) return fail(ctx, LOSA_ERR_INVALID_ARG, "losa_block_merge: NULL pointer");
  hipStream_t st = as_stream(stream);
  StageTimer timer(ctx, st, LOSA_STAGE_BLOCK);
  hipError_t e = launch_block_merge(st, ctx->cfg.dtype, ctx->sh, batch, q, k_b, v_b, o_p, lse_p, out, o_b, lse_b);
  if (e != hipSuccess) return hip_fail(ctx, "block_merge launch", e);
  return LOSA_OK;
}

losa_status losa_step(losa_ctx* ctx, void* stream, const losa_kv* kv, int32_t step_index, const void* h_cur,
                      const void* h_prev, const void* q, losa_select_mode mode, float param, int32_t topk_pages,
                      void* o_p, float* lse_p, uint8_t* mask, int32_t* sel_count) {
  if (!ctx) return LOSA_ERR_INVALID_ARG;
  int msp;
  const bool dense = step_index == 0;
  losa_status s = check_kv(ctx, kv, !dense, &msp);
  if (s != LOSA_OK) return s;
  if (step_index < 0) return fail(ctx, LOSA_ERR_INVALID_ARG, "step_index is negative");
  if (!q || !o_p || !lse_p) return fail(ctx, LOSA_ERR_INVALID_ARG, "losa_step: NULL pointer");
  hipStream_t st = as_stream(stream);
  const KvView view = view_of(kv, msp);
  if (dense)
    return sparse_attn_impl(ctx, st, view, kv->batch, msp, q, nullptr, nullptr, nullptr, nullptr, 0, 0, false,
                            (float*)o_p, lse_p);
  if (!h_cur || !h_prev) return fail(ctx, LOSA_ERR_INVALID_ARG, "losa_step: h_cur / h_prev are NULL");
  if (topk_pages < 1 || topk_pages > ctx->cfg.max_topk_pages)
    return fail(ctx, LOSA_ERR_INVALID_ARG, "topk_pages %d outside 1..max_topk_pages (%d)", topk_pages,
                ctx->cfg.max_topk_pages);
  uint8_t* mk = mask ? mask : ctx->mask;
  int32_t* sc = sel_count ? sel_count : ctx->sel_count;
  // Where the scoring kernel can rank the locality scores itself, the locality launch only
  // computes them: its end-of-kernel hand-over (store, wait, ticket, reload, rank) drops out
  // of the step's chain of dependent launches.
  InKernelRanking ranking{ctx->delta, (int)mode, 0, 0.f, mk, ctx->active_idx, ctx->active_count};
  const bool rank_in_scores = ctx->rank_in_scores && ctx->cfg.dtype == LOSA_BF16 && ctx->sh.B <= 256;
  if (rank_in_scores) {
    s = parse_select(ctx, (int)mode, param, &ranking.n, &ranking.tau);
    if (s != LOSA_OK) return s;
    StageTimer timer(ctx, st, LOSA_STAGE_LOCALITY);
    hipError_t e = launch_locality_delta(st, ctx->cfg.dtype, h_cur, h_prev, kv->batch, ctx->sh.B, ctx->sh.H, ctx->delta);
    if (e != hipSuccess) return hip_fail(ctx, "locality_delta launch", e);
  } else {
    s = select_active_impl(ctx, st, kv->batch, h_cur, h_prev, (int)mode, param, ctx->delta, mk, ctx->active_idx,
                           ctx->active_count);
    if (s != LOSA_OK) return s;
  }
  const int cap = ctx->sh.max_pages;
  const bool fuse_prepare = ctx->cfg.dtype == LOSA_BF16;   // the selection kernel also builds the attention inputs
  // the host knows |A| in the top-n modes, so selection and attention can be shaped for n*G rows
  const bool counted = mode == LOSA_SEL_TOPK || mode == LOSA_SEL_FRACTION;
  const int rows_upper = counted ? select_count(ctx, (int)mode, param) * ctx->sh.G : 0;
  // Up to 64 query rows per KV head: the attention workgroups build the union of the per-row picks
  // themselves, and the selection kernel ends with the row bitmaps.  With a count only the device
  // knows, the selection kernel does so for the heads it finds with at most 64 rows, and the attention
  // launch for those heads takes their row-tile counts from the device; heads with more rows get the
  // union list and the many-row launch as before.
  const bool union_counted = fuse_prepare && counted && rows_upper >= 1 && rows_upper <= 64 && ctx->union_in_attention;
  const bool union_on_device = fuse_prepare && !counted && ctx->sh.rows_max <= 256 && ctx->union_in_attention;
  const bool union_in_attn = union_counted || union_on_device;
  const UnionInKernel uni{ctx->rowmaps, sc, union_on_device};
  s = score_pages_impl(ctx, st, view, kv->batch, msp, q, ctx->active_idx, ctx->active_count, topk_pages, nullptr,
                       ctx->sel_pages, sc, cap, fuse_prepare, rows_upper, rank_in_scores ? &ranking : nullptr,
                       union_in_attn);
  if (s != LOSA_OK) return s;
  return sparse_attn_impl(ctx, st, view, kv->batch, msp, q, ctx->active_idx, ctx->active_count, ctx->sel_pages, sc,
                          cap, rows_upper, fuse_prepare, (float*)o_p, lse_p, union_in_attn ? &uni : nullptr);
}

}  // extern "C"
