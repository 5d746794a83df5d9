// Internal declarations shared by the translation units of liblosa.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "losa.h"

namespace losa {

constexpr int kWave = 64;

// Device view of the ragged page table, passed to kernels by value.
struct KvView {
  const void* k_pages;
  const void* v_pages;
  void* meta;
  const int32_t* page_indptr;
  const int32_t* page_indices;
  const int32_t* seq_lens;
  int32_t num_pages;
  int32_t seq_page_limit;   // the host's upper bound on pages per sequence (grids and register tiles are sized by it)
};

// Static problem shape, passed to kernels by value.
struct Shape {
  int32_t max_pages;   // row stride of the score matrix / bitmap sizing (config.max_pages_per_seq)
  int32_t rows_max;    // B * G: rows of one KV head when every token is active
  int32_t Hkv, Hq, G, d, H, g, B;
  float sm_scale;
};

// Pages of sequence b that the kernels look at: those the page table lists, that hold at least
// one of the sequence's tokens (a table may list pages reserved ahead of the tokens: their
// metadata was never written), and that the launch was sized for.
__device__ __forceinline__ int seq_pages(const KvView& kv, const Shape& sh, int b) {
  const int listed = kv.page_indptr[b + 1] - kv.page_indptr[b];
  const int filled = (kv.seq_lens[b] + sh.g - 1) >> (sh.g == 16 ? 4 : 5);   // g is 16 or 32
  return max(0, min(min(listed, filled), min(sh.max_pages, kv.seq_page_limit)));
}

// Split-K partials of the attention: item = ((b*Hkv + j)*nchunk + c), row r < rows.
struct Partials {
  float* o;   // [items, rows, d]   un-normalised sum_t exp(s_t - m) v_t
  float* m;   // [items, rows]      running max of the scaled scores
  float* l;   // [items, rows]      sum_t exp(s_t - m)
  int rows;   // rows per item in this launch: an upper bound on the query rows of a KV head
};

// Prepared inputs of the matrix-core attention kernel, per (sequence, KV head) = `head`.
constexpr int kEntryShift = 26;   // entry = physical page id | (valid tokens << 26)
struct AttnPrepared {
  int32_t* entries;   // [heads, max_pages]
  uint16_t* q_act;    // [heads, rows_max, d] bfloat16: query rows of the active tokens, gathered
  int32_t* ucount;    // [heads] entries in the list
  int32_t* mrows;     // [heads] query rows (|A| * G)
};
// The other way the matrix-core kernel can get its page list (sparse steps of losa_step with at
// most 64 query rows per KV head): the selection kernel leaves only the per-row pick bitmaps, and
// every attention workgroup ORs them, ranks the union and resolves its own pages itself while it
// starts up.  That takes the selection kernel's serial tail (bitmap hand-over to one workgroup per
// head, union, list) out of the chain of launches.  When the host does not know the row count
// (threshold / cumulative-mass selection) the selection kernel decides per (sequence, KV head),
// by the count it finds, which of the two forms it leaves, and the attention launch takes each
// head's row-tile count from the device (rows_on_device).
constexpr int kUnionRows = 64;   // row slots per bitmap word in that layout (the most rows the split-pages shape serves)
struct UnionInKernel {
  const uint32_t* rowmaps;   // [heads][words, kUnionRows] pick bitmaps, word-major: slot r of word w is row r's
                             // word w, slots past the head's row count are zero; NULL: use AttnPrepared::entries.
                             // A head's region is union_region_words() wide (it can hold the row-major form too).
  int32_t* sel_count;        // [heads] out: pages in the union (written by the head's first workgroup)
  bool rows_on_device;       // host side only: launch the form that sizes itself by AttnPrepared::mrows
};
// 32-bit words of one (sequence, KV head) region of the row-bitmap buffer: `words` per row, for the
// larger of the block's row count and the word-major layout's 64 slots
__host__ __device__ inline size_t union_region_words(int rows_max, int words) {
  return (size_t)words * (size_t)(rows_max > kUnionRows ? rows_max : kUnionRows);
}

// ---- losa_api.hip
// Sets `n` ints to zero with a small fill kernel (safe to record into a captured graph).
hipError_t launch_zero_ints(hipStream_t st, int32_t* p, int n);
// Records the error text losa_last_error(NULL) returns on this thread; returns `st`.
losa_status set_thread_error(losa_status st, const char* fmt, ...);

// ---- select_active.hip
// fused: score per token + ranking by the last workgroup of each sequence (tickets: [batch] ints, zero on entry)
hipError_t launch_locality_select(hipStream_t st, int dtype, const void* h_cur, const void* h_prev, int batch, int B,
                                  int H, int mode, int n, float tau, float* delta, uint8_t* mask, int32_t* active_idx,
                                  int32_t* active_count, int32_t* tickets);
// One shared page set per (sequence, KV head): top pages of the scores max-reduced over the head's rows.
hipError_t launch_shared_select(hipStream_t st, const KvView& kv, const Shape& sh, int batch, int max_seq_pages,
                                const int32_t* active_count, const float* scores, int topk, int32_t* sel_pages,
                                int32_t* sel_count, int cap);
// Locality scores only (no ranking): for the step whose scoring kernel ranks them itself.
hipError_t launch_locality_delta(hipStream_t st, int dtype, const void* h_cur, const void* h_prev, int batch, int B,
                                 int H, float* delta);

// ---- page_bounds.hip
hipError_t launch_page_bounds(hipStream_t st, int dtype, const KvView& kv, const Shape& sh, int batch,
                              int first_page, int num_pages_in_range);

// ---- score_pages.hip
constexpr int kMaxSelectPages = 1024 * 16;   // pages per sequence the register-resident top-k handles
// ranking != NULL (bfloat16, B <= 256): the scoring workgroups derive the
// active set from `delta` themselves and write mask / active_idx / active_count; the active_idx /
// active_count arguments are then outputs of this launch, not inputs.
struct InKernelRanking {
  const float* delta;
  int mode, n;
  float tau;
  uint8_t* mask;
  int32_t* active_idx;
  int32_t* active_count;
};
hipError_t launch_page_scores(hipStream_t st, int dtype, const KvView& kv, const Shape& sh, int batch, int max_seq_pages,
                              const void* q, const int32_t* active_idx, const int32_t* active_count,
                              float* scores, int32_t* tickets, int32_t* sel_count, const AttnPrepared* prep,
                              const InKernelRanking* ranking, long workgroups_per_round);
hipError_t launch_select_pages(hipStream_t st, const KvView& kv, const Shape& sh, int batch, int max_seq_pages,
                               const void* q, const int32_t* active_idx, const int32_t* active_count,
                               const float* scores, int topk, int32_t* topk_out, int32_t* sel_pages,
                               int32_t* sel_count, int cap, uint32_t* rowmaps, int32_t* tickets,
                               const AttnPrepared* prep, int rows_hint, long workgroups_per_round,
                               bool bitmaps_only = false);

// ---- sparse_attn.hip (element-generic kernel, merge) and sparse_attn_mfma.hip (bfloat16 matrix-core kernel)
// Both deal the 32-token tiles of a (sequence, KV head) page list round-robin to `nchunk` work items.
// launch_attn_merge: prep != NULL means the partials came from the matrix-core kernel.
hipError_t launch_attn_generic(hipStream_t st, int dtype, const KvView& kv, const Shape& sh, int batch,
                               const void* q, const int32_t* active_idx, const int32_t* active_count,
                               const int32_t* sel_pages, const int32_t* sel_count, int cap, int nchunk,
                               const Partials& part);
hipError_t launch_attn_prepare(hipStream_t st, const KvView& kv, const Shape& sh, int batch, const void* q,
                               const int32_t* active_idx, const int32_t* active_count, const int32_t* sel_pages,
                               const int32_t* sel_count, int cap, const AttnPrepared& prep);
// The attention kernel's form above 64 query rows per KV head.
enum ManyRowForm : int {
  kManyRowsIndependent = 0,   // 4 wavefronts of 64 rows, each loading every tile itself; P as a bfloat16 pair
  kManyRowsSharedHalf = 1,    // 8 wavefronts of 32 rows, tiles shared through LDS, value product in half precision
  kManyRowsSharedPair = 2     // the same sharing, P as a bfloat16 pair (values keep bfloat16's range)
};
// e0/e1 (both or neither): events bound to the dispatch itself, for exact kernel timing.
hipError_t launch_attn_mfma(hipStream_t st, const KvView& kv, const Shape& sh, int batch, const AttnPrepared& prep,
                            int nchunk, int rows_upper, const Partials& part, hipEvent_t e0, hipEvent_t e1,
                            int m_lo = 0, int m_hi = 0x7fffffff,   // serves (sequence, head) pairs with m_lo < rows <= m_hi
                            const UnionInKernel* uni = nullptr, int many_rows = kManyRowsSharedHalf);
hipError_t launch_attn_merge(hipStream_t st, const KvView& kv, const Shape& sh, int batch,
                             const int32_t* active_idx, const int32_t* active_count,
                             const int32_t* sel_count, int cap, int nchunk, const AttnPrepared* prep,
                             const Partials& part, float* o_p, float* lse_p, int rows_hint);

// ---- block_merge.hip
hipError_t launch_block_merge(hipStream_t st, int dtype, const Shape& sh, int batch, const void* q, const void* k_b,
                              const void* v_b, const float* o_p, const float* lse_p, float* out, float* o_b,
                              float* lse_b);

}  // namespace losa
