// QUEST page scoring, per-query top pages and their union per KV head
// (paper: Preliminaries, Sparse Attention Algorithms for LLMs; Methodology, eq. quest_union).
//
//   page_scores   s[b,j,r,p] = sum_c max(q_c*min_c, q_c*max_c)   r = a*G + hg over the active slots a
//   topk_union    per row r: exact top-K by 4-pass radix select on order-preserving keys
//                 (ties: smaller page), bits OR-ed into the KV head's page bitmap
//   union_compact bitmap -> ascending page list + count
//
// Everything that decides a set is integer work on float bit patterns: no float atomics,
// so the outcome does not depend on scheduling.
#include "losa_device.h"
#include "losa_internal.h"

namespace losa {

constexpr int kScorePages = 32;  // pages per workgroup in page_scores
constexpr int kScoreRows = 32;   // query rows staged at a time

template <typename T, int D>
__global__ __launch_bounds__(256) void page_scores_kernel(KvView kv, Shape sh, const T* __restrict__ q,
                                                          const int32_t* __restrict__ active_idx,
                                                          const int32_t* __restrict__ active_count,
                                                          float* __restrict__ scores, uint32_t* __restrict__ bitmap) {
  constexpr int V = Vec16<T>::n;
  constexpr int PT = kScorePages, RC = kScoreRows;
  __shared__ float mn[PT][D + 1];
  __shared__ float mx[PT][D + 1];
  __shared__ float qs[RC][D];
  const int b = blockIdx.z, j = blockIdx.y, p0 = blockIdx.x * PT, tid = threadIdx.x;
  const int words = (sh.max_pages + 31) / 32;
  if (blockIdx.x == 0)
    for (int w = tid; w < words; w += 256) bitmap[((size_t)b * sh.Hkv + j) * words + w] = 0u;
  const int base = kv.page_indptr[b];
  const int P = min(kv.page_indptr[b + 1] - base, sh.max_pages);
  if (p0 >= P) return;
  const int n = min(active_count[b], sh.B);
  const int M = n * sh.G;
  if (M <= 0) return;

  constexpr int VPR = D / V;  // vectors per metadata row
  for (int v = tid; v < PT * 2 * VPR; v += 256) {
    const int pg = v / (2 * VPR), rem = v % (2 * VPR), which = rem / VPR, cv = rem % VPR;
    float f[V];
#pragma unroll
    for (int e = 0; e < V; ++e) f[e] = 0.f;
    if (p0 + pg < P) {
      const int phys = kv.page_indices[base + p0 + pg];
      if ((unsigned)phys < (unsigned)kv.num_pages) {
        const uint4 raw = reinterpret_cast<const uint4*>((const T*)kv.meta + (((size_t)phys * sh.Hkv + j) * 2 + which) * D)[cv];
        widen16(raw, f, T());
      }
    }
    float* dst = which ? &mx[pg][cv * V] : &mn[pg][cv * V];
#pragma unroll
    for (int e = 0; e < V; ++e) dst[e] = f[e];
  }

  const int pg = tid % PT, rs = tid / PT;  // 8 row lanes
  for (int r0 = 0; r0 < M; r0 += RC) {
    __syncthreads();
    for (int v = tid; v < RC * VPR; v += 256) {
      const int rr = v / VPR, cv = v % VPR, r = r0 + rr;
      float f[V];
#pragma unroll
      for (int e = 0; e < V; ++e) f[e] = 0.f;
      if (r < M) {
        const int a = r / sh.G, hg = r % sh.G;
        const int tok = active_idx[(size_t)b * sh.B + a];
        if ((unsigned)tok < (unsigned)sh.B) {
          const uint4 raw = reinterpret_cast<const uint4*>(q + (((size_t)b * sh.B + tok) * sh.Hq + j * sh.G + hg) * D)[cv];
          widen16(raw, f, T());
        }
      }
#pragma unroll
      for (int e = 0; e < V; ++e) qs[rr][cv * V + e] = f[e];
    }
    __syncthreads();
    for (int rr = rs; rr < RC && r0 + rr < M; rr += 256 / PT) {
      float s = 0.f;
#pragma unroll 8
      for (int c = 0; c < D; ++c) {
        const float qv = qs[rr][c];
        s += fmaxf(qv * mn[pg][c], qv * mx[pg][c]);
      }
      if (p0 + pg < P)
        scores[(((size_t)b * sh.Hkv + j) * sh.rows_max + r0 + rr) * sh.max_pages + p0 + pg] = s;
    }
  }
}

// float -> uint32 whose unsigned order is the float order (-0 and +0 made equal first).
__device__ __forceinline__ uint32_t order_key(float f) {
  f += 0.0f;
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(256) void topk_union_kernel(KvView kv, Shape sh, const int32_t* __restrict__ active_count,
                                                         const float* __restrict__ scores, int topk,
                                                         int32_t* __restrict__ topk_out,
                                                         uint32_t* __restrict__ bitmap) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t s_bucket;
  __shared__ int s_need;
  __shared__ int scan[17];
  const int r = blockIdx.x, j = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const int n = min(active_count[b], sh.B);
  if (r >= n * sh.G) return;
  const int P = min(kv.page_indptr[b + 1] - kv.page_indptr[b], sh.max_pages);
  const int a = r / sh.G, h = j * sh.G + r % sh.G;
  int32_t* out = topk_out ? topk_out + (((size_t)b * sh.B + a) * sh.Hq + h) * topk : nullptr;
  const int Kp = min(topk, P);
  const float* row = scores + (((size_t)b * sh.Hkv + j) * sh.rows_max + r) * sh.max_pages;
  const bool all = Kp >= P;
  uint32_t prefix = 0u, pmask = 0u;
  int need = Kp;
  if (!all) {
    // K-th largest key, one byte per pass from the top
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      hist[tid] = 0u;
      __syncthreads();
      for (int p = tid; p < P; p += 256) {
        const uint32_t key = order_key(row[p]);
        if ((key & pmask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
      }
      __syncthreads();
      if (tid == 0) {
        int cum = 0, bkt = 255;
        for (; bkt > 0; --bkt) {
          const int c = (int)hist[bkt];
          if (cum + c >= need) break;
          cum += c;
        }
        s_bucket = (uint32_t)bkt;
        s_need = need - cum;
      }
      __syncthreads();
      prefix |= s_bucket << shift;
      pmask |= 0xFFu << shift;
      need = s_need;
      __syncthreads();
    }
  }
  // picks in page order: every key above the K-th, plus the first `need` keys equal to it
  const int words = (sh.max_pages + 31) / 32;
  uint32_t* bm = bitmap + ((size_t)b * sh.Hkv + j) * words;
  int base_sel = 0, base_eq = 0;
  for (int p0 = 0; p0 < P; p0 += 256) {
    const int p = p0 + tid;
    const bool in = p < P;
    const uint32_t key = in ? order_key(row[p]) : 0u;
    const int gt = in && (all || key > prefix);
    const int eq = in && !all && key == prefix;
    int tot_eq, tot_sel;
    const int eq_rank = base_eq + block_exclusive_scan(eq, scan, &tot_eq);
    const int sel = gt || (eq && eq_rank < need);
    const int pos = base_sel + block_exclusive_scan(sel, scan, &tot_sel);
    const unsigned long long ball = __ballot(sel);
    const int lane = tid & 63;
    if (lane == 0 && (uint32_t)ball) atomicOr(&bm[(p0 + (tid & ~63)) / 32], (uint32_t)ball);
    if (lane == 32 && (uint32_t)(ball >> 32)) atomicOr(&bm[(p0 + (tid & ~63)) / 32 + 1], (uint32_t)(ball >> 32));
    if (sel && out) out[pos] = p;
    base_eq += tot_eq;
    base_sel += tot_sel;
  }
  if (out)
    for (int k = base_sel + tid; k < topk; k += 256) out[k] = -1;
}

__global__ __launch_bounds__(256) void union_compact_kernel(KvView kv, Shape sh, const uint32_t* __restrict__ bitmap,
                                                            int32_t* __restrict__ sel_pages,
                                                            int32_t* __restrict__ sel_count, int cap) {
  __shared__ int scan[17];
  const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int P = kv.page_indptr[b + 1] - kv.page_indptr[b];
  const int words = (sh.max_pages + 31) / 32, wordsP = (min(P, sh.max_pages) + 31) / 32;
  const uint32_t* bm = bitmap + ((size_t)b * sh.Hkv + j) * words;
  int32_t* out = sel_pages + ((size_t)b * sh.Hkv + j) * cap;
  int base_out = 0;
  for (int w0 = 0; w0 < wordsP; w0 += 256) {
    const int w = w0 + tid;
    uint32_t bits = w < wordsP ? bm[w] : 0u;
    int total;
    int pos = base_out + block_exclusive_scan(__popc(bits), scan, &total);
    while (bits) {
      const int bit = __ffs((int)bits) - 1;
      if (pos < cap) out[pos] = w * 32 + bit;
      ++pos;
      bits &= bits - 1u;
    }
    base_out += total;
  }
  if (tid == 0) sel_count[b * sh.Hkv + j] = min(base_out, cap);
}

hipError_t launch_page_scores(hipStream_t st, int dtype, const KvView& kv, const Shape& sh, int batch,
                              int max_seq_pages, const void* q, const int32_t* active_idx,
                              const int32_t* active_count, float* scores, uint32_t* bitmap) {
  if (batch <= 0) return hipSuccess;
  dim3 grid((max_seq_pages + kScorePages - 1) / kScorePages, sh.Hkv, batch);
  if (grid.x == 0) grid.x = 1;
  if (dtype == LOSA_BF16) {
    if (sh.d == 128)
      page_scores_kernel<bf16_t, 128><<<grid, 256, 0, st>>>(kv, sh, (const bf16_t*)q, active_idx, active_count, scores, bitmap);
    else
      page_scores_kernel<bf16_t, 64><<<grid, 256, 0, st>>>(kv, sh, (const bf16_t*)q, active_idx, active_count, scores, bitmap);
  } else {
    if (sh.d == 128)
      page_scores_kernel<float, 128><<<grid, 256, 0, st>>>(kv, sh, (const float*)q, active_idx, active_count, scores, bitmap);
    else
      page_scores_kernel<float, 64><<<grid, 256, 0, st>>>(kv, sh, (const float*)q, active_idx, active_count, scores, bitmap);
  }
  return hipGetLastError();
}

hipError_t launch_topk_union(hipStream_t st, const KvView& kv, const Shape& sh, int batch, int max_seq_pages,
                             const int32_t* active_count, const float* scores, int topk, int32_t* topk_out,
                             uint32_t* bitmap) {
  (void)max_seq_pages;
  if (batch <= 0) return hipSuccess;
  dim3 grid(sh.rows_max, sh.Hkv, batch);
  topk_union_kernel<<<grid, 256, 0, st>>>(kv, sh, active_count, scores, topk, topk_out, bitmap);
  return hipGetLastError();
}

hipError_t launch_union_compact(hipStream_t st, const KvView& kv, const Shape& sh, int batch, int max_seq_pages,
                                const int32_t* active_count, const uint32_t* bitmap, int32_t* sel_pages,
                                int32_t* sel_count, int cap) {
  (void)max_seq_pages;
  (void)active_count;
  if (batch <= 0) return hipSuccess;
  dim3 grid(sh.Hkv, batch);
  union_compact_kernel<<<grid, 256, 0, st>>>(kv, sh, bitmap, sel_pages, sel_count, cap);
  return hipGetLastError();
}

}  // namespace losa
