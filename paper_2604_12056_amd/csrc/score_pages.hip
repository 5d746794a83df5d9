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

// Matrix-core page scoring for bfloat16.  Since max >= min per channel,
//   max(q*min, q*max) = q+ * max + q- * min      with q+ = max(q,0), q- = min(q,0),
// and one of the two terms is exactly zero, so each channel contributes the same exact
// product either way: the score matrix of a KV head is the dense contraction
//   S^T [pages x rows] = [max | min] (pages x 2d) . [Q+ | Q-]^T (2d x rows).
// A wavefront takes 16 pages: its A operands are the 16 metadata rows read straight from
// memory (one 16-byte load per lane and k-step, 8 KiB per wavefront all in flight at once);
// the B operands are the sign-split query fragments.  Output leaves the matrix core as 4
// consecutive pages per lane and query row: one 16-byte store.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

template <int D>
__global__ __launch_bounds__(256) void page_scores_mfma_kernel(KvView kv, Shape sh, const bf16_t* __restrict__ q,
                                                               const int32_t* __restrict__ active_idx,
                                                               const int32_t* __restrict__ active_count,
                                                               float* __restrict__ scores,
                                                               uint32_t* __restrict__ bitmap) {
  constexpr int KS = D / 32;
  const int b = blockIdx.z, j = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6, l16 = lane & 15, qd = lane >> 4;
  const int words = (sh.max_pages + 31) / 32;
  if (blockIdx.x == 0)
    for (int w = tid; w < words; w += 256) bitmap[((size_t)b * sh.Hkv + j) * words + w] = 0u;
  const int base = kv.page_indptr[b];
  const int P = min(kv.page_indptr[b + 1] - base, sh.max_pages);
  const int p0 = blockIdx.x * 64 + wave * 16;
  if (p0 >= P) return;
  const int M = min(active_count[b], sh.B) * sh.G;
  if (M <= 0) return;

  // A operands: metadata rows of page p0 + l16 (a valid page is read for lanes past P, never stored)
  const int pg = min(p0 + l16, P - 1);
  int phys = kv.page_indices[base + pg];
  if ((unsigned)phys >= (unsigned)kv.num_pages) phys = 0;
  const bf16_t* mrow = (const bf16_t*)kv.meta + ((size_t)phys * sh.Hkv + j) * 2 * D;
  bf16x8_t amin[KS], amax[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    amin[ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(mrow + ks * 32 + qd * 8));
    amax[ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(mrow + D + ks * 32 + qd * 8));
  }
  const bool vec_ok = (sh.max_pages & 3) == 0 && p0 + 16 <= P;
  float* out_base = scores + ((size_t)b * sh.Hkv + j) * sh.rows_max * sh.max_pages;

  for (int r0 = 0; r0 < M; r0 += 16) {
    const int r = r0 + l16;
    uint4 raw[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) raw[ks] = make_uint4(0u, 0u, 0u, 0u);
    if (r < M) {
      const int a = r / sh.G, hg = r % sh.G;
      const int tok = active_idx[(size_t)b * sh.B + a];
      if ((unsigned)tok < (unsigned)sh.B) {
        const bf16_t* qrow = q + (((size_t)b * sh.B + tok) * sh.Hq + j * sh.G + hg) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) raw[ks] = *reinterpret_cast<const uint4*>(qrow + ks * 32 + qd * 8);
      }
    }
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      // per 16-bit half: all-ones where the sign bit is set
      auto neg_mask = [](uint32_t x) { return ((x >> 15) & 0x00010001u) * 0xFFFFu; };
      const uint4 x = raw[ks];
      const uint4 mk = make_uint4(neg_mask(x.x), neg_mask(x.y), neg_mask(x.z), neg_mask(x.w));
      const uint4 qneg = make_uint4(x.x & mk.x, x.y & mk.y, x.z & mk.z, x.w & mk.w);
      const uint4 qpos = make_uint4(x.x & ~mk.x, x.y & ~mk.y, x.z & ~mk.z, x.w & ~mk.w);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(amax[ks], __builtin_bit_cast(bf16x8_t, qpos), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(amin[ks], __builtin_bit_cast(bf16x8_t, qneg), acc, 0, 0, 0);
    }
    // acc[e] = score of page p0 + 4*qd + e for query row r0 + l16
    if (r < M) {
      float* dst = out_base + (size_t)r * sh.max_pages + p0 + 4 * qd;
      if (vec_ok) {
        *reinterpret_cast<f32x4_t*>(dst) = acc;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (p0 + 4 * qd + e < P) dst[e] = acc[e];
      }
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

// Register-resident variant for P <= 256*E pages: thread t owns the E consecutive pages
// [t*E, t*E+E), keys are read from memory once.  Per radix pass: LDS histogram of the
// still-matching keys, then a block-wide suffix scan over the 256 buckets finds the bucket
// holding the K-th largest key (no serial walk).  The picks of the row are assembled as a
// bitmap in LDS and OR-ed into the KV head's bitmap one word at a time.
template <int E>
__global__ __launch_bounds__(256) void topk_union_reg_kernel(KvView kv, Shape sh,
                                                             const int32_t* __restrict__ active_count,
                                                             const float* __restrict__ scores, int topk,
                                                             int32_t* __restrict__ topk_out,
                                                             uint32_t* __restrict__ bitmap) {
  constexpr int WORDS = 256 * E / 32;
  __shared__ uint32_t hist[256];
  __shared__ uint32_t rowbits[WORDS];
  __shared__ uint32_t s_bucket;
  __shared__ int s_need;
  __shared__ int scan[17];
  const int r = blockIdx.x, j = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const int n = min(active_count[b], sh.B);
  if (r >= n * sh.G) return;
  const int P = min(kv.page_indptr[b + 1] - kv.page_indptr[b], sh.max_pages);
  if (P <= 0) return;
  const int a = r / sh.G, h = j * sh.G + r % sh.G;
  int32_t* out = topk_out ? topk_out + (((size_t)b * sh.B + a) * sh.Hq + h) * topk : nullptr;
  const int Kp = min(topk, P);
  const float* row = scores + (((size_t)b * sh.Hkv + j) * sh.rows_max + r) * sh.max_pages;
  const int p_first = tid * E;

  uint32_t key[E];
  if (p_first + E <= P && (sh.max_pages & 3) == 0) {
#pragma unroll
    for (int i = 0; i < E; i += 4) {
      const float4 v = *reinterpret_cast<const float4*>(row + p_first + i);
      key[i] = order_key(v.x);
      key[i + 1] = order_key(v.y);
      key[i + 2] = order_key(v.z);
      key[i + 3] = order_key(v.w);
    }
  } else {
#pragma unroll
    for (int i = 0; i < E; ++i) key[i] = p_first + i < P ? order_key(row[p_first + i]) : 0u;
  }
  const int nmine = max(0, min(E, P - p_first));   // pages of this thread that exist

  for (int w = tid; w < WORDS; w += 256) rowbits[w] = 0u;
  const bool all = Kp >= P;
  uint32_t prefix = 0u, pmask = 0u;
  int need = Kp;
  if (!all) {
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      hist[tid] = 0u;
      __syncthreads();
#pragma unroll
      for (int i = 0; i < E; ++i)
        if (i < nmine && (key[i] & pmask) == prefix) atomicAdd(&hist[(key[i] >> shift) & 255u], 1u);
      __syncthreads();
      // thread t looks at bucket 255-t: its inclusive prefix over t is the count of keys in buckets >= 255-t
      const int c = (int)hist[255 - tid];
      int total;
      const int above = block_exclusive_scan(c, scan, &total);   // keys in strictly higher buckets
      if (above < need && above + c >= need) {
        s_bucket = (uint32_t)(255 - tid);
        s_need = need - above;
      }
      __syncthreads();
      prefix |= s_bucket << shift;
      pmask |= 0xFFu << shift;
      need = s_need;
    }
  } else {
    __syncthreads();
  }
  // picks: keys above the K-th, plus the first `need` keys equal to it in page order
  int my_eq = 0, my_gt = 0;
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const bool in = i < nmine;
    my_gt += in && (all || key[i] > prefix);
    my_eq += in && !all && key[i] == prefix;
  }
  int tot_eq, tot_sel;
  int eq_rank = block_exclusive_scan(my_eq, scan, &tot_eq);
  int my_sel = my_gt + max(0, min(my_eq, need - eq_rank));
  int pos = block_exclusive_scan(my_sel, scan, &tot_sel);
  uint32_t bits[(E + 31) / 32];
#pragma unroll
  for (int w = 0; w < (E + 31) / 32; ++w) bits[w] = 0u;
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const bool in = i < nmine;
    bool sel = in && (all || key[i] > prefix);
    if (in && !all && key[i] == prefix) {
      sel = eq_rank < need;
      ++eq_rank;
    }
    if (sel) {
      bits[i / 32] |= 1u << ((p_first + i) & 31);
      if (out) out[pos] = p_first + i;
      ++pos;
    }
  }
  if (E >= 32) {
#pragma unroll
    for (int w = 0; w < (E + 31) / 32; ++w)
      if (bits[w]) rowbits[p_first / 32 + w] = bits[w];   // this thread owns whole words
  } else {
    if (bits[0]) atomicOr(&rowbits[p_first / 32], bits[0]);
  }
  __syncthreads();
  const int words = (sh.max_pages + 31) / 32;
  uint32_t* bm = bitmap + ((size_t)b * sh.Hkv + j) * words;
  for (int w = tid; w < WORDS && w < words; w += 256)
    if (rowbits[w]) atomicOr(&bm[w], rowbits[w]);
  if (out)
    for (int k = tot_sel + tid; k < topk; k += 256) out[k] = -1;
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
    dim3 mgrid((max_seq_pages + 63) / 64, sh.Hkv, batch);
    if (mgrid.x == 0) mgrid.x = 1;
    if (sh.d == 128)
      page_scores_mfma_kernel<128><<<mgrid, 256, 0, st>>>(kv, sh, (const bf16_t*)q, active_idx, active_count, scores, bitmap);
    else
      page_scores_mfma_kernel<64><<<mgrid, 256, 0, st>>>(kv, sh, (const bf16_t*)q, active_idx, active_count, scores, bitmap);
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
  if (batch <= 0) return hipSuccess;
  dim3 grid(sh.rows_max, sh.Hkv, batch);
  const int pages = max_seq_pages < sh.max_pages ? max_seq_pages : sh.max_pages;
  if (pages <= 256 * 8)
    topk_union_reg_kernel<8><<<grid, 256, 0, st>>>(kv, sh, active_count, scores, topk, topk_out, bitmap);
  else if (pages <= 256 * 32)
    topk_union_reg_kernel<32><<<grid, 256, 0, st>>>(kv, sh, active_count, scores, topk, topk_out, bitmap);
  else
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
