// Paged sparse prefix attention for the active queries, split over page chunks
// (paper: Preliminaries, Attention Decomposition With Online Softmax; Methodology, eq. update_rule).
//
// Work item = (sequence b, KV head j, block of query rows, chunk of the KV head's page list).
// Each item keeps a running (max, sum, un-normalised output) per row and writes it as a
// partial; attn_merge combines the chunks of a row in chunk order with the same
// log-sum-exp rule the paper uses to merge prefix and block parts, normalises, and writes
// (o_p, lse_p) at the active token's row.  No float atomics anywhere: results do not
// depend on scheduling.
//
// This file holds the float-mode kernel (vector ALUs, K/V tiles staged in LDS, float64
// accumulation) and the merge kernel both precisions share; bfloat16 inputs always take the
// matrix-core kernel.
#include <math.h>

#include <type_traits>

#include "losa_device.h"
#include "losa_internal.h"

namespace losa {

constexpr int kRowBlock = 32;  // query rows per work item (generic kernel)
constexpr int kTileTok = 32;   // tokens per LDS tile

// Accumulation type of the generic kernel.  bfloat16 inputs: float (products are exact, the
// 2e-2 bound is far away).  float inputs: double, because the float mode's 1e-4 bound is
// within reach of float summation error once outlier channels push |q.k| into the hundreds.
template <typename T> struct AccOf { typedef float type; };
template <> struct AccOf<float> { typedef double type; };

template <typename T, int D, int GP>
__global__ __launch_bounds__(256) void attn_partials_generic_kernel(
    KvView kv, Shape sh, const T* __restrict__ q, const int32_t* __restrict__ active_idx,
    const int32_t* __restrict__ active_count, const int32_t* __restrict__ sel_pages,
    const int32_t* __restrict__ sel_count, int cap, int nchunk, int nrb, Partials part) {
  constexpr int V = Vec16<T>::n;
  constexpr int VPR = D / V;           // 16-byte vectors per key row
  constexpr int PPT = kTileTok / GP;   // pages per tile
  constexpr int VPC = GP / V;          // 16-byte vectors per value channel row of a page
  constexpr int CPT = D / 8;           // output channels per thread
  __shared__ float qs[kRowBlock][D + 1];
  __shared__ float ks[kTileTok][D + 1];
  __shared__ float vs[kTileTok][D + 1];
  __shared__ typename AccOf<T>::type ps[kRowBlock][kTileTok + 1];
  __shared__ int tok_ok[kTileTok];

  const int chunk = blockIdx.x, j = blockIdx.y / nrb, rb = blockIdx.y % nrb, b = blockIdx.z, tid = threadIdx.x;
  const int n = active_idx ? min(active_count[b], sh.B) : sh.B;
  const int M = min(n * sh.G, part.rows), r0 = rb * kRowBlock;
  if (r0 >= M) return;
  const int base = kv.page_indptr[b];
  const int P = seq_pages(kv, sh, b);
  const int L = kv.seq_lens[b];
  const int32_t* list = sel_pages ? sel_pages + ((size_t)b * sh.Hkv + j) * cap : nullptr;
  const int U = list ? min(sel_count[b * sh.Hkv + j], cap) : P;
  const int ntiles = (U + PPT - 1) / PPT;
  if (chunk >= ntiles) return;   // tiles are dealt round-robin: chunk, chunk + nchunk, ...
  const int c1 = U;

  for (int v = tid; v < kRowBlock * VPR; v += 256) {
    const int rr = v / VPR, cv = v % VPR, r = r0 + rr;
    float f[V];
#pragma unroll
    for (int e = 0; e < V; ++e) f[e] = 0.f;
    if (r < M) {
      const int a = r / sh.G, hg = r % sh.G;
      const int tok = active_idx ? active_idx[(size_t)b * sh.B + a] : a;
      if ((unsigned)tok < (unsigned)sh.B) {
        const uint4 raw = reinterpret_cast<const uint4*>(q + (((size_t)b * sh.B + tok) * sh.Hq + j * sh.G + hg) * D)[cv];
        widen16(raw, f, T());
      }
    }
#pragma unroll
    for (int e = 0; e < V; ++e) qs[rr][cv * V + e] = f[e];
  }

  typedef typename AccOf<T>::type Acc;
  const int row = tid / 8, sub = tid % 8;
  float m = -INFINITY;   // running reference point of the exponentials (any value near the max works)
  Acc l = 0, acc[CPT];
#pragma unroll
  for (int k = 0; k < CPT; ++k) acc[k] = 0;

  for (int tile = chunk; tile < ntiles; tile += nchunk) {
    const int pp = tile * PPT;
    __syncthreads();
    // ---- stage one tile of keys (token-major pages) and values (channel-major pages)
    for (int v = tid; v < kTileTok * VPR; v += 256) {
      const int ts = v / VPR, cv = v % VPR;
      const int lp = pp + ts / GP, tin = ts % GP;
      float f[V];
#pragma unroll
      for (int e = 0; e < V; ++e) f[e] = 0.f;
      int ok = 0;
      if (lp < c1) {
        const int logical = list ? list[lp] : lp;
        if ((unsigned)logical < (unsigned)P && logical * GP + tin < L) {
          const int phys = kv.page_indices[base + logical];
          if ((unsigned)phys < (unsigned)kv.num_pages) {
            ok = 1;
            const uint4 raw = reinterpret_cast<const uint4*>((const T*)kv.k_pages + (((size_t)phys * sh.Hkv + j) * GP + tin) * D)[cv];
            widen16(raw, f, T());
          }
        }
      }
      if (cv == 0) tok_ok[ts] = ok;
#pragma unroll
      for (int e = 0; e < V; ++e) ks[ts][cv * V + e] = f[e];
    }
    for (int v = tid; v < PPT * D * VPC; v += 256) {
      const int pgi = v / (D * VPC), rem = v % (D * VPC), c = rem / VPC, tv = rem % VPC;
      const int lp = pp + pgi;
      float f[V];
#pragma unroll
      for (int e = 0; e < V; ++e) f[e] = 0.f;
      int logical = -1;
      if (lp < c1) {
        logical = list ? list[lp] : lp;
        if ((unsigned)logical < (unsigned)P) {
          const int phys = kv.page_indices[base + logical];
          if ((unsigned)phys < (unsigned)kv.num_pages) {
            const uint4 raw = reinterpret_cast<const uint4*>((const T*)kv.v_pages + (((size_t)phys * sh.Hkv + j) * D + c) * GP)[tv];
            widen16(raw, f, T());
          } else {
            logical = -1;
          }
        } else {
          logical = -1;
        }
      }
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const int tin = tv * V + e;
        const bool ok = logical >= 0 && logical * GP + tin < L;
        vs[pgi * GP + tin][c] = ok ? f[e] : 0.f;   // slots past the sequence end may hold NaN
      }
    }
    __syncthreads();
    // ---- scores of this thread's row against 4 tokens
    Acc s[4];
    float tmax = -INFINITY;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int ts = sub + 8 * k;
      Acc dot = 0;
#pragma unroll 8
      for (int c = 0; c < D; ++c) dot += (Acc)qs[row][c] * (Acc)ks[ts][c];
      s[k] = tok_ok[ts] ? dot * (Acc)sh.sm_scale : (Acc)-INFINITY;
      tmax = fmaxf(tmax, (float)s[k]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 1, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 2, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 4, 64));
    const float m_new = fmaxf(m, tmax);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const Acc alpha = exp_acc((Acc)m - (Acc)m_use);
    Acc psum = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const Acc p = exp_acc(s[k] - (Acc)m_use);
      ps[row][sub + 8 * k] = p;
      psum += p;
    }
    psum += __shfl_xor(psum, 1, 64);
    psum += __shfl_xor(psum, 2, 64);
    psum += __shfl_xor(psum, 4, 64);
    l = l * alpha + psum;
    m = m_new;
    __syncthreads();
    // ---- output channels sub, sub+8, ... of this thread's row
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      Acc a = acc[k] * alpha;
#pragma unroll 8
      for (int ts = 0; ts < kTileTok; ++ts) a += (Acc)ps[row][ts] * (Acc)vs[ts][sub + 8 * k];
      acc[k] = a;
    }
  }
  const int r = r0 + row;
  if (r < M) {
    const size_t item = ((size_t)b * sh.Hkv + j) * nchunk + chunk;
    const size_t prow = item * part.rows + r;
#pragma unroll
    for (int k = 0; k < CPT; ++k) part.o[prow * D + sub + 8 * k] = (float)acc[k];
    if (sub == 0) {
      part.m[prow] = m;
      part.l[prow] = (float)l;
    }
  }
}

// Combine the chunk partials of one query row with the log-sum-exp rule, normalise, and
// write (o_p, lse_p) at the active token's row.  256 threads = CL chunk lanes x D/4 channel
// quads: every chunk lane sums its chunks c = lane, lane+CL, ... (independent loads), then
// the lanes are added in a fixed order, so the result does not depend on scheduling.
// LOG2: partial maxima are in log2 units (scores scaled by sm_scale*log2(e)) and sums are
// float; otherwise natural units and double sums (the element-generic kernel, which also
// serves the float mode).
template <int D, bool LOG2>
__global__ __launch_bounds__(256) void attn_merge_kernel(KvView kv, Shape sh, const int32_t* __restrict__ active_idx,
                                                         const int32_t* __restrict__ active_count,
                                                         const int32_t* __restrict__ sel_count, int cap, int nchunk,
                                                         const int32_t* __restrict__ ucount,
                                                         const int32_t* __restrict__ mrows, Partials part,
                                                         float* __restrict__ o_p, float* __restrict__ lse_p,
                                                         int rows_known) {
  typedef typename std::conditional<LOG2, float, double>::type Acc;
  constexpr int C4 = D / 4, CL = 256 / C4;
  __shared__ Acc red[CL][D];
  __shared__ Acc lred[CL];
  __shared__ float wmax[CL];
  const int r = blockIdx.x, j = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  // A grid sized without knowing the row count (threshold / cumulative-mass selection) has a
  // workgroup for every possible row: those look at the count first and leave, instead of
  // fetching partials nobody wrote (a block of 224 possible rows with 35 active ones would fetch
  // six times what it needs).
  if (!rows_known) {
    const int M0 = mrows ? mrows[b * sh.Hkv + j] : (active_idx ? min(active_count[b], sh.B) : sh.B) * sh.G;
    if (r >= M0) return;
  }
  // The first KSPEC chunks of this thread are fetched before it is known how many chunks are
  // live (slots exist for all nchunk work items): together with the counts below this makes
  // the kernel one memory round trip deep instead of three.
  constexpr int KSPEC = 8;
  float pm_s[KSPEC], pl_s[KSPEC];
  float4 po_s[KSPEC];
  {
    const int cl = tid / C4, c4 = tid % C4;
    const size_t item0 = ((size_t)b * sh.Hkv + j) * nchunk;
#pragma unroll
    for (int k = 0; k < KSPEC; ++k) {
      const int c = min(cl + CL * k, nchunk - 1);
      const size_t prow = (item0 + c) * part.rows + r;
      pm_s[k] = part.m[prow];
      pl_s[k] = part.l[prow];
      po_s[k] = reinterpret_cast<const float4*>(part.o + prow * D)[c4];
    }
  }
  // the token of this row, fetched alongside (its slot exists whatever the active count is)
  const int tok_early = active_idx ? active_idx[(size_t)b * sh.B + min(r / sh.G, sh.B - 1)] : r / sh.G;
  int M, U;
  if (ucount) {   // prepared by the matrix-core path
    M = min(mrows[b * sh.Hkv + j], sh.rows_max);
    U = min(ucount[b * sh.Hkv + j], sh.max_pages);
  } else {
    M = (active_idx ? min(active_count[b], sh.B) : sh.B) * sh.G;
    const int P = seq_pages(kv, sh, b);
    U = sel_count ? min(sel_count[b * sh.Hkv + j], cap) : P;
  }
  if (r >= min(M, part.rows)) return;
  const int hg = r % sh.G;
  const int tok = tok_early;   // r < M <= B*G here, so the index above was not clamped
  if ((unsigned)tok >= (unsigned)sh.B) return;
  const int ppt = 32 / sh.g;
  const int ntiles = (U + ppt - 1) / ppt;
  const int live = min(nchunk, ntiles);   // work item c exists iff tile c does
  const size_t item0 = ((size_t)b * sh.Hkv + j) * nchunk;

  // thread (cl, c4) owns chunks cl, cl+CL, ... and channel quad c4
  const int cl = tid / C4, c4 = tid % C4;
  float mk[KSPEC];
#pragma unroll
  for (int k = 0; k < KSPEC; ++k) mk[k] = cl + CL * k < live ? pm_s[k] : -INFINITY;
  float mx = -INFINITY;
#pragma unroll
  for (int k = 0; k < KSPEC; ++k) mx = fmaxf(mx, mk[k]);
  for (int c = cl + CL * KSPEC; c < live; c += CL) mx = fmaxf(mx, part.m[(item0 + c) * part.rows + r]);
  if (c4 == 0) wmax[cl] = mx;
  __syncthreads();
  float m_tot = -INFINITY;
#pragma unroll
  for (int k = 0; k < CL; ++k) m_tot = fmaxf(m_tot, wmax[k]);
  const size_t orow = ((size_t)b * sh.B + tok) * sh.Hq + j * sh.G + hg;
  if (!(m_tot > -1.0e29f)) {   // no valid token at all: the neutral element of the merge
    if (tid < C4) reinterpret_cast<float4*>(o_p + orow * D)[tid] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (tid == 0) lse_p[orow] = -INFINITY;
    return;
  }
  Acc ax = 0, ay = 0, az = 0, aw = 0, lacc = 0;
#pragma unroll
  for (int k = 0; k < KSPEC; ++k) {
    if (cl + CL * k < live) {   // slots past `live` hold leftovers of earlier launches: never touch their values
      const float dm = mk[k] - m_tot;
      const Acc w = LOG2 ? (Acc)exp2f(dm) : (Acc)exp((double)dm);
      ax += w * (Acc)po_s[k].x;
      ay += w * (Acc)po_s[k].y;
      az += w * (Acc)po_s[k].z;
      aw += w * (Acc)po_s[k].w;
      lacc += w * (Acc)pl_s[k];
    }
  }
  for (int c = cl + CL * KSPEC; c < live; c += CL) {
    const size_t prow = (item0 + c) * part.rows + r;
    const float dm = part.m[prow] - m_tot;
    const Acc w = LOG2 ? (Acc)exp2f(dm) : (Acc)exp((double)dm);
    const float4 v = reinterpret_cast<const float4*>(part.o + prow * D)[c4];
    ax += w * (Acc)v.x;
    ay += w * (Acc)v.y;
    az += w * (Acc)v.z;
    aw += w * (Acc)v.w;
    lacc += w * (Acc)part.l[prow];
  }
  red[cl][c4 * 4 + 0] = ax;
  red[cl][c4 * 4 + 1] = ay;
  red[cl][c4 * 4 + 2] = az;
  red[cl][c4 * 4 + 3] = aw;
  if (c4 == 0) lred[cl] = lacc;
  __syncthreads();
  if (tid < D) {
    Acc o = 0, l = 0;
#pragma unroll
    for (int k = 0; k < CL; ++k) {
      o += red[k][tid];
      l += lred[k];
    }
    o_p[orow * D + tid] = (float)(o / l);
    if (tid == 0)
      lse_p[orow] = LOG2 ? (m_tot + log2f((float)l)) * 0.6931471805599453f : (float)((double)m_tot + log((double)l));
  }
}

template <typename T, int D>
static hipError_t launch_generic(hipStream_t st, const KvView& kv, const Shape& sh, int batch, const void* q,
                                 const int32_t* active_idx, const int32_t* active_count, const int32_t* sel_pages,
                                 const int32_t* sel_count, int cap, int nchunk, const Partials& part) {
  const int nrb = (sh.rows_max + kRowBlock - 1) / kRowBlock;
  dim3 grid(nchunk, sh.Hkv * nrb, batch);
  if (sh.g == 16)
    attn_partials_generic_kernel<T, D, 16><<<grid, 256, 0, st>>>(kv, sh, (const T*)q, active_idx, active_count,
                                                                 sel_pages, sel_count, cap, nchunk, nrb, part);
  else
    attn_partials_generic_kernel<T, D, 32><<<grid, 256, 0, st>>>(kv, sh, (const T*)q, active_idx, active_count,
                                                                 sel_pages, sel_count, cap, nchunk, nrb, part);
  return hipGetLastError();
}

hipError_t launch_attn_generic(hipStream_t st, int dtype, const KvView& kv, const Shape& sh, int batch, const void* q,
                               const int32_t* active_idx, const int32_t* active_count, const int32_t* sel_pages,
                               const int32_t* sel_count, int cap, int nchunk, const Partials& part) {
  if (batch <= 0 || nchunk <= 0) return hipSuccess;
  if (dtype != LOSA_F32) return hipErrorInvalidValue;   // bfloat16 takes the matrix-core kernel
  return sh.d == 128 ? launch_generic<float, 128>(st, kv, sh, batch, q, active_idx, active_count, sel_pages, sel_count,
                                                  cap, nchunk, part)
                     : launch_generic<float, 64>(st, kv, sh, batch, q, active_idx, active_count, sel_pages, sel_count,
                                                 cap, nchunk, part);
}

hipError_t launch_attn_merge(hipStream_t st, const KvView& kv, const Shape& sh, int batch, const int32_t* active_idx,
                             const int32_t* active_count, const int32_t* sel_count, int cap, int nchunk,
                             const AttnPrepared* prep, const Partials& part, float* o_p, float* lse_p, int rows_hint) {
  if (batch <= 0) return hipSuccess;
  // rows_hint: an upper bound on the active rows per KV head the host happens to know (0: none);
  // rows past it get no workgroup (they would only fetch partials speculatively and exit)
  dim3 grid(rows_hint >= 1 && rows_hint < sh.rows_max ? rows_hint : sh.rows_max, sh.Hkv, batch);
  const int32_t* uc = prep ? prep->ucount : nullptr;
  const int32_t* mr = prep ? prep->mrows : nullptr;
  const int known = rows_hint >= 1 || !active_idx;   // (no list of active tokens: every row exists)
  if (sh.d == 128) {
    if (prep)
      attn_merge_kernel<128, true><<<grid, 256, 0, st>>>(kv, sh, active_idx, active_count, sel_count, cap, nchunk, uc, mr, part, o_p, lse_p, known);
    else
      attn_merge_kernel<128, false><<<grid, 256, 0, st>>>(kv, sh, active_idx, active_count, sel_count, cap, nchunk, uc, mr, part, o_p, lse_p, known);
  } else {
    if (prep)
      attn_merge_kernel<64, true><<<grid, 256, 0, st>>>(kv, sh, active_idx, active_count, sel_count, cap, nchunk, uc, mr, part, o_p, lse_p, known);
    else
      attn_merge_kernel<64, false><<<grid, 256, 0, st>>>(kv, sh, active_idx, active_count, sel_count, cap, nchunk, uc, mr, part, o_p, lse_p, known);
  }
  return hipGetLastError();
}

}  // namespace losa
