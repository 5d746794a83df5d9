// Split-K paged sparse prefix attention on the gfx950 matrix cores, bfloat16 inputs
// (paper: Preliminaries, Attention Decomposition With Online Softmax; Methodology, eq. update_rule).
//
// One wavefront owns up to R*16 query rows of one KV head and walks 32-token tiles of that
// head's page list with v_mfma_f32_16x16x32_bf16:
//
//   S^T = K_tile . Q^T      A operand = 16 keys x 32 channels, read straight from the
//                           token-major key page (each lane one 16-byte load);
//                           B operand = the query fragment, resident in registers.
//   O^T += V_tile^T . P^T   A operand = 16 channels x 32 tokens, read straight from the
//                           channel-major value page (two 8-byte loads per lane);
//                           B operand = P^T, which is exactly how S^T leaves the matrix core
//                           (lane = query column, 4+4 tokens), so probabilities never cross
//                           lanes and the per-row rescale factor is lane-local as well.
//
// The k-index of the second product is a permutation of the 32 tokens of a tile (slot e<4:
// token 4*(lane/16)+e of the first 16-token half, slot e>=4: the same of the second half);
// both operands use it, which is all a contraction needs.
//
// No LDS and no barrier in the main loop: K/V go global -> registers in operand layout, one
// tile ahead.  Two work shapes:
//   split-pages (rows <= 64): the four wavefronts of a workgroup take interleaved tiles of
//       the same chunk and combine their (max, sum, O) through LDS at the end, so one
//       partial leaves the workgroup;
//   split-rows (rows > 64, e.g. the dense initialisation): the four wavefronts take four
//       64-row blocks and all walk the same tiles (served by the CU's L1 after the first).
// Chunks are equal shares of the *actual* list length read from device memory, so every
// workgroup of a (sequence, head) gets the same number of tiles whatever the union size is.
#include <math.h>

#include "losa_device.h"
#include "losa_internal.h"

namespace losa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(8))) float f32x8_t;

constexpr float kNegBig = -1.0e30f;   // finite stand-in for "no token seen yet"

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D, int R>
struct MergeSlot {   // LDS image of one wavefront's state
  static constexpr int kStride = D + 4;   // +4 floats: 16-byte row writes of 16 lanes land on distinct banks
  static constexpr int kFloats = R * 16 * (kStride + 2);
};

template <int D, int GP, int R, bool SPLIT_PAGES>
__global__ __launch_bounds__(256) void attn_mfma_kernel(KvView kv, Shape sh, const bf16_t* __restrict__ q,
                                                        const int32_t* __restrict__ active_idx,
                                                        const int32_t* __restrict__ active_count,
                                                        const int32_t* __restrict__ sel_pages,
                                                        const int32_t* __restrict__ sel_count, int cap, int nchunk,
                                                        int nrbg, Partials part, float scale_log2e) {
  constexpr int KS = D / 32;    // k-steps of the score product
  constexpr int NT = D / 16;    // channel tiles of the output
  constexpr int PPT = 32 / GP;  // pages per 32-token tile
  extern __shared__ float lds[];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, qd = lane >> 4;
  const int chunk = blockIdx.x, b = blockIdx.z;
  const int j = SPLIT_PAGES ? blockIdx.y : blockIdx.y / nrbg;
  const int rb = SPLIT_PAGES ? 0 : (blockIdx.y % nrbg) * 4 + wave;

  const int n_act = active_idx ? min(active_count[b], sh.B) : sh.B;
  const int M = n_act * sh.G;
  if (M <= 0) return;
  if (!SPLIT_PAGES && rb * (R * 16) >= M) return;   // no barrier is used in this shape

  const int base = kv.page_indptr[b];
  const int P = min(kv.page_indptr[b + 1] - base, sh.max_pages);
  const int L = kv.seq_lens[b];
  const int32_t* list = sel_pages ? sel_pages + ((size_t)b * sh.Hkv + j) * cap : nullptr;
  const int U = list ? min(sel_count[b * sh.Hkv + j], cap) : P;
  const int ntiles = (U + PPT - 1) / PPT;
  const int tpc = (ntiles + nchunk - 1) / nchunk;   // tiles per chunk: equal shares of the real list
  const int tile0 = chunk * tpc;
  const int tile1 = min(ntiles, tile0 + tpc);
  if (tile0 >= tile1) return;

  const int wstart = SPLIT_PAGES ? wave : 0, wstride = SPLIT_PAGES ? 4 : 1;
  const int wfirst = tile0 + wstart;
  const int ntw = wfirst < tile1 ? (tile1 - wfirst + wstride - 1) / wstride : 0;   // this wavefront's tiles

  // ---- query fragments (B operand of the score product), zero for rows past M
  bf16x8_t qf[R][KS];
#pragma unroll
  for (int mt = 0; mt < R; ++mt) {
    const int rg = rb * (R * 16) + mt * 16 + l16;
    const bf16_t* qrow = nullptr;
    if (rg < M) {
      const int a = rg / sh.G, hg = rg % sh.G;
      const int tok = active_idx ? active_idx[(size_t)b * sh.B + a] : a;
      if ((unsigned)tok < (unsigned)sh.B) qrow = q + (((size_t)b * sh.B + tok) * sh.Hq + j * sh.G + hg) * D;
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 raw = make_uint4(0u, 0u, 0u, 0u);
      if (qrow) raw = *reinterpret_cast<const uint4*>(qrow + ks * 32 + qd * 8);
      qf[mt][ks] = __builtin_bit_cast(bf16x8_t, raw);
    }
  }

  float m_run[R], l_run[R];
  f32x4_t o[R][NT];
#pragma unroll
  for (int mt = 0; mt < R; ++mt) {
    m_run[mt] = kNegBig;
    l_run[mt] = 0.f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) o[mt][nt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
  }

  // ---- page ids of this wavefront's next 64 pages, one per lane (refilled every 64/PPT tiles)
  int pg_phys = 0, pg_valid = 0;
  auto fetch_pages = [&](int first_local_tile) {
    const int n = first_local_tile + lane / PPT;
    const int lp = (wfirst + n * wstride) * PPT + lane % PPT;
    int phys = 0, valid = 0;
    if (n < ntw && lp < U) {
      const int logical = list ? list[lp] : lp;
      if ((unsigned)logical < (unsigned)P) {
        const int ph = kv.page_indices[base + logical];
        if ((unsigned)ph < (unsigned)kv.num_pages) {
          phys = ph;
          valid = max(0, min(GP, L - logical * GP));
        }
      }
    }
    pg_phys = phys;
    pg_valid = valid;
  };

  struct Tile {
    bf16x8_t k[2][KS];
    uint2 v[NT][2];
    int nv[2];
  };

  auto load_tile = [&](Tile& t, int n) {
    const int slot = (n * PPT) & 63;
    const bf16_t *kA, *kB, *vA, *vB;
    if (GP == 16) {
      const int pa = __builtin_amdgcn_readlane(pg_phys, slot), pb = __builtin_amdgcn_readlane(pg_phys, slot + 1);
      t.nv[0] = __builtin_amdgcn_readlane(pg_valid, slot);
      t.nv[1] = __builtin_amdgcn_readlane(pg_valid, slot + 1);
      const size_t ta = (size_t)pa * sh.Hkv + j, tb = (size_t)pb * sh.Hkv + j;
      kA = (const bf16_t*)kv.k_pages + ta * (GP * D);
      kB = (const bf16_t*)kv.k_pages + tb * (GP * D);
      vA = (const bf16_t*)kv.v_pages + ta * (GP * D);
      vB = (const bf16_t*)kv.v_pages + tb * (GP * D);
    } else {
      const int pa = __builtin_amdgcn_readlane(pg_phys, slot);
      const int nv = __builtin_amdgcn_readlane(pg_valid, slot);
      t.nv[0] = min(nv, 16);
      t.nv[1] = max(nv - 16, 0);
      const size_t ta = (size_t)pa * sh.Hkv + j;
      kA = (const bf16_t*)kv.k_pages + ta * (GP * D);
      kB = kA + 16 * D;
      vA = (const bf16_t*)kv.v_pages + ta * (GP * D);
      vB = vA + 16;
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      t.k[0][ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(kA + l16 * D + ks * 32 + qd * 8));
      t.k[1][ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(kB + l16 * D + ks * 32 + qd * 8));
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      t.v[nt][0] = *reinterpret_cast<const uint2*>(vA + (nt * 16 + l16) * GP + qd * 4);
      t.v[nt][1] = *reinterpret_cast<const uint2*>(vB + (nt * 16 + l16) * GP + qd * 4);
    }
  };

  auto compute_tile = [&](Tile& t) {
    const bool full = (t.nv[0] == 16) && (t.nv[1] == 16);
    if (!full) {
      // slots past the end of the sequence may hold anything: clear them in V (0 * NaN = NaN)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        const int cnt = max(0, min(4, t.nv[hf] - qd * 4));
        const unsigned long long keep = cnt >= 4 ? ~0ull : ((1ull << (16 * cnt)) - 1ull);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          t.v[nt][hf].x &= (unsigned)keep;
          t.v[nt][hf].y &= (unsigned)(keep >> 32);
        }
      }
    }
#pragma unroll
    for (int mt = 0; mt < R; ++mt) {
      f32x4_t sA = {0.f, 0.f, 0.f, 0.f}, sB = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sA = __builtin_amdgcn_mfma_f32_16x16x32_bf16(t.k[0][ks], qf[mt][ks], sA, 0, 0, 0);
        sB = __builtin_amdgcn_mfma_f32_16x16x32_bf16(t.k[1][ks], qf[mt][ks], sB, 0, 0, 0);
      }
      float s[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s[e] = sA[e] * scale_log2e;
        s[4 + e] = sB[e] * scale_log2e;
      }
      if (!full) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (qd * 4 + (e & 3) >= t.nv[e >> 2]) s[e] = -INFINITY;
      }
      float tmax = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float m_new = fmaxf(m_run[mt], tmax);
      const float alpha = fast_exp2(m_run[mt] - m_new);
      m_run[mt] = m_new;
      f32x8_t p;
#pragma unroll
      for (int e = 0; e < 8; ++e) p[e] = fast_exp2(s[e] - m_new);
      // P as a bfloat16 pair hi + lo (16 mantissa bits): one bfloat16 alone costs 2^-9 of the
      // spread of V per row, which outlier value channels push past the 2e-2 bound.
      const bf16x8_t p_hi = __builtin_convertvector(p, bf16x8_t);
      const f32x8_t hi_f = __builtin_convertvector(p_hi, f32x8_t);
      const bf16x8_t p_lo = __builtin_convertvector(p - hi_f, bf16x8_t);
      const f32x8_t lo_f = __builtin_convertvector(p_lo, f32x8_t);
      // the row sum uses the same rounded values the products see
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) psum += hi_f[e] + lo_f[e];
      l_run[mt] = l_run[mt] * alpha + psum;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        o[mt][nt] *= alpha;
        const bf16x8_t vv = __builtin_bit_cast(bf16x8_t, make_uint4(t.v[nt][0].x, t.v[nt][0].y, t.v[nt][1].x, t.v[nt][1].y));
        o[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vv, p_hi, o[mt][nt], 0, 0, 0);
        o[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vv, p_lo, o[mt][nt], 0, 0, 0);
      }
    }
  };

  // ---- main loop, one tile of lookahead in registers
  constexpr int TPR = 64 / PPT;   // tiles per page-id refill
  Tile t0, t1;
  if (ntw > 0) {
    fetch_pages(0);
    load_tile(t0, 0);
  }
  for (int n = 0; n < ntw; n += 2) {
    if (n + 1 < ntw) {
      if (((n + 1) % TPR) == 0) fetch_pages(n + 1);
      load_tile(t1, n + 1);
    }
    compute_tile(t0);
    if (n + 2 < ntw) {
      if (((n + 2) % TPR) == 0) fetch_pages(n + 2);
      load_tile(t0, n + 2);
    }
    if (n + 1 < ntw) compute_tile(t1);
  }

  // each lane summed its own tokens; rows are spread over the 4 lane groups
#pragma unroll
  for (int mt = 0; mt < R; ++mt) {
    l_run[mt] += __shfl_xor(l_run[mt], 16, 64);
    l_run[mt] += __shfl_xor(l_run[mt], 32, 64);
  }

  if (SPLIT_PAGES) {
    // ---- deterministic tree over the 4 wavefronts through LDS: (1->0, 3->2), then 2->0
    typedef MergeSlot<D, R> Slot;
    auto put = [&](float* slot) {
      float* so = slot;
      float* sm = slot + R * 16 * Slot::kStride;
      float* sl = sm + R * 16;
#pragma unroll
      for (int mt = 0; mt < R; ++mt) {
        const int r = mt * 16 + l16;
        if (qd == 0) {
          sm[r] = m_run[mt];
          sl[r] = l_run[mt];
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          *reinterpret_cast<f32x4_t*>(so + r * Slot::kStride + nt * 16 + qd * 4) = o[mt][nt];
      }
    };
    auto take = [&](const float* slot) {
      const float* so = slot;
      const float* sm = slot + R * 16 * Slot::kStride;
      const float* sl = sm + R * 16;
#pragma unroll
      for (int mt = 0; mt < R; ++mt) {
        const int r = mt * 16 + l16;
        const float m_o = sm[r], l_o = sl[r];
        const float m_n = fmaxf(m_run[mt], m_o);
        const float wa = fast_exp2(m_run[mt] - m_n), wb = fast_exp2(m_o - m_n);
        m_run[mt] = m_n;
        l_run[mt] = l_run[mt] * wa + l_o * wb;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const f32x4_t other = *reinterpret_cast<const f32x4_t*>(so + r * Slot::kStride + nt * 16 + qd * 4);
          o[mt][nt] = o[mt][nt] * wa + other * wb;
        }
      }
    };
    float* slot0 = lds;
    float* slot1 = lds + Slot::kFloats;
    if (wave == 1) put(slot0);
    if (wave == 3) put(slot1);
    __syncthreads();
    if (wave == 0) take(slot0);
    if (wave == 2) take(slot1);
    __syncthreads();
    if (wave == 2) put(slot0);
    __syncthreads();
    if (wave != 0) return;
    take(slot0);
  }

  // ---- partial of this (sequence, head, chunk): un-normalised O, running max (log2 units), sum
  const size_t item = ((size_t)b * sh.Hkv + j) * nchunk + chunk;
#pragma unroll
  for (int mt = 0; mt < R; ++mt) {
    const int rg = rb * (R * 16) + mt * 16 + l16;
    if (rg < M) {
      const size_t prow = item * sh.rows_max + rg;
      if (qd == 0) {
        part.m[prow] = m_run[mt];
        part.l[prow] = l_run[mt];
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        *reinterpret_cast<f32x4_t*>(part.o + prow * D + nt * 16 + qd * 4) = o[mt][nt];
    }
  }
}

template <int D, int GP, int R, bool SPLIT>
static hipError_t launch_one(hipStream_t st, const KvView& kv, const Shape& sh, int batch, const void* q,
                             const int32_t* active_idx, const int32_t* active_count, const int32_t* sel_pages,
                             const int32_t* sel_count, int cap, int nchunk, const Partials& part) {
  const int nrbg = SPLIT ? 1 : (sh.rows_max + R * 16 * 4 - 1) / (R * 16 * 4);
  const size_t lds_bytes = SPLIT ? 2 * MergeSlot<D, R>::kFloats * sizeof(float) : 0;
  auto kern = attn_mfma_kernel<D, GP, R, SPLIT>;
  if (lds_bytes > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds_bytes);
    if (e != hipSuccess) return e;
  }
  const float scale_log2e = sh.sm_scale * 1.4426950408889634f;
  dim3 grid(nchunk, sh.Hkv * nrbg, batch);
  kern<<<grid, 256, lds_bytes, st>>>(kv, sh, (const bf16_t*)q, active_idx, active_count, sel_pages, sel_count, cap,
                                     nchunk, nrbg, part, scale_log2e);
  return hipGetLastError();
}

template <int D, int GP>
static hipError_t launch_dg(hipStream_t st, const KvView& kv, const Shape& sh, int batch, const void* q,
                            const int32_t* ai, const int32_t* ac, const int32_t* sp, const int32_t* sc, int cap,
                            int nchunk, int rows_upper, const Partials& part) {
  if (rows_upper <= 16) return launch_one<D, GP, 1, true>(st, kv, sh, batch, q, ai, ac, sp, sc, cap, nchunk, part);
  if (rows_upper <= 32) return launch_one<D, GP, 2, true>(st, kv, sh, batch, q, ai, ac, sp, sc, cap, nchunk, part);
  if (rows_upper <= 48) return launch_one<D, GP, 3, true>(st, kv, sh, batch, q, ai, ac, sp, sc, cap, nchunk, part);
  if (rows_upper <= 64) return launch_one<D, GP, 4, true>(st, kv, sh, batch, q, ai, ac, sp, sc, cap, nchunk, part);
  return launch_one<D, GP, 4, false>(st, kv, sh, batch, q, ai, ac, sp, sc, cap, nchunk, part);
}

hipError_t launch_attn_mfma(hipStream_t st, const KvView& kv, const Shape& sh, int batch, const void* q,
                            const int32_t* active_idx, const int32_t* active_count, const int32_t* sel_pages,
                            const int32_t* sel_count, int cap, int nchunk, int rows_upper, const Partials& part) {
  if (batch <= 0 || nchunk <= 0) return hipSuccess;
  if (sh.d == 128) {
    if (sh.g == 16)
      return launch_dg<128, 16>(st, kv, sh, batch, q, active_idx, active_count, sel_pages, sel_count, cap, nchunk, rows_upper, part);
    return launch_dg<128, 32>(st, kv, sh, batch, q, active_idx, active_count, sel_pages, sel_count, cap, nchunk, rows_upper, part);
  }
  if (sh.g == 16)
    return launch_dg<64, 16>(st, kv, sh, batch, q, active_idx, active_count, sel_pages, sel_count, cap, nchunk, rows_upper, part);
  return launch_dg<64, 32>(st, kv, sh, batch, q, active_idx, active_count, sel_pages, sel_count, cap, nchunk, rows_upper, part);
}

}  // namespace losa
