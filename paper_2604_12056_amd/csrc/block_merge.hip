// Dense in-block attention and the final online-softmax merge with the cached prefix
// statistics (paper: Methodology, Computation of the Suffix Tokens and Final Output;
// Preliminaries, eq. full_attn and Attention Decomposition With Online Softmax):
//
//   s_b = sm_scale * q_i . k_b[t]   over the B tokens of the block (bidirectional)
//   L_b = ln sum_t exp(s_b),  o_b = sum_t exp(s_b - L_b) v_b[t]
//   O_i = (e^{L_p} o_p + e^{L_b} o_b) / (e^{L_p} + e^{L_b})
//
// B << L, so this is a few KiB per head and launch-latency bound.  Two kernels: a matrix-core
// one for bfloat16 blocks of up to 64 tokens (below), and an element-generic one (vector ALUs,
// one workgroup per (sequence, query head, 32 query tokens), keys and values of the block staged
// through LDS 32 tokens at a time; float accumulation for bfloat16 inputs, double for float
// inputs) for everything else.
#include <math.h>

#include <type_traits>

#include "losa_device.h"
#include "losa_internal.h"

namespace losa {

template <typename T, int D>
__global__ __launch_bounds__(256) void block_merge_kernel(Shape sh, const T* __restrict__ q, const T* __restrict__ k_b,
                                                          const T* __restrict__ v_b, const float* __restrict__ o_p,
                                                          const float* __restrict__ lse_p, float* __restrict__ out,
                                                          float* __restrict__ o_b, float* __restrict__ lse_b) {
  typedef typename std::conditional<std::is_same<T, float>::value, double, float>::type Acc;
  constexpr int V = Vec16<T>::n, VPR = D / V, CPT = D / 8, RB = 32, TK = 32;
  __shared__ float qs[RB][D + 1];
  __shared__ float ks[TK][D + 1];
  __shared__ float vs[TK][D + 1];
  __shared__ Acc ps[RB][TK + 1];
  const int rb = blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const int j = h / sh.G, r0 = rb * RB;
  if (r0 >= sh.B) return;

  for (int v = tid; v < RB * VPR; v += 256) {
    const int rr = v / VPR, cv = v % VPR, i = r0 + rr;
    float f[V];
#pragma unroll
    for (int e = 0; e < V; ++e) f[e] = 0.f;
    if (i < sh.B) {
      const uint4 raw = reinterpret_cast<const uint4*>(q + (((size_t)b * sh.B + i) * sh.Hq + h) * D)[cv];
      widen16(raw, f, T());
    }
#pragma unroll
    for (int e = 0; e < V; ++e) qs[rr][cv * V + e] = f[e];
  }
  const int row = tid / 8, sub = tid % 8;
  float m = -INFINITY;
  Acc l = 0, acc[CPT];
#pragma unroll
  for (int k = 0; k < CPT; ++k) acc[k] = 0;

  for (int t0 = 0; t0 < sh.B; t0 += TK) {
    __syncthreads();
    for (int v = tid; v < TK * VPR; v += 256) {
      const int ts = v / VPR, cv = v % VPR, t = t0 + ts;
      float fk[V], fv[V];
#pragma unroll
      for (int e = 0; e < V; ++e) fk[e] = fv[e] = 0.f;
      if (t < sh.B) {
        const size_t base = (((size_t)b * sh.B + t) * sh.Hkv + j) * D;
        widen16(reinterpret_cast<const uint4*>(k_b + base)[cv], fk, T());
        widen16(reinterpret_cast<const uint4*>(v_b + base)[cv], fv, T());
      }
#pragma unroll
      for (int e = 0; e < V; ++e) {
        ks[ts][cv * V + e] = fk[e];
        vs[ts][cv * V + e] = fv[e];
      }
    }
    __syncthreads();
    Acc s[4];
    float tmax = -INFINITY;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int ts = sub + 8 * k;
      Acc dot = 0;
#pragma unroll 8
      for (int c = 0; c < D; ++c) dot += (Acc)qs[row][c] * (Acc)ks[ts][c];
      s[k] = t0 + ts < sh.B ? dot * (Acc)sh.sm_scale : (Acc)-INFINITY;
      tmax = fmaxf(tmax, (float)s[k]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 1, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 2, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 4, 64));
    const float m_new = fmaxf(m, tmax);
    const Acc alpha = exp_acc((Acc)m - (Acc)m_new);   // m_new is finite: the block holds at least one token
    Acc psum = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const Acc p = exp_acc(s[k] - (Acc)m_new);
      ps[row][sub + 8 * k] = p;
      psum += p;
    }
    psum += __shfl_xor(psum, 1, 64);
    psum += __shfl_xor(psum, 2, 64);
    psum += __shfl_xor(psum, 4, 64);
    l = l * alpha + psum;
    m = m_new;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      Acc a = acc[k] * alpha;
#pragma unroll 8
      for (int ts = 0; ts < TK; ++ts) a += (Acc)ps[row][ts] * (Acc)vs[ts][sub + 8 * k];
      acc[k] = a;
    }
  }
  const int i = r0 + row;
  if (i >= sh.B) return;
  // ---- merge with the cached prefix statistics of this row
  const size_t orow = ((size_t)b * sh.B + i) * sh.Hq + h;
  const Acc Lb = (Acc)m + log_acc(l);
  const float Lp = lse_p[orow];
  const Acc Lm = Lb > (Acc)Lp ? Lb : (Acc)Lp;
  const Acc wb = exp_acc(Lb - Lm), wp = exp_acc((Acc)Lp - Lm);   // Lp = -inf (empty prefix) gives wp = 0
  const Acc inv = (Acc)1 / (wb + wp);
#pragma unroll
  for (int k = 0; k < CPT; ++k) {
    const int c = sub + 8 * k;
    const Acc ob = acc[k] / l;
    const Acc op = wp > 0 ? (Acc)o_p[orow * D + c] : (Acc)0;
    out[orow * D + c] = (float)((ob * wb + op * wp) * inv);
    if (o_b) o_b[orow * D + c] = (float)ob;
  }
  if (lse_b && sub == 0) lse_b[orow] = (float)Lb;
}

// Matrix-core form for bfloat16 blocks of up to 64 tokens (the block sizes the paper uses:
// 16, 32, 64).  One workgroup per (sequence, query head); wavefront w takes query rows
// 16w..16w+15 against all keys of the block.  Same transposed products and token order as the
// prefix kernel: S^T = K . Q^T leaves every lane with 8 consecutive tokens of its query row,
// which is the B operand of O^T += V^T . P^T; the values are staged once per workgroup into LDS
// in channel-major order (the block's V arrives token-major), so the A operand of the second
// product is one 16-byte LDS read.  All scores of a row fit in registers (at most 64 keys), so
// the softmax is two-pass, no running rescale.  P goes in as a bfloat16 pair hi + lo, as there.
typedef __attribute__((ext_vector_type(8))) __bf16 bm_bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float bm_f32x4_t;
typedef __attribute__((ext_vector_type(8))) float bm_f32x8_t;

template <int D>
__global__ __launch_bounds__(256) void block_merge_mfma_kernel(Shape sh, const bf16_t* __restrict__ q,
                                                               const bf16_t* __restrict__ k_b,
                                                               const bf16_t* __restrict__ v_b,
                                                               const float* __restrict__ o_p,
                                                               const float* __restrict__ lse_p, float* __restrict__ out,
                                                               float* __restrict__ o_b, float* __restrict__ lse_b) {
  constexpr int KS = D / 32, NT = D / 16, VPR = D / 8, TPAD = 64 + 8;   // tokens per LDS row (16-byte aligned rows)
  __shared__ __attribute__((aligned(16))) bf16_t vT[D][TPAD];
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6, l16 = lane & 15, qd = lane >> 4;
  const int j = h / sh.G, B = sh.B;   // B <= 64 (launcher)

  // ---- values of the block, transposed into LDS; tokens past B are zero
  for (int idx = tid; idx < 64 * VPR; idx += 256) {
    const int t = idx / VPR, cv = idx % VPR;
    uint4 raw = make_uint4(0u, 0u, 0u, 0u);
    if (t < B) raw = reinterpret_cast<const uint4*>(v_b + (((size_t)b * B + t) * sh.Hkv + j) * D)[cv];
    const uint32_t wds[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vT[cv * 8 + 2 * e][t] = (bf16_t)(wds[e] & 0xFFFFu);
      vT[cv * 8 + 2 * e + 1][t] = (bf16_t)(wds[e] >> 16);
    }
  }
  // ---- queries (B operand) and keys (A operands) straight from global memory in operand layout
  const int r0 = wave * 16;
  const int row = min(r0 + l16, B - 1);
  bm_bf16x8_t qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks] = __builtin_bit_cast(bm_bf16x8_t, *reinterpret_cast<const uint4*>(
                                                 q + (((size_t)b * B + row) * sh.Hq + h) * D + ks * 32 + qd * 8));
  const int ntile = (B + 31) / 32;   // 1 or 2 tiles of 32 keys
  // row i of half hh of a tile is its token 8*(i/4) + 4*hh + (i%4): lane group qd then ends up with
  // tokens 8*qd .. 8*qd+7 of the tile (half 0 gives +0..3, half 1 gives +4..7)
  bm_bf16x8_t kf[2][2][KS];
#pragma unroll
  for (int tl = 0; tl < 2; ++tl)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int t = 32 * tl + 8 * (l16 >> 2) + 4 * hh + (l16 & 3);
      const bf16_t* kr = k_b + (((size_t)b * B + min(t, B - 1)) * sh.Hkv + j) * D;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        kf[tl][hh][ks] = __builtin_bit_cast(bm_bf16x8_t, *reinterpret_cast<const uint4*>(kr + ks * 32 + qd * 8));
    }
  // the prefix statistics this row will be merged with: requested now, used at the very end
  const size_t orow_early = ((size_t)b * B + row) * sh.Hq + h;
  const float Lp = lse_p[orow_early];
  bm_f32x4_t op[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) op[nt] = *reinterpret_cast<const bm_f32x4_t*>(o_p + orow_early * D + nt * 16 + 4 * qd);
  __syncthreads();
  if (r0 >= B) return;

  const float scale_log2e = sh.sm_scale * 1.4426950408889634f;
  float s[2][8];
#pragma unroll
  for (int tl = 0; tl < 2; ++tl) {
    bm_f32x4_t sc0 = {0.f, 0.f, 0.f, 0.f}, sc1 = {0.f, 0.f, 0.f, 0.f};
    if (tl < ntile) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tl][0][ks], qf[ks], sc0, 0, 0, 0);
        sc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tl][1][ks], qf[ks], sc1, 0, 0, 0);
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int t0 = 32 * tl + 8 * qd + e, t1 = t0 + 4;
      s[tl][e] = t0 < B ? sc0[e] * scale_log2e : -INFINITY;       // log2 units from here on
      s[tl][4 + e] = t1 < B ? sc1[e] * scale_log2e : -INFINITY;
    }
  }
  float m = -INFINITY;
#pragma unroll
  for (int tl = 0; tl < 2; ++tl)
#pragma unroll
    for (int e = 0; e < 8; ++e) m = fmaxf(m, s[tl][e]);
  m = __uint_as_float(across_rows(__float_as_uint(m), [](uint32_t a, uint32_t c) {
    return __float_as_uint(fmaxf(__uint_as_float(a), __uint_as_float(c)));
  }));   // finite: the block holds at least one token
  bm_f32x4_t o[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) o[nt] = (bm_f32x4_t){0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
#pragma unroll
  for (int tl = 0; tl < 2; ++tl) {
    if (tl >= ntile) break;
    float pv[8];
    uint32_t pb[8];
    bm_f32x8_t lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pv[e] = __builtin_amdgcn_exp2f(s[tl][e] - m);
      l += pv[e];
      pb[e] = __float_as_uint(pv[e]);
      lo[e] = pv[e] - __uint_as_float(pb[e] & 0xFFFF0000u);
    }
    uint4 hi_bits;
    hi_bits.x = __builtin_amdgcn_perm(pb[1], pb[0], 0x07060302u);
    hi_bits.y = __builtin_amdgcn_perm(pb[3], pb[2], 0x07060302u);
    hi_bits.z = __builtin_amdgcn_perm(pb[5], pb[4], 0x07060302u);
    hi_bits.w = __builtin_amdgcn_perm(pb[7], pb[6], 0x07060302u);
    const bm_bf16x8_t p_hi = __builtin_bit_cast(bm_bf16x8_t, hi_bits);
    const bm_bf16x8_t p_lo = __builtin_convertvector(lo, bm_bf16x8_t);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const bm_bf16x8_t vf = __builtin_bit_cast(
          bm_bf16x8_t, *reinterpret_cast<const uint4*>(&vT[nt * 16 + l16][32 * tl + 8 * qd]));
      o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, p_hi, o[nt], 0, 0, 0);
      o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, p_lo, o[nt], 0, 0, 0);
    }
  }
  l = __uint_as_float(across_rows(__float_as_uint(l), [](uint32_t a, uint32_t c) {
    return __float_as_uint(__uint_as_float(a) + __uint_as_float(c));
  }));

  // ---- merge with the cached prefix statistics of this row (lane: row l16, channels 4*qd.. of each tile)
  const int i = r0 + l16;
  if (i >= B) return;
  const size_t orow = ((size_t)b * B + i) * sh.Hq + h;
  const float Lb = (m + log2f(l)) * 0.6931471805599453f;
  const float Lm = fmaxf(Lb, Lp);
  const float wb = expf(Lb - Lm), wp = expf(Lp - Lm);   // Lp = -inf (empty prefix) gives wp = 0
  const float inv = 1.0f / (wb + wp), inv_l = 1.0f / l;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const size_t at = orow * D + nt * 16 + 4 * qd;
    bm_f32x4_t ob = o[nt] * inv_l;
    const bm_f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
    const bm_f32x4_t opv = wp > 0.f ? op[nt] : zero;   // an empty prefix may hold anything in o_p, NaN included
    *reinterpret_cast<bm_f32x4_t*>(out + at) = (ob * wb + opv * wp) * inv;
    if (o_b) *reinterpret_cast<bm_f32x4_t*>(o_b + at) = ob;
  }
  if (lse_b && qd == 0) lse_b[orow] = Lb;
}

hipError_t launch_block_merge(hipStream_t st, int dtype, const Shape& sh, int batch, const void* q, const void* k_b,
                              const void* v_b, const float* o_p, const float* lse_p, float* out, float* o_b,
                              float* lse_b) {
  if (batch <= 0) return hipSuccess;
  if (dtype == LOSA_BF16 && sh.B <= 64) {
    dim3 mgrid(sh.Hq, batch);
    if (sh.d == 128)
      block_merge_mfma_kernel<128><<<mgrid, 256, 0, st>>>(sh, (const bf16_t*)q, (const bf16_t*)k_b, (const bf16_t*)v_b, o_p, lse_p, out, o_b, lse_b);
    else
      block_merge_mfma_kernel<64><<<mgrid, 256, 0, st>>>(sh, (const bf16_t*)q, (const bf16_t*)k_b, (const bf16_t*)v_b, o_p, lse_p, out, o_b, lse_b);
    return hipGetLastError();
  }
  dim3 grid((sh.B + 31) / 32, sh.Hq, batch);
  if (dtype == LOSA_BF16) {
    if (sh.d == 128)
      block_merge_kernel<bf16_t, 128><<<grid, 256, 0, st>>>(sh, (const bf16_t*)q, (const bf16_t*)k_b, (const bf16_t*)v_b, o_p, lse_p, out, o_b, lse_b);
    else
      block_merge_kernel<bf16_t, 64><<<grid, 256, 0, st>>>(sh, (const bf16_t*)q, (const bf16_t*)k_b, (const bf16_t*)v_b, o_p, lse_p, out, o_b, lse_b);
  } else {
    if (sh.d == 128)
      block_merge_kernel<float, 128><<<grid, 256, 0, st>>>(sh, (const float*)q, (const float*)k_b, (const float*)v_b, o_p, lse_p, out, o_b, lse_b);
    else
      block_merge_kernel<float, 64><<<grid, 256, 0, st>>>(sh, (const float*)q, (const float*)k_b, (const float*)v_b, o_p, lse_p, out, o_b, lse_b);
  }
  return hipGetLastError();
}

}  // namespace losa
