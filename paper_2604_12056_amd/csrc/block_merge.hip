// Dense in-block attention and the final online-softmax merge with the cached prefix
// statistics (paper: Methodology, Computation of the Suffix Tokens and Final Output;
// Preliminaries, eq. full_attn and Attention Decomposition With Online Softmax):
//
//   s_b = sm_scale * q_i . k_b[t]   over the B tokens of the block (bidirectional)
//   L_b = ln sum_t exp(s_b),  o_b = sum_t exp(s_b - L_b) v_b[t]
//   O_i = (e^{L_p} o_p + e^{L_b} o_b) / (e^{L_p} + e^{L_b})
//
// B << L, so this is a few KiB per head and launch-latency bound: one workgroup per
// (sequence, query head, 32 query tokens), keys and values of the block staged through LDS
// 32 tokens at a time, vector ALUs.  Accumulation type as in the element-generic attention
// kernel: float for bfloat16 inputs, double for float inputs.
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

hipError_t launch_block_merge(hipStream_t st, int dtype, const Shape& sh, int batch, const void* q, const void* k_b,
                              const void* v_b, const float* o_p, const float* lse_p, float* out, float* o_b,
                              float* lse_b) {
  if (batch <= 0) return hipSuccess;
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
