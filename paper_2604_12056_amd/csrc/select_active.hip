// Locality score and locality pruning (paper: eq. mse_locality; Methodology, Locality Pruning).
//
//   delta[r] = (1/H) * sum_c (h_cur[r,c] - h_prev[r,c])^2      one workgroup per block token
//   A        = top-n tokens by delta, {delta > tau}, or the smallest set of top tokens that
//              carries a fraction tau of the block's total delta
//
// The score is a pure streaming read of 2*H elements per token (16-byte loads, a wavefront
// reduction in DPP / lane-swap steps, one LDS hop).  The ranking is by counting: with B <= 1024 tokens,
// rank_i = #{j : delta_j > delta_i or (delta_j == delta_i and j < i)} is B compares per
// thread out of LDS, cheaper than any sort and deterministic under ties.
#include "losa_device.h"
#include "losa_internal.h"

namespace losa {

// Both steps in one launch: one workgroup per block token computes its score; the workgroup
// that draws the last ticket of a sequence ranks the B scores and writes the active set
// (mode < 0: scores only - the step's scoring kernel then does the ranking itself).
// Scores travel in agent-scope atomic stores (written through to memory, completion awaited
// before the ticket is drawn) and the ranking workgroup reads them with agent-scope atomic
// loads, which are served from the coherence point, never from a line this compute unit or
// its die's L2 fetched earlier: several sequences' scores share a 128-byte line (B * 4 < 128,
// or any 32 tokens of a block), so a ranking workgroup of another sequence may have pulled
// the line in before all of this sequence's scores were written.
template <typename T>
__global__ __launch_bounds__(256) void locality_select_kernel(const T* __restrict__ h_cur, const T* __restrict__ h_prev,
                                                              int H, int B, int mode, int n, float tau,
                                                              float* __restrict__ delta, uint8_t* __restrict__ mask,
                                                              int32_t* __restrict__ active_idx,
                                                              int32_t* __restrict__ active_count,
                                                              int32_t* __restrict__ tickets) {
  constexpr int V = Vec16<T>::n;
  __shared__ float part[4];
  __shared__ float sd[1024];
  __shared__ int scan[17];
  __shared__ int s_last;
  const int row = blockIdx.x, b = row / B, tid = threadIdx.x;
  const uint4* pa = reinterpret_cast<const uint4*>(h_cur + (size_t)row * H);
  const uint4* pb = reinterpret_cast<const uint4*>(h_prev + (size_t)row * H);
  const int nvec = H / V;
  float acc = 0.f;
  constexpr int UN = 4;   // vectors of each operand in flight per thread
  for (int v0 = tid; v0 < nvec; v0 += 256 * UN) {
    uint4 x[UN], y[UN];
#pragma unroll
    for (int k = 0; k < UN; ++k) {   // clamped, so that all loads go out before the first is used
      const int v = min(v0 + 256 * k, nvec - 1);
      x[k] = pa[v];
      y[k] = pb[v];
    }
#pragma unroll
    for (int k = 0; k < UN; ++k) {
      float fx[V], fy[V];
      widen16(x[k], fx, T());
      widen16(y[k], fy, T());
      float part_k = 0.f;
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const float df = fx[e] - fy[e];
        part_k = fmaf(df, df, part_k);
      }
      acc += v0 + 256 * k < nvec ? part_k : 0.f;
    }
  }
  acc = wave_sum(acc);
  if ((tid & 63) == 0) part[tid >> 6] = acc;
  __syncthreads();
  if (mode < 0) {   // scores only: whoever ranks them runs in a later launch
    if (tid == 0) delta[row] = (part[0] + part[1] + part[2] + part[3]) / (float)H;
    return;
  }
  if (tid == 0) {
    const float d = (part[0] + part[1] + part[2] + part[3]) / (float)H;
    __hip_atomic_store(&delta[row], d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_s_waitcnt(0);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    s_last = __hip_atomic_fetch_add(&tickets[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == B - 1;
  }
  __syncthreads();
  if (!s_last) return;
  if (tid == 0) tickets[b] = 0;
  // ---- ranking by counting, B <= 1024: thread i handles tokens i, i+256, ...
  for (int i = tid; i < B; i += 256)
    sd[i] = __hip_atomic_load(&delta[(size_t)b * B + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (mode == LOSA_SEL_MASS) {
    // Cumulative-mass rule: scores in descending order, summed in that order in float; A is
    // the shortest prefix whose sum reaches tau * total.  Done as rank -> sorted copy -> one
    // sequential pass, so the float sums are taken in a defined order.
    __shared__ float sorted[1024];
    __shared__ int s_n;
    for (int i = tid; i < B; i += 256) {
      const float di = sd[i];
      int rank = 0;
      for (int k = 0; k < B; ++k) {
        const float dk = sd[k];
        rank += (int)(dk > di) | ((int)(dk == di) & (int)(k < i));   // bitwise: no branch per element
      }
      sorted[rank] = di;
    }
    __syncthreads();
    if (tid == 0) {
      float total = 0.f;
      for (int k = 0; k < B; ++k) total += sorted[k];
      const float target = tau * total;
      int cnt = 0;
      if (total > 0.f) {
        float run = 0.f;
        cnt = B;
        for (int k = 0; k < B; ++k) {
          run += sorted[k];
          if (run >= target) {
            cnt = k + 1;
            break;
          }
        }
        if (!(tau > 0.f)) cnt = 0;
      }
      s_n = cnt;
    }
    __syncthreads();
    n = s_n;
  }
  int base_out = 0;
  for (int i0 = 0; i0 < B; i0 += 256) {
    const int i = i0 + tid;
    int act = 0;
    if (i < B) {
      const float di = sd[i];
      if (mode == LOSA_SEL_THRESHOLD) {
        act = di > tau;
      } else {
        int rank = 0;
        for (int k = 0; k < B; ++k) {
          const float dk = sd[k];
          rank += (int)(dk > di) | ((int)(dk == di) & (int)(k < i));   // bitwise: no branch per element
        }
        act = rank < n;
      }
      mask[(size_t)b * B + i] = (uint8_t)act;
    }
    int total;
    const int pos = base_out + block_exclusive_scan(act, scan, &total);
    if (act) active_idx[(size_t)b * B + pos] = i;
    base_out += total;
  }
  for (int i = base_out + tid; i < B; i += 256) active_idx[(size_t)b * B + i] = -1;
  if (tid == 0) active_count[b] = base_out;
}

hipError_t launch_locality_select(hipStream_t st, int dtype, const void* h_cur, const void* h_prev, int batch, int B,
                                  int H, int mode, int n, float tau, float* delta, uint8_t* mask, int32_t* active_idx,
                                  int32_t* active_count, int32_t* tickets) {
  if (batch <= 0) return hipSuccess;
  if (dtype == LOSA_BF16)
    locality_select_kernel<bf16_t><<<batch * B, 256, 0, st>>>((const bf16_t*)h_cur, (const bf16_t*)h_prev, H, B, mode, n,
                                                              tau, delta, mask, active_idx, active_count, tickets);
  else
    locality_select_kernel<float><<<batch * B, 256, 0, st>>>((const float*)h_cur, (const float*)h_prev, H, B, mode, n,
                                                             tau, delta, mask, active_idx, active_count, tickets);
  return hipGetLastError();
}

hipError_t launch_locality_delta(hipStream_t st, int dtype, const void* h_cur, const void* h_prev, int batch, int B,
                                 int H, float* delta) {
  return launch_locality_select(st, dtype, h_cur, h_prev, batch, B, H, /*mode=*/-1, 0, 0.f, delta, nullptr, nullptr,
                                nullptr, nullptr);
}

}  // namespace losa
