// Locality score and locality pruning (paper: eq. mse_locality; Methodology, Locality Pruning).
//
//   delta[r] = (1/H) * sum_c (h_cur[r,c] - h_prev[r,c])^2      one workgroup per block token
//   A        = top-n tokens by delta, or {delta > tau}          one workgroup per sequence
//
// The score kernel is a pure streaming read of 2*H elements per token (16-byte loads,
// wavefront butterfly + one LDS hop).  The ranking is by counting: with B <= 1024 tokens,
// rank_i = #{j : delta_j > delta_i or (delta_j == delta_i and j < i)} is B compares per
// thread out of LDS, cheaper than any sort and deterministic under ties.
#include "losa_device.h"
#include "losa_internal.h"

namespace losa {

template <typename T>
__global__ __launch_bounds__(256) void locality_delta_kernel(const T* __restrict__ h_cur,
                                                             const T* __restrict__ h_prev, int H,
                                                             float* __restrict__ delta) {
  constexpr int V = Vec16<T>::n;
  __shared__ float part[4];
  const int row = blockIdx.x;
  const uint4* a = reinterpret_cast<const uint4*>(h_cur + (size_t)row * H);
  const uint4* b = reinterpret_cast<const uint4*>(h_prev + (size_t)row * H);
  const int nvec = H / V;
  float acc = 0.f;
  for (int v = threadIdx.x; v < nvec; v += 256) {
    const uint4 x = a[v], y = b[v];
    float fx[V], fy[V];
    widen16(x, fx, T());
    widen16(y, fy, T());
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const float df = fx[e] - fy[e];
      acc = fmaf(df, df, acc);
    }
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) delta[row] = (part[0] + part[1] + part[2] + part[3]) / (float)H;
}

__global__ __launch_bounds__(1024) void rank_select_kernel(const float* __restrict__ delta, int B, int mode, int n,
                                                           float tau, uint8_t* __restrict__ mask,
                                                           int32_t* __restrict__ active_idx,
                                                           int32_t* __restrict__ active_count) {
  __shared__ float sd[1024];
  __shared__ int scan[17];
  const int b = blockIdx.x, i = threadIdx.x;
  const float di = (i < B) ? delta[(size_t)b * B + i] : 0.f;
  if (i < B) sd[i] = di;
  __syncthreads();
  int act = 0;
  if (i < B) {
    if (mode == LOSA_SEL_THRESHOLD) {
      act = di > tau;
    } else {
      int rank = 0;
      for (int j = 0; j < B; ++j) {
        const float dj = sd[j];
        rank += (dj > di) || (dj == di && j < i);
      }
      act = rank < n;
    }
  }
  int total;
  const int pos = block_exclusive_scan(act, scan, &total);
  if (i < B) {
    mask[(size_t)b * B + i] = (uint8_t)act;
    if (i >= total) active_idx[(size_t)b * B + i] = -1;
  }
  __syncthreads();
  if (act) active_idx[(size_t)b * B + pos] = i;
  if (i == 0) active_count[b] = total;
}

// Both steps in one launch: one workgroup per block token computes its score; the workgroup
// that draws the last ticket of a sequence ranks the B scores and writes the active set.
// Scores travel in agent-scope atomic stores (written through to memory) and the ranking
// workgroup reads them with plain loads: every score has one writer in this launch, no
// reader before the ticket, and the caches were invalidated when the launch began.
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
  for (int v = tid; v < nvec; v += 256) {
    const uint4 x = pa[v], y = pb[v];
    float fx[V], fy[V];
    widen16(x, fx, T());
    widen16(y, fy, T());
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const float df = fx[e] - fy[e];
      acc = fmaf(df, df, acc);
    }
  }
  acc = wave_sum(acc);
  if ((tid & 63) == 0) part[tid >> 6] = acc;
  __syncthreads();
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
  for (int i = tid; i < B; i += 256) sd[i] = delta[(size_t)b * B + i];
  __syncthreads();
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
          rank += (dk > di) || (dk == di && k < i);
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

hipError_t launch_locality_delta(hipStream_t st, int dtype, const void* h_cur, const void* h_prev, int rows, int H,
                                 float* delta) {
  if (rows <= 0) return hipSuccess;
  if (dtype == LOSA_BF16)
    locality_delta_kernel<bf16_t><<<rows, 256, 0, st>>>((const bf16_t*)h_cur, (const bf16_t*)h_prev, H, delta);
  else
    locality_delta_kernel<float><<<rows, 256, 0, st>>>((const float*)h_cur, (const float*)h_prev, H, delta);
  return hipGetLastError();
}

hipError_t launch_rank_select(hipStream_t st, const float* delta, int batch, int B, int mode, int n, float tau,
                              uint8_t* mask, int32_t* active_idx, int32_t* active_count) {
  if (batch <= 0) return hipSuccess;
  const int threads = ((B + 63) / 64) * 64;
  rank_select_kernel<<<batch, threads, 0, st>>>(delta, B, mode, n, tau, mask, active_idx, active_count);
  return hipGetLastError();
}

}  // namespace losa
