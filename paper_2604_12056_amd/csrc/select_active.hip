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
