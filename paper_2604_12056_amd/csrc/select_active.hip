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
#include <math.h>

#include <mutex>

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

// ---------------------------------------------------------------------------------------------
// Allocation-free variant of losa_select_active: the per-sequence ticket counters, which the
// other entry point keeps in the caller's workspace, live in a device array of this library.
// Every GPU holds its own copy of the array (at its own address) until the process ends.
namespace {

constexpr int kStaticMaxBatch = 4096;   // sequences per call: 16 KiB of ticket counters per GPU
constexpr int kStaticMaxBlock = 1024;   // tokens per block the ranking holds in LDS
constexpr int kStaticMaxDevices = 64;

static __device__ __align__(256) int32_t scratch[kStaticMaxBatch];

std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[kStaticMaxDevices] = {};   // device address of `scratch` per GPU; NULL: not resolved yet

// The device address of `scratch` on the current GPU (in host code the array's name is only a
// handle for this lookup, never an address a kernel may be given).
losa_status static_scratch(int32_t** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return losa::set_thread_error(LOSA_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kStaticMaxDevices)
    return losa::set_thread_error(LOSA_ERR_UNSUPPORTED, "device index %d outside 0..%d", dev, kStaticMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    int32_t* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return losa::set_thread_error(LOSA_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LOSA_OK;
}

}  // namespace

extern "C" losa_status losa_select_active_static(void* stream, int32_t dtype, int32_t batch, int32_t block_size,
                                                 int32_t hidden_size, const void* h_cur, const void* h_prev,
                                                 losa_select_mode mode, float param, float* delta, uint8_t* mask,
                                                 int32_t* active_idx, int32_t* active_count) {
  using losa::set_thread_error;
  if (dtype != LOSA_BF16 && dtype != LOSA_F32) return set_thread_error(LOSA_ERR_INVALID_ARG, "dtype must be LOSA_BF16 or LOSA_F32");
  if (batch < 1 || block_size < 1 || hidden_size < 1)
    return set_thread_error(LOSA_ERR_INVALID_ARG, "batch, block_size and hidden_size must be >= 1");
  if (batch > kStaticMaxBatch)
    return set_thread_error(LOSA_ERR_UNSUPPORTED, "batch %d is above the %d sequences the static scratch holds counters for",
                            batch, kStaticMaxBatch);
  if (block_size > kStaticMaxBlock)
    return set_thread_error(LOSA_ERR_UNSUPPORTED, "block_size %d is above %d", block_size, kStaticMaxBlock);
  if (hidden_size % 8 != 0) return set_thread_error(LOSA_ERR_UNSUPPORTED, "hidden_size must be a multiple of 8");
  if (!h_cur || !h_prev || !delta || !mask || !active_idx || !active_count)
    return set_thread_error(LOSA_ERR_INVALID_ARG, "losa_select_active_static: NULL pointer");
  int n = 0;
  float tau = 0.f;
  const int B = block_size;
  if (mode == LOSA_SEL_TOPK) {
    if (!(param >= 0.f)) return set_thread_error(LOSA_ERR_INVALID_ARG, "top-k parameter must be >= 0");
    n = param >= (float)B ? B : (int)param;
  } else if (mode == LOSA_SEL_FRACTION) {
    if (!(param >= 0.f && param <= 1.f)) return set_thread_error(LOSA_ERR_INVALID_ARG, "fraction must be in [0,1]");
    n = (int)floorf(param * (float)B + 0.5f);
    n = n < 1 ? 1 : (n > B ? B : n);
  } else if (mode == LOSA_SEL_THRESHOLD) {
    if (param != param) return set_thread_error(LOSA_ERR_INVALID_ARG, "threshold is NaN");
    tau = param;
  } else if (mode == LOSA_SEL_MASS) {
    if (!(param >= 0.f && param <= 1.f)) return set_thread_error(LOSA_ERR_INVALID_ARG, "mass fraction must be in [0,1]");
    tau = param;
  } else {
    return set_thread_error(LOSA_ERR_INVALID_ARG, "unknown select mode %d", (int)mode);
  }
  int32_t* tickets = nullptr;
  const losa_status ss = static_scratch(&tickets);
  if (ss != LOSA_OK) return ss;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  // The counters must start at zero.  A completed launch leaves them so, but the array is shared
  // by every call on this GPU and an earlier launch may have been abandoned half-way; they are
  // cleared with a fill kernel (which, unlike a memset node, replays correctly in a captured graph).
  hipError_t e = losa::launch_zero_ints(st, tickets, batch);
  if (e != hipSuccess) return set_thread_error(LOSA_ERR_HIP, "ticket clear launch: %s", hipGetErrorString(e));
  e = losa::launch_locality_select(st, dtype, h_cur, h_prev, batch, B, hidden_size, (int)mode, n, tau, delta, mask,
                                   active_idx, active_count, tickets);
  if (e != hipSuccess) return set_thread_error(LOSA_ERR_HIP, "locality_select launch: %s", hipGetErrorString(e));
  return LOSA_OK;
}
