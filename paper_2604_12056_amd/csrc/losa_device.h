// Device-side helpers: element widening, 16-byte vector access, wavefront / block reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace losa {

typedef uint16_t bf16_t;  // bfloat16 bit pattern

__device__ __forceinline__ float bf16_to_f32(uint32_t bits) { return __uint_as_float(bits << 16); }

// Elements held by one 16-byte vector of T.
template <typename T> struct Vec16;
template <> struct Vec16<bf16_t> { static constexpr int n = 8; };
template <> struct Vec16<float> { static constexpr int n = 4; };

// Widen one 16-byte vector to floats.
__device__ __forceinline__ void widen16(const uint4& v, float (&f)[8], bf16_t) {
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
  f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}
__device__ __forceinline__ void widen16(const uint4& v, float (&f)[4], float) {
  f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
  f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
}

template <typename T> __device__ __forceinline__ float load_elem(const T* p);
template <> __device__ __forceinline__ float load_elem<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <> __device__ __forceinline__ float load_elem<float>(const float* p) { return *p; }

// ---- cross-lane traffic without LDS round trips: DPP row operations inside each row of 16
// lanes, then the two lane-swap instructions across rows.
// DPP controls (CDNA ISA, "DPP_CTRL"): row_shr:n = 0x110+n, row_ror:n = 0x120+n,
// row_bcast15 = 0x142 (lane 15 of each row to the next row), row_bcast31 = 0x143.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ int dpp_move(int v) {   // lanes without a source, or masked out, get 0
  return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xF, false);
}

// Combines the four rows once every lane of a row already holds that row's result.
template <typename F>
__device__ __forceinline__ uint32_t across_rows(uint32_t v, F op) {
  const auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  const uint32_t h = op(a[0], a[1]);
  const auto c = __builtin_amdgcn_permlane32_swap(h, h, false, false);
  return op(c[0], c[1]);
}
template <typename F>
__device__ __forceinline__ uint32_t wave_all_reduce(uint32_t v, F op) {
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x121, 0xF, 0xF, false));
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x122, 0xF, 0xF, false));
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x124, 0xF, 0xF, false));
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x128, 0xF, 0xF, false));
  return across_rows(v, op);
}
__device__ __forceinline__ float wave_sum(float v) {
  return __uint_as_float(wave_all_reduce(__float_as_uint(v), [](uint32_t a, uint32_t b) {
    return __float_as_uint(__uint_as_float(a) + __uint_as_float(b));
  }));
}
__device__ __forceinline__ float wave_max(float v) {
  return __uint_as_float(wave_all_reduce(__float_as_uint(v), [](uint32_t a, uint32_t b) {
    return __float_as_uint(fmaxf(__uint_as_float(a), __uint_as_float(b)));
  }));
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
  return wave_all_reduce(v, [](uint32_t a, uint32_t b) { return a < b ? a : b; });
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  return wave_all_reduce(v, [](uint32_t a, uint32_t b) { return a > b ? a : b; });
}
// Inclusive prefix sum over the 64 lanes.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += dpp_move<0x111>(v);
  v += dpp_move<0x112>(v);
  v += dpp_move<0x114>(v);
  v += dpp_move<0x118>(v);         // scanned inside each row of 16
  v += dpp_move<0x142, 0xA>(v);    // rows 1 and 3 take the total of the row before them
  v += dpp_move<0x143, 0xC>(v);    // rows 2 and 3 take the total of the first 32 lanes
  return v;
}

__device__ __forceinline__ float exp_acc(float x) { return expf(x); }
__device__ __forceinline__ double exp_acc(double x) { return exp(x); }
__device__ __forceinline__ float log_acc(float x) { return logf(x); }
__device__ __forceinline__ double log_acc(double x) { return log(x); }

// Exclusive prefix sum of one int per thread over a block of up to 1024 threads.
// `wave_tot` is LDS scratch of 17 ints.  Returns the exclusive prefix; *total gets the block sum.
// Every thread of the block must call it.
__device__ __forceinline__ int block_exclusive_scan(int v, int* wave_tot, int* total) {
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  const int incl = wave_inclusive_scan(v);
  if (lane == 63) wave_tot[wid] = incl;
  __syncthreads();
  int base = 0, sum = 0;
  for (int w = 0; w < nw; ++w) {
    const int t = wave_tot[w];
    base += w < wid ? t : 0;
    sum += t;
  }
  *total = sum;
  __syncthreads();   // scratch may be reused by the next call
  return base + incl - v;
}

}  // namespace losa
