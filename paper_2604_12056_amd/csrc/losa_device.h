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

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
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
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(incl, o, 64);
    if (lane >= o) incl += t;
  }
  if (lane == 63) wave_tot[wid] = incl;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int w = 0; w < nw; ++w) { int t = wave_tot[w]; wave_tot[w] = run; run += t; }
    wave_tot[16] = run;
  }
  __syncthreads();
  const int base = wave_tot[wid];
  *total = wave_tot[16];
  __syncthreads();   // scratch may be reused by the next call
  return base + incl - v;
}

}  // namespace losa
