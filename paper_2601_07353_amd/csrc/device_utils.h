// Wavefront (64 lanes) and workgroup (256 threads) reduction helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace talon {

__device__ __forceinline__ float wave_max_f32(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ int wave_sum_i32(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    unsigned long long w = __shfl_xor(v, o);
    v = w > v ? w : v;
  }
  return v;
}

// Inclusive prefix sum across the 64 lanes of a wavefront.
__device__ __forceinline__ int wave_inclusive_scan_i32(int v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int w = __shfl_up(v, o);
    if (lane >= o) v += w;
  }
  return v;
}

// Workgroup-wide helpers for 256 threads.  `scratch` points at >= 8 values of T in LDS.
// Every helper starts and ends with a barrier, so scratch can be reused back to back.
__device__ __forceinline__ float block_max_f32(float v, float* scratch) {
  v = wave_max_f32(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(scratch[0], scratch[1]), fmaxf(scratch[2], scratch[3]));
}

__device__ __forceinline__ double block_sum_f64(double v, double* scratch) {
  v = wave_sum_f64(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  return (scratch[0] + scratch[1]) + (scratch[2] + scratch[3]);
}

__device__ __forceinline__ int block_sum_i32(int v, int* scratch) {
  v = wave_sum_i32(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v,
                                                            unsigned long long* scratch) {
  v = wave_max_u64(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long a = scratch[0] > scratch[1] ? scratch[0] : scratch[1];
  unsigned long long b = scratch[2] > scratch[3] ? scratch[2] : scratch[3];
  return a > b ? a : b;
}

// Exclusive prefix sum over the 256 threads; *total receives the workgroup sum.
__device__ __forceinline__ int block_exclusive_scan_i32(int v, int* scratch, int* total) {
  const int incl = wave_inclusive_scan_i32(v);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 63) scratch[wave] = incl;
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    if (w < wave) base += scratch[w];
  *total = scratch[0] + scratch[1] + scratch[2] + scratch[3];
  return base + incl - v;
}

// Order-preserving maps from IEEE bit patterns to unsigned integers.
__device__ __forceinline__ uint32_t sortable_u32(float x) {
  x = x + 0.0f;  // -0.0 -> +0.0 so that the two zeros tie
  uint32_t u = __float_as_uint(x);
  return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

__device__ __forceinline__ float unsortable_f32(uint32_t s) {
  uint32_t u = (s >> 31) ? (s ^ 0x80000000u) : ~s;
  return __uint_as_float(u);
}

__device__ __forceinline__ unsigned long long sortable_u64(double x) {
  x = x + 0.0;
  unsigned long long u = (unsigned long long)__double_as_longlong(x);
  return u ^ ((u >> 63) ? 0xFFFFFFFFFFFFFFFFull : 0x8000000000000000ull);
}

}  // namespace talon
