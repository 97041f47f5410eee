// Wavefront (64 lanes) and workgroup (256 threads) reduction helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace talon {

// ---- cross-lane moves without the LDS crossbar: DPP inside a row of 16 lanes, lane-swap
// instructions across rows.  Each helper returns the value held by the partner lane.
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <- lane 7-i of its group of 8
constexpr int kDppMirror = 0x140;     // lane i <- lane 15-i of its row

// All-reduce over the 64 lanes; OP(a, b) must be commutative and associative on 32-bit ints
// reinterpreted by the caller.  The two swap steps return {own, partner} in some order.
#define TALON_WAVE_ALLREDUCE_32(v, COMBINE)                                   \
  do {                                                                        \
    v = COMBINE(v, dpp_i32<kDppXor1>(v));                                     \
    v = COMBINE(v, dpp_i32<kDppXor2>(v));                                     \
    v = COMBINE(v, dpp_i32<kDppHalfMirror>(v));                               \
    v = COMBINE(v, dpp_i32<kDppMirror>(v));                                   \
    auto p16_ = __builtin_amdgcn_permlane16_swap(v, v, false, false);         \
    v = COMBINE(static_cast<int>(p16_[0]), static_cast<int>(p16_[1]));        \
    auto p32_ = __builtin_amdgcn_permlane32_swap(v, v, false, false);         \
    v = COMBINE(static_cast<int>(p32_[0]), static_cast<int>(p32_[1]));        \
  } while (0)

__device__ __forceinline__ int combine_max_f32(int a, int b) {
  return __float_as_int(fmaxf(__int_as_float(a), __int_as_float(b)));
}
__device__ __forceinline__ int combine_add_i32(int a, int b) { return a + b; }

__device__ __forceinline__ float wave_max_f32(float x) {
  int v = __float_as_int(x);
  TALON_WAVE_ALLREDUCE_32(v, combine_max_f32);
  return __int_as_float(v);
}

__device__ __forceinline__ int wave_sum_i32(int v) {
  TALON_WAVE_ALLREDUCE_32(v, combine_add_i32);
  return v;
}

__device__ __forceinline__ int combine_max_i32(int a, int b) { return a > b ? a : b; }
__device__ __forceinline__ int wave_max_i32(int v) {
  TALON_WAVE_ALLREDUCE_32(v, combine_max_i32);
  return v;
}

// 64-bit all-reduces move the two halves separately.
#define TALON_WAVE_ALLREDUCE_64(T, x, COMBINE)                                               \
  do {                                                                                       \
    union { T t; int w[2]; } a_, b_;                                                         \
    a_.t = x;                                                                                \
    b_.w[0] = dpp_i32<kDppXor1>(a_.w[0]); b_.w[1] = dpp_i32<kDppXor1>(a_.w[1]);              \
    a_.t = COMBINE(a_.t, b_.t);                                                              \
    b_.w[0] = dpp_i32<kDppXor2>(a_.w[0]); b_.w[1] = dpp_i32<kDppXor2>(a_.w[1]);              \
    a_.t = COMBINE(a_.t, b_.t);                                                              \
    b_.w[0] = dpp_i32<kDppHalfMirror>(a_.w[0]); b_.w[1] = dpp_i32<kDppHalfMirror>(a_.w[1]);  \
    a_.t = COMBINE(a_.t, b_.t);                                                              \
    b_.w[0] = dpp_i32<kDppMirror>(a_.w[0]); b_.w[1] = dpp_i32<kDppMirror>(a_.w[1]);          \
    a_.t = COMBINE(a_.t, b_.t);                                                              \
    {                                                                                        \
      auto l_ = __builtin_amdgcn_permlane16_swap(a_.w[0], a_.w[0], false, false);            \
      auto h_ = __builtin_amdgcn_permlane16_swap(a_.w[1], a_.w[1], false, false);            \
      a_.w[0] = l_[0]; a_.w[1] = h_[0]; b_.w[0] = l_[1]; b_.w[1] = h_[1];                    \
      a_.t = COMBINE(a_.t, b_.t);                                                            \
    }                                                                                        \
    {                                                                                        \
      auto l_ = __builtin_amdgcn_permlane32_swap(a_.w[0], a_.w[0], false, false);            \
      auto h_ = __builtin_amdgcn_permlane32_swap(a_.w[1], a_.w[1], false, false);            \
      a_.w[0] = l_[0]; a_.w[1] = h_[0]; b_.w[0] = l_[1]; b_.w[1] = h_[1];                    \
      a_.t = COMBINE(a_.t, b_.t);                                                            \
    }                                                                                        \
    x = a_.t;                                                                                \
  } while (0)

__device__ __forceinline__ double combine_add_f64(double a, double b) { return a + b; }
__device__ __forceinline__ unsigned long long combine_max_u64(unsigned long long a, unsigned long long b) {
  return a > b ? a : b;
}

// Note: the lane order of the additions is fixed, so the sum is reproducible run to run.
__device__ __forceinline__ double wave_sum_f64(double x) {
  TALON_WAVE_ALLREDUCE_64(double, x, combine_add_f64);
  return x;
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long x) {
  TALON_WAVE_ALLREDUCE_64(unsigned long long, x, combine_max_u64);
  return x;
}

// Inclusive prefix sum across the 64 lanes of a wavefront (all lanes active): a
// Kogge-Stone scan inside each row of 16 lanes (row_shr 1, 2, 4, 8; lanes shifted in from
// outside the row read 0), then the last lane of row 0/2 is added to row 1/3 (row_bcast:15)
// and lane 31 to rows 2 and 3 (row_bcast:31).
__device__ __forceinline__ int wave_inclusive_scan_i32(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);  // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);  // row_bcast:15 -> rows 1, 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);  // row_bcast:31 -> rows 2, 3
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
