// Attainable-rate probes for the two rooflines the library is measured against (no
// counterpart in the paper): a streaming read of a buffer (what fraction of the HBM figure a
// plain kernel reaches on this part) and a register-resident bf16 MFMA loop (what the matrix
// pipes sustain at the clocks they actually run at).  Two more probes time, in cycles of the
// shader clock, what the tree-attention step is made of: the issue cost of its vector and
// matrix instructions with one and two wavefronts per SIMD, and the rate at which a compute
// unit moves K/V tiles from an L2-resident window into LDS.
#include "talon_internal.h"

namespace talon {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// Every thread folds 16-byte vectors (8 loads in flight) into one word; the result is stored
// only if it has an unlikely value, so the loads cannot be dropped and nothing is written.
__global__ __launch_bounds__(kThreads) void read_probe_kernel(const uint4* p, size_t n_vec, uint32_t* sink) {
  const size_t stride = static_cast<size_t>(gridDim.x) * kThreads;
  size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
  uint32_t acc = 0u;
  for (; i + 7 * stride < n_vec; i += 8 * stride) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n_vec; i += stride) { const uint4 v = p[i]; acc ^= v.x ^ v.y ^ v.z ^ v.w; }
  if (acc == 0x9E3779B9u) sink[0] = acc;
}

// Four independent accumulator chains per wavefront, operands in registers.
__global__ __launch_bounds__(kThreads) void mfma_probe_kernel(int iters, float* sink) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = static_cast<__bf16>(0.001f * static_cast<float>((threadIdx.x + e) & 7));
    b[e] = static_cast<__bf16>(0.002f * static_cast<float>((threadIdx.x * 3 + e) & 7));
  }
  floatx16 c0, c1, c2, c3;
#pragma unroll
  for (int r = 0; r < 16; ++r) { c0[r] = 0.f; c1[r] = 0.f; c2[r] = 0.f; c3[r] = 0.f; }
  for (int i = 0; i < iters; ++i) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
  if (s == 123456.789f) sink[0] = s;
}


// ---- issue-rate probe.  One workgroup of 4 or 8 wavefronts (one or two per SIMD); every
// wavefront runs `iters` rounds of one instruction mix and stores the cycles it took.
// MODE 0: 32 independent exp2; 1: 32 independent fma; 2: 16 matrix instructions over 4
// accumulators; 3: 16 matrix instructions over 1 accumulator; 4: 16 matrix instructions with 32
// (fma, exp2) pairs between them.
template <int MODE>
__global__ __launch_bounds__(512) void issue_probe_kernel(unsigned long long* cycles, float* sink, int iters) {
  float x[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) x[i] = 0.001f * static_cast<float>(threadIdx.x + i);
  floatx16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) { a[e] = static_cast<__bf16>(0.5f + static_cast<float>(threadIdx.x & 7)); b[e] = static_cast<__bf16>(0.25f); }
  __syncthreads();
  const unsigned long long t0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
    if constexpr (MODE == 0) {
#pragma unroll
      for (int i = 0; i < 32; ++i) x[i] = __builtin_amdgcn_exp2f(x[i]);
    } else if constexpr (MODE == 1) {
#pragma unroll
      for (int i = 0; i < 32; ++i) x[i] = __builtin_fmaf(x[i], 0.999f, 0.001f);
    } else if constexpr (MODE == 2) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i & 3], 0, 0, 0);
    } else if constexpr (MODE == 3) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[0], 0, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i & 3], 0, 0, 0);
        x[2 * i] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[2 * i], 0.999f, 0.001f));
        x[2 * i + 1] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[2 * i + 1], 0.999f, 0.001f));
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
      }
    }
  }
  const unsigned long long t1 = __builtin_readcyclecounter();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i) s += x[i];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  if (s == 123456.789f) sink[0] = s;
  if ((threadIdx.x & 63) == 0) cycles[threadIdx.x >> 6] = t1 - t0;
}

// ---- tile-load probe.  256 workgroups (one per compute unit) of 4 or 8 wavefronts; in every
// round each wavefront issues LOADS direct-to-LDS loads of 1 KB (16 bytes per lane) from a
// 64 KB window of its workgroup (it stays in the L2), waits for them, and stores the cycles of
// all rounds.  With `with_mfma` sixteen matrix instructions are issued around the loads.
template <int LOADS, bool WITH_MFMA>
__global__ __launch_bounds__(512) void tile_load_probe_kernel(const uint16_t* src, unsigned long long* cycles, float* sink, int iters) {
  extern __shared__ __attribute__((aligned(16))) uint16_t probe_smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
  const uint16_t* base = src + static_cast<size_t>(blockIdx.x) * 32768;   // 64 KB of bf16 per workgroup
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
      (__attribute__((address_space(3))) void*)(probe_smem))) + static_cast<uint32_t>(wave * LOADS * 1024);
  floatx16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) { a[e] = static_cast<__bf16>(0.5f + static_cast<float>(lane & 7)); b[e] = static_cast<__bf16>(0.25f); }
  __syncthreads();
  const unsigned long long t0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
    // byte offset inside the window: four 16 KB quarters in turn, this wavefront's LOADS KB of a quarter
    const uint32_t off = static_cast<uint32_t>((it & 3) * 16384 + ((wave * LOADS) & 15) * 1024 + lane * 16);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if constexpr (WITH_MFMA) acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i & 3], 0, 0, 0);
      if (i % (16 / LOADS) == 0) {
        const uint32_t j = static_cast<uint32_t>(i / (16 / LOADS));
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :: "v"((off + j * 1024u) & 65535u), "s"(base), "s"(lds0 + j * 1024u) : "memory", "m0");
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  const unsigned long long t1 = __builtin_readcyclecounter();
  float s = static_cast<float>(probe_smem[threadIdx.x]);
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  if (s == 123456.789f) sink[0] = s;
  if (lane == 0) cycles[blockIdx.x * 8 + wave] = t1 - t0;
}

}  // namespace

hipError_t launch_read_probe(const void* buf, size_t bytes, void* sink, hipStream_t s) {
  hipLaunchKernelGGL(read_probe_kernel, dim3(2048), dim3(kThreads), 0, s, static_cast<const uint4*>(buf), bytes / 16,
                     static_cast<uint32_t*>(sink));
  return hipGetLastError();
}

hipError_t launch_mfma_probe(int workgroups, int iters, void* sink, hipStream_t s) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(kThreads), 0, s, iters, static_cast<float*>(sink));
  return hipGetLastError();
}

hipError_t launch_issue_probe(int mode, int waves, int iters, void* cycles, void* sink, hipStream_t s) {
  unsigned long long* c = static_cast<unsigned long long*>(cycles);
  float* k = static_cast<float*>(sink);
  const dim3 block(64 * waves);
  switch (mode) {
    case 0: hipLaunchKernelGGL(issue_probe_kernel<0>, dim3(1), block, 0, s, c, k, iters); break;
    case 1: hipLaunchKernelGGL(issue_probe_kernel<1>, dim3(1), block, 0, s, c, k, iters); break;
    case 2: hipLaunchKernelGGL(issue_probe_kernel<2>, dim3(1), block, 0, s, c, k, iters); break;
    case 3: hipLaunchKernelGGL(issue_probe_kernel<3>, dim3(1), block, 0, s, c, k, iters); break;
    default: hipLaunchKernelGGL(issue_probe_kernel<4>, dim3(1), block, 0, s, c, k, iters); break;
  }
  return hipGetLastError();
}

template <int LOADS, bool WITH_MFMA>
static hipError_t launch_tile_load_probe_t(int waves, int iters, const void* window, void* cycles, void* sink, hipStream_t s) {
  auto kern = tile_load_probe_kernel<LOADS, WITH_MFMA>;
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3(256), dim3(64 * waves), 65536, s, static_cast<const uint16_t*>(window),
                     static_cast<unsigned long long*>(cycles), static_cast<float*>(sink), iters);
  return hipGetLastError();
}

hipError_t launch_tile_load_probe(int loads, bool with_mfma, int waves, int iters, const void* window, void* cycles, void* sink, hipStream_t s) {
  if (loads == 4) return with_mfma ? launch_tile_load_probe_t<4, true>(waves, iters, window, cycles, sink, s)
                                   : launch_tile_load_probe_t<4, false>(waves, iters, window, cycles, sink, s);
  return with_mfma ? launch_tile_load_probe_t<8, true>(waves, iters, window, cycles, sink, s)
                   : launch_tile_load_probe_t<8, false>(waves, iters, window, cycles, sink, s);
}

}  // namespace talon
