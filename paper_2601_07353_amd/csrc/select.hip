// Stand-alone budget selection kernel (one workgroup per sequence; the work is in
// select_device.h) and the tree-mask kernel.
#include "select_device.h"

namespace talon {

namespace {

__global__ __launch_bounds__(kThreads) void select_kernel(SelectArgs a) {
  __shared__ unsigned long long s_key[kSelectKeySlots];
  __shared__ int s_hist[256];
  __shared__ unsigned long long s_red_u64[8];
  __shared__ int s_red_i32[8];
  __shared__ int s_misc[2];

  const talon_tree_state& st = a.st;
  const int b = blockIdx.x;
  const uint32_t status = st.status[b];
  const int F = st.frontier_count[b];
  if ((status & kDoneMask) || F <= 0) return;
  if (status & TALON_STATUS_BAD_ROW) {  // a row of this layer could not be normalised: stop here
    if (threadIdx.x == 0) st.frontier_count[b] = 0;
    return;
  }
  const SelectLds lds{s_key, s_hist, s_red_u64, s_red_i32, s_misc};
  select_sequence<false>(a, b, F, st.frontier_begin[b], status, lds, nullptr);
}

// Tree attention mask: bit j of row i set iff j is i or an ancestor of i (Fig. 5(b), App. B).
// One workgroup per sequence, one thread per node walking its parent chain in LDS.
__global__ __launch_bounds__(kThreads) void mask_kernel(talon_tree_state st, uint64_t* mask) {
  __shared__ int s_parent[TALON_N_MAX];
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int n = st.n_nodes[b];
  const int words = st.N_pad / 64;
  const size_t base = static_cast<size_t>(b) * st.N_pad;
  if (tid < st.N_pad) s_parent[tid] = tid < n ? st.parent[base + tid] : -1;
  __syncthreads();
  if (tid >= st.N_pad) return;
  uint64_t w0 = 0, w1 = 0, w2 = 0, w3 = 0;
  if (tid < n) {
    int j = tid;
    for (int step = 0; step < TALON_N_MAX && j >= 0; ++step) {
      const uint64_t bit = 1ull << (j & 63);
      const int q = j >> 6;
      w0 |= q == 0 ? bit : 0ull;
      w1 |= q == 1 ? bit : 0ull;
      w2 |= q == 2 ? bit : 0ull;
      w3 |= q == 3 ? bit : 0ull;
      j = s_parent[j];
    }
  }
  uint64_t* row = mask + (base + tid) * words;
  row[0] = w0;
  if (words > 1) row[1] = w1;
  if (words > 2) row[2] = w2;
  if (words > 3) row[3] = w3;
}

}  // namespace

hipError_t launch_select(const SelectArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(select_kernel, dim3(a.st.B), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_mask(const talon_tree_state& st, uint64_t* mask, hipStream_t s) {
  hipLaunchKernelGGL(mask_kernel, dim3(st.B), dim3(kThreads), 0, s, st, mask);
  return hipGetLastError();
}

}  // namespace talon
