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
  select_sequence<false>(a, b, F, st.frontier_begin[b], status, lds);
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

// Alg. 1, last step: T <- Top-N(T by p(u)).  One workgroup per sequence, one thread per node.
// Order: (path confidence descending, node id ascending): a key of 64 bits, the order-preserving
// image of the fp64 log confidence with its low 8 bits replaced by 255 - id.  (Dropping 8 of
// the 52 mantissa bits only matters for confidences closer than 2^-44 relative, far below
// what decides anything here.)  A node's confidence never exceeds its parent's and the parent
// has the smaller id, so the kept set is closed under "parent of".  Kept nodes keep their
// order; arrays are compacted in place.
__global__ __launch_bounds__(kThreads) void prune_kernel(talon_tree_state st, int n_keep, int32_t* kept_ids) {
  static_assert(TALON_N_MAX <= kThreads && TALON_N_MAX <= 256, "one thread per node, 8-bit ids");
  __shared__ __attribute__((aligned(16))) unsigned long long s_key[TALON_N_MAX];
  __shared__ int s_new[TALON_N_MAX];
  __shared__ int s_red[8];
  const int b = blockIdx.x;
  const int i = threadIdx.x;
  const int n = st.n_nodes[b];
  const size_t base = static_cast<size_t>(b) * st.N_pad;
  int token = 0, parent = -1, depth = 0;
  float prob = 0.f;
  double logp = 0.0;
  unsigned long long key = 0ull;
  if (i < n) {
    token = st.token[base + i]; parent = st.parent[base + i]; depth = st.depth[base + i];
    prob = st.prob[base + i]; logp = st.logp[base + i];
    key = (sortable_u64(logp) & ~0xFFull) | static_cast<unsigned long long>(255 - i);
    if ((key >> 8) == 0ull) key |= 0x100ull;   // never the "no node" key
  }
  s_key[i] = key;
  __syncthreads();
  int rank = 0;
  if (i < n) {
    const ulonglong2* kp = reinterpret_cast<const ulonglong2*>(s_key);
    for (int j = 0; j < TALON_N_MAX / 2; j += 8) {
      ulonglong2 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = kp[j + u];
#pragma unroll
      for (int u = 0; u < 8; ++u) rank += ((v[u].x > key) ? 1 : 0) + ((v[u].y > key) ? 1 : 0);
    }
  }
  const bool keep = i < n && rank < n_keep;
  int total;
  const int pos = block_exclusive_scan_i32(keep ? 1 : 0, s_red, &total);
  s_new[i] = keep ? pos : -1;
  __syncthreads();   // every thread has read its node; the new ids are known
  if (keep) {
    st.token[base + pos] = token;
    st.parent[base + pos] = parent < 0 ? -1 : s_new[parent];
    st.depth[base + pos] = depth;
    st.prob[base + pos] = prob;
    st.logp[base + pos] = logp;
    kept_ids[base + pos] = i;
  }
  if (i < st.N_pad && i >= total) kept_ids[base + i] = -1;
  if (i == 0) {
    st.n_nodes[b] = total;
    st.frontier_begin[b] = total;
    st.frontier_count[b] = 0;
    st.status[b] = st.status[b] | TALON_STATUS_DONE_BUDGET;
  }
}

}  // namespace

hipError_t launch_prune(const talon_tree_state& st, int n_keep, int32_t* kept_ids, hipStream_t s) {
  hipLaunchKernelGGL(prune_kernel, dim3(st.B), dim3(kThreads), 0, s, st, n_keep, kept_ids);
  return hipGetLastError();
}

hipError_t launch_select(const SelectArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(select_kernel, dim3(a.st.B), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_mask(const talon_tree_state& st, uint64_t* mask, hipStream_t s) {
  hipLaunchKernelGGL(mask_kernel, dim3(st.B), dim3(kThreads), 0, s, st, mask);
  return hipGetLastError();
}

}  // namespace talon
