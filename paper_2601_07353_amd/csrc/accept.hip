// Verification outcome at temperature 0 (App. B "Token-Tree Verification", step (2); Sec. 2:
// the verifier accepts the longest matched prefix): from the target model's greedy token
// after every tree node, the longest root path on which every drafted token is the target's
// own choice, the token the target adds after it, and the move of the accepted tokens' keys
// and values into the prefix cache.
//
// The target's greedy tokens come from the vocabulary scan of expand.hip run with k = 1 over
// all nodes of every tree (a frontier that covers nodes 0 .. n-1); this file holds the small
// kernels around it.
#include "device_utils.h"
#include "talon_internal.h"

namespace talon {

namespace {

// Frontier that covers every node of every tree, a clean status word per sequence, and zero
// row tickets for the scan.
__global__ __launch_bounds__(kThreads) void all_nodes_frontier_kernel(talon_tree_state st, int32_t* begin, int32_t* count,
                                                                       uint32_t* status, int32_t* ticket) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i < st.B * st.N_pad) ticket[i] = 0;
  if (i < st.B) { begin[i] = 0; count[i] = st.n_nodes[i]; status[i] = 0u; }
}

// One workgroup per sequence, one thread per node.  A node is on the accepted path iff every
// edge from the root down to it carries the target's greedy token of the edge's upper end;
// such nodes form one chain (siblings carry distinct tokens), one per depth.
__global__ __launch_bounds__(kThreads) void accept_kernel(talon_tree_state st, const int32_t* target_token,
                                                          const uint32_t* scan_status, int32_t* path,
                                                          int32_t* accept_len, int32_t* bonus_token) {
  static_assert(TALON_N_MAX <= kThreads, "one thread per node");
  __shared__ int s_parent[TALON_N_MAX];
  __shared__ int s_target[TALON_N_MAX];
  __shared__ unsigned char s_match[TALON_N_MAX];
  __shared__ int s_red[8];
  const int b = blockIdx.x;
  const int i = threadIdx.x;
  const int n = st.n_nodes[b];
  const size_t base = static_cast<size_t>(b) * st.N_pad;
  int tok = -1;
  if (i < n) {
    s_parent[i] = st.parent[base + i];
    s_target[i] = target_token[base + i];
    tok = st.token[base + i];
  }
  __syncthreads();
  if (i < n) s_match[i] = (i == 0) || (tok == s_target[s_parent[i]]);
  __syncthreads();
  bool valid = i < n;
  int steps = 0;   // depth of node i
  for (int j = i; valid && j > 0 && steps < TALON_N_MAX; ++steps) {
    valid = s_match[j] != 0;
    j = s_parent[j];
  }
  // the deepest valid node ends the path
  int key = valid ? ((steps << 16) | i) : -1;
  key = wave_max_i32(key);
  if ((i & 63) == 0) s_red[i >> 6] = key;
  __syncthreads();
  key = max(max(s_red[0], s_red[1]), max(s_red[2], s_red[3]));
  const int len = key >> 16;          // accepted draft tokens (the root is not counted)
  const int last = key & 0xFFFF;
  if (valid) path[base + steps] = i;
  if (i < st.N_pad && i > len) path[base + i] = -1;
  if (i == 0) {
    accept_len[b] = len;
    bonus_token[b] = s_target[last];
    if (scan_status[b] & TALON_STATUS_BAD_ROW) atomicOr(&st.status[b], TALON_STATUS_BAD_ROW);
  }
}

// Block (j, b) copies the K and V rows of the j-th accepted node of sequence b (all KV heads)
// to position prefix_len[b] + j of the prefix cache.
__global__ __launch_bounds__(kThreads) void compact_kv_kernel(const uint16_t* k_tree, const uint16_t* v_tree,
                                                              const int32_t* path, const int32_t* accept_len,
                                                              const int32_t* prefix_len, int32_t* new_prefix_len,
                                                              uint16_t* k_prefix, uint16_t* v_prefix, int N_pad, int Hkv,
                                                              int Dh, int capacity, int64_t sb, int64_t st_, int64_t sh) {
  const int j = blockIdx.x;
  const int b = blockIdx.y;
  const int len = accept_len[b];
  int L = prefix_len[b];
  L = L < 0 ? 0 : L;
  if (j == 0 && threadIdx.x == 0) {
    const int want = L + len + 1;
    new_prefix_len[b] = want < capacity ? want : capacity;
  }
  if (j > len || L + j >= capacity) return;
  const int node = path[static_cast<size_t>(b) * N_pad + j];
  if (node < 0 || node >= N_pad) return;
  const int cpr = Dh / 8;                       // 16-byte chunks per head row
  const int chunks = Hkv * cpr;
  const size_t src = (static_cast<size_t>(b) * N_pad + node) * Hkv * Dh;
  const int64_t dst = static_cast<int64_t>(b) * sb + static_cast<int64_t>(L + j) * st_;
  for (int c = threadIdx.x; c < 2 * chunks; c += kThreads) {
    const bool is_v = c >= chunks;
    const int cc = is_v ? c - chunks : c;
    const int h = cc / cpr, q = cc - h * cpr;
    const uint4 v = *reinterpret_cast<const uint4*>((is_v ? v_tree : k_tree) + src + static_cast<size_t>(h) * Dh + q * 8);
    *reinterpret_cast<uint4*>((is_v ? v_prefix : k_prefix) + dst + static_cast<int64_t>(h) * sh + q * 8) = v;
  }
}

}  // namespace

hipError_t launch_all_nodes_frontier(const talon_tree_state& st, int32_t* begin, int32_t* count, uint32_t* status,
                                     int32_t* ticket, hipStream_t s) {
  const int n = st.B * st.N_pad;
  hipLaunchKernelGGL(all_nodes_frontier_kernel, dim3((n + kThreads - 1) / kThreads), dim3(kThreads), 0, s, st, begin, count,
                     status, ticket);
  return hipGetLastError();
}

hipError_t launch_accept(const talon_tree_state& st, const int32_t* target_token, const uint32_t* scan_status,
                         int32_t* path, int32_t* accept_len, int32_t* bonus_token, hipStream_t s) {
  hipLaunchKernelGGL(accept_kernel, dim3(st.B), dim3(kThreads), 0, s, st, target_token, scan_status, path, accept_len,
                     bonus_token);
  return hipGetLastError();
}

hipError_t launch_compact_kv(const uint16_t* k_tree, const uint16_t* v_tree, const int32_t* path, const int32_t* accept_len,
                             const int32_t* prefix_len, int32_t* new_prefix_len, uint16_t* k_prefix, uint16_t* v_prefix,
                             int B, int N_pad, int Hkv, int Dh, int capacity, int64_t sb, int64_t st_, int64_t sh,
                             hipStream_t s) {
  hipLaunchKernelGGL(compact_kv_kernel, dim3(N_pad, B), dim3(kThreads), 0, s, k_tree, v_tree, path, accept_len, prefix_len,
                     new_prefix_len, k_prefix, v_prefix, N_pad, Hkv, Dh, capacity, sb, st_, sh);
  return hipGetLastError();
}

}  // namespace talon
