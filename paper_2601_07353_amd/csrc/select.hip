// Hybrid allocation of the remaining node budget for one layer (Sec. 5.2; Alg. 2 "Hybrid
// Expansion Strategy" and "Budget Check"), one workgroup per sequence, all candidates of
// the layer resident in LDS:
//   score(u) = logp[v] + edge_logp(v, rank)                    (log of p(u) = p(v) P(w|x<=v))
//   layer < init_layers: keep the K_init best                   (Eq. 5)
//   else: anchor m_d = max score, keep score >= log(mu) + m_d   (Eq. 4)
//   more than R = N - |T| left: keep the R best                 (budget check)
// The R-th best score is found by an 8-pass radix select over order-preserving 64-bit
// images of the fp64 scores; equal scores are taken in (parent, rank) order.  Kept
// candidates are appended by a prefix-sum compaction, which yields node ids ordered
// (parent ascending, rank ascending) without a sort.
#include "device_utils.h"
#include "talon_internal.h"

namespace talon {

namespace {

constexpr int kMaxCand = TALON_N_MAX * TALON_K_MAX;  // frontier <= N-1 rows of k candidates
constexpr int kPerThread = kMaxCand / kThreads;      // 16 consecutive candidates per thread

__device__ __forceinline__ double unsortable_f64(unsigned long long s) {
  const unsigned long long u = (s >> 63) ? (s ^ 0x8000000000000000ull) : ~s;
  return __longlong_as_double(static_cast<long long>(u));
}

__global__ __launch_bounds__(kThreads) void select_kernel(SelectArgs a) {
  __shared__ unsigned long long s_key[kThreads * (kPerThread + 1)];
  __shared__ int s_hist[256];
  __shared__ unsigned long long s_red_u64[8];
  __shared__ int s_red_i32[8];
  __shared__ int s_digit, s_remaining;

  const talon_tree_state& st = a.st;
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const uint32_t status = st.status[b];
  const int F = st.frontier_count[b];
  if ((status & kDoneMask) || F <= 0) return;
  if (status & TALON_STATUS_BAD_ROW) {  // a row of this layer could not be normalised: stop here
    if (tid == 0) st.frontier_count[b] = 0;
    return;
  }
  const int fb = st.frontier_begin[b];
  const int n = st.n_nodes[b];
  const int d = st.depth_cur[b];
  const int R = st.N - n;
  const int k = a.k;
  const int C = F * k;
  const size_t base = static_cast<size_t>(b) * st.N_pad;

  // Thread t owns the `per` consecutive candidates [t*per, t*per+per) of the flat
  // (parent, rank) order.  Its LDS slots start at t*stride with stride odd, so that the
  // 64-bit accesses of a wavefront fall on distinct banks.
  const int per = (C + kThreads - 1) / kThreads;
  const int stride = per | 1;
  const int c_begin = tid * per;
  unsigned long long* my = s_key + tid * stride;

  // ---- path scores of the pool, as sortable keys (0 = no candidate)
  unsigned long long anchor_key = 0ull;
  for (int i = 0; i < per; ++i) {
    const int c = c_begin + i;
    unsigned long long key = 0ull;
    if (c < C) {
      const int p = c / k;
      const size_t ci = (base + fb + p) * k + (c - p * k);
      const double s = st.logp[base + fb + p] + a.cand_edge_logp[ci];
      if (a.cand_token[ci] >= 0 && s == s) {
        key = sortable_u64(s);
        if (key == 0ull) key = 1ull;
      }
    }
    my[i] = key;
    anchor_key = key > anchor_key ? key : anchor_key;
  }
  anchor_key = block_max_u64(anchor_key, s_red_u64);

  const bool init = d < a.init_layers;
  const int limit = init ? (a.K_init < R ? a.K_init : R) : R;
  unsigned long long thr_key = 1ull;
  if (!init && anchor_key != 0ull) {
    thr_key = sortable_u64(a.log_mu + unsortable_f64(anchor_key));
    if (thr_key == 0ull) thr_key = 1ull;
  }

  int n_pass_local = 0;
  for (int i = 0; i < per; ++i) n_pass_local += (my[i] >= thr_key) ? 1 : 0;
  const int n_pass = block_sum_i32(n_pass_local, s_red_i32);

  unsigned long long T = thr_key;     // keep key > T, and the first need_eq keys == T
  int need_eq = 0x7FFFFFFF;
  if (n_pass > limit) {
    // ---- radix select: the limit-th largest key, 8 bits per pass from the top
    unsigned long long prefix = 0ull;
    int remaining = limit;
    for (int pass = 0; pass < 8; ++pass) {
      const int shift = 56 - 8 * pass;
      s_hist[tid] = 0;
      __syncthreads();
      for (int i = 0; i < per; ++i) {
        const unsigned long long key = my[i];
        const bool match = pass == 0 || ((key ^ prefix) >> ((shift + 8) & 63)) == 0ull;
        if (match && key != 0ull) atomicAdd(&s_hist[static_cast<int>(key >> shift) & 255], 1);
      }
      __syncthreads();
      if (tid < 64) {
        // lane l owns digits 255-4l .. 252-4l, walked from the largest digit down
        int h[4], lane_sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) { h[j] = s_hist[255 - 4 * tid - j]; lane_sum += h[j]; }
        const int incl = wave_inclusive_scan_i32(lane_sum);
        const unsigned long long hit = __ballot(incl >= remaining);
        const int first = __ffsll(static_cast<long long>(hit)) - 1;
        if (tid == first) {
          int before = incl - lane_sum;
          int dg = 255 - 4 * tid;
#pragma unroll
          for (int j = 0; j < 3; ++j) {
            if (before + h[j] < remaining) { before += h[j]; --dg; } else break;
          }
          s_digit = dg;
          s_remaining = remaining - before;
        }
      }
      __syncthreads();
      prefix |= static_cast<unsigned long long>(s_digit) << shift;
      remaining = s_remaining;
      __syncthreads();
    }
    T = prefix;
    need_eq = remaining;
  }

  // ---- keep flags, ranks among equal keys, compaction
  int eq_local = 0;
  for (int i = 0; i < per; ++i) eq_local += (my[i] == T) ? 1 : 0;
  int eq_total;
  int eq_rank = block_exclusive_scan_i32(eq_local, s_red_i32, &eq_total);
  unsigned int keep_bits = 0u;
  int keep_local = 0;
  for (int i = 0; i < per; ++i) {
    const unsigned long long key = my[i];
    bool keep = key > T;
    if (key == T) { keep = eq_rank < need_eq; ++eq_rank; }
    if (key == 0ull) keep = false;
    if (keep) { keep_bits |= 1u << i; ++keep_local; }
  }
  int n_keep;
  int pos = block_exclusive_scan_i32(keep_local, s_red_i32, &n_keep);
  for (int i = 0; i < per; ++i) {
    if (keep_bits & (1u << i)) {
      const int c = c_begin + i;
      const int p = c / k;
      const size_t ci = (base + fb + p) * k + (c - p * k);
      const size_t o = base + n + pos;
      st.token[o] = a.cand_token[ci];
      st.parent[o] = fb + p;
      st.depth[o] = d + 1;
      st.prob[o] = a.cand_prob[ci];
      st.logp[o] = st.logp[base + fb + p] + a.cand_edge_logp[ci];
      ++pos;
    }
  }
  if (tid == 0) {
    const int n_new = n + n_keep;
    st.n_nodes[b] = n_new;
    st.frontier_begin[b] = n;
    st.frontier_count[b] = n_keep;
    st.depth_cur[b] = d + 1;
    uint32_t s = status;
    if (n_new >= st.N) s |= TALON_STATUS_DONE_BUDGET;
    else if (d + 1 >= a.max_depth) s |= TALON_STATUS_DONE_DEPTH;
    st.status[b] = s;
  }
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
