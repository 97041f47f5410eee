// Budget selection of one layer for one sequence, as a workgroup-wide device function shared
// by the stand-alone select kernel and by the vocab-scan kernel that runs it in its tail.
//
// Hybrid allocation of the remaining node budget (Sec. 5.2; Alg. 2 "Hybrid Expansion
// Strategy" and "Budget Check"), all candidates of the layer resident in LDS:
//   score(u) = logp[v] + edge_logp(v, rank)                    (log of p(u) = p(v) P(w|x<=v))
//   layer < init_layers: keep the K_init best                   (Eq. 5)
//   else: anchor m_d = max score, keep score >= log(mu) + m_d   (Eq. 4)
//   more than R = N - |T| left: keep the R best                 (budget check)
// The R-th best score is found by an 8-pass radix select over order-preserving 64-bit
// images of the fp64 scores; equal scores are taken in (parent, rank) order.  Kept
// candidates are appended by a prefix-sum compaction, which yields node ids ordered
// (parent ascending, rank ascending) without a sort.
#pragma once

#include "device_utils.h"
#include "talon_internal.h"

namespace talon {

constexpr int kMaxCand = 4096;                       // candidates of one layer: frontier rows * k (checked on the host)
constexpr int kPerThread = kMaxCand / kThreads;      // at most 16 consecutive candidates per thread
constexpr int kSelectKeySlots = kThreads * (kPerThread + 1);

// LDS the selection needs; the caller provides it (the scan kernel carves it out of buffers
// that are idle by then).
struct SelectLds {
  unsigned long long* key;      // [kSelectKeySlots]
  int* hist;                    // [256]
  unsigned long long* red_u64;  // [8]
  int* red_i32;                 // [8]
  int* misc;                    // [2]
};

__device__ __forceinline__ double unsortable_f64(unsigned long long s) {
  const unsigned long long u = (s >> 63) ? (s ^ 0x8000000000000000ull) : ~s;
  return __longlong_as_double(static_cast<long long>(u));
}

// AGENT: the candidates, and the tree state of earlier layers, may have been written by other
// workgroups of the same launch, and what is written here may be read by others before the
// launch ends: such data is read and written at the device-coherent level.
template <bool AGENT, typename T>
__device__ __forceinline__ T ld(const T* p) {
  if constexpr (AGENT) return __hip_atomic_load(const_cast<T*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return *p;
}

template <bool AGENT, typename T>
__device__ __forceinline__ void st_(T* p, T v) {
  if constexpr (AGENT) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = v;
}

// Runs on all 256 threads of the workgroup.  F, fb: the frontier being expanded.  Returns, in
// thread 0, the new frontier as begin + (count << 32), count 0 if the sequence is done.
// n_known / d_known (>= 0): |T| and the layer index when the caller knows them (a launch that
// started the tree itself: the frontier is the newest F nodes, so |T| = fb + F); otherwise
// they are read from the tree state.  Either way the selection costs dependent memory round
// trips, which is what its time is made of, so it avoids every one it can: the token, edge
// probability and path score of a thread's first kRegCand candidates stay in registers from
// the scoring pass to the append.
constexpr int kRegCand = 4;
template <bool AGENT>
__device__ __forceinline__ unsigned long long select_sequence(const SelectArgs& a, int b, int F, int fb,
                                                              uint32_t status, const SelectLds& lds,
                                                              int n_known = -1, int d_known = -1) {
  const talon_tree_state& st = a.st;
  // (the thread index is taken afresh, through an empty asm statement: a caller that inlines this
  // into a long kernel would otherwise keep the per-thread addresses computed from it alive, or
  // spilled, across all of its own code)
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  unsigned long long* s_key = lds.key;
  int* s_hist = lds.hist;
  unsigned long long* s_red_u64 = lds.red_u64;
  int* s_red_i32 = lds.red_i32;
  int& s_digit = lds.misc[0];
  int& s_remaining = lds.misc[1];
  const int n = n_known >= 0 ? n_known : ld<AGENT, int32_t>(st.n_nodes + b);
  const int d = d_known >= 0 ? d_known : ld<AGENT, int32_t>(st.depth_cur + b);
  const int R = st.N - n;
  const int k = a.k;
  const int C = F * k;
  const size_t base = static_cast<size_t>(b) * st.N_pad;

  // One frontier row in a top-K-initialised layer (the first layer of every tree): the row's
  // candidates are already in key order (edge log-probability falls with the rank, ties in
  // rank order), so the K_init best of the pool are simply its first ones.
  if (F == 1 && d < a.init_layers && k <= 64) {
    const int limit = a.K_init < R ? a.K_init : R;
    const size_t ci = (base + fb) * k + tid;
    int tok = -1;
    float pr = 0.f;
    double score = 0.0;
    if (tid < k) {
      tok = ld<AGENT, int32_t>(a.cand_token + ci);
      pr = ld<AGENT, float>(a.cand_prob + ci);
      score = ld<AGENT, double>(st.logp + base + fb) + ld<AGENT, double>(a.cand_edge_logp + ci);
    }
    if (tid < 64) {   // the first wavefront holds the whole row
      const bool valid = tid < k && tok >= 0 && score == score;
      const unsigned long long vb = __ballot(valid);
      // candidates are valid up to the first invalid one (missing candidates sit at the end)
      const int n_valid = vb == ~0ull ? 64 : __builtin_ctzll(~vb);
      const int n_keep = n_valid < limit ? n_valid : limit;
      if (a.cap_hit && tid == 0 && n_keep >= k) st_<true, uint32_t>(a.cap_hit, 1u);   // the row's last candidate is kept
      if (tid < n_keep) {
        const size_t o = base + n + tid;
        st.token[o] = tok;
        st_<AGENT, int32_t>(st.parent + o, fb);
        st.depth[o] = d + 1;
        st.prob[o] = pr;
        st_<AGENT, double>(st.logp + o, score);
      }
      if (tid == 0) {
        const int n_new = n + n_keep;
        uint32_t s = status;
        if (n_new >= st.N) s |= TALON_STATUS_DONE_BUDGET;
        else if (d + 1 >= a.max_depth) s |= TALON_STATUS_DONE_DEPTH;
        st_<AGENT, int32_t>(st.n_nodes + b, n_new);
        st_<AGENT, int32_t>(st.frontier_begin + b, n);
        st_<AGENT, int32_t>(st.frontier_count + b, n_keep);
        st_<AGENT, int32_t>(st.depth_cur + b, d + 1);
        st_<AGENT, uint32_t>(st.status + b, s);
        return static_cast<unsigned long long>(static_cast<uint32_t>(n)) |
               (static_cast<unsigned long long>((s & kDoneMask) ? 0 : n_keep) << 32);
      }
    }
    return 0ull;
  }

  // Thread t owns the `per` consecutive candidates [t*per, t*per+per) of the flat
  // (parent, rank) order.  Its LDS slots start at t*stride with stride odd, so that the
  // 64-bit accesses of a wavefront fall on distinct banks.
  const int per = (C + kThreads - 1) / kThreads;
  const int stride = per | 1;
  const int c_begin = tid * per;
  unsigned long long* my = s_key + tid * stride;

  // ---- path scores of the pool, as sortable keys (0 = no candidate)
  // Loads first, arithmetic after, four candidates at a time: the loads of a group are all in
  // flight together (one memory round trip per group, not one per candidate).
  unsigned long long anchor_key = 0ull;
  int tok_r[kRegCand];
  float prob_r[kRegCand];
  double score_r[kRegCand];
  auto score_group = [&](int i0, int (&tok)[kRegCand], float (&prob)[kRegCand], double (&score)[kRegCand]) {
    double edge[kRegCand], plogp[kRegCand];
    // (no branch around the loads: a slot past the end reads candidate 0 of the frontier and
    // drops it, so that nothing makes the compiler wait between two slots)
#pragma unroll
    for (int u = 0; u < kRegCand; ++u) {
      const int c = c_begin + i0 + u;
      const bool have = i0 + u < per && c < C;
      const int cc = have ? c : 0;
      const int p = cc / k;
      const size_t ci = (base + fb + p) * k + (cc - p * k);
      const int t_ = ld<AGENT, int32_t>(a.cand_token + ci);
      const float pr_ = ld<AGENT, float>(a.cand_prob + ci);
      plogp[u] = ld<AGENT, double>(st.logp + base + fb + p);
      edge[u] = ld<AGENT, double>(a.cand_edge_logp + ci);
      tok[u] = have ? t_ : -1;
      prob[u] = pr_;
    }
#pragma unroll
    for (int u = 0; u < kRegCand; ++u) {
      if (i0 + u < per) {
        const double sc = plogp[u] + edge[u];
        score[u] = sc;
        unsigned long long key = 0ull;
        if (tok[u] >= 0 && sc == sc) {
          key = sortable_u64(sc);
          if (key == 0ull) key = 1ull;
        }
        my[i0 + u] = key;
        anchor_key = key > anchor_key ? key : anchor_key;
      }
    }
  };
  score_group(0, tok_r, prob_r, score_r);
  for (int i0 = kRegCand; i0 < per; i0 += kRegCand) {
    int tok_x[kRegCand];
    float prob_x[kRegCand];
    double score_x[kRegCand];
    score_group(i0, tok_x, prob_x, score_x);
  }
  anchor_key = block_max_u64(anchor_key, s_red_u64);

  const bool init = d < a.init_layers;
  const int limit = init ? (a.K_init < R ? a.K_init : R) : R;
  unsigned long long thr_key = 1ull;
  if (!init && anchor_key != 0ull) {
    thr_key = sortable_u64(a.log_mu + unsortable_f64(anchor_key));
    if (thr_key == 0ull) thr_key = 1ull;
  }

  // candidates that pass the gate, and the lowest of their keys
  int n_pass_local = 0;
  unsigned long long inv_low = 0ull;   // max of ~key over the passing keys
  for (int i = 0; i < per; ++i) {
    const unsigned long long key = my[i];
    if (key >= thr_key) { ++n_pass_local; inv_low = ~key > inv_low ? ~key : inv_low; }
  }
  n_pass_local = wave_sum_i32(n_pass_local);
  inv_low = wave_max_u64(inv_low);
  __syncthreads();
  if ((tid & 63) == 0) { s_red_i32[tid >> 6] = n_pass_local; s_red_u64[tid >> 6] = inv_low; }
  __syncthreads();
  const int n_pass = s_red_i32[0] + s_red_i32[1] + s_red_i32[2] + s_red_i32[3];

  unsigned long long T = thr_key;     // keep key > T, and the first need_eq keys == T
  int need_eq = 0x7FFFFFFF;
  if (n_pass > limit) {
    // ---- radix select: the limit-th largest key, 8 bits per pass from the top.
    // Path scores of one layer lie close together, so their keys share their leading bits.
    // The keys are first moved to the range they span: key' = (key - lowest + 1) << s with s
    // such that the largest key' has its top bit set (order and ties are preserved, keys
    // below the gate become 0 = no candidate).  The digits of key' are spread over the bins,
    // and the search usually ends after two or three passes: as soon as the bin that holds
    // the limit-th key holds exactly as many keys as are still wanted.
    unsigned long long a01 = s_red_u64[0] > s_red_u64[1] ? s_red_u64[0] : s_red_u64[1];
    unsigned long long a23 = s_red_u64[2] > s_red_u64[3] ? s_red_u64[2] : s_red_u64[3];
    const unsigned long long low_key = ~(a01 > a23 ? a01 : a23);
    const int sh = __clzll(static_cast<long long>(anchor_key - low_key + 1ull));
    for (int i = 0; i < per; ++i) {
      const unsigned long long key = my[i];
      my[i] = key >= thr_key ? (key - low_key + 1ull) << sh : 0ull;
    }
    unsigned long long prefix = 0ull;
    int remaining = limit;
    T = 0ull;
    need_eq = 0;
    bool found = false;
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
          int j = 0;
#pragma unroll
          for (; j < 3; ++j) {
            if (before + h[j] < remaining) { before += h[j]; --dg; } else break;
          }
          const int want = remaining - before;
          // the bin holds exactly the keys still wanted: all of them are kept
          s_digit = dg | ((h[j] == want) ? 256 : 0);
          s_remaining = want;
        }
      }
      __syncthreads();
      const int dg = s_digit;
      prefix |= static_cast<unsigned long long>(dg & 255) << shift;
      remaining = s_remaining;
      __syncthreads();
      if (dg & 256) {   // keep every key >= prefix (lower digits zero): none equals prefix - 1 with a claim
        T = prefix != 0ull ? prefix - 1ull : 0ull;   // prefix 0: every candidate left is kept
        need_eq = 0;
        found = true;
        break;
      }
    }
    if (!found) { T = prefix; need_eq = remaining; }
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
    if (keep && a.cap_hit && (c_begin + i) % k == k - 1) st_<true, uint32_t>(a.cap_hit, 1u);   // a row's last candidate
  }
  int n_keep;
  int pos = block_exclusive_scan_i32(keep_local, s_red_i32, &n_keep);
#pragma unroll
  for (int i = 0; i < kRegCand; ++i) {
    if (i < per && (keep_bits & (1u << i))) {
      const int p = (c_begin + i) / k;
      const size_t o = base + n + pos;
      st.token[o] = tok_r[i];
      st_<AGENT, int32_t>(st.parent + o, fb + p);   // read again by the in-launch mask build
      st.depth[o] = d + 1;
      st.prob[o] = prob_r[i];
      st_<AGENT, double>(st.logp + o, score_r[i]);
      ++pos;
    }
  }
  for (int i = kRegCand; i < per; ++i) {
    if (keep_bits & (1u << i)) {
      const int c = c_begin + i;
      const int p = c / k;
      const size_t ci = (base + fb + p) * k + (c - p * k);
      const size_t o = base + n + pos;
      st.token[o] = ld<AGENT, int32_t>(a.cand_token + ci);
      st_<AGENT, int32_t>(st.parent + o, fb + p);
      st.depth[o] = d + 1;
      st.prob[o] = ld<AGENT, float>(a.cand_prob + ci);
      st_<AGENT, double>(st.logp + o, ld<AGENT, double>(st.logp + base + fb + p) + ld<AGENT, double>(a.cand_edge_logp + ci));
      ++pos;
    }
  }
  if (tid == 0) {
    const int n_new = n + n_keep;
    uint32_t s = status;
    if (n_new >= st.N) s |= TALON_STATUS_DONE_BUDGET;
    else if (d + 1 >= a.max_depth) s |= TALON_STATUS_DONE_DEPTH;
    st_<AGENT, int32_t>(st.n_nodes + b, n_new);
    st_<AGENT, int32_t>(st.frontier_begin + b, n);     // per-sequence words are rewritten layer after layer,
    st_<AGENT, int32_t>(st.frontier_count + b, n_keep);   // possibly from different compute dies in one launch
    st_<AGENT, int32_t>(st.depth_cur + b, d + 1);
    st_<AGENT, uint32_t>(st.status + b, s);
    return static_cast<unsigned long long>(static_cast<uint32_t>(n)) |
           (static_cast<unsigned long long>((s & kDoneMask) ? 0 : n_keep) << 32);
  }
  return 0ull;
}

}  // namespace talon
