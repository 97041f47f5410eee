// One layer of Alg. 2 with the pool exactly as the listing writes it (Sec. 5.2, Alg. 2 "Hybrid
// Expansion Strategy" and "Budget Check"): S_d holds every token of every frontier row, not a
// fixed number per row.  This is the slow, general form (any budget up to TALON_N_MAX); the
// fast path caps a row at k <= TALON_K_MAX candidates, which is the same tree whenever
// k >= N - |T|.
//
// A layer never takes more than `limit` nodes (the remaining budget R_d, or min(K_init, R_d) on
// a top-K layer), so a row can contribute at most `limit` of them, and inside a row the path
// score rises with the logit.  Two kernels after the vocabulary scan (row maximum and
// log-sum-exp; on top-K layers also the K_init best of every row):
//   (plan    in both, per sequence: anchor m_d = best path score of the pool (a row's best
//            candidate is its largest logit), gate threshold log(mu) + m_d  (Eq. 4), limit)
//   collect  per frontier row: the tokens that pass the gate, at most `limit` of them, the
//            best by (logit descending, token ascending) -- a radix select over the row when
//            more pass; rows of a narrow layer are streamed in parts by several workgroups
//   select   per sequence: the `limit` best of what the rows kept, by (path score descending,
//            parent ascending, in-row rank ascending), appended in (parent, rank) order
// Keys are unique ((logit, token) inside a row, (score, parent, token) inside a layer), so
// every radix select ends with exactly the wanted number of keys and no tie handling.
#include <type_traits>

#include "device_utils.h"
#include "talon_internal.h"

namespace talon {

namespace {

__device__ __forceinline__ double key_to_f64(unsigned long long s) {
  const unsigned long long u = (s >> 63) ? (s ^ 0x8000000000000000ull) : ~s;
  return __longlong_as_double(static_cast<long long>(u));
}

// Histogram of 8-bit digits in LDS, fed one wavefront-wide call at a time.  Keys of one row
// often share their leading digits: when all lanes that count hit the same bin, their number
// is added by one lane, and runs of such calls on the same bin are added up in a register
// first (flush() hands the rest over; call it before the histogram is read).
struct WaveHist {
  int* hist;
  int pend_digit = -1;
  int pend_count = 0;
  __device__ __forceinline__ explicit WaveHist(int* h) : hist(h) {}
  __device__ __forceinline__ void flush() {
    if (pend_count > 0 && (threadIdx.x & 63) == 0) atomicAdd(&hist[pend_digit], pend_count);
    pend_count = 0;
    pend_digit = -1;
  }
  __device__ __forceinline__ void add(bool c, int digit) {
    const unsigned long long m = __ballot(c);
    if (m == 0ull) return;
    const int lead = __ffsll(static_cast<long long>(m)) - 1;
    const int d0 = __builtin_amdgcn_readlane(digit, lead);
    const unsigned long long same = __ballot(c && digit == d0);
    if (same == m) {
      if (d0 != pend_digit) { flush(); pend_digit = d0; }
      pend_count += __popcll(m);
    } else if (c) {
      atomicAdd(&hist[digit], 1);
    }
  }
};

// One slot of a counter in LDS for every lane with c set (-1 for the others): one atomic per
// wavefront, the lanes' slots in lane order.
__device__ __forceinline__ int claim_slots(int* counter, bool c) {
  const unsigned long long m = __ballot(c);
  if (m == 0ull) return -1;
  const int lane = threadIdx.x & 63;
  const int lead = __ffsll(static_cast<long long>(m)) - 1;
  int base = 0;
  if (lane == lead) base = atomicAdd(counter, __popcll(m));
  base = __shfl(base, lead);
  return c ? base + __popcll(m & ((1ull << lane) - 1ull)) : -1;
}

// Walks the 256 bins from the largest digit down to the bin that holds the `remaining`-th
// key.  Returns that digit, plus 256 if the bin holds exactly the keys still wanted (then
// all of them are kept and the search is over); *s_want = keys wanted from the bin.  Starts
// with a barrier (the histogram is complete) and ends with one (the result is visible); the
// caller places another before the histogram or the result words are written again.
__device__ __forceinline__ int find_bin(const int* s_hist, int remaining, int* s_digit, int* s_want) {
  const int tid = threadIdx.x;
  __syncthreads();
  if (tid < 64) {   // lane l owns digits 255-4l .. 252-4l
    int h[4], lane_sum = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) { h[j] = s_hist[255 - 4 * tid - j]; lane_sum += h[j]; }
    const int incl = wave_inclusive_scan_i32(lane_sum);
    const unsigned long long hit = __ballot(incl >= remaining);
    const int first = hit ? __ffsll(static_cast<long long>(hit)) - 1 : 63;
    if (tid == first) {
      int before = incl - lane_sum;
      int dg = 255 - 4 * tid;
      int j = 0;
#pragma unroll
      for (; j < 3; ++j) {
        if (before + h[j] < remaining) { before += h[j]; --dg; } else break;
      }
      const int want = remaining - before;
      *s_digit = dg | ((h[j] == want) ? 256 : 0);
      *s_want = want;
    }
  }
  __syncthreads();
  return *s_digit;
}

// What a layer does for sequence b, from the tree state and the scan's row statistics; computed
// by every workgroup that works on the sequence (the same value in all of them and in all
// threads; the tree state changes only in the select kernel, which is a later launch).
// s_plan: one LiteralPlan in LDS.
// NT: threads of the workgroup; s_red: NT / 64 values of LDS.
// s_rows (optional, NT / 64 + 1 values of LDS): the last of them receives the number of frontier
// rows of all sequences that this layer expands.
template <int NT>
__device__ __forceinline__ LiteralPlan make_plan(const LiteralArgs& a, int b, unsigned long long* s_red,
                                                 LiteralPlan* s_plan, int* s_rows = nullptr) {
  const talon_tree_state& st = a.st;
  const int tid = threadIdx.x;
  const uint32_t status = st.status[b];
  const int F = st.frontier_count[b];
  const int n = st.n_nodes[b];
  const int R = st.N - n;
  int rows_t = 0;   // thread t: the rows of sequence t (loads issued here, used at the barrier below)
  if (s_rows && tid < st.B) {
    const uint32_t st_t = st.status[tid];
    const int f_t = st.frontier_count[tid];
    const int n_t = st.n_nodes[tid];
    rows_t = ((st_t & (kDoneMask | TALON_STATUS_BAD_ROW)) || f_t <= 0 || st.N - n_t <= 0) ? 0 : f_t;
  }

  LiteralPlan p;
  p.thr = 0.0; p.active = 0; p.F = F; p.fb = 0; p.n = n; p.d = 0; p.limit = 0; p.status = status; p.pad = 0;
  // finished, nothing to expand, or a row of this layer could not be normalised
  if ((status & (kDoneMask | TALON_STATUS_BAD_ROW)) || F <= 0 || R <= 0) return p;
  const int fb = st.frontier_begin[b];
  const int d = st.depth_cur[b];
  const size_t base = static_cast<size_t>(b) * st.N_pad;
  unsigned long long key = 0ull;
  for (int j = tid; j < F; j += NT) {
    const size_t row = base + fb + j;
    const double s = st.logp[row] + (static_cast<double>(a.top_logit[row * a.k_scan]) - a.row_lse[row]);
    if (s == s) {
      unsigned long long ks = sortable_u64(s);
      if (ks == 0ull) ks = 1ull;
      key = ks > key ? ks : key;
    }
  }
  key = wave_max_u64(key);
  if (s_rows) rows_t = wave_sum_i32(rows_t);
  if ((tid & 63) == 0) {
    s_red[tid >> 6] = key;
    if (s_rows) s_rows[tid >> 6] = rows_t;
  }
  __syncthreads();
  if (tid == 0) {
    if (s_rows) {
      int sum = 0;
#pragma unroll
      for (int w = 0; w < NT / 64; ++w) sum += s_rows[w];
      s_rows[NT / 64] = sum;
    }
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) key = s_red[w] > key ? s_red[w] : key;
    const bool init = d < a.init_layers;
    p.active = 1; p.fb = fb; p.d = d;
    p.limit = init ? (a.K_init < R ? a.K_init : R) : R;
    p.thr = (init || key == 0ull) ? -__builtin_huge_val() : a.log_mu + key_to_f64(key);
    *s_plan = p;
  }
  __syncthreads();
  return *s_plan;
}

template <int EPL>
__device__ __forceinline__ float vec_elem(const uint4& v, int e) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  if constexpr (EPL == 4) {
    return __uint_as_float(w[e]);
  } else {
    const uint32_t word = w[e >> 1];
    return __uint_as_float((e & 1) ? (word & 0xFFFF0000u) : (word << 16));
  }
}

constexpr int kCollectThreads = 1024;   // many wavefronts per workgroup, to have enough loads in flight
constexpr int kHistCopies = 32;
constexpr int kLdsKeys = 2048;   // keys that a search finishes on in LDS
constexpr int kVecAhead = 4;     // 16-byte loads a thread has in flight
constexpr int kPoolLds = 4096;   // survivors of a layer that the budget check holds in LDS
constexpr int kFinCap = 256;     // keys of the last bin that the budget check ranks by counting

// Rows and chunks cross workgroups (and the per-XCD L2 caches) inside the launch: what one
// workgroup leaves for another is written and read at agent scope, and a ticket is taken only
// after the stores before it have been performed.
template <typename T>
__device__ __forceinline__ void st_agent(T* p, T v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
template <typename T>
__device__ __forceinline__ T ld_agent(const T* p) { return __hip_atomic_load(const_cast<T*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void stores_done() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <int NT>
__device__ __forceinline__ unsigned long long block_max_u64_nt(unsigned long long v, unsigned long long* scratch) {
  v = wave_max_u64(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long m = scratch[0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) m = scratch[w] > m ? scratch[w] : m;
  return m;
}

// Exclusive prefix sum over the NT threads; *total receives the workgroup sum.
template <int NT>
__device__ __forceinline__ int block_exclusive_scan_nt(int v, int* scratch, int* total) {
  const int incl = wave_inclusive_scan_i32(v);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 63) scratch[wave] = incl;
  __syncthreads();
  int base = 0, sum = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) {
    const int x = scratch[w];
    if (w < wave) base += x;
    sum += x;
  }
  *total = sum;
  return base + incl - v;
}

// LDS of the two kernels.
struct CollectLds {   // while rows are streamed
  int rep[256 * kHistCopies];
  unsigned long long bin[kLdsKeys];
};
struct SelectLds2 {   // the budget check
  unsigned long long pool[kPoolLds];
  unsigned char pool_j[kPoolLds];
  int cnt[256], off[256], kj[256];
  double lp[256], lse[256];
  unsigned long long kkey[256];
  unsigned long long fin_hi[kFinCap], fin_lo[kFinCap];
};
struct CommonLds {
  int hist[256];
  unsigned long long lo;
  int digit, want, count, nbin, flag, nkeep, nfin;
  int red_i32[kCollectThreads / 64];
  int rows[kCollectThreads / 64 + 1];
  unsigned long long red_u64[kCollectThreads / 64];
  LiteralPlan plan;
};

// The `want` largest of the n <= kLdsKeys keys in `keys` (LDS, unique), written to out[0..want)
// in any order: a radix select from the top byte down, all in LDS.  want < n.
template <int NT>
__device__ __forceinline__ void lds_select(const unsigned long long* keys, int n, int want, unsigned long long* out,
                                           CommonLds& cm) {
  const int tid = threadIdx.x;
  unsigned long long prefix = 0ull;
  int remaining = want;
  for (int sh = 56; sh >= 0; sh -= 8) {
    if (tid < 256) cm.hist[tid] = 0;
    __syncthreads();
    WaveHist wh(cm.hist);
    for (int base = 0; base < n; base += NT) {
      const int i = base + tid;
      const unsigned long long key = i < n ? keys[i] : 0ull;
      const bool c = i < n && (sh == 56 || ((key ^ prefix) >> (sh + 8)) == 0ull);
      wh.add(c, static_cast<int>(key >> sh) & 255);
    }
    wh.flush();
    const int r = find_bin(cm.hist, remaining, &cm.digit, &cm.want);
    prefix |= static_cast<unsigned long long>(r & 255) << sh;
    remaining = cm.want;
    __syncthreads();
    if (r & 256) break;
  }
  if (tid == 0) cm.count = 0;
  __syncthreads();
  for (int base = 0; base < n; base += NT) {
    const int i = base + tid;
    const unsigned long long key = i < n ? keys[i] : 0ull;
    const int slot = claim_slots(&cm.count, i < n && key >= prefix);
    if (slot >= 0 && slot < want) out[slot] = key;
  }
  __syncthreads();
}

// ---- the budget check of one sequence, on the NT threads of a workgroup: the `limit` best of what the rows kept, by (path score descending,
// parent ascending, token ascending), appended in (parent, in-row order).
template <int NT>
__device__ __forceinline__ void literal_select(const LiteralArgs& a, int b, const LiteralPlan& p, SelectLds2& L,
                                               CommonLds& cm) {
  const talon_tree_state& st = a.st;
  const int tid = threadIdx.x;
  const int F = p.F < 256 ? p.F : 256;
  const size_t base = static_cast<size_t>(b) * st.N_pad;
  const unsigned long long* rows = a.row_key + (base + p.fb) * kLiteralRowCap;
  int c_own = 0;
  if (tid < F) {
    const size_t row = base + p.fb + tid;
    c_own = a.row_count[row];
    L.lp[tid] = st.logp[row];
    L.lse[tid] = a.row_lse[row];
  }
  if (tid < 256) L.cnt[tid] = c_own;
  if (tid == 0) cm.nkeep = 0;
  int total;
  const int my_off = block_exclusive_scan_nt<NT>(c_own, cm.red_i32, &total);
  if (tid < 256) L.off[tid] = my_off;
  __syncthreads();

  // The pool in LDS, rows one after the other, when it fits (it does unless many rows are
  // flat); otherwise every pass reads it from memory, row by row.
  const bool dense = total <= kPoolLds;
  if (dense) {
    // One pool position per thread and round: the row of a position is the last one that starts
    // at or before it (rows without survivors start where the next one does, and the last row
    // that starts at or before a position below `total` has some).
    for (int i0 = 0; i0 < total; i0 += NT) {
      const int i = i0 + tid;
      if (i < total) {
        int lo_j = 0, hi_j = F - 1;
        while (lo_j < hi_j) {
          const int mid = (lo_j + hi_j + 1) >> 1;
          if (L.off[mid] <= i) lo_j = mid; else hi_j = mid - 1;
        }
        L.pool[i] = rows[static_cast<size_t>(lo_j) * kLiteralRowCap + (i - L.off[lo_j])];
        L.pool_j[i] = static_cast<unsigned char>(lo_j);
      }
    }
    __syncthreads();
  }
  // f(valid, row j, key): the same number of calls in every thread
  auto for_each = [&](auto&& f) {
    if (dense) {
      for (int i0 = 0; i0 < total; i0 += NT) {
        const int i = i0 + tid;
        const bool valid = i < total;
        f(valid, valid ? static_cast<int>(L.pool_j[i]) : 0, valid ? L.pool[i] : 0ull);
      }
    } else {
      for (int j = 0; j < F; ++j) {
        const bool valid = tid < L.cnt[j];
        f(valid, j, valid ? rows[static_cast<size_t>(j) * kLiteralRowCap + tid] : 0ull);
      }
    }
  };
  // path score of a candidate as a sortable key, and the order among equal scores (parent
  // ascending, then token ascending = in-row rank ascending) as a second key
  auto score_key = [&](int j, unsigned long long key) {
    return sortable_u64(L.lp[j] + (static_cast<double>(unsortable_f32(static_cast<uint32_t>(key >> 32))) - L.lse[j]));
  };
  auto order_key = [&](int j, unsigned long long key) {
    return ((static_cast<unsigned long long>(255 - j) << 32) | (key & 0xFFFFFFFFull)) << 24;
  };

  unsigned long long pre_hi = 0ull, pre_lo = 0ull, low = 0ull;
  int sh = 0;
  const bool cut = total > p.limit;
  if (cut) {
    // move the score keys to the range they span, so that their digits spread over the bins
    unsigned long long mx = 0ull, inv_mn = 0ull;
    for_each([&](bool valid, int j, unsigned long long key) {
      if (valid) {
        const unsigned long long hi = score_key(j, key);
        mx = hi > mx ? hi : mx;
        inv_mn = ~hi > inv_mn ? ~hi : inv_mn;
      }
    });
    mx = block_max_u64_nt<NT>(mx, cm.red_u64);
    low = ~block_max_u64_nt<NT>(inv_mn, cm.red_u64);
    sh = __clzll(static_cast<long long>(mx - low + 1ull));
    int remaining = p.limit;
    for (int pass = 0; pass < 13; ++pass) {
      const bool first_key = pass < 8;
      const int shift = first_key ? 56 - 8 * pass : 56 - 8 * (pass - 8);
      if (tid < 256) cm.hist[tid] = 0;
      __syncthreads();
      WaveHist wh(cm.hist);
      for_each([&](bool valid, int j, unsigned long long key) {
        const unsigned long long hi = (score_key(j, key) - low + 1ull) << sh;
        const unsigned long long lo2 = order_key(j, key);
        bool match;
        int digit;
        if (first_key) {
          match = pass == 0 || ((hi ^ pre_hi) >> (shift + 8)) == 0ull;
          digit = static_cast<int>(hi >> shift) & 255;
        } else {
          match = hi == pre_hi && (pass == 8 || ((lo2 ^ pre_lo) >> (shift + 8)) == 0ull);
          digit = static_cast<int>(lo2 >> shift) & 255;
        }
        wh.add(valid && match, digit);
      });
      wh.flush();
      const int r = find_bin(cm.hist, remaining, &cm.digit, &cm.want);
      const int population = cm.hist[r & 255];
      if (first_key) pre_hi |= static_cast<unsigned long long>(r & 255) << shift;
      else pre_lo |= static_cast<unsigned long long>(r & 255) << shift;
      remaining = cm.want;
      __syncthreads();
      if (r & 256) break;
      if (population <= kFinCap) {
        // The bin fits one key per thread: rank its keys by counting and take the cut from
        // there.  (Scores of bf16 rows tie in whole groups, and a cut inside such a group
        // would otherwise walk every remaining digit of both keys.)
        if (tid == 0) cm.nfin = 0;
        __syncthreads();
        for_each([&](bool valid, int j, unsigned long long key) {
          const unsigned long long hi = (score_key(j, key) - low + 1ull) << sh;
          const unsigned long long lo2 = order_key(j, key);
          const bool in_bin = valid && (first_key ? ((hi ^ pre_hi) >> shift) == 0ull
                                                  : (hi == pre_hi && ((lo2 ^ pre_lo) >> shift) == 0ull));
          const int slot = claim_slots(&cm.nfin, in_bin);
          if (slot >= 0 && slot < kFinCap) { L.fin_hi[slot] = hi; L.fin_lo[slot] = lo2; }
        });
        __syncthreads();
        const int nf = cm.nfin < kFinCap ? cm.nfin : kFinCap;
        if (tid < nf) {
          const unsigned long long mh = L.fin_hi[tid], ml = L.fin_lo[tid];
          int rank = 0;
          int i = 0;
          for (; i + 8 <= nf; i += 8) {   // eight broadcast reads in flight: the loop is bound by LDS latency
            unsigned long long oh[8], ol[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) { oh[u] = L.fin_hi[i + u]; ol[u] = L.fin_lo[i + u]; }
#pragma unroll
            for (int u = 0; u < 8; ++u) rank += (oh[u] > mh || (oh[u] == mh && ol[u] > ml)) ? 1 : 0;
          }
          for (; i < nf; ++i) {
            const unsigned long long oh = L.fin_hi[i], ol = L.fin_lo[i];
            rank += (oh > mh || (oh == mh && ol > ml)) ? 1 : 0;
          }
          if (rank == remaining - 1) { cm.red_u64[0] = mh; cm.red_u64[1] = ml; }   // keys are unique: one thread
        }
        __syncthreads();
        pre_hi = cm.red_u64[0];
        pre_lo = cm.red_u64[1];
        __syncthreads();
        break;
      }
    }
  }

  // kept candidates, in any order
  for_each([&](bool valid, int j, unsigned long long key) {
    bool keep = valid;
    if (cut && valid) {
      const unsigned long long hi = (score_key(j, key) - low + 1ull) << sh;
      keep = hi > pre_hi || (hi == pre_hi && order_key(j, key) >= pre_lo);
    }
    const int slot = claim_slots(&cm.nkeep, keep);
    if (slot >= 0 && slot < 256) { L.kkey[slot] = key; L.kj[slot] = j; }
  });
  __syncthreads();
  const int n_keep = cm.nkeep < p.limit ? cm.nkeep : p.limit;

  // node ids in (parent ascending, in-row rank ascending) order: rank by counting
  if (tid < n_keep) {
    const int myj = L.kj[tid];
    const unsigned long long myk = L.kkey[tid];
    int rank = 0;
    int i = 0;
    for (; i + 8 <= n_keep; i += 8) {
      int oj[8];
      unsigned long long ok[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) { oj[u] = L.kj[i + u]; ok[u] = L.kkey[i + u]; }
#pragma unroll
      for (int u = 0; u < 8; ++u) rank += (oj[u] < myj || (oj[u] == myj && ok[u] > myk)) ? 1 : 0;
    }
    for (; i < n_keep; ++i) {
      const int oj = L.kj[i];
      rank += (oj < myj || (oj == myj && L.kkey[i] > myk)) ? 1 : 0;
    }
    const float lg = unsortable_f32(static_cast<uint32_t>(myk >> 32));
    const double edge = static_cast<double>(lg) - L.lse[myj];
    const size_t o = base + p.n + rank;
    st.token[o] = static_cast<int32_t>(0xFFFFFFFFu - static_cast<uint32_t>(myk));
    st.parent[o] = p.fb + myj;
    st.depth[o] = p.d + 1;
    st.prob[o] = __expf(static_cast<float>(edge));
    st.logp[o] = L.lp[myj] + edge;
  }
  if (tid == 0) {
    const int n_new = p.n + n_keep;
    uint32_t s = p.status;
    if (n_new >= st.N) s |= TALON_STATUS_DONE_BUDGET;
    else if (p.d + 1 >= a.max_depth) s |= TALON_STATUS_DONE_DEPTH;
    st.n_nodes[b] = n_new;
    st.frontier_begin[b] = p.n;
    st.frontier_count[b] = n_keep;
    st.depth_cur[b] = p.d + 1;
    st.status[b] = s;
  }
}

// Rows of a layer.  grid (workgroups per sequence, B): the workgroups of a sequence take its work
// items in turn.  An item is a frontier row, or one of up to kLiteralChunks equal parts of a row
// when the sequence has fewer rows than workgroups (a flat row, of which thousands of tokens
// pass the gate, keeps one workgroup busy for tens of microseconds).  A part is streamed once
// to count what passes the gate (and to keep it, if it fits: the common case, one pass).  If
// more than `cap` pass, a radix select finds the cap-th largest key of the part: 8 bits per
// pass, until the bin that holds the cut is small enough for LDS; one more pass then writes the
// keys above that bin and gathers the bin, and the search ends in LDS.  bf16 logits carry 16
// significant bits, so the two low bytes of their images are skipped.  The workgroup that
// finishes the last part of a row merges the parts' survivors (at most kLiteralChunks * cap <=
// kLdsKeys keys) into the row's.
template <int EPL>
__global__ __launch_bounds__(kCollectThreads) void literal_collect_kernel(LiteralArgs a) {
  constexpr int NT = kCollectThreads;
  __shared__ CollectLds s_c;
  __shared__ CommonLds s_cm;
  int* s_rep = s_c.rep;
  unsigned long long* s_bin = s_c.bin;
  int* s_hist = s_cm.hist;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  if (static_cast<int>(blockIdx.x) >= a.st.frontier_count[b] * kLiteralChunks) return;   // more workgroups than items
  const LiteralPlan p = make_plan<NT>(a, b, s_cm.red_u64, &s_cm.plan, s_cm.rows);
  if (!p.active) return;
  const int nvec = (a.vocab + EPL - 1) / EPL;
  // parts per row: none while the layer's rows (all sequences) keep every compute unit busy as
  // they are; otherwise as many as that takes, while a part keeps at least 2048 vectors
  int chunks = 256 / s_cm.rows[NT / 64];
  {
    const int per_seq = static_cast<int>(gridDim.x) / p.F;   // every part needs a workgroup of its own
    chunks = chunks < per_seq ? chunks : per_seq;
    const int by_size = nvec / 2048;
    chunks = chunks < by_size ? chunks : by_size;
    chunks = chunks < 1 ? 1 : (chunks > kLiteralChunks ? kLiteralChunks : chunks);
    if (chunks * p.limit > kLdsKeys) chunks = kLdsKeys / p.limit;   // what a merge holds in LDS (limit <= 255)
    if (chunks < 1) chunks = 1;
  }
  const int vec_per_chunk = (nvec + chunks - 1) / chunks;
  const size_t seq_base = static_cast<size_t>(b) * a.st.N_pad;

  auto collect_item = [&](const int j, const int c) {
  const int node = p.fb + j;
  const size_t out_row = seq_base + node;
  const int in_row = a.row_mode == TALON_ROWS_BY_FRONTIER ? j : node;
  const uint4* row = reinterpret_cast<const uint4*>(
      static_cast<const char*>(a.logits) +
      (static_cast<int64_t>(b) * a.seq_stride + static_cast<int64_t>(in_row) * a.row_stride) * (16 / EPL));
  unsigned long long* row_out = a.row_key + out_row * kLiteralRowCap;

  const int cap = p.limit;
  if (p.d < a.init_layers && a.k_scan >= cap) {
    // top-K layer: the pool's K_init best hold at most K_init tokens of one row, and the scan
    // has already ranked that many (logit descending, token ascending; missing ones last)
    if (c != 0) return;
    unsigned long long key = 0ull;
    bool have = false;
    if (tid < cap) {
      const int tok = a.scan_token[out_row * a.k_scan + tid];
      have = tok >= 0;
      key = (static_cast<unsigned long long>(sortable_u32(a.top_logit[out_row * a.k_scan + tid])) << 32) |
            static_cast<unsigned long long>(0xFFFFFFFFu - static_cast<uint32_t>(tok));
    }
    if (have) row_out[tid] = key;
    if (tid < 64) {   // cap <= 64 here: candidates are valid up to the first missing one
      const unsigned long long vb = __ballot(have);
      if (tid == 0) a.row_count[out_row] = vb == ~0ull ? 64 : __builtin_ctzll(~vb);
    }
    return;
  }

  const int copy = tid & (kHistCopies - 1);
  auto clear_copies = [&]() {
    for (int i = tid; i < 256 * kHistCopies; i += NT) s_rep[i] = 0;
  };
  auto sum_copies = [&]() {   // s_hist[bin] = sum of the copies; barriers before and after
    __syncthreads();
    if (tid < 256) {
      int sum = 0;
#pragma unroll 8
      for (int r = 0; r < kHistCopies; ++r) sum += s_rep[tid * kHistCopies + ((r + tid) & (kHistCopies - 1))];
      s_hist[tid] = sum;
    }
    __syncthreads();
  };
  if (tid == 0) {
    s_cm.count = 0;
    s_cm.nbin = 0;
    // Inside a row the path score log p(v) + (logit - lse_v) rises with the logit, so the gate
    // is a bound on the logit: the smallest logit image whose score passes, by bisection with
    // the very expression the score is computed with.
    const double lp = a.st.logp[out_row], lse = a.row_lse[out_row], thr = p.thr;
    auto passes = [&](uint32_t k32) { return lp + (static_cast<double>(unsortable_f32(k32)) - lse) >= thr; };
    uint32_t l = 0x007FFFFFu, h = 0xFF800000u;   // images of -inf and +inf
    uint32_t res = 0xFFFFFFFFu;
    if (passes(h)) {
      while (l < h) {
        const uint32_t mid = l + ((h - l) >> 1);
        if (passes(mid)) h = mid; else l = mid + 1u;
      }
      res = l;
    }
    s_cm.lo = static_cast<unsigned long long>(res) << 32;
    s_cm.digit = 0;
  }
  __syncthreads();
  const unsigned long long lo = s_cm.lo;
  const float x_lo = unsortable_f32(static_cast<uint32_t>(lo >> 32));   // logit >= x_lo: passes the gate

  // The scan has ranked the row's k_scan best tokens.  Those that pass the gate are the first
  // of them; if not all pass, no other token of the row does, and the row is settled
  // without reading it again (the rule for peaked rows, and for rows far below the anchor).
  // Every part of the row comes to the same conclusion; the first one writes.
  if (a.k_scan >= 2 && tid < 64) {
    unsigned long long key = 0ull;
    bool ok = false;
    if (tid < a.k_scan) {
      const int tok = a.scan_token[out_row * a.k_scan + tid];
      key = (static_cast<unsigned long long>(sortable_u32(a.top_logit[out_row * a.k_scan + tid])) << 32) |
            static_cast<unsigned long long>(0xFFFFFFFFu - static_cast<uint32_t>(tok));
      ok = tok >= 0 && key >= lo;
    }
    const unsigned long long vb = __ballot(ok);
    const int n_pass = vb == ~0ull ? 64 : __builtin_ctzll(~vb);   // the passing candidates come first
    if (n_pass < a.k_scan) {
      const int m = n_pass < cap ? n_pass : cap;
      if (c == 0) {
        if (tid < m) row_out[tid] = key;
        if (tid == 0) a.row_count[out_row] = m;
      }
      if (tid == 0) s_cm.digit = 1;
    }
  }
  __syncthreads();
  if (s_cm.digit) return;
  clear_copies();
  __syncthreads();

  // where this part's survivors go: the row's own slots, or the part's slots (cap of them)
  const bool whole = chunks == 1;
  unsigned long long* out = whole ? row_out
                                  : a.part_key + static_cast<size_t>(b) * a.part_keys_per_seq +
                                        (static_cast<size_t>(j) * chunks + c) * cap;
  int* out_count = whole ? a.row_count + out_row : a.part_count + out_row * kLiteralChunks + c;
  const int v_begin = c * vec_per_chunk;
  const int v_end = v_begin + vec_per_chunk < nvec ? v_begin + vec_per_chunk : nvec;

  auto key64 = [](uint32_t k32, uint32_t tk) { return (static_cast<unsigned long long>(k32) << 32) | tk; };

  // (compiled twice: for a whole row, whose loop and stores are the plain ones, and for a part)
  auto stream_part = [&](auto whole_tag) {
  constexpr bool WHOLE = decltype(whole_tag)::value;
  // f(passes, logit image, ~token) for every logit of the part, the same number of calls in every
  // lane of a wavefront; vectors in which no lane holds a passing logit are skipped whole.
  // (logit >= x_lo is the gate: the float order and the order of the images agree.)  The
  // 64-bit key (image << 32 | ~token) is put together only where a key is stored.
  auto for_each_key = [&](auto&& f) {
    for (int base = v_begin; base < v_end; base += kVecAhead * NT) {
      uint4 raw[kVecAhead];
#pragma unroll
      for (int u = 0; u < kVecAhead; ++u) {
        const int vi = base + u * NT + tid;
        raw[u] = vi < v_end ? row[vi] : make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int u = 0; u < kVecAhead; ++u) {
        const int vi = base + u * NT + tid;
        const int t0 = vi * EPL;
        // a vector past the end of a whole row holds no token below the vocabulary size; past the
        // end of a part it may
        const bool here = WHOLE || vi < v_end;
        float x[EPL];
        bool any = false;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          x[e] = vec_elem<EPL>(raw[u], e);
          any = any || (here && t0 + e < a.vocab && x[e] >= x_lo);
        }
        if (__ballot(any) == 0ull) continue;
#pragma unroll
        for (int e = 0; e < EPL; ++e)
          f(here && t0 + e < a.vocab && x[e] >= x_lo, sortable_u32(x[e]), 0xFFFFFFFFu - static_cast<uint32_t>(t0 + e));
      }
    }
  };
  // a row's own slots are read by the next launch; a part's by another workgroup of this one
  auto put_key = [&](int slot, unsigned long long key) {
    if constexpr (WHOLE) out[slot] = key; else st_agent(out + slot, key);
  };
  auto put_count = [&](int n) {
    if constexpr (WHOLE) *out_count = n; else st_agent(out_count, n);
  };
  // first pass: count what passes the gate, keep it if it fits, histogram of the top digit
  // (slots are claimed only until the part has overflowed; after that a wavefront just counts)
  {
    bool overflow = false;
    for_each_key([&](bool cnd, uint32_t k32, uint32_t tk) {
      if (cnd) atomicAdd(&s_rep[static_cast<int>(k32 >> 24) * kHistCopies + copy], 1);
      if (!overflow) {
        const int slot = claim_slots(&s_cm.count, cnd);
        if (slot >= 0 && slot < cap) put_key(slot, key64(k32, tk));
        overflow = __ballot(slot >= cap) != 0ull;
      }
    });
  }
  sum_copies();
  {
    const int v = wave_sum_i32(tid < 256 ? s_hist[tid] : 0);
    if (tid < 256 && (tid & 63) == 0) s_cm.red_i32[tid >> 6] = v;
    __syncthreads();
  }
  const int total = s_cm.red_i32[0] + s_cm.red_i32[1] + s_cm.red_i32[2] + s_cm.red_i32[3];
  __syncthreads();
  if (total <= cap) {
    if (tid == 0) put_count(total);
    return;
  }

  // more than the layer can take: the cap-th largest key
  unsigned long long prefix = 0ull;
  int remaining = cap;
  int shift = 56;
  bool in_lds = false, found = false;
  for (int pass = 0; pass < 8; ++pass) {
    shift = 56 - 8 * pass;
    if (EPL == 8 && (pass == 2 || pass == 3)) {
      // the low half of a bf16 logit's image is all zeros (positive) or all ones (negative)
      if (!(prefix >> 63)) prefix |= 0xFFull << shift;
      continue;
    }
    if (pass > 0) {
      clear_copies();
      __syncthreads();
      const uint32_t pre32 = static_cast<uint32_t>(prefix >> 32), pre_tk = static_cast<uint32_t>(prefix);
      if (pass < 4) {        // a byte of the logit image
        const int s32 = shift - 32;
        for_each_key([&](bool ok, uint32_t k32, uint32_t) {
          if (ok && ((k32 ^ pre32) >> (s32 + 8)) == 0u) atomicAdd(&s_rep[((k32 >> s32) & 255u) * kHistCopies + copy], 1);
        });
      } else {               // a byte of ~token, among equal logits
        for_each_key([&](bool ok, uint32_t k32, uint32_t tk) {
          if (ok && k32 == pre32 && (pass == 4 || ((tk ^ pre_tk) >> (shift + 8)) == 0u))
            atomicAdd(&s_rep[((tk >> shift) & 255u) * kHistCopies + copy], 1);
        });
      }
      sum_copies();
    }
    const int r = find_bin(s_hist, remaining, &s_cm.digit, &s_cm.want);
    const int population = s_hist[r & 255];
    prefix |= static_cast<unsigned long long>(r & 255) << shift;
    remaining = s_cm.want;
    __syncthreads();
    if (r & 256) { found = true; break; }
    if (population <= kLdsKeys) { in_lds = true; break; }
  }

  if (tid == 0) s_cm.count = 0;
  __syncthreads();
  if (found || !in_lds) {
    // every key >= prefix (its lower digits zero) is kept
    const unsigned long long T = prefix > lo ? prefix : lo;
    const uint32_t T32 = static_cast<uint32_t>(T >> 32), T_tk = static_cast<uint32_t>(T);
    for_each_key([&](bool ok, uint32_t k32, uint32_t tk) {
      const int slot = claim_slots(&s_cm.count, ok && (k32 > T32 || (k32 == T32 && tk >= T_tk)));
      if (slot >= 0 && slot < cap) put_key(slot, key64(k32, tk));
    });
    __syncthreads();
    if (tid == 0) put_count(s_cm.count < cap ? s_cm.count : cap);
    return;
  }

  // keys above the bin are kept; the bin itself goes to LDS, where the search continues
  {
    const uint32_t pre32 = static_cast<uint32_t>(prefix >> 32), pre_tk = static_cast<uint32_t>(prefix);
    const bool logit_stage = shift >= 32;
    const int s32 = logit_stage ? shift - 32 : 0;
    for_each_key([&](bool ok, uint32_t k32, uint32_t tk) {
      bool above, inbin;
      if (logit_stage) {
        const uint32_t hi_part = k32 >> s32, bin = pre32 >> s32;
        above = hi_part > bin;
        inbin = hi_part == bin;
      } else {
        const uint32_t hi_part = tk >> shift, bin = pre_tk >> shift;
        above = k32 > pre32 || (k32 == pre32 && hi_part > bin);
        inbin = k32 == pre32 && hi_part == bin;
      }
      const int slot = claim_slots(&s_cm.count, ok && above);
      if (slot >= 0 && slot < cap) put_key(slot, key64(k32, tk));
      const int slot2 = claim_slots(&s_cm.nbin, ok && inbin);
      if (slot2 >= 0 && slot2 < kLdsKeys) s_bin[slot2] = key64(k32, tk);
    });
  }
  __syncthreads();
  const int nbin = s_cm.nbin < kLdsKeys ? s_cm.nbin : kLdsKeys;
  bool done = false;
  for (int sh2 = shift - 8; sh2 >= 0 && !done; sh2 -= 8) {
    if (tid < 256) s_hist[tid] = 0;
    __syncthreads();
    WaveHist wh(s_hist);
    for (int base = 0; base < nbin; base += NT) {
      const int i = base + tid;
      const unsigned long long key = i < nbin ? s_bin[i] : 0ull;
      const bool cnd = i < nbin && ((key ^ prefix) >> (sh2 + 8)) == 0ull;
      wh.add(cnd, static_cast<int>(key >> sh2) & 255);
    }
    wh.flush();
    const int r = find_bin(s_hist, remaining, &s_cm.digit, &s_cm.want);
    prefix |= static_cast<unsigned long long>(r & 255) << sh2;
    remaining = s_cm.want;
    __syncthreads();
    done = (r & 256) != 0;
  }
  for (int i = tid; i < nbin; i += NT) {
    const unsigned long long key = s_bin[i];
    if (key >= prefix) {
      const int slot = atomicAdd(&s_cm.count, 1);
      if (slot < cap) put_key(slot, key);
    }
  }
  __syncthreads();
  if (tid == 0) put_count(s_cm.count < cap ? s_cm.count : cap);
  };
  if (whole) { stream_part(std::true_type{}); return; }
  stream_part(std::false_type{});

  // ---- the last part of the row to finish merges the parts' survivors into the row's
  stores_done();
  __syncthreads();
  if (tid == 0) {
    const int old = __hip_atomic_fetch_add(a.row_ticket + out_row, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last_one = old == chunks - 1;
    if (last_one) st_agent(a.row_ticket + out_row, 0);   // as the next launch wants it
    s_cm.flag = last_one;
  }
  __syncthreads();
  if (!s_cm.flag) return;
  int cnt_c = 0;
  if (tid < chunks) cnt_c = ld_agent(a.part_count + out_row * kLiteralChunks + tid);
  int total;
  const int off_c = block_exclusive_scan_nt<NT>(cnt_c, s_cm.red_i32, &total);
  if (tid < chunks) { s_hist[tid] = off_c; s_hist[16 + tid] = cnt_c; }
  __syncthreads();
  const unsigned long long* parts = a.part_key + static_cast<size_t>(b) * a.part_keys_per_seq +
                                    static_cast<size_t>(j) * chunks * cap;
  // (total <= chunks * cap <= kLdsKeys)
  for (int i = tid; i < total; i += NT) {
    int cc = 0;
    while (cc + 1 < chunks && s_hist[cc + 1] <= i) ++cc;
    // parts without survivors share their offset with the next one: the last part that starts at or before i has some
    const unsigned long long key = ld_agent(parts + static_cast<size_t>(cc) * cap + (i - s_hist[cc]));
    if (total <= cap) row_out[i] = key;
    else s_bin[i] = key;
  }
  __syncthreads();
  if (total <= cap) {
    if (tid == 0) a.row_count[out_row] = total;
    return;
  }
  lds_select<NT>(s_bin, total, cap, row_out, s_cm);
  if (tid == 0) a.row_count[out_row] = cap;
  };

  const int n_items = p.F * chunks;
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    collect_item(item / chunks, item - (item / chunks) * chunks);
    __syncthreads();   // the LDS is reused by the next item
  }
}

// One workgroup per sequence: the budget check over what the rows kept.
template <int NT>
__global__ __launch_bounds__(NT) void literal_select_kernel(LiteralArgs a) {
  __shared__ SelectLds2 s_s;
  __shared__ CommonLds s_cm;
  const int b = blockIdx.x;
  const LiteralPlan p = make_plan<NT>(a, b, s_cm.red_u64, &s_cm.plan);
  if (!p.active) {
    // a row of this layer could not be normalised: the sequence stops here
    if (threadIdx.x == 0 && (p.status & TALON_STATUS_BAD_ROW) && !(p.status & kDoneMask) && p.F > 0) a.st.frontier_count[b] = 0;
    return;
  }
  literal_select<NT>(a, b, p, s_s, s_cm);
}

}  // namespace

hipError_t launch_literal_layer(const LiteralArgs& a, int dtype, hipStream_t s) {
  // Workgroups per sequence: two per compute unit over all sequences, at least 32; a sequence
  // with more rows than that has its workgroups take rows in turn, one with fewer cuts its
  // rows into parts.  Launches that find nothing to do stay short.
  int per_seq = 512 / a.st.B;
  if (per_seq < 32) per_seq = 32;
  const int most = (a.st.N > 1 ? a.st.N - 1 : 1) * kLiteralChunks;
  const dim3 grid(per_seq < most ? per_seq : most, a.st.B);
  if (dtype == TALON_DTYPE_F32) hipLaunchKernelGGL(literal_collect_kernel<4>, grid, dim3(kCollectThreads), 0, s, a);
  else hipLaunchKernelGGL(literal_collect_kernel<8>, grid, dim3(kCollectThreads), 0, s, a);
  // (four wavefronts: on 8 or 16 the barriers between the passes cost more than the shorter loops save)
  hipLaunchKernelGGL(literal_select_kernel<kThreads>, dim3(a.st.B), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace talon
