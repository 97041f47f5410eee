// One layer of Alg. 2 with the pool exactly as the listing writes it (Sec. 5.2, Alg. 2 "Hybrid
// Expansion Strategy" and "Budget Check"): S_d holds every token of every frontier row, not a
// fixed number per row.  This is the slow, general form (any budget up to TALON_N_MAX); the
// fast path caps a row at k <= TALON_K_MAX candidates, which is the same tree whenever
// k >= N - |T|.
//
// A layer never takes more than `limit` nodes (the remaining budget R_d, or min(K_init, R_d) on
// a top-K layer), so a row can contribute at most `limit` of them, and inside a row the path
// score rises with the logit.  Three kernels after the vocabulary scan (k = 1: row maximum and
// log-sum-exp):
//   plan     per sequence: anchor m_d = best path score of the pool (a row's best candidate is
//            its largest logit), gate threshold log(mu) + m_d  (Eq. 4), limit
//   collect  per frontier row: the tokens that pass the gate, at most `limit` of them, the
//            best by (logit descending, token ascending) -- a radix select over the row when
//            more pass
//   select   per sequence: the `limit` best of what the rows kept, by (path score descending,
//            parent ascending, in-row rank ascending), appended in (parent, rank) order
// Keys are unique ((logit, token) inside a row, (score, parent, token) inside a layer), so
// every radix select ends with exactly the wanted number of keys and no tie handling.
#include "device_utils.h"
#include "talon_internal.h"

namespace talon {

namespace {

__device__ __forceinline__ double key_to_f64(unsigned long long s) {
  const unsigned long long u = (s >> 63) ? (s ^ 0x8000000000000000ull) : ~s;
  return __longlong_as_double(static_cast<long long>(u));
}

// Adds one to s_hist[digit] for every lane with c set.  Keys of one row often share their
// leading digits: when all lanes that count hit the same bin, one of them adds their number.
__device__ __forceinline__ void hist_add(int* s_hist, bool c, int digit) {
  const unsigned long long m = __ballot(c);
  if (m == 0ull) return;
  const int lead = __ffsll(static_cast<long long>(m)) - 1;
  const int d0 = __shfl(digit, lead);
  const unsigned long long same = __ballot(c && digit == d0);
  if (same == m) {
    if (static_cast<int>(threadIdx.x & 63) == lead) atomicAdd(&s_hist[d0], __popcll(m));
  } else if (c) {
    atomicAdd(&s_hist[digit], 1);
  }
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

__global__ __launch_bounds__(kThreads) void literal_plan_kernel(LiteralArgs a) {
  __shared__ unsigned long long s_red[8];
  const talon_tree_state& st = a.st;
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const uint32_t status = st.status[b];
  const int F = st.frontier_count[b];
  LiteralPlan p;
  p.thr = 0.0; p.active = 0; p.F = 0; p.fb = 0; p.n = 0; p.d = 0; p.limit = 0; p.status = status; p.pad = 0;
  const int n = st.n_nodes[b];
  const int R = st.N - n;
  if ((status & kDoneMask) || F <= 0 || R <= 0) {
    if (tid == 0) a.plan[b] = p;
    return;
  }
  if (status & TALON_STATUS_BAD_ROW) {   // a row of this layer could not be normalised: stop here
    if (tid == 0) { st.frontier_count[b] = 0; a.plan[b] = p; }
    return;
  }
  const int fb = st.frontier_begin[b];
  const int d = st.depth_cur[b];
  const size_t base = static_cast<size_t>(b) * st.N_pad;
  unsigned long long key = 0ull;
  for (int j = tid; j < F; j += kThreads) {
    const size_t row = base + fb + j;
    const double s = st.logp[row] + (static_cast<double>(a.top_logit[row]) - a.row_lse[row]);
    if (s == s) {
      unsigned long long ks = sortable_u64(s);
      if (ks == 0ull) ks = 1ull;
      key = ks > key ? ks : key;
    }
  }
  key = block_max_u64(key, s_red);
  if (tid == 0) {
    const bool init = d < a.init_layers;
    p.active = 1; p.F = F; p.fb = fb; p.n = n; p.d = d;
    p.limit = init ? (a.K_init < R ? a.K_init : R) : R;
    p.thr = (init || key == 0ull) ? -__builtin_huge_val() : a.log_mu + key_to_f64(key);
    a.plan[b] = p;
  }
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

// One workgroup per frontier row.  EPL: logits per 16-byte vector (4 fp32, 8 bf16).
template <int EPL>
__global__ __launch_bounds__(kThreads) void literal_collect_kernel(LiteralArgs a) {
  __shared__ int s_hist[256];
  __shared__ unsigned long long s_lo;
  __shared__ int s_digit, s_want, s_count;
  const int b = blockIdx.y;
  const int j = blockIdx.x;
  const LiteralPlan p = a.plan[b];
  if (!p.active || j >= p.F) return;
  const int tid = threadIdx.x;
  const int node = p.fb + j;
  const size_t out_row = static_cast<size_t>(b) * a.st.N_pad + node;
  const int in_row = a.row_mode == TALON_ROWS_BY_FRONTIER ? j : node;
  const uint4* row = reinterpret_cast<const uint4*>(
      static_cast<const char*>(a.logits) +
      (static_cast<int64_t>(b) * a.seq_stride + static_cast<int64_t>(in_row) * a.row_stride) * (16 / EPL));
  const int nvec = (a.vocab + EPL - 1) / EPL;
  unsigned long long* out = a.row_key + out_row * kLiteralRowCap;

  s_hist[tid] = 0;
  if (tid == 0) {
    s_count = 0;
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
    s_lo = static_cast<unsigned long long>(res) << 32;
  }
  __syncthreads();
  const unsigned long long lo = s_lo;
  const int cap = p.limit;

  // f(valid, key) for every logit of the row; the same number of calls in every lane
  auto for_each_key = [&](auto&& f) {
    for (int base = 0; base < nvec; base += 4 * kThreads) {
      uint4 raw[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int vi = base + u * kThreads + tid;
        raw[u] = vi < nvec ? row[vi] : make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int t0 = (base + u * kThreads + tid) * EPL;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const int token = t0 + e;
          const unsigned long long key = (static_cast<unsigned long long>(sortable_u32(vec_elem<EPL>(raw[u], e))) << 32) |
                                         static_cast<unsigned long long>(0xFFFFFFFFu - static_cast<uint32_t>(token));
          f(token < a.vocab, key);
        }
      }
    }
  };

  // first pass: count what passes the gate, keep it if it fits, histogram of the top digit
  for_each_key([&](bool ok, unsigned long long key) {
    const bool c = ok && key >= lo;
    hist_add(s_hist, c, static_cast<int>(key >> 56));
    if (c) {
      const int slot = atomicAdd(&s_count, 1);
      if (slot < kLiteralRowCap) out[slot] = key;
    }
  });
  __syncthreads();
  const int total = s_count;
  if (total <= cap) {
    if (tid == 0) a.row_count[out_row] = total;
    return;
  }

  // more than the layer can take: the cap-th largest key, 8 bits per pass
  unsigned long long prefix = 0ull;
  int remaining = cap;
  for (int pass = 0; pass < 8; ++pass) {
    const int shift = 56 - 8 * pass;
    if (pass > 0) {
      s_hist[tid] = 0;
      __syncthreads();
      for_each_key([&](bool ok, unsigned long long key) {
        const bool c = ok && key >= lo && ((key ^ prefix) >> (shift + 8)) == 0ull;
        hist_add(s_hist, c, static_cast<int>(key >> shift) & 255);
      });
    }
    const int r = find_bin(s_hist, remaining, &s_digit, &s_want);
    prefix |= static_cast<unsigned long long>(r & 255) << shift;
    remaining = s_want;
    __syncthreads();
    if (r & 256) break;
  }
  const unsigned long long T = prefix > lo ? prefix : lo;
  if (tid == 0) s_count = 0;
  __syncthreads();
  for_each_key([&](bool ok, unsigned long long key) {
    if (ok && key >= T) {
      const int slot = atomicAdd(&s_count, 1);
      if (slot < cap) out[slot] = key;
    }
  });
  __syncthreads();
  if (tid == 0) a.row_count[out_row] = s_count < cap ? s_count : cap;
}

// One workgroup per sequence.
__global__ __launch_bounds__(kThreads) void literal_select_kernel(LiteralArgs a) {
  __shared__ int s_hist[256];
  __shared__ int s_cnt[256];
  __shared__ double s_lp[256];
  __shared__ double s_lse[256];
  __shared__ unsigned long long s_red_u64[8];
  __shared__ int s_red_i32[8];
  __shared__ int s_digit, s_want, s_nkeep;
  __shared__ unsigned long long s_kkey[256];
  __shared__ int s_kj[256];
  const talon_tree_state& st = a.st;
  const int b = blockIdx.x;
  const LiteralPlan p = a.plan[b];
  if (!p.active) return;
  const int tid = threadIdx.x;
  const int F = p.F < 256 ? p.F : 256;
  const size_t base = static_cast<size_t>(b) * st.N_pad;
  int c_own = 0;
  if (tid < F) {
    const size_t row = base + p.fb + tid;
    c_own = a.row_count[row];
    s_lp[tid] = st.logp[row];
    s_lse[tid] = a.row_lse[row];
  }
  s_cnt[tid] = c_own;
  if (tid == 0) s_nkeep = 0;
  const int total = block_sum_i32(c_own, s_red_i32);

  // candidate (row j, slot tid): its path score as a sortable key, and the order among equal
  // scores (parent ascending, then token ascending = in-row rank ascending) as a second key
  auto candidate = [&](int j, unsigned long long* k64, unsigned long long* hi, unsigned long long* lo2) {
    const bool valid = tid < s_cnt[j];
    const unsigned long long key = valid ? a.row_key[(base + p.fb + j) * kLiteralRowCap + tid] : 0ull;
    const double score = s_lp[j] + (static_cast<double>(unsortable_f32(static_cast<uint32_t>(key >> 32))) - s_lse[j]);
    *k64 = key;
    *hi = sortable_u64(score);
    *lo2 = ((static_cast<unsigned long long>(255 - j) << 32) | (key & 0xFFFFFFFFull)) << 24;
    return valid;
  };

  unsigned long long pre_hi = 0ull, pre_lo = 0ull, low = 0ull;
  int sh = 0;
  const bool cut = total > p.limit;
  if (cut) {
    // move the score keys to the range they span, so that their digits spread over the bins
    unsigned long long mx = 0ull, inv_mn = 0ull;
    for (int j = 0; j < F; ++j) {
      unsigned long long k64, hi, lo2;
      if (candidate(j, &k64, &hi, &lo2)) { mx = hi > mx ? hi : mx; inv_mn = ~hi > inv_mn ? ~hi : inv_mn; }
    }
    mx = block_max_u64(mx, s_red_u64);
    low = ~block_max_u64(inv_mn, s_red_u64);
    sh = __clzll(static_cast<long long>(mx - low + 1ull));
    int remaining = p.limit;
    for (int pass = 0; pass < 13; ++pass) {
      const bool first_key = pass < 8;
      const int shift = first_key ? 56 - 8 * pass : 56 - 8 * (pass - 8);
      s_hist[tid] = 0;
      __syncthreads();
      for (int j = 0; j < F; ++j) {
        unsigned long long k64, hi, lo2;
        const bool valid = candidate(j, &k64, &hi, &lo2);
        hi = (hi - low + 1ull) << sh;
        bool match;
        int digit;
        if (first_key) {
          match = pass == 0 || ((hi ^ pre_hi) >> (shift + 8)) == 0ull;
          digit = static_cast<int>(hi >> shift) & 255;
        } else {
          match = hi == pre_hi && (pass == 8 || ((lo2 ^ pre_lo) >> (shift + 8)) == 0ull);
          digit = static_cast<int>(lo2 >> shift) & 255;
        }
        hist_add(s_hist, valid && match, digit);
      }
      const int r = find_bin(s_hist, remaining, &s_digit, &s_want);
      if (first_key) pre_hi |= static_cast<unsigned long long>(r & 255) << shift;
      else pre_lo |= static_cast<unsigned long long>(r & 255) << shift;
      remaining = s_want;
      __syncthreads();
      if (r & 256) break;
    }
  }

  // kept candidates, in any order
  __syncthreads();
  for (int j = 0; j < F; ++j) {
    unsigned long long k64, hi, lo2;
    const bool valid = candidate(j, &k64, &hi, &lo2);
    bool keep = valid;
    if (cut) {
      hi = (hi - low + 1ull) << sh;
      keep = valid && (hi > pre_hi || (hi == pre_hi && lo2 >= pre_lo));
    }
    if (keep) {
      const int slot = atomicAdd(&s_nkeep, 1);
      if (slot < 256) { s_kkey[slot] = k64; s_kj[slot] = j; }
    }
  }
  __syncthreads();
  const int n_keep = s_nkeep < p.limit ? s_nkeep : p.limit;

  // node ids in (parent ascending, in-row rank ascending) order: rank by counting
  if (tid < n_keep) {
    const int myj = s_kj[tid];
    const unsigned long long myk = s_kkey[tid];
    int rank = 0;
    for (int i = 0; i < n_keep; ++i) {
      const int oj = s_kj[i];
      rank += (oj < myj || (oj == myj && s_kkey[i] > myk)) ? 1 : 0;
    }
    const float lg = unsortable_f32(static_cast<uint32_t>(myk >> 32));
    const double edge = static_cast<double>(lg) - s_lse[myj];
    const size_t o = base + p.n + rank;
    st.token[o] = static_cast<int32_t>(0xFFFFFFFFu - static_cast<uint32_t>(myk));
    st.parent[o] = p.fb + myj;
    st.depth[o] = p.d + 1;
    st.prob[o] = __expf(static_cast<float>(edge));
    st.logp[o] = s_lp[myj] + edge;
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

}  // namespace

hipError_t launch_literal_layer(const LiteralArgs& a, int dtype, hipStream_t s) {
  hipLaunchKernelGGL(literal_plan_kernel, dim3(a.st.B), dim3(kThreads), 0, s, a);
  const dim3 grid(a.st.N > 1 ? a.st.N - 1 : 1, a.st.B);
  if (dtype == TALON_DTYPE_F32) hipLaunchKernelGGL(literal_collect_kernel<4>, grid, dim3(kThreads), 0, s, a);
  else hipLaunchKernelGGL(literal_collect_kernel<8>, grid, dim3(kThreads), 0, s, a);
  hipLaunchKernelGGL(literal_select_kernel, dim3(a.st.B), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace talon
