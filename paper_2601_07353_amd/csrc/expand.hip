// Vocabulary scan: per frontier row, softmax statistics and the k largest logits in one
// pass over the row (candidate pool of Eq. 3 restricted to each parent's k best tokens;
// Alg. 2 "gather" loop).  HBM-bandwidth bound: every logit is read exactly once.
//
// Work decomposition.  A row is cut into chunks of 16 KiB (8192 bf16 / 4096 f32 logits).
// A fixed-size grid walks the (row, chunk) items of every unfinished sequence with a grid
// stride, so the launch needs no host knowledge of the frontier sizes.  A workgroup
// holds its whole chunk in registers (4 x 16-byte loads per thread, all in flight at
// once) and produces a partial result: chunk max, sum of exp relative to that max, and
// the chunk's k best (logit, token) keys.  The workgroup that completes a row's last
// chunk (atomic ticket) merges the partials into the row's outputs.
//
// Exactness.  Ordering is by the 64-bit integer key (sortable(logit) << 32 | ~token), so
// the order (logit descending, token ascending) is exact.  Per chunk, each wavefront finds
// the k-th largest of its 64 per-lane maxima; every element of the chunk's top k is >=
// that value, so only those are pushed to an LDS candidate list (a handful per chunk on
// ordinary rows).  Rows with so many ties that the list overflows take an exact k-round
// arg-max instead.
#include "device_utils.h"
#include "talon_internal.h"

namespace talon {

namespace {

constexpr float kNegInf = -__builtin_huge_valf();

// Phase timestamps (100 MHz wall clock) of workgroup 0, and of the merging workgroup for
// phases >= 8; compiled only into tuning builds with -DTALON_PHASE_TIMING.
#ifdef TALON_PHASE_TIMING
__device__ unsigned long long g_phase[16];
#define PHASE(i) do { if (threadIdx.x == 0 && (blockIdx.x == 0 || ((i) >= 8 && (i) <= 9))) g_phase[i] = wall_clock64(); } while (0)
#else
#define PHASE(i) do { } while (0)
#endif

template <int EPL>
struct RowVec;
template <>
struct RowVec<4> {  // f32: one 16-byte vector = 4 logits
  __device__ static void load(const void* row, int e0, int vocab, float* x) {
    const float* p = static_cast<const float*>(row);
    if (e0 + 4 <= vocab) {
      const float4 v = *reinterpret_cast<const float4*>(p + e0);
      x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] = (e0 + e < vocab) ? p[e0 + e] : kNegInf;
    }
  }
};
template <>
struct RowVec<8> {  // bf16: one 16-byte vector = 8 logits
  __device__ static void load(const void* row, int e0, int vocab, float* x) {
    const uint16_t* p = static_cast<const uint16_t*>(row);
    if (e0 + 8 <= vocab) {
      const uint4 v = *reinterpret_cast<const uint4*>(p + e0);
      x[0] = __uint_as_float(v.x << 16); x[1] = __uint_as_float(v.x & 0xFFFF0000u);
      x[2] = __uint_as_float(v.y << 16); x[3] = __uint_as_float(v.y & 0xFFFF0000u);
      x[4] = __uint_as_float(v.z << 16); x[5] = __uint_as_float(v.z & 0xFFFF0000u);
      x[6] = __uint_as_float(v.w << 16); x[7] = __uint_as_float(v.w & 0xFFFF0000u);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        x[e] = (e0 + e < vocab) ? __uint_as_float(static_cast<uint32_t>(p[e0 + e]) << 16) : kNegInf;
    }
  }
};

// Partial results cross workgroups (and the per-XCD L2 caches) inside one launch.  They are
// written and read with agent-scope atomic accesses, which go to the device-coherent level
// directly, so no whole-cache write-back or invalidate is needed around the ticket.
template <typename T>
__device__ __forceinline__ void store_agent(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ T load_agent(const T* p) {
  return __hip_atomic_load(const_cast<T*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Number of keys in s[0..n) greater than key (LDS broadcast reads, 8 in flight).
__device__ __forceinline__ int count_greater(const unsigned long long* s, int n, unsigned long long key) {
  int r = 0;
  int j = 0;
  for (; j + 8 <= n; j += 8) {
    unsigned long long v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = s[j + u];
#pragma unroll
    for (int u = 0; u < 8; ++u) r += (v[u] > key) ? 1 : 0;
  }
  for (; j < n; ++j) r += (s[j] > key) ? 1 : 0;
  return r;
}

__device__ __forceinline__ unsigned long long make_key(float x, int token) {
  return (static_cast<unsigned long long>(sortable_u32(x)) << 32) |
         static_cast<unsigned long long>(0xFFFFFFFFu - static_cast<uint32_t>(token));
}

template <int EPL>
__global__ __launch_bounds__(kThreads) void expand_kernel(ExpandArgs a) {
  constexpr int NX = kScanTiles * EPL;          // logits per thread per chunk
  constexpr int CHUNK = kThreads * NX;          // logits per chunk
  __shared__ int s_prefix[TALON_B_MAX + 1];     // exclusive prefix of frontier sizes
  __shared__ unsigned long long s_keys[kMergeCap];  // chunk candidates, later merge staging
  __shared__ unsigned long long s_red_u64[8];
  __shared__ double s_red_f64[8];
  __shared__ float s_red_f32[8];
  __shared__ int s_red_i32[8];
  __shared__ float s_wmax[4];
  __shared__ double s_wsum[4];
  __shared__ int s_ncand;
  __shared__ int s_last;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  PHASE(0);

  // ---- frontier sizes of all sequences -> item map (identical in every workgroup)
  {
    int run = 0;  // B <= 1024: each thread owns up to 4 consecutive sequences
    int cnt[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int b = tid * 4 + j;
      int c = 0;
      if (b < a.B) {  // both loads are issued together; the select below is register-only
        const uint32_t stat = a.status[b];
        const int fc = a.frontier_count[b];
        c = (stat & kDoneMask) ? 0 : fc;
      }
      cnt[j] = c;
      run += c;
    }
    int total;
    int base = block_exclusive_scan_i32(run, s_red_i32, &total);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int b = tid * 4 + j;
      if (b < a.B) s_prefix[b] = base;
      base += cnt[j];
    }
    if (tid == 0) s_prefix[a.B] = total;
    __syncthreads();
  }
  PHASE(1);
  const int total_rows = s_prefix[a.B];
  const long long n_items = static_cast<long long>(total_rows) * a.chunks;
  const int k = a.k;

  for (long long item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int rg = static_cast<int>(item / a.chunks);
    const int ch = static_cast<int>(item - static_cast<long long>(rg) * a.chunks);
    int lo = 0, hi = a.B;  // largest b with s_prefix[b] <= rg
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_prefix[mid] <= rg) lo = mid; else hi = mid;
    }
    const int b = lo;
    const int local = rg - s_prefix[b];
    const int node = a.frontier_begin[b] + local;
    const int in_row = a.row_mode == TALON_ROWS_BY_FRONTIER ? local : node;
    const size_t esz = EPL == 4 ? 4 : 2;
    const char* row = static_cast<const char*>(a.logits) +
                      (static_cast<int64_t>(b) * a.seq_stride + static_cast<int64_t>(in_row) * a.row_stride) * esz;
    const int out_row = b * a.N_pad + node;

    if (tid == 0) s_ncand = 0;

    // ---- the whole chunk into registers
    float x[NX];
    const int c0 = ch * CHUNK;
#pragma unroll
    for (int j = 0; j < kScanTiles; ++j)
      RowVec<EPL>::load(row, c0 + (j * kThreads + tid) * EPL, a.vocab, x + j * EPL);

    // ---- per-wavefront max and sum of exp relative to it
    float lane_max = kNegInf;
#pragma unroll
    for (int i = 0; i < NX; ++i) lane_max = fmaxf(lane_max, x[i]);
    PHASE(2);
    const float wmax = wave_max_f32(lane_max);
    float lane_sum = 0.f;
    if (wmax != kNegInf) {
#pragma unroll
      for (int i = 0; i < NX; ++i) lane_sum += __expf(x[i] - wmax);
    }
    const double wsum = wave_sum_f64(static_cast<double>(lane_sum));
    if (lane == 0) { s_wmax[wave] = wmax; s_wsum[wave] = wsum; }

    // ---- k-th largest lane maximum of this wavefront: lower bound of the chunk's top k
    float tau = kNegInf;
    {
      float v = lane_max;
      int cnt = 0;
      for (int r = 0; r < k; ++r) {
        const float cur = wave_max_f32(v);
        const unsigned long long eq = __ballot(v == cur);
        cnt += __popcll(eq);
        tau = cur;
        if (cnt >= k) break;
        v = (v == cur) ? kNegInf : v;
      }
    }
    PHASE(3);
    __syncthreads();  // s_ncand = 0 visible; previous iteration's readers of s_keys are done

    // ---- push every logit >= tau (rare: about k per wavefront on ordinary rows)
#pragma unroll
    for (int j = 0; j < kScanTiles; ++j) {
      bool any = false;
#pragma unroll
      for (int e = 0; e < EPL; ++e) any |= (x[j * EPL + e] >= tau);
      if (any) {
        const int e0 = c0 + (j * kThreads + tid) * EPL;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          if (x[j * EPL + e] >= tau && e0 + e < a.vocab) {
            const int slot = atomicAdd(&s_ncand, 1);
            if (slot < kCandCap) s_keys[slot] = make_key(x[j * EPL + e], e0 + e);
          }
        }
      }
    }
    __syncthreads();
    PHASE(4);
    const int ncand = s_ncand;
    unsigned long long* pk = a.part_keys + (static_cast<size_t>(out_row) * a.chunks + ch) * k;

    if (ncand <= kCandCap) {
      // rank by counting: keys are distinct (distinct tokens)
      for (int i = tid; i < ncand; i += kThreads) {
        const unsigned long long ki = s_keys[i];
        const int r = count_greater(s_keys, ncand, ki);
        if (r < k) store_agent(pk + r, ki);
      }
      if (tid >= ncand && tid < k) store_agent(pk + tid, 0ull);  // fewer than k logits in this chunk
    } else {
      // heavy ties: exact k rounds of workgroup arg-max over the registers
      unsigned long long prev = ~0ull;
      for (int r = 0; r < k; ++r) {
        unsigned long long best = 0ull;
#pragma unroll
        for (int j = 0; j < kScanTiles; ++j) {
          const int e0 = c0 + (j * kThreads + tid) * EPL;
#pragma unroll
          for (int e = 0; e < EPL; ++e) {
            if (e0 + e < a.vocab) {
              const unsigned long long key = make_key(x[j * EPL + e], e0 + e);
              if (key < prev && key > best) best = key;
            }
          }
        }
        best = block_max_u64(best, s_red_u64);
        if (tid == 0) store_agent(pk + r, best);
        prev = best;
        if (best == 0ull) {
          if (tid > r && tid < k) store_agent(pk + tid, 0ull);
          break;
        }
      }
    }

    PHASE(5);
    // ---- chunk statistics
    if (tid == 0) {
      const float m = fmaxf(fmaxf(s_wmax[0], s_wmax[1]), fmaxf(s_wmax[2], s_wmax[3]));
      double sum = 0.0;
#pragma unroll
      for (int w = 0; w < 4; ++w)
        if (s_wmax[w] != kNegInf) sum += s_wsum[w] * exp(static_cast<double>(s_wmax[w]) - static_cast<double>(m));
      store_agent(a.part_max + static_cast<size_t>(out_row) * a.chunks + ch, m);
      store_agent(a.part_sum + static_cast<size_t>(out_row) * a.chunks + ch, sum);
    }

    PHASE(6);
    // ---- ticket: the workgroup that finishes the row's last chunk merges the row
    // every partial store of this workgroup has completed before the ticket is taken
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (tid == 0) {
      const int old = __hip_atomic_fetch_add(&a.ticket[out_row], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_last = (old == a.chunks - 1) ? 1 : 0;
    }
    __syncthreads();
    PHASE(7);
    if (s_last) {
      PHASE(8);
      const float* pm = a.part_max + static_cast<size_t>(out_row) * a.chunks;
      const double* ps = a.part_sum + static_cast<size_t>(out_row) * a.chunks;
      const unsigned long long* keys = a.part_keys + static_cast<size_t>(out_row) * a.chunks * k;
      const int nkeys = a.chunks * k;
      for (int i = tid; i < nkeys; i += kThreads) s_keys[i] = load_agent(keys + i);
      float m = kNegInf;
      for (int c = tid; c < a.chunks; c += kThreads) m = fmaxf(m, load_agent(pm + c));
      m = block_max_f32(m, s_red_f32);  // barrier inside: s_keys staged
      double sum = 0.0;
      for (int c = tid; c < a.chunks; c += kThreads) {
        const float mc = load_agent(pm + c);
        if (mc != kNegInf) sum += load_agent(ps + c) * exp(static_cast<double>(mc) - static_cast<double>(m));
      }
      sum = block_sum_f64(sum, s_red_f64);
      PHASE(9);
      const double lse = static_cast<double>(m) + log(sum);
      const int valid = a.vocab < k ? a.vocab : k;
      const size_t ob = static_cast<size_t>(out_row) * k;
      for (int i = tid; i < nkeys; i += kThreads) {
        const unsigned long long ki = s_keys[i];
        if (ki == 0ull) continue;
        const int r = count_greater(s_keys, nkeys, ki);
        if (r < k) {
          const float lg = unsortable_f32(static_cast<uint32_t>(ki >> 32));
          const double edge = static_cast<double>(lg) - lse;
          a.cand_token[ob + r] = static_cast<int32_t>(0xFFFFFFFFu - static_cast<uint32_t>(ki));
          a.cand_logit[ob + r] = lg;
          a.cand_edge_logp[ob + r] = edge;
          a.cand_prob[ob + r] = static_cast<float>(exp(edge));
        }
      }
      if (tid >= valid && tid < k) {
        a.cand_token[ob + tid] = -1;
        a.cand_logit[ob + tid] = kNegInf;
        a.cand_edge_logp[ob + tid] = -__builtin_huge_val();
        a.cand_prob[ob + tid] = 0.f;
      }
      if (tid == 0) {
        a.row_max[out_row] = m;
        a.row_lse[out_row] = lse;
        if (!(fabs(lse) <= 1.7e308)) atomicOr(&a.status[b], TALON_STATUS_BAD_ROW);
        store_agent(a.ticket + out_row, 0);  // leave the workspace clean for the next layer
      }
    }
    __syncthreads();  // s_keys / s_last are reused by the next item
    PHASE(10);
  }
  PHASE(11);
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(uint32_t* p, size_t n) {
  for (size_t i = blockIdx.x * static_cast<size_t>(kThreads) + threadIdx.x; i < n;
       i += static_cast<size_t>(gridDim.x) * kThreads)
    p[i] = 0u;
}

__global__ __launch_bounds__(kThreads) void tree_init_kernel(talon_tree_state st, const int32_t* root_token) {
  const int b = blockIdx.x * kThreads + threadIdx.x;
  if (b >= st.B) return;
  const size_t o = static_cast<size_t>(b) * st.N_pad;
  st.token[o] = root_token[b];
  st.parent[o] = -1;
  st.depth[o] = 0;
  st.prob[o] = 1.f;
  st.logp[o] = 0.0;
  st.n_nodes[b] = 1;
  st.frontier_begin[b] = 0;
  st.frontier_count[b] = 1;
  st.depth_cur[b] = 0;
  st.status[b] = st.N <= 1 ? TALON_STATUS_DONE_BUDGET : 0u;
}

}  // namespace

int expand_chunk_elems(int dtype) { return dtype == TALON_DTYPE_F32 ? kChunkBytes / 4 : kChunkBytes / 2; }

hipError_t launch_expand(const ExpandArgs& a, int dtype, int grid, hipStream_t s) {
  if (dtype == TALON_DTYPE_F32)
    hipLaunchKernelGGL(expand_kernel<4>, dim3(grid), dim3(kThreads), 0, s, a);
  else
    hipLaunchKernelGGL(expand_kernel<8>, dim3(grid), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

#ifdef TALON_PHASE_TIMING
extern "C" int talon_debug_read_phases(unsigned long long* host16) {
  return static_cast<int>(hipMemcpyFromSymbol(host16, HIP_SYMBOL(g_phase), sizeof(unsigned long long) * 16));
}
#endif

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 4;
  int grid = static_cast<int>((n + kThreads - 1) / kThreads);
  if (grid > 1024) grid = 1024;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(kThreads), 0, s, static_cast<uint32_t*>(p), n);
  return hipGetLastError();
}

hipError_t launch_tree_init(const talon_tree_state& st, const int32_t* root_token, hipStream_t s) {
  hipLaunchKernelGGL(tree_init_kernel, dim3((st.B + kThreads - 1) / kThreads), dim3(kThreads), 0, s, st,
                     root_token);
  return hipGetLastError();
}

}  // namespace talon
