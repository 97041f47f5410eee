// Vocabulary scan: per frontier row, softmax statistics and the k largest logits in one
// pass over the row (candidate pool of Eq. 3 restricted to each parent's k best tokens;
// Alg. 2 "gather" loop).  HBM-bandwidth bound: every logit is read exactly once.
//
// Work decomposition.  A row is a sequence of 16 KiB blocks (8192 bf16 / 4096 f32 logits);
// a block is what one workgroup holds in registers at a time (4 x 16-byte loads per
// thread).  A row is cut into `chunks` runs of consecutive blocks; one (row, chunk) item is
// streamed by one workgroup.  The number of chunks per row is chosen on the device from the total number
// of frontier rows of the launch (few rows: many short chunks, so that a one-row layer
// still spreads over the chip; many rows: one long chunk per row, so that the per-item
// fixed work vanishes).  A fixed-size grid walks the items with a grid stride; nothing
// about the frontier sizes is needed on the host.
//
// Inside a workgroup the four wavefronts stream independently, without barriers:
//   - softmax: every lane keeps its own running max and a double-precision running sum of
//     exp(logit - max), rescaled only when its max grows (rare after the first blocks);
//   - top-k: every wavefront keeps its k best keys so far and a threshold tau.  The first
//     group of 4 tiles sets tau from the 64 per-lane maxima, to a value that at least k of
//     them reach.  A lane whose 16-byte vector holds a logit that
//     reaches tau drops the whole vector into an LDS buffer (a few instructions, no
//     per-logit work); when the buffer runs full, and at the end, the buffered vectors are
//     expanded, ranked against the k best, and tau rises to the new k-th best.  After such
//     a cut a later logit EQUAL to the k-th best cannot enter (the wavefront meets tokens
//     in ascending id order, so it loses the tie): tau becomes the next float above it,
//     and rows full of ties cost nothing extra.
// The workgroup then merges its four lists and statistics.  With one chunk per row it
// writes the row's outputs directly; otherwise it stores a partial result and the
// workgroup that completes the row's last chunk (atomic ticket) merges the partials.
//
// Three ways to run it.  Scan only (talon_expand_layer).  Scan with the budget selection
// (Sec. 5.2, Alg. 2 "Hybrid Expansion Strategy" and "Budget Check") in its tail: the
// workgroup that writes the last row of a sequence's frontier selects for that sequence, one
// launch per layer (talon_expand_select_layer).  Or one launch for the whole loop of Alg. 2
// (talon_expand_tree): the grid walks the layers and enters the next one when all selections
// of the current one are published.
//
// Exactness.  Ordering is by the 64-bit integer key (sortable(logit) << 32 | ~token), so
// the order (logit descending, token ascending) is exact; floating point only enters the
// softmax statistics.
#include "select_device.h"

// Time-stamp marks exist only in tuning builds (-DTALON_TUNING pulls in tuning.h).
#ifdef TALON_TUNING
#define TALON_TUNING_MARKS
#include "tuning.h"
#else
#define TL_MARK(d, i) do { } while (0)
#define TL_ANY(d, i) do { } while (0)
#endif

namespace talon {

namespace {

constexpr float kNegInf = -__builtin_huge_valf();
constexpr int kHitTrigger = 64;                  // buffered vectors that trigger a cut before the next tile
constexpr int kHitCap = kHitTrigger + 64;        // a tile adds at most 64 vectors
constexpr int kSubBatch = 32;                    // vectors expanded per ranking round (two lanes per vector)
constexpr int kSubKeys = kSubBatch * 8 + TALON_K_MAX + 16;  // keys ranked per round (<= 8 logits per vector) + zero padding

// One 16-byte vector of a logits row, with -inf in the lanes past the end of the row.
template <int EPL>
__device__ __forceinline__ uint4 load_vec(const char* row, int e0, int vocab) {
  if (e0 + EPL <= vocab) return *reinterpret_cast<const uint4*>(row + static_cast<size_t>(e0) * (16 / EPL));
  uint32_t w[4];
  if constexpr (EPL == 4) {
    const uint32_t* p = reinterpret_cast<const uint32_t*>(row);
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = (e0 + e < vocab) ? p[e0 + e] : 0xFF800000u;
  } else {
    const uint16_t* p = reinterpret_cast<const uint16_t*>(row);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t lo = (e0 + 2 * q < vocab) ? p[e0 + 2 * q] : 0xFF80u;
      const uint32_t hi = (e0 + 2 * q + 1 < vocab) ? p[e0 + 2 * q + 1] : 0xFF80u;
      w[q] = lo | (hi << 16);
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

template <int EPL>
__device__ __forceinline__ void unpack_vec(const uint4& v, float* x) {
  if constexpr (EPL == 4) {
    x[0] = __uint_as_float(v.x); x[1] = __uint_as_float(v.y);
    x[2] = __uint_as_float(v.z); x[3] = __uint_as_float(v.w);
  } else {
    x[0] = __uint_as_float(v.x << 16); x[1] = __uint_as_float(v.x & 0xFFFF0000u);
    x[2] = __uint_as_float(v.y << 16); x[3] = __uint_as_float(v.y & 0xFFFF0000u);
    x[4] = __uint_as_float(v.z << 16); x[5] = __uint_as_float(v.z & 0xFFFF0000u);
    x[6] = __uint_as_float(v.w << 16); x[7] = __uint_as_float(v.w & 0xFFFF0000u);
  }
}

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

// Release half of a ticket: every global store and atomic this wavefront has issued so far
// has been performed at the device-coherent level when this returns.  A workgroup-scope
// fence does not give that (the compiler emits no wait on the vector memory counter for
// it), and without the wait a ticket's atomic can overtake the partial results it
// announces, even those of its own wavefront.  An agent-scope fence would also write the
// whole L2 back, which nothing here needs: everything that crosses workgroups is stored at
// agent scope.  Every wavefront of the workgroup calls this before the barrier that
// precedes the ticket.
__device__ __forceinline__ void stores_performed() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Number of keys in s[0..n) greater than key (LDS broadcast reads, 4 in flight).
__device__ __forceinline__ int count_greater(const unsigned long long* s, int n, unsigned long long key) {
  int r = 0;
  int j = 0;
  for (; j + 4 <= n; j += 4) {
    unsigned long long v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = s[j + u];
#pragma unroll
    for (int u = 0; u < 4; ++u) r += (v[u] > key) ? 1 : 0;
  }
  for (; j < n; ++j) r += (s[j] > key) ? 1 : 0;
  return r;
}

// Number of keys in s[0..n) greater than key, for a 16-byte aligned array padded with zero keys
// to a multiple of 16 keys: 8 two-key LDS broadcast reads in flight per round.
__device__ __forceinline__ int count_greater_pad16(const unsigned long long* s, int n, unsigned long long key) {
  const ulonglong2* kp = reinterpret_cast<const ulonglong2*>(s);
  int r = 0;
  for (int j = 0; j < n; j += 16) {
    ulonglong2 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = kp[(j >> 1) + u];
#pragma unroll
    for (int u = 0; u < 8; ++u) r += ((v[u].x > key) ? 1 : 0) + ((v[u].y > key) ? 1 : 0);
  }
  return r;
}

// Number of keys greater than `key` in a list sorted in descending order (zeros, if any, at
// the end): binary search.
__device__ __forceinline__ int count_greater_sorted(const unsigned long long* s, int n, unsigned long long key) {
  int lo = 0, hi = n;   // invariant: s[i] > key for i < lo, s[i] <= key for i >= hi
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (s[mid] > key) lo = mid + 1; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ unsigned long long make_key(float x, int token) {
  return (static_cast<unsigned long long>(sortable_u32(x)) << 32) |
         static_cast<unsigned long long>(0xFFFFFFFFu - static_cast<uint32_t>(token));
}

// Smallest float greater than x (x finite or -inf, not NaN): "v > x" is "v >= float_above(x)".
__device__ __forceinline__ float float_above(float x) {
  x = x + 0.0f;
  const uint32_t u = __float_as_uint(x);
  return __uint_as_float((u >> 31) ? u - 1u : u + 1u);
}

__device__ __forceinline__ float key_logit(unsigned long long key) {
  return unsortable_f32(static_cast<uint32_t>(key >> 32));
}

// log of a softmax denominator (1 <= sum <= vocabulary size, or 0 / inf / NaN for a row that
// cannot be normalised): sum = 2^e * f with f in [0.5, 1), log(sum) = e*ln2 + log(f); the
// second term is small, so single precision gives it to about 1e-7 absolute.
__device__ __forceinline__ double log_of_sum(double sum) {
  if (!(sum > 0.0) || !(sum <= 1.7e308)) return log(sum);
  int e;
  const double f = frexp(sum, &e);
  return static_cast<double>(e) * 0.69314718055994530942 + static_cast<double>(__logf(static_cast<float>(f)));
}

constexpr int kCandCap = 512;   // keys of a row merge that can still be among the k best, after the filter below

// Write the outputs of one row from its candidate keys (in LDS) and softmax statistics.
// `keys` holds `lists` lists of k keys, each sorted in descending order, zero keys in unused
// slots and up to the next multiple of 16.  s_cand: kCandCap + 16 keys of LDS, 16-byte aligned.
// FUSED: the candidates are read by another workgroup of this launch (the one that runs the
// sequence's selection), so they are stored at the device-coherent level.
// Returns whether the row could not be normalised (the same value in every thread).
template <bool FUSED>
__device__ __forceinline__ bool write_row(const ExpandArgs& a, int b, int out_row, const unsigned long long* keys,
                                          int lists, float m, double sum, unsigned long long* s_cand, int* s_nc) {
  // (thread index taken afresh, through an empty asm statement: addresses derived from it are
  // then computed here, at their use, instead of being kept alive or spilled across the
  // caller's streaming loop)
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int k = a.k;
  const double lse = static_cast<double>(m) + log_of_sum(sum);
  const size_t ob = static_cast<size_t>(out_row) * k;
  const int nkeys = lists * k;
  auto emit = [&](unsigned long long ki, int r) {
    const float lg = key_logit(ki);
    const double edge = static_cast<double>(lg) - lse;
    const int32_t tok = static_cast<int32_t>(0xFFFFFFFFu - static_cast<uint32_t>(ki));
    const float pr = __expf(static_cast<float>(edge));
    a.cand_logit[ob + r] = lg;
    if constexpr (FUSED) {
      store_agent(a.cand_token + ob + r, tok);
      store_agent(a.cand_edge_logp + ob + r, edge);
      store_agent(a.cand_prob + ob + r, pr);
    } else {
      a.cand_token[ob + r] = tok;
      a.cand_edge_logp[ob + r] = edge;
      a.cand_prob[ob + r] = pr;
    }
  };
  if (lists == 1) {   // a single sorted list: a key's position is its rank
    for (int i = tid; i < k; i += kThreads) {
      const unsigned long long ki = keys[i];
      if (ki != 0ull) emit(ki, i);
    }
  } else {
    // Rank by counting keys greater than mine.  First a filter: with q = ceil(k / lists), the
    // q-th key of every list is >= T = their minimum, so at least k keys are >= T and only keys
    // >= T can be among the k best; usually that leaves little more than k of the lists * k keys.
    bool done = false;
    if (lists <= 64) {
      const int q = (k + lists - 1) / lists;
      const int lane = tid & 63;
      unsigned long long inv = 0ull;   // ~key of this lane's list (0 beyond the lists: no effect on the max)
      if (lane < lists) inv = ~keys[lane * k + q - 1];
      const unsigned long long T = ~wave_max_u64(inv);   // 0 if a list is shorter than q: no filter then
      if (tid == 0) *s_nc = 0;
      __syncthreads();
      for (int i = tid; i < nkeys; i += kThreads) {
        const unsigned long long ki = keys[i];
        if (ki != 0ull && ki >= T) {
          const int slot = atomicAdd(s_nc, 1);
          if (slot < kCandCap) s_cand[slot] = ki;
        }
      }
      __syncthreads();
      const int nc = *s_nc;
      if (nc <= kCandCap) {
        if (tid < 16) s_cand[nc + tid] = 0ull;
        __syncthreads();
        for (int j = tid; j < nc; j += kThreads) {
          const unsigned long long ki = s_cand[j];
          const int r = count_greater_pad16(s_cand, nc, ki);
          if (r < k) emit(ki, r);
        }
        done = true;
      }
    }
    if (!done) {   // every key against every key
      for (int i = tid; i < nkeys; i += kThreads) {
        const unsigned long long ki = keys[i];
        if (ki == 0ull) continue;
        const int r = count_greater_pad16(keys, nkeys, ki);
        if (r < k) emit(ki, r);
      }
    }
  }
  const int valid = a.vocab < k ? a.vocab : k;
  if (tid >= valid && tid < k) {
    a.cand_logit[ob + tid] = kNegInf;
    if constexpr (FUSED) {
      store_agent(a.cand_token + ob + tid, -1);
      store_agent(a.cand_edge_logp + ob + tid, -__builtin_huge_val());
      store_agent(a.cand_prob + ob + tid, 0.f);
    } else {
      a.cand_token[ob + tid] = -1;
      a.cand_edge_logp[ob + tid] = -__builtin_huge_val();
      a.cand_prob[ob + tid] = 0.f;
    }
  }
  const bool bad = !(fabs(lse) <= 1.7e308);
  if (tid == 0) {
    a.row_max[out_row] = m;
    a.row_lse[out_row] = lse;
    if (bad) atomicOr(&a.status[b], TALON_STATUS_BAD_ROW);
  }
  return bad;
}

// How a launch is used: scan only; scan with the selection in its tail (one layer per launch);
// or one launch that walks all layers.
constexpr int kModeSplit = 0, kModeFused = 1, kModeTree = 2;

// One layer: returns the number of frontier rows it found (0: every sequence is finished).
template <int EPL, int MODE>
__device__ __forceinline__ int expand_body(const ExpandArgs& a, const int launch_idx) {
  constexpr bool FUSED = MODE != kModeSplit;
  constexpr bool TREE = MODE == kModeTree;
  constexpr int NX = kScanTiles * EPL;          // logits per thread per block
  constexpr int BLOCK = kThreads * NX;          // logits per block
  __shared__ int s_prefix[TALON_B_MAX + 1];     // exclusive prefix of frontier sizes
  __shared__ int s_begin[TALON_B_MAX];          // first frontier node of every sequence
  // One LDS pool: the scan's buffers (buffered vectors per wavefront, their tile*64+lane tags,
  // ranking scratch per wavefront; the vector buffers double as row-merge staging) and, in
  // fused mode, the key array and histogram of the budget selection, which runs when the
  // scan buffers are idle.
  constexpr int kHitvBytes = sizeof(uint4) * 4 * kHitCap;
  constexpr int kHithBytes = sizeof(int) * 4 * kHitCap;
  constexpr int kCkBytes = sizeof(unsigned long long) * 4 * kSubKeys;
  constexpr int kScanBytes = kHitvBytes + kHithBytes + kCkBytes;
  constexpr int kSelBytes = sizeof(unsigned long long) * kSelectKeySlots + sizeof(int) * 256;
  constexpr int kPoolBytes = (FUSED && kSelBytes > kScanBytes) ? kSelBytes : kScanBytes;
  __shared__ __attribute__((aligned(16))) unsigned char s_pool[kPoolBytes];
  uint4 (*s_hitv)[kHitCap] = reinterpret_cast<uint4 (*)[kHitCap]>(s_pool);
  int (*s_hith)[kHitCap] = reinterpret_cast<int (*)[kHitCap]>(s_pool + kHitvBytes);
  unsigned long long (*s_ck)[kSubKeys] = reinterpret_cast<unsigned long long (*)[kSubKeys]>(s_pool + kHitvBytes + kHithBytes);
  __shared__ unsigned long long s_red_u64[8];
  __shared__ int s_misc[2];
  __shared__ __attribute__((aligned(16))) unsigned long long s_topw[4][TALON_K_MAX]; // k best keys of each wavefront, sorted
  __shared__ int s_part[4][64];                         // partial ranks of the list merge
  __shared__ unsigned long long s_top[TALON_K_MAX];
  __shared__ double s_red_f64[8];
  __shared__ float s_red_f32[8];
  __shared__ int s_red_i32[8];
  __shared__ float s_wmax[4];
  __shared__ double s_wsum[4];
  __shared__ int s_wcnt[4];
  __shared__ int s_last;
  static_assert(kScanBytes >= static_cast<int>(sizeof(unsigned long long)) * kMergeCap,
                "the scan buffers double as the row-merge staging array");
  static_assert(kScanBytes >= static_cast<int>(sizeof(unsigned long long)) * (kMergeCap + kCandCap + 16),
                "... and hold the filtered candidates of a row merge behind it");
  unsigned long long* s_keys = reinterpret_cast<unsigned long long*>(s_pool);
  unsigned long long* s_cand = s_keys + kMergeCap;
  __shared__ int s_nc;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;

  // ---- frontier sizes of all sequences -> item map (identical in every workgroup)
  __shared__ int s_gave_up;
  {
    static_assert(TALON_B_MAX <= kThreads, "one thread per sequence");
    if (TREE && tid == 0) s_gave_up = 0;
    if constexpr (TREE) __syncthreads();
    int c = 0;
    if (tid < a.B) {
      if (TREE && a.root_token && launch_idx == 0) {   // fresh trees: the frontier is the root
        s_begin[tid] = 0;
        c = 1;
      } else if constexpr (TREE) {   // {begin, count} in one 8-byte load
        const unsigned long long* dp = a.desc + (launch_idx * a.B + tid);
        unsigned long long d2 = ld<TREE, unsigned long long>(dp);
        if constexpr (TREE) {
          // the selection of the layer before stores this word when all it wrote has been
          // performed: wait for it (bounded)
          if (!(d2 & kDescReady)) {
            const unsigned long long t0 = wall_clock64();
            do {
              if (wall_clock64() - t0 > a.spin_ticks) { s_gave_up = 1; break; }
              __builtin_amdgcn_s_sleep(2);
              d2 = ld<true, unsigned long long>(dp);
            } while (!(d2 & kDescReady));
          }
        }
        s_begin[tid] = static_cast<int>(static_cast<uint32_t>(d2));
        c = static_cast<int>(static_cast<uint32_t>(d2 >> 32) & 0x7FFFFFFFu);
      } else {  // the loads are issued together; the select below is register-only
        // (In a launch of one layer with the selection in its tail, that selection rewrites this
        // state while workgroups of the same launch may still be starting, and every workgroup
        // must see the same item map: a workgroup says below that it has read the state, and a
        // selection touches nothing before every workgroup of the grid has said so.)
        const uint32_t stat = a.status[tid];
        const int fc = a.frontier_count[tid];
        s_begin[tid] = a.frontier_begin[tid];
        c = (stat & kDoneMask) ? 0 : fc;
      }
      // a finished sequence gets no selection in this launch: carry its empty frontier over
      if (TREE && blockIdx.x == 0 && c == 0 && launch_idx + 1 < a.N_pad)
        st_<true, unsigned long long>(a.desc + ((launch_idx + 1) * a.B + tid),
                                      kDescReady | static_cast<unsigned long long>(static_cast<uint32_t>(s_begin[tid])));
    }
    int total;
    const int base = block_exclusive_scan_i32(c, s_red_i32, &total);
    if (tid < a.B) s_prefix[tid] = base;
    if (tid == 0) s_prefix[a.B] = total;
    __syncthreads();
    if constexpr (TREE) {
      if (s_gave_up) return -1;
    }
  }
  const int total_rows = s_prefix[a.B];
  if (total_rows == 0) return 0;   // (nothing will be selected in this launch: nobody waits for anybody)
  if constexpr (FUSED && !TREE) {
    // this workgroup has read the frontier (the loads fed the prefix sums that thread 0 has
    // waited for at the barrier above)
    if (tid == 0) __hip_atomic_fetch_add(a.exit_ticket + kStartedWord, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  const int k = a.k;

  // ---- chunks per row from the width of this layer
  const int blocks_per_row = a.chunks;
  int chunks = (a.target_items + total_rows - 1) / total_rows;
  {   // ... and at least as many as give every workgroup of the grid an item in the first round
    const int fill = static_cast<int>(gridDim.x) / total_rows;
    chunks = fill > chunks ? fill : chunks;
  }
  chunks = chunks < 1 ? 1 : (chunks > blocks_per_row ? blocks_per_row : chunks);
  const int bpc = (blocks_per_row + chunks - 1) / chunks;   // blocks per chunk
  chunks = (blocks_per_row + bpc - 1) / bpc;
  const long long n_items = static_cast<long long>(total_rows) * chunks;
  uint4* hitv = s_hitv[wave];
  int* hith = s_hith[wave];
  unsigned long long* ck = s_ck[wave];
  unsigned long long* topw = s_topw[wave];

  for (long long item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int rg = static_cast<int>(item / chunks);
    const int ch = static_cast<int>(item - static_cast<long long>(rg) * chunks);
    int lo = 0, hi = a.B;  // largest b with s_prefix[b] <= rg
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_prefix[mid] <= rg) lo = mid; else hi = mid;
    }
    const int b = lo;
    const int local = rg - s_prefix[b];
    const int fbegin = s_begin[b];
    const int node = fbegin + local;
    const int in_row = a.row_mode == TALON_ROWS_BY_FRONTIER ? local : node;
    const char* row = static_cast<const char*>(a.logits) +
                      (static_cast<int64_t>(b) * a.seq_stride + static_cast<int64_t>(in_row) * a.row_stride) * (16 / EPL);
    const int out_row = b * a.N_pad + node;
    const int blk0 = ch * bpc;
    const int blk1 = blk0 + bpc < blocks_per_row ? blk0 + bpc : blocks_per_row;

    // ---- wavefront-local streaming state
    int cnt = 0;            // buffered vectors
    int tcnt = 0;           // keys in topw (<= k)
    float tau = __builtin_huge_valf();   // a vector is buffered iff one of its logits is >= tau (set by the first step)
    float m_l = kNegInf;    // this lane's running max
    double s_l = 0.0;       // this lane's running sum of exp(logit - m_l)

    // A tile is one 16-byte vector per thread (256 * EPL logits); a block is 4 tiles, and the
    // scan advances by groups of 4 tiles.  A group that lies wholly inside the row is loaded
    // with plain vector loads; the group at the ragged end of the row (only in the row's last
    // chunk) with guarded loads that return -inf past the end.
    const int t0 = blk0 * kScanTiles;
    const int tiles_in_row = (a.vocab + kThreads * EPL - 1) / (kThreads * EPL);
    const int full_tiles = a.vocab / (kThreads * EPL);
    const int t1 = blk1 * kScanTiles < tiles_in_row ? blk1 * kScanTiles : tiles_in_row;
    const char* lane_ptr = row + static_cast<size_t>(tid) * 16;
    constexpr size_t kTileBytes = static_cast<size_t>(kThreads) * 16;

    // Buffer this lane's vector if one of its logits reaches tau.  Returns false (and buffers
    // nothing) when the wavefront's buffer has no room for all hits of the tile.
    auto buffer_hits = [&](const uint4& raw, float vmax, int tile) -> bool {
      const bool hit = vmax >= tau;
      const unsigned long long bal = __ballot(hit);
      if (bal != 0ull) {
        const int nh = __popcll(bal);
        if (cnt + nh > kHitCap) return false;
        const int pos = cnt + __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(bal >> 32),
                                                        __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(bal), 0));
        if (hit) { hitv[pos] = raw; hith[pos] = tile * 64 + lane; }
        cnt += nh;
      }
      return true;
    };

    // First threshold of an item: the largest value with a 16-bit (sign, exponent, 7 mantissa
    // bits) pattern that at least k of the 64 lane maxima of its first group reach, found
    // bit by bit on the order-preserving integer image of the maxima (-inf if fewer than k
    // lanes hold a logit).  For bf16 logits this is the k-th largest lane maximum itself.
    auto first_threshold = [&](float v) {
      const uint32_t u = sortable_u32(v);
      uint32_t prefix = 0u;
#pragma unroll
      for (int bit = 31; bit >= 16; --bit) {
        const uint32_t cand = prefix | (1u << bit);
        if (__popcll(__ballot(u >= cand)) >= k) prefix = cand;
      }
      tau = prefix <= 0x007FFFFFu ? kNegInf : unsortable_f32(prefix);   // at or below the image of -inf
    };

    // Streaming state machine.  A step is a group of 4 tiles.  Tiles whose hits do not fit the
    // buffer are deferred, together with all later tiles of the group, to the single slow
    // section below, which cuts the buffer and then re-reads them.
    // One group of 4 tiles of this thread: plain vector loads where the group lies wholly inside
    // the row, guarded loads (-inf past the end) at the ragged end.
    auto load_group = [&](int t, uint4 (&r)[kScanTiles]) {
      if (t + kScanTiles <= full_tiles) {
#pragma unroll
        for (int q = 0; q < kScanTiles; ++q)
          r[q] = *reinterpret_cast<const uint4*>(lane_ptr + (t + q) * kTileBytes);
      } else {
#pragma unroll
        for (int q = 0; q < kScanTiles; ++q)
          r[q] = load_vec<EPL>(row, ((t + q) * kThreads + tid) * EPL, a.vocab);
      }
    };
    int tb = t0;
    bool done = false;
    // With the selection in the launch the kernel runs three workgroups per compute unit and has
    // registers to spare: the loads of the next group are issued before the current one is
    // processed, so that a chunk of several blocks does not pay the memory latency per block.
    // The scan-only launch runs four workgroups per compute unit on 128 registers and relies on
    // those for the overlap.
    constexpr bool PREFETCH = FUSED;
    uint4 raw_next[kScanTiles];
    if constexpr (PREFETCH) {
      if (tb < t1) load_group(tb, raw_next);
    }
    while (!done) {
      uint32_t deferred = 0;   // bit q: tile def_base + q still has to be buffered
      int def_base = tb;
      bool force = false;
      if (tb < t1) {
        uint4 raw[kScanTiles];
        if constexpr (PREFETCH) {
#pragma unroll
          for (int q = 0; q < kScanTiles; ++q) raw[q] = raw_next[q];
          if (tb + kScanTiles < t1) load_group(tb + kScanTiles, raw_next);
        } else {
          load_group(tb, raw);
        }
        // lane maxima of the 4 tiles first; the running max moves at most once per group
        float vmax4[kScanTiles];
#pragma unroll
        for (int q = 0; q < kScanTiles; ++q) {
          float x[EPL];
          unpack_vec<EPL>(raw[q], x);
          float vmax = x[0];
#pragma unroll
          for (int e = 1; e < EPL; ++e) vmax = fmaxf(vmax, x[e]);
          vmax4[q] = vmax;
        }
        const float gmax = fmaxf(fmaxf(vmax4[0], vmax4[1]), fmaxf(vmax4[2], vmax4[3]));
        if (gmax > m_l) {
          s_l = (m_l == kNegInf) ? 0.0 : s_l * static_cast<double>(__expf(m_l - gmax));
          m_l = gmax;
        }
        // sum of 2^(x*log2e - c) with c = fl(m*log2e); the rounding of c is a common factor
        // 2^(c - m*log2e) of the whole group, applied once below
        const float kLog2e = 1.4426950408889634f;
        const float mm = (m_l == kNegInf) ? 0.f : m_l;
        const float c = mm * kLog2e;
        const float c_err = __builtin_fmaf(mm, kLog2e, -c);   // m*log2e - c, exact
        float acc = 0.f;
#pragma unroll
        for (int q = 0; q < kScanTiles; ++q) {
          // unpack again from the raw vector instead of keeping the 4 * EPL floats of the
          // maximum pass alive (the empty asm hides the value's origin from the optimiser)
          uint4 r = raw[q];
          asm volatile("" : "+v"(r.x), "+v"(r.y), "+v"(r.z), "+v"(r.w));
          float x[EPL];
          unpack_vec<EPL>(r, x);
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc += __builtin_amdgcn_exp2f(__builtin_fmaf(x[e], kLog2e, -c));
        }
        s_l += static_cast<double>(acc * __builtin_amdgcn_exp2f(-c_err));
        if (tb == t0) { first_threshold(gmax); force = true; }
#pragma unroll
        for (int q = 0; q < kScanTiles; ++q)
          if (deferred != 0u || !buffer_hits(raw[q], vmax4[q], tb + q)) deferred |= 1u << q;
        tb += kScanTiles;
      } else {
        force = cnt > 0;
        done = true;
      }

      if (force || deferred != 0u || cnt > kHitTrigger) {
        // ---- slow section: cut the buffer to the k best; then buffer the deferred tiles
        while (true) {
          // Expand the buffered vectors, rank their logits that reach tau together with the k
          // best so far, keep the k best.  Every buffered token id is below every id still to
          // come (deferred tiles included), so afterwards a logit equal to the k-th best loses
          // the tie and tau becomes the next float above it.
          for (int base = 0; base < cnt; base += kSubBatch) {
            constexpr int HPL = EPL / 2;   // logits per lane: a lane expands half a vector
            float x[HPL];
            int e0 = 0;
            uint32_t hbits = 0;
            if (base + (lane >> 1) < cnt) {
              const int slot = base + (lane >> 1), half = lane & 1;
              const uint2 raw = reinterpret_cast<const uint2*>(&hitv[slot])[half];
              const int hdr = hith[slot];
              e0 = (((hdr >> 6) * 4 + wave) * 64 + (hdr & 63)) * EPL + half * HPL;
              if constexpr (EPL == 4) {
                x[0] = __uint_as_float(raw.x); x[1] = __uint_as_float(raw.y);
              } else {
                x[0] = __uint_as_float(raw.x << 16); x[1] = __uint_as_float(raw.x & 0xFFFF0000u);
                x[2] = __uint_as_float(raw.y << 16); x[3] = __uint_as_float(raw.y & 0xFFFF0000u);
              }
#pragma unroll
              for (int e = 0; e < HPL; ++e)
                if (x[e] >= tau && e0 + e < a.vocab) hbits |= 1u << e;
            }
            const int nh = __popc(hbits);
            const int incl = wave_inclusive_scan_i32(nh);
            const int total = __builtin_amdgcn_readlane(incl, 63);
            if (lane < tcnt) ck[lane] = topw[lane];
            int pos = tcnt + incl - nh;
#pragma unroll
            for (int e = 0; e < HPL; ++e)
              if (hbits & (1u << e)) ck[pos++] = make_key(x[e], e0 + e);
            const int n = tcnt + total;
            if (lane < 16) ck[n + lane] = 0ull;   // zero keys up to the next multiple of 16
            // LDS operations of one wavefront complete in order: ck is complete before it is read
            for (int i = lane; i < n; i += 64) {
              const unsigned long long key = ck[i];
              const int r = count_greater_pad16(ck, n, key);
              if (r < k) topw[r] = key;
            }
            tcnt = n < k ? n : k;
            if (tcnt >= k) tau = fmaxf(tau, key_logit(topw[k - 1]));
          }
          cnt = 0;
          if (tcnt >= k) tau = float_above(key_logit(topw[k - 1]));
          if (deferred == 0u) break;
#pragma unroll 1
          for (int q = 0; q < kScanTiles; ++q) {
            if (!((deferred >> q) & 1u)) continue;
            const int tile = def_base + q;
            const uint4 raw = load_vec<EPL>(row, (tile * kThreads + tid) * EPL, a.vocab);
            float x[EPL];
            unpack_vec<EPL>(raw, x);
            float vmax = x[0];
#pragma unroll
            for (int e = 1; e < EPL; ++e) vmax = fmaxf(vmax, x[e]);
            if (!buffer_hits(raw, vmax, tile)) break;   // full again: cut first
            deferred &= ~(1u << q);
          }
        }
      }
    }

    // ---- wavefront statistics
    {
      const float wmax = wave_max_f32(m_l);
      // rescale factors are <= 1 and only need fp32 accuracy: their error is relative to a part of the sum
      const double sl = (m_l == kNegInf) ? 0.0 : s_l * static_cast<double>(__expf(m_l - wmax));
      const double wsum = wave_sum_f64(sl);
      if (lane == 0) { s_wmax[wave] = wmax; s_wsum[wave] = wsum; s_wcnt[wave] = tcnt; }
      static_assert(TALON_K_MAX == 64, "a list has one slot per lane");
      if (lane >= tcnt) topw[lane] = 0ull;   // unused slots of the list: zero keys
    }
    __syncthreads();

    // ---- merge the four lists (each <= k keys, zero keys in the unused slots) into the
    // chunk's k best, sorted.  Lane 16w+i of every wavefront holds key i of list w; wavefront v
    // counts how many keys of list v are greater; the four counts add up to the rank.
    const int ctot = s_wcnt[0] + s_wcnt[1] + s_wcnt[2] + s_wcnt[3];
    if (k <= 16) {
      const unsigned long long mkey = s_topw[lane >> 4][lane & 15];
      s_part[wave][lane] = count_greater_pad16(s_topw[wave], 16, mkey);
      __syncthreads();
      if (wave == 0) {
        const int r = s_part[0][lane] + s_part[1][lane] + s_part[2][lane] + s_part[3][lane];
        if (mkey != 0ull && r < k) s_top[r] = mkey;
        if (lane >= ctot && lane < k) s_top[lane] = 0ull;   // fewer than k logits in this chunk
      }
    } else {
      // long lists: thread t holds key t % 64 of its own wavefront's list and counts against all four
      const unsigned long long mkey = s_topw[wave][lane];
      int r = 0;
#pragma unroll 1   // a rare path: keep it small in registers
      for (int w = 0; w < 4; ++w) r += count_greater_pad16(s_topw[w], 64, mkey);
      if (mkey != 0ull && r < k) s_top[r] = mkey;
      if (tid >= ctot && tid < k) s_top[tid] = 0ull;
    }
    const float cm = fmaxf(fmaxf(s_wmax[0], s_wmax[1]), fmaxf(s_wmax[2], s_wmax[3]));
    double csum = 0.0;
#pragma unroll
    for (int w = 0; w < 4; ++w)
      if (s_wmax[w] != kNegInf) csum += s_wsum[w] * static_cast<double>(__expf(s_wmax[w] - cm));
    __syncthreads();

    bool row_written = false;   // this workgroup has just written a whole row's outputs
    bool row_bad = false;       // ... and the row could not be normalised
    // Alg. 2 line 1 inside the single launch: T = {x_t}, p(x_t) = 1, d = 0.  The workgroup that
    // writes the root's row (and then runs the sequence's first selection) sets the state up.
    auto start_tree = [&]() {
      if constexpr (TREE) {
        if (a.root_token && launch_idx == 0) {
          if (tid == 0) {
            const talon_tree_state& st = a.sel.st;
            const size_t o = static_cast<size_t>(b) * st.N_pad;
            store_agent(st.token + o, a.root_token[b]);
            store_agent(st.parent + o, -1);
            store_agent(st.depth + o, 0);
            store_agent(st.prob + o, 1.f);
            store_agent(st.logp + o, 0.0);
            store_agent(st.n_nodes + b, 1);
            store_agent(st.frontier_begin + b, 0);
            store_agent(st.frontier_count + b, 1);
            store_agent(st.depth_cur + b, 0);
            store_agent(st.status + b, 0u);
          }
          __syncthreads();
        }
      }
    };
    if (chunks == 1) {
      start_tree();
      row_bad = write_row<FUSED>(a, b, out_row, s_top, 1, cm, csum, s_cand, &s_nc);
      row_written = true;
    } else {
      unsigned long long* pk = a.part_keys + (static_cast<size_t>(out_row) * blocks_per_row + ch) * k;
      if (tid < k) store_agent(pk + tid, s_top[tid]);
      if (tid == 0) {
        store_agent(a.part_max + static_cast<size_t>(out_row) * blocks_per_row + ch, cm);
        store_agent(a.part_sum + static_cast<size_t>(out_row) * blocks_per_row + ch, csum);
      }
      // every partial store of this workgroup has completed before the ticket is taken
      stores_performed();
      __syncthreads();
      if (tid == 0) {
        const int old = __hip_atomic_fetch_add(&a.ticket[out_row], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (old == chunks - 1) ? 1 : 0;
      }
      __syncthreads();
      if (s_last) {
        const float* pm = a.part_max + static_cast<size_t>(out_row) * blocks_per_row;
        const double* ps = a.part_sum + static_cast<size_t>(out_row) * blocks_per_row;
        const unsigned long long* keys = a.part_keys + static_cast<size_t>(out_row) * blocks_per_row * k;
        const int nkeys = chunks * k;
        const int nkeys_pad = (nkeys + 15) & ~15;   // zero keys rank below every real key
        // softmax statistics of the row: every wavefront merges the chunk statistics on its own
        // (one chunk per lane, more only for very long rows), so that no workgroup-wide
        // reduction is needed.  All loads of the first sweep are issued before any is used.
        float mc0 = kNegInf;
        double sc0 = 0.0;
        if (lane < chunks) { mc0 = load_agent(pm + lane); sc0 = load_agent(ps + lane); }
        const unsigned long long key0 = tid < nkeys ? load_agent(keys + tid) : 0ull;
        if (tid < nkeys_pad) s_keys[tid] = key0;
        for (int i = tid + kThreads; i < nkeys_pad; i += kThreads) s_keys[i] = i < nkeys ? load_agent(keys + i) : 0ull;
        float m = mc0;
        for (int c = lane + 64; c < chunks; c += 64) m = fmaxf(m, load_agent(pm + c));
        m = wave_max_f32(m);
        double sum = (mc0 != kNegInf) ? sc0 * static_cast<double>(__expf(mc0 - m)) : 0.0;
        for (int c = lane + 64; c < chunks; c += 64) {
          const float mc = load_agent(pm + c);
          if (mc != kNegInf) sum += load_agent(ps + c) * static_cast<double>(__expf(mc - m));
        }
        sum = wave_sum_f64(sum);
        __syncthreads();   // s_keys is staged
        start_tree();
        row_bad = write_row<FUSED>(a, b, out_row, s_keys, chunks, m, sum, s_cand, &s_nc);
        if (tid == 0) store_agent(a.ticket + out_row, 0);  // leave the workspace clean for the next layer
        row_written = true;
      }
    }
    if constexpr (FUSED) {
      if (row_written) {
        // ---- sequence ticket: the workgroup that writes the last row of a sequence's frontier
        // runs that sequence's budget selection
        const int F = s_prefix[b + 1] - s_prefix[b];
        if (F > 1) {
          stores_performed();
          __syncthreads();
          if (tid == 0) {
            // low 16 bits: rows written; above: how many of them could not be normalised
            const int old = __hip_atomic_fetch_add(&a.seq_ticket[b], row_bad ? 0x10001 : 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const bool last = (old & 0xFFFF) == F - 1;
            s_last = last ? ((old >> 16) != 0 || row_bad ? 2 : 1) : 0;
            if (last) store_agent(a.seq_ticket + b, 0);
          }
        } else {
          stores_performed();   // the selection reads the row's candidates back from global memory
          if (tid == 0) s_last = row_bad ? 2 : 1;   // a one-row frontier: the workgroup that wrote the row selects right away
        }
        __syncthreads();
        if constexpr (!TREE) {
          if (s_last) {
            // One layer per launch: the selection rewrites the state the item map is made from.
            // Wait until every workgroup of the grid has read it (workgroups that have not
            // started yet start as others leave; only the at most B selecting workgroups wait,
            // so the others always get their turn).  The wait is bounded like the single
            // launch's: a workgroup that gives up marks the sequence aborted and selects nothing.
            if (tid == 0) {
              const unsigned long long t0 = wall_clock64();
              while (load_agent(a.exit_ticket + kStartedWord) != gridDim.x) {
                if (wall_clock64() - t0 > a.spin_ticks) { s_last = 3; break; }
                __builtin_amdgcn_s_sleep(2);
              }
            }
            __syncthreads();
          }
        }
        if (s_last == 3) {
          if (tid == 0) atomicOr(&a.status[b], static_cast<uint32_t>(TALON_STATUS_ABORTED));
        } else if (s_last) {
          TL_ANY(launch_idx, 2);
          // A launch that started the tree itself knows the sequence's status (nothing but a
          // row that cannot be normalised can have touched it), its size and its layer
          // without asking memory.
          const bool own = TREE && a.root_token != nullptr;
          const uint32_t status = own ? (s_last == 2 ? static_cast<uint32_t>(TALON_STATUS_BAD_ROW) : 0u)
                                      : __hip_atomic_load(&a.status[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          unsigned long long next = static_cast<unsigned long long>(static_cast<uint32_t>(fbegin));   // count 0
          if (status & TALON_STATUS_BAD_ROW) {   // a row could not be normalised: stop the sequence here
            if (tid == 0) st_<TREE, int32_t>(a.sel.st.frontier_count + b, 0);
          } else {
            const SelectLds lds{reinterpret_cast<unsigned long long*>(s_pool),
                                reinterpret_cast<int*>(s_pool + sizeof(unsigned long long) * kSelectKeySlots),
                                s_red_u64, s_red_i32, s_misc};
            next = select_sequence<true>(a.sel, b, F, fbegin, status, lds, own ? fbegin + F : -1,
                                         own ? launch_idx : -1);
          }
          if constexpr (TREE) {
            // everything this layer wrote for the sequence has been performed before the
            // descriptor that lets the grid into the next layer is stored
            stores_performed();
            __syncthreads();
            if (tid == 0 && launch_idx + 1 < a.N_pad)
              st_<true, unsigned long long>(a.desc + ((launch_idx + 1) * a.B + b), next | kDescReady);
            TL_ANY(launch_idx, 3);
          }   // (a launch of one layer leaves no descriptor: the next call starts from the public state)
        }
        if constexpr (!TREE) {
          if (s_last) {
            // the last selection of the launch puts the two counters back to zero (every
            // workgroup has started by now, so nobody counts after this)
            if (tid == 0) {
              int active = 0;
              for (int q = 0; q < a.B; ++q) active += (s_prefix[q + 1] > s_prefix[q]) ? 1 : 0;
              const uint32_t done_before = __hip_atomic_fetch_add(a.exit_ticket + kSelectedWord, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              if (static_cast<int>(done_before) + 1 == active) {
                store_agent(a.exit_ticket + kStartedWord, 0u);
                store_agent(a.exit_ticket + kSelectedWord, 0u);
              }
            }
          }
        }
      }
    }
    __syncthreads();  // s_keys / s_top / s_w* are reused by the next item
  }
  return total_rows;
}

// With the selection in its tail the kernel needs about 160 vector registers: three
// workgroups per compute unit instead of four, rather than spilling.
template <int EPL, int MODE>
__global__ __launch_bounds__(kThreads, MODE == kModeSplit ? 4 : 3) void expand_kernel(ExpandArgs a) {
  static_assert(MODE != kModeTree, "the single-launch loop has its own kernel");
  expand_body<EPL, MODE>(a, a.launch_idx);
}

// All layers in one launch.  The grid must be resident as a whole (the host sizes it from the
// occupancy of this kernel): a workgroup waits, between two layers, for the selections of the
// layer it has just left, which other workgroups run.  The wait is bounded; a workgroup that
// gives up marks every sequence TALON_STATUS_ABORTED and leaves, and so do all others.
template <int EPL>
__global__ __launch_bounds__(kThreads, 3) void expand_tree_kernel(ExpandArgs a) {
  __shared__ int s_go;
  // a launch that is only wanted when an earlier one of the same call has raised its flag
  if (a.run_if && load_agent(a.run_if) == 0u) return;
  bool gave_up = false;
  // One pass more than there are layers: the pass after the last layer finds every sequence
  // finished (depth cap or budget), which is also the proof that every selection is
  // published.  A pass starts by waiting for the descriptors of its layer.
  int d = 0;
  for (; d <= a.layers; ++d) {
    TL_MARK(d, 0);
    const int rows = expand_body<EPL, kModeTree>(a, d);
    TL_MARK(d, 1);
    if (rows < 0) {   // the wait for a descriptor ran out
      for (int b = threadIdx.x; b < a.B; b += kThreads) atomicOr(&a.status[b], TALON_STATUS_ABORTED);
      gave_up = true;
      break;
    }
    if (rows == 0) break;   // uniform over the grid: every workgroup reads the same descriptors
  }
  TL_MARK(31, 0);
  // ---- exit ticket: this workgroup has finished with the tickets and layer counters (all its
  // own updates of them have completed).  The answer is needed only after the masks.
  stores_performed();
  __syncthreads();
  // Two levels: workgroup i counts in group i % kExitGroups; the last of a group counts the
  // group.  Low 16 bits: arrivals; above: how many of them gave up.
  const uint32_t group = blockIdx.x % kExitGroups;
  const uint32_t group_size = (gridDim.x - group + kExitGroups - 1) / kExitGroups;
  const uint32_t n_groups = gridDim.x < kExitGroups ? gridDim.x : kExitGroups;
  uint32_t left_before = 0u;
  if (threadIdx.x == 0)
    left_before = __hip_atomic_fetch_add(a.exit_ticket + 1 + group, gave_up ? 0x10001u : 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  // ---- ancestor masks (Fig. 5(b), App. B): every selection of every layer is published by
  // now.  Bit j of row i is set iff j is i or an ancestor of i; one thread per node walks its
  // parent chain in LDS.
  __shared__ int s_par[TALON_N_MAX];
  const talon_tree_state& st = a.sel.st;
  const int words = st.N_pad / 64;
  for (int b = blockIdx.x; a.tree_mask && !gave_up && b < a.B; b += gridDim.x) {
    const int tid = threadIdx.x;
    const int n = load_agent(st.n_nodes + b);
    const size_t base = static_cast<size_t>(b) * st.N_pad;
    __syncthreads();
    if (tid < st.N_pad) s_par[tid] = tid < n ? load_agent(st.parent + base + tid) : -1;
    __syncthreads();
    if (tid < st.N_pad) {
      uint64_t w[4] = {0, 0, 0, 0};
      if (tid < n) {
        int j = tid;
        for (int step = 0; step < TALON_N_MAX && j >= 0; ++step) {
          const uint64_t bit = 1ull << (j & 63);
          const int q = j >> 6;
#pragma unroll
          for (int u = 0; u < 4; ++u) w[u] |= q == u ? bit : 0ull;
          j = s_par[j];
        }
      }
      uint64_t* row = a.tree_mask + (base + tid) * words;
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (u < words) row[u] = w[u];
    }
  }
  TL_MARK(31, 1);
  // ---- the last workgroup to leave puts the counters back to zero for the next launch; if
  // any workgroup gave up, tickets may be half taken: clear them all, and mark every sequence
  // (a tree started late in the launch may have overwritten the mark)
  if (threadIdx.x == 0) {
    int go = 0;
    if ((left_before & 0xFFFFu) == group_size - 1u) {   // last of its group
      const bool bad = (left_before >> 16) != 0u || gave_up;
      const uint32_t groups_before = __hip_atomic_fetch_add(a.exit_ticket, bad ? 0x10001u : 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((groups_before & 0xFFFFu) == n_groups - 1u) go = ((groups_before >> 16) != 0u || bad) ? 2 : 1;
    }
    s_go = go;
  }
  __syncthreads();
  if (s_go == 0) return;
  const int t = threadIdx.x;
  // descriptors of the layers this launch has written (all of them if a workgroup gave up)
  const int used = s_go == 2 ? a.N_pad - 1 : (d + 1 < a.N_pad ? d + 1 : a.N_pad - 1);
  for (int i = t; i < used * a.B; i += kThreads) store_agent(a.desc + a.B + i, 0ull);
  if (s_go == 2) {
    for (int i = t; i < a.B * a.N_pad; i += kThreads) store_agent(a.ticket + i, 0);
    for (int i = t; i < a.B; i += kThreads) {
      store_agent(a.seq_ticket + i, 0);
      atomicOr(&a.status[i], TALON_STATUS_ABORTED);
    }
  }
  for (int i = t; i < kExitWords; i += kThreads) store_agent(a.exit_ticket + i, 0u);
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

// Start of a fused call that continues trees already begun: frontier descriptors of its first
// layer from the public tree state, none for the later layers; zero tickets (nothing leaves
// them taken, but a caller may hand over a workspace that other launch forms have used).
__global__ void fused_init_kernel(talon_tree_state st, unsigned long long* desc, int32_t* ticket, int32_t* seq_ticket,
                                  FusedInitArgs f) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (f.mode == kInitRestoreIf && *f.flag == 0u) return;
  if (f.mode == kInitSave && f.clear && i <= kExitWords) f.clear[i] = 0u;   // (the grid has at least 256 threads)
  if (i >= st.B * st.N_pad) return;
  ticket[i] = 0;
  if (i >= st.B) { desc[i] = 0ull; return; }
  seq_ticket[i] = 0;
  if (f.mode == kInitSave) {
    f.saved[i] = st.n_nodes[i];
    f.saved[st.B + i] = st.frontier_begin[i];
    f.saved[2 * st.B + i] = st.frontier_count[i];
    f.saved[3 * st.B + i] = st.depth_cur[i];
    f.saved[4 * st.B + i] = static_cast<int32_t>(st.status[i]);
  } else if (f.mode == kInitRestoreIf) {
    st.n_nodes[i] = f.saved[i];
    st.frontier_begin[i] = f.saved[st.B + i];
    st.frontier_count[i] = f.saved[2 * st.B + i];
    st.depth_cur[i] = f.saved[3 * st.B + i];
    st.status[i] = static_cast<uint32_t>(f.saved[4 * st.B + i]);
  }
  const uint32_t count = (st.status[i] & kDoneMask) ? 0u : static_cast<uint32_t>(st.frontier_count[i]);
  desc[i] = kDescReady | (static_cast<unsigned long long>(count) << 32) | static_cast<uint32_t>(st.frontier_begin[i]);
}

hipError_t launch_fused_init(const talon_tree_state& st, const ExpandArgs& a, const FusedInitArgs& f, hipStream_t s) {
  const int n = st.B * st.N_pad;
  hipLaunchKernelGGL(fused_init_kernel, dim3((n + 255) / 256), dim3(256), 0, s, st, a.desc, a.ticket, a.seq_ticket, f);
  return hipGetLastError();
}

hipError_t launch_expand_tree(const ExpandArgs& a, int dtype, int grid, hipStream_t s) {
  if (dtype == TALON_DTYPE_F32) hipLaunchKernelGGL(expand_tree_kernel<4>, dim3(grid), dim3(kThreads), 0, s, a);
  else hipLaunchKernelGGL(expand_tree_kernel<8>, dim3(grid), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

// Workgroups of the single-launch kernel that the current device holds at once.
int expand_tree_max_grid(int dtype) {
  int dev = 0, per_cu = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
  const hipError_t e = dtype == TALON_DTYPE_F32
      ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, expand_tree_kernel<4>, kThreads, 0)
      : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, expand_tree_kernel<8>, kThreads, 0);
  if (e != hipSuccess) return 0;
  return per_cu * prop.multiProcessorCount;
}

hipError_t launch_expand(const ExpandArgs& a, int dtype, int grid, bool fused, hipStream_t s) {
  if (dtype == TALON_DTYPE_F32) {
    if (fused) hipLaunchKernelGGL((expand_kernel<4, kModeFused>), dim3(grid), dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL((expand_kernel<4, kModeSplit>), dim3(grid), dim3(kThreads), 0, s, a);
  } else {
    if (fused) hipLaunchKernelGGL((expand_kernel<8, kModeFused>), dim3(grid), dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL((expand_kernel<8, kModeSplit>), dim3(grid), dim3(kThreads), 0, s, a);
  }
  return hipGetLastError();
}

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
