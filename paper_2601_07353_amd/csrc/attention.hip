// Tree attention (App. B "Tree Attention"; mask of Fig. 5(b)): every tree node attends to
// the whole prefix KV cache plus the tree keys on its own root-to-node path.
//
// Dense contraction on bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulation, fp32 online
// softmax in base-2 units.
//
// Tiling.  The G = Hq/Hkv query heads that share a KV head are packed with the tree nodes
// into one row dimension (row = node * G + head-in-group), so one K/V tile read from HBM
// feeds G * n query rows.  A workgroup (NW = 4 or 8 wavefronts) owns 32*NW packed rows of one
// (sequence, KV head) and a contiguous range of 64-key tiles (split-KV); each wavefront
// owns one block of 32 rows.  K and V tiles are staged through LDS (double buffered, one
// barrier per tile).  Both products are computed transposed so that a query is a lane:
//   S^T[key][query] = K . Q^T        A = K fragment (LDS, 16-byte reads), B = Q^T (registers)
//   O^T[dh][query] += V^T . P^T      A = V^T fragment (LDS transpose reads), B = P^T
// With this orientation the S^T accumulator registers of a lane are already the P^T operand
// of that lane's query (up to a fixed permutation of the 16 keys of a step, applied to the
// V^T operand as well), and every softmax statistic is a per-lane scalar.
//
// The ancestor mask is applied in-tile and only to the tree tiles (the last N_pad/64 tiles
// of a sequence); prefix tiles need no mask except the ragged last one.
//
// Split-KV partial results (unnormalised O, running max, denominator) go to a workspace
// and are merged by a second kernel; with a single split the output is written directly.
#include <stdlib.h>

#include <type_traits>

#include "device_utils.h"
#include "talon_internal.h"
#ifdef TALON_TUNING
#include "tuning.h"
#endif

namespace talon {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef short short4v __attribute__((ext_vector_type(4)));

constexpr int kKeyTile = 64;
#ifndef TALON_AHEAD_PV
#define TALON_AHEAD_PV 2
#endif
constexpr int kAheadPV = TALON_AHEAD_PV;   // V^T fragments (two reads each) read ahead
constexpr float kNegInfF = -__builtin_huge_valf();

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// 16 bytes per lane from global memory straight into LDS: lane l of the wavefront lands at
// lds_base + 16*l (lds_base wave-uniform).  Written as inline assembly on purpose: for the
// builtin of the same instruction the compiler waits for ALL outstanding loads before the
// next LDS read of any address, which exposes the whole memory latency inside every step;
// here the only waits are the explicit ones of tile_landed().  (Loads complete in order, so
// a compiler-inserted wait for one of its own loads can only wait longer, never less.)
// Same with the address split into a wave-uniform base (scalar registers) and a 32-bit
// per-lane byte offset: the per-tile address arithmetic then runs on the scalar unit.
__device__ __forceinline__ void global_to_lds_16(const uint16_t* uniform_base, uint32_t lane_byte_offset,
                                                 const uint16_t* lds_base) {
  const uint32_t lds_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
      (__attribute__((address_space(3))) void*)(lds_base)));
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(lane_byte_offset), "s"(uniform_base), "s"(lds_addr) : "memory", "m0");
}

__device__ __forceinline__ void global_to_lds_16(const uint16_t* src, const uint16_t* lds_base) {
  const uint32_t lds_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
      (__attribute__((address_space(3))) void*)(lds_base)));
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(src), "s"(lds_addr) : "memory", "m0");
}

// LDS image of one 64-key tile: rows of DH bf16 without padding (the tiles are written by
// direct global-to-LDS loads, which place the 64 lanes of a wavefront back to back).  Bank
// conflicts are avoided by permuting the 16-byte chunks of every row, differently for K
// (read as 16-byte fragments, 16 consecutive key rows at one chunk index) and for V (read
// with the transposing load, 4 consecutive key rows by 32 bytes).
template <int DH>
struct Smem {
  static constexpr int CPR = DH / 8;                     // 16-byte chunks per key row
  static constexpr int T_ELEMS = kKeyTile * DH;          // one tensor, one tile
  static constexpr int MASK_BYTES = 256 * (TALON_N_MAX / 64) * 8;   // ancestor words of the workgroup's rows (at most 256)
  static constexpr int BYTES = 4 * T_ELEMS * 2 + MASK_BYTES;        // two K stages, two V stages, the mask words
  __device__ static int kswz(int row) { return DH == 128 ? (row & 15) : ((row >> 1) & 7); }
  __device__ static int vswz(int row) { return DH == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }
};

template <int DH, int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void tree_attention_kernel(AttnArgs a) {
  constexpr int RB = 1;             // 32-row blocks per wavefront
  constexpr int kWgThreads = 64 * NW;
  using SM = Smem<DH>;
  constexpr int DSTEPS = DH / 16;   // MFMA steps over the head dimension for S^T
  constexpr int DB = DH / 32;       // 32-row blocks of O^T
  constexpr int CPR = DH / 8;       // 16-byte chunks per key row
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps LDS bases in scalar registers
  const int l32 = lane & 31;
  const int h = lane >> 5;

  // Workgroup -> work item.  The hardware deals consecutive workgroup ids round-robin to the
  // 8 XCDs, each with its own L2.  The row tiles of one (sequence, KV head, split) read the
  // same K/V tiles, so they are given ids that are congruent modulo 8 and adjacent in time:
  // they share one L2 and the tile is fetched from HBM once, not once per row tile.
  const int per_xcd = (a.total_items + 7) / 8;
  const int item = static_cast<int>(blockIdx.x % 8) * per_xcd + static_cast<int>(blockIdx.x / 8);
  if (item >= a.total_items) return;
  const int rt = item % a.row_tiles;
  const int split = (item / a.row_tiles) % a.splits;
  const int bg = item / (a.row_tiles * a.splits);
  const int b = bg / a.Hkv;
  const int g = bg - b * a.Hkv;
  const int G = a.G;
  const int n = a.n_nodes[b];
  int L = a.prefix_len[b];
  L = L < 0 ? 0 : (L > a.max_prefix_len ? a.max_prefix_len : L);
  const int rows = n * G;
  const int row0 = rt * (32 * NW * RB);
  if (row0 >= rows) return;

  const int nPT = (L + kKeyTile - 1) / kKeyTile;
  const int nTT = (n + kKeyTile - 1) / kKeyTile;
  const int T = nPT + nTT;
  const int t_begin = split * a.tiles_per_split;
  const int t_end = (t_begin + a.tiles_per_split < T) ? t_begin + a.tiles_per_split : T;
  const int words = a.N_pad / 64;

  // ---- this lane's queries (one per row block): which node and head each is
  const int wrow0 = row0 + wave * 32 * RB;
  bf16x8 bq[RB][DSTEPS];   // Q^T operands, loaded in the prologue below
  int node_rb[RB];
  bool valid_rb[RB];
  size_t orow_rb[RB];  // (b*N_pad + node)*Hq + head
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int rho = wrow0 + 32 * rb + l32;
    const bool valid = rho < rows;
    const int node = valid ? rho / G : 0;
    const int j = valid ? rho - node * G : 0;
    node_rb[rb] = node;
    valid_rb[rb] = valid;
    orow_rb[rb] = (static_cast<size_t>(b) * a.N_pad + node) * a.Hq + g * G + j;
  }

  float m_run[RB], l_run[RB];
  floatx16 o[DB][RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    m_run[rb] = kNegInfF;
    l_run[rb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][rb][r] = 0.f;
  }

  // ---- global -> register -> LDS staging of one 64-key tile of K and V
  const uint16_t* kp_base = a.k_prefix + static_cast<int64_t>(b) * a.kv_stride_b + static_cast<int64_t>(g) * a.kv_stride_h;
  const uint16_t* vp_base = a.v_prefix + static_cast<int64_t>(b) * a.kv_stride_b + static_cast<int64_t>(g) * a.kv_stride_h;
  const size_t tree_stride = static_cast<size_t>(a.Hkv) * DH;
  const uint16_t* kt_base = a.k_tree + (static_cast<size_t>(b) * a.N_pad * a.Hkv + g) * DH;
  const uint16_t* vt_base = a.v_tree + (static_cast<size_t>(b) * a.N_pad * a.Hkv + g) * DH;

  // One tile of K and V goes from global memory straight into LDS (no staging registers):
  // every wavefront issues 16-byte-per-lane loads whose 64 lanes land back to back in LDS,
  // i.e. whole key rows; the lane picks the global chunk that belongs at its LDS slot under
  // the row's chunk permutation.  A key past the end of its segment reads the segment's last
  // key instead: its score is masked to -inf below, so its probability is exactly 0 and the
  // (finite) value row it brought along adds nothing.
  constexpr int ROWS_PER_LOAD = 64 / CPR;                 // key rows per wavefront load
  // With eight wavefronts only the last four issue tile loads (twice as many each).  A compute
  // unit's address path takes a step's 32 KB in about 512 cycles whoever issues them, and a
  // wavefront waits at its loads for its turn: with half of the wavefronts loading, the other
  // half never waits there (measured: 16384 keys 2.6 % faster; two or one loading wavefronts
  // are slower again, and which half loads makes no difference).
  constexpr int LW = NW == 8 ? NW / 2 : NW;   // wavefronts that issue tile loads
  constexpr int LOADS = kKeyTile / ROWS_PER_LOAD / LW;    // loads per loading wavefront, tile and tensor
  static_assert(LOADS >= 1, "every loading wavefront loads at least one group of key rows");
  const int lwave = wave - (NW - LW);                     // the loaders are the last LW wavefronts
  const bool loader = lwave >= 0 && lwave < LW;           // wave-uniform
  // LDS: two K stages then two V stages.
  unsigned long long* s_mask = reinterpret_cast<unsigned long long*>(smem + 4 * SM::T_ELEMS);
  auto stage_k = [&](int st_) { return smem + st_ * SM::T_ELEMS; };
  auto stage_v = [&](int st_) { return smem + (2 + st_) * SM::T_ELEMS; };
  auto load_tensor = [&](int t, const uint16_t* pre_base, const uint16_t* tree_base, uint16_t* dst, bool is_k) {
    const bool is_prefix = t < nPT;
    const int key0 = (is_prefix ? t : t - nPT) * kKeyTile;
    const int last = (is_prefix ? L : n) - 1;
    const size_t stride = is_prefix ? static_cast<size_t>(a.kv_stride_t) : tree_stride;
    const uint16_t* base = is_prefix ? pre_base : tree_base;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int row0_ = (lwave * LOADS + i) * ROWS_PER_LOAD;
      const int row = row0_ + lane / CPR;
      const int cslot = lane % CPR;
      int key = key0 + row;
      key = key < last ? key : last;
      const int chunk = cslot ^ (is_k ? SM::kswz(row) : SM::vswz(row));
      const uint16_t* src = base + static_cast<size_t>(key) * stride + chunk * 8;
      global_to_lds_16(src, dst + row0_ * DH);
    }
  };
  // Fast path for a prefix tile that lies wholly below the prefix length: no clamping, and
  // the address is a per-lane base plus tile and load offsets (no 64-bit multiplies).
  const int lrow = lane / CPR;                       // key row of this lane inside one load
  const size_t tile_step = static_cast<size_t>(kKeyTile) * a.kv_stride_t;       // elements between tiles
  // Byte offset of this lane's chunk inside a tile, per load.  Where a loading wavefront has
  // four loads per tensor (half of the wavefronts load), there are no registers to spare for
  // eight offsets: the first row of a load goes into the wave-uniform base address and the lane
  // offset is put together at the load.  The first row u of a load is a multiple of
  // ROWS_PER_LOAD and lrow is below it, so kswz(u + lrow) = kswz(u) ^ kswz(lrow) and
  // vswz(u + lrow) = vswz(lrow).
  constexpr bool kOffsetsAtLoad = LW != NW;
  uint32_t koff[kOffsetsAtLoad ? 1 : LOADS], voff[kOffsetsAtLoad ? 1 : LOADS];
  uint32_t lane_row_bytes = 0, kchunk_bytes = 0;
  if constexpr (kOffsetsAtLoad) {
    lane_row_bytes = static_cast<uint32_t>(lrow) * static_cast<uint32_t>(a.kv_stride_t) * 2u;
    kchunk_bytes = static_cast<uint32_t>(((lane % CPR) ^ SM::kswz(lrow)) * 16);
    koff[0] = 0;
    voff[0] = lane_row_bytes + static_cast<uint32_t>(((lane % CPR) ^ SM::vswz(lrow)) * 16);
  } else {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int row = (lwave * LOADS + i) * ROWS_PER_LOAD + lrow;
      const uint32_t row_bytes = static_cast<uint32_t>(row) * static_cast<uint32_t>(a.kv_stride_t) * 2u;
      koff[i] = row_bytes + static_cast<uint32_t>(((lane % CPR) ^ SM::kswz(row)) * 16);
      voff[i] = row_bytes + static_cast<uint32_t>(((lane % CPR) ^ SM::vswz(row)) * 16);
    }
  }
  auto load_full_prefix = [&](int t, int kst, int vst, bool want_k, bool want_v) {
    const uint16_t* kt_ = kp_base + static_cast<size_t>(t) * tile_step;   // wave-uniform
    const uint16_t* vt_ = vp_base + static_cast<size_t>(t) * tile_step;
    uint16_t* sK = stage_k(kst) + lwave * LOADS * ROWS_PER_LOAD * DH;
    uint16_t* sV = stage_v(vst) + lwave * LOADS * ROWS_PER_LOAD * DH;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      if constexpr (kOffsetsAtLoad) {
        const int u = (lwave * LOADS + i) * ROWS_PER_LOAD;                            // wave-uniform
        const size_t row_elems = static_cast<size_t>(u) * a.kv_stride_t;
        if (want_k) global_to_lds_16(kt_ + row_elems, lane_row_bytes + (kchunk_bytes ^ static_cast<uint32_t>(SM::kswz(u) * 16)),
                                     sK + i * ROWS_PER_LOAD * DH);
        if (want_v) global_to_lds_16(vt_ + row_elems, voff[0], sV + i * ROWS_PER_LOAD * DH);
      } else {
        if (want_k) global_to_lds_16(kt_, koff[i], sK + i * ROWS_PER_LOAD * DH);
        if (want_v) global_to_lds_16(vt_, voff[i], sV + i * ROWS_PER_LOAD * DH);
      }
    }
  };
  auto is_full_prefix = [&](int t) { return t < nPT && (t + 1) * kKeyTile <= L; };
  auto load_k = [&](int t, int st_) {
    if (!loader) return;
    if (is_full_prefix(t)) load_full_prefix(t, st_, 0, true, false);
    else load_tensor(t, kp_base, kt_base, stage_k(st_), true);
  };
  auto load_v = [&](int t, int st_) {
    if (!loader) return;
    if (is_full_prefix(t)) load_full_prefix(t, 0, st_, false, true);
    else load_tensor(t, vp_base, vt_base, stage_v(st_), false);
  };
  auto tile_landed = [&]() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };

  const float c2 = a.scale_log2e;

  // S^T = K . Q^T for the 64 keys of one K stage
  auto qk = [&](const uint16_t* sK, floatx16 (&s)[2][RB]) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][rb][r] = 0.f;
      const int krow_i = 32 * kb + l32;
      const uint16_t* krow = sK + krow_i * DH;
      const int ksw = SM::kswz(krow_i);
#pragma unroll
      for (int ds = 0; ds < DSTEPS; ++ds) {
        const bf16x8 ak = as_bf16x8(*reinterpret_cast<const uint4*>(krow + ((2 * ds + h) ^ ksw) * 8));
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          s[kb][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, bq[rb][ds], s[kb][rb], 0, 0, 0);
      }
    }
  };

  // Mask of tile t: ancestor bits on tree tiles, length bound on the ragged prefix tile.
  auto mask_scores = [&](int t, floatx16 (&s)[2][RB]) {
    const bool is_prefix = t < nPT;
    const int key0 = (is_prefix ? t : t - nPT) * kKeyTile;
    const bool full = is_prefix && key0 + kKeyTile <= L;
    if (full) return;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      unsigned long long allow;
      if (is_prefix) allow = (1ull << (L - key0)) - 1ull;
      else allow = s_mask[(wave * 32 * RB + 32 * rb + l32) * words + (t - nPT)];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const uint32_t w = static_cast<uint32_t>(allow >> (32 * kb)) >> (4 * h);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int bit = 8 * (r / 4) + (r % 4);
          if (!((w >> bit) & 1u)) s[kb][rb][r] = kNegInfF;
        }
      }
    }
  };

  // One pipelined step for tile t = t_begin + i, whose (masked) scores are already in s:
  //   start the loads of K(t+2) and V(t+1); compute the scores of tile t+1 into s_nxt (matrix
  //   pipe) while the softmax of tile t runs (vector pipe); then O^T += V(t)^T . P^T.
  const int nt = t_end - t_begin;
  auto step = [&](int i, floatx16 (&s)[2][RB], floatx16 (&s_nxt)[2][RB], auto has_next) {
    constexpr bool kHasNext = decltype(has_next)::value;   // a tile t+1 exists in this split
    const int t = t_begin + i;
    if (i + 2 < nt) load_k(t + 2, i & 1);          // the stage K(t) has just left
    if constexpr (kHasNext) load_v(t + 1, (i + 1) & 1);
    const uint16_t* sV = stage_v(i & 1);
    static_assert(RB == 1, "the pipelined step is written for one row block per wavefront");

    // ---- online softmax (base 2), per query = per lane pair (lane, lane ^ 32); s holds the
    // masked scores of tile t
    bf16x8 pb[2][2][RB];
    float mx = kNegInfF;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][0][r]);
    {
      const int mi = __float_as_int(mx);
      const auto sw = __builtin_amdgcn_permlane32_swap(mi, mi, false, false);   // {own, lane ^ 32} in some order
      mx = fmaxf(__int_as_float(static_cast<int>(sw[0])), __int_as_float(static_cast<int>(sw[1])));
    }
    const float m_new = fmaxf(m_run[0], mx * c2);
    const float m_safe = m_new == kNegInfF ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run[0] - m_safe);
    m_run[0] = m_new;
    if (__ballot(alpha != 1.f) != 0ull) {   // after the first tiles the running max rarely moves
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][0][r] *= alpha;
    }
    // From here to the mask of the next tile there is no branch: the matrix instructions of
    // the next tile's scores and the exponentials of this tile are independent and are
    // scheduled against each other.
    if constexpr (kHasNext) qk(stage_k((i + 1) & 1), s_nxt);
    {
      float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
          bf16x8 pk;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][0][8 * sp + e], c2, -m_safe));
            if (e & 1) sum1 += p; else sum0 += p;
            pk[e] = static_cast<__bf16>(p);
          }
          pb[kb][sp][0] = pk;
        }
      }
      l_run[0] = l_run[0] * alpha + (sum0 + sum1);
    }
    // (Which of them goes where is left to the compiler's scheduler: an explicit pattern of one
    // fragment read, one matrix instruction and a handful of vector instructions, repeated, was
    // measured 3-4 % slower at 8192 and 16384 keys.)
    if constexpr (kHasNext) mask_scores(t + 1, s_nxt);

    // ---- O^T += V^T . P^T
    {
      const int i16 = lane & 15;
      const int dhblk = (lane >> 4) & 1;
      const int vrow_l = 4 * h + (i16 >> 2);          // + 32*kb + 16*sp (+ 8 for the second read)
      const int vsw = SM::vswz(vrow_l);               // the added row offsets are multiples of 8
      const int vch = 2 * dhblk + ((i16 & 3) >> 1);   // + 4*db: chunk of this lane's 4 values
      const int vsub = (i16 & 1) * 4;                 // element offset inside the chunk
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const uint16_t* vp = sV + (32 * kb + 16 * sp + vrow_l) * DH + ((4 * db + vch) ^ vsw) * 8 + vsub;
            const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) short4v*)(vp));
            const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) short4v*)(vp + 8 * DH));
            typedef short short8v __attribute__((ext_vector_type(8)));
            const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            const bf16x8 av = __builtin_bit_cast(bf16x8, both);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
              o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pb[kb][sp][rb], o[db][rb], 0, 0, 0);
          }
        }
      }
      // the transposing reads of a V^T fragment (two per matrix instruction) run two matrix
      // instructions ahead
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAheadPV, 0);
#pragma unroll
      for (int g_ = 0; g_ < 4 * DB - kAheadPV; ++g_) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, kAheadPV, 0);
    }
    // loads of K(t+2), V(t+1) have landed; every wavefront is done with K(t+1) and V(t)
    tile_landed();
  };

  // Prologue.  Three kinds of loads start the workgroup: the first K/V tiles (global to LDS),
  // this lane's queries (registers) and the ancestor words of the workgroup's rows (LDS, so that
  // inside the loop the only global loads are the tile loads, whose waits are all explicit).
  // They are issued back to back, tiles first, and waited for together: one memory round trip
  // instead of three.
  if (nt > 0) {
    load_k(t_begin, 0);
    load_v(t_begin, 0);
    if (nt > 1) load_k(t_begin + 1, 1);
  }
  // ---- this lane's queries (loaded here, after the tile loads have been issued)
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const uint16_t* qp = a.q + orow_rb[rb] * DH + 8 * h;
#pragma unroll
    for (int ds = 0; ds < DSTEPS; ++ds) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (valid_rb[rb]) v = *reinterpret_cast<const uint4*>(qp + 16 * ds);
      bq[rb][ds] = as_bf16x8(v);
    }
  }
  for (int idx = tid; idx < 32 * NW * RB * words; idx += kWgThreads) {
    const int r = idx / words;
    const int rho = row0 + r;
    unsigned long long wv = 0ull;
    if (rho < rows) wv = a.mask[(static_cast<size_t>(b) * a.N_pad + rho / G) * words + (idx - r * words)];
    s_mask[idx] = wv;
  }
  // Make the compiler wait for the query loads here, in straight-line code: otherwise it
  // places its wait for them at their first use inside the loop, where it would also wait
  // for every tile load in flight (see global_to_lds_16).
  {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    static_assert(RB == 1 && (DSTEPS == 8 || DSTEPS == 4), "one statement names every query fragment");
    u32x4 qv[DSTEPS];
#pragma unroll
    for (int ds = 0; ds < DSTEPS; ++ds) qv[ds] = __builtin_bit_cast(u32x4, bq[0][ds]);
    if constexpr (DSTEPS == 8)
      asm volatile("" : "+v"(qv[0]), "+v"(qv[1]), "+v"(qv[2]), "+v"(qv[3]), "+v"(qv[4]), "+v"(qv[5]), "+v"(qv[6]), "+v"(qv[7]));
    else
      asm volatile("" : "+v"(qv[0]), "+v"(qv[1]), "+v"(qv[2]), "+v"(qv[3]));
#pragma unroll
    for (int ds = 0; ds < DSTEPS; ++ds) bq[0][ds] = __builtin_bit_cast(bf16x8, qv[ds]);
  }

  floatx16 s_a[2][RB], s_b[2][RB];
  if (nt > 0) {
    tile_landed();
    qk(stage_k(0), s_a);
    mask_scores(t_begin, s_a);
    __syncthreads();   // K stage 0 is free for K(t_begin + 2)
  }
  {
    constexpr std::true_type more{};
    constexpr std::false_type last{};
    int i = 0;
    for (; i + 2 < nt; i += 2) {   // two steps per trip so that the score registers swap roles
      step(i, s_a, s_b, more);
      step(i + 1, s_b, s_a, more);
    }
    if (i + 1 < nt) {
      step(i, s_a, s_b, more);
      step(i + 1, s_b, s_a, last);
    } else if (i < nt) {
      step(i, s_a, s_b, last);
    }
  }

  // ---- epilogue
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float l_tot;
    {
      const int li = __float_as_int(l_run[rb]);
      const auto sw = __builtin_amdgcn_permlane32_swap(li, li, false, false);
      l_tot = __int_as_float(static_cast<int>(sw[0])) + __int_as_float(static_cast<int>(sw[1]));
    }
    // Where this lane's row goes is worked out again here, from a lane index the compiler cannot
    // trace back: otherwise it keeps the output addresses alive (or spills them) across the loop.
    int l32_e = l32;
    asm volatile("" : "+v"(l32_e));
    const int rho_e = wrow0 + 32 * rb + l32_e;
    if (rho_e >= rows) continue;
    const int node_e = rho_e / G;
    const size_t orow_e = (static_cast<size_t>(b) * a.N_pad + node_e) * a.Hq + g * G + (rho_e - node_e * G);
    if (a.splits == 1) {
      const float inv = 1.f / l_tot;
      uint16_t* op = a.out + orow_e * DH;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = static_cast<__bf16>(o[db][rb][4 * q4 + e] * inv);
          *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * q4 + 4 * h) = v;
        }
      }
      if (a.out_lse && h == 0) a.out_lse[orow_e] = (m_run[rb] + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    } else {
      // Partial O^T of a (KV head, split), normalised by the split's own denominator and rounded
      // to bf16 (half the bytes of the round trip through memory; the rounding, 2^-9 relative
      // per split, is below that of the final bf16 output), laid out in slabs of 8 head-dim
      // values: [DH / 8][rows_pad][8], so that the 64 lanes of a store (32 rows x 2 halves of a
      // slab entry) cover 512 consecutive bytes; row-major would give 8-byte pieces.
      const int rho = rho_e;
      const size_t pblock = (static_cast<size_t>(bg) * a.splits + split) * a.rows_pad;
      const size_t prow = pblock + rho;
      uint16_t* po = a.part_o + pblock * DH + static_cast<size_t>(rho) * 8 + 4 * h;
      const float inv_l = l_tot > 0.f ? 1.f / l_tot : 0.f;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = static_cast<__bf16>(o[db][rb][4 * q4 + e] * inv_l);
          *reinterpret_cast<bf16x4*>(po + static_cast<size_t>(4 * db + q4) * a.rows_pad * 8) = v;
        }
      }
      if (h == 0) {
        a.part_m[prow] = m_run[rb];
        a.part_l[prow] = l_tot;
      }
    }
  }
}

// Merge of the split-KV partial results (O_s normalised by its own l_s):
// out = sum_s 2^(m_s - M) l_s O_s / sum_s 2^(m_s - M) l_s.
// One thread per (packed row, 4 head-dim values).  A workgroup takes 256 / (DH / 4) rows.  It
// reads the partial results in their slab order (thread = (slab, row, half): consecutive
// threads, consecutive addresses) and turns its results through LDS to write whole output
// rows.
template <int DH>
__global__ __launch_bounds__(kThreads) void tree_attention_combine_kernel(AttnArgs a) {
  constexpr int QPR = DH / 4;            // threads per row
  constexpr int RPW = kThreads / QPR;    // rows per workgroup
  __shared__ bf16x4 s_out[RPW][QPR];
  const int bg = blockIdx.y;
  const int b = bg / a.Hkv;
  const int g = bg - b * a.Hkv;
  const int rows = a.n_nodes[b] * a.G;
  const int t = threadIdx.x;
  const int h = t & 1;
  const int r = (t >> 1) % RPW;
  const int slab = t / (2 * RPW);        // 8 head-dim values: c = 2 * slab + h
  const int c = 2 * slab + h;
  const int rho = blockIdx.x * RPW + r;
  // Every split of a row tile that has rows stores a partial result (one without key tiles stores
  // a maximum of -inf), and the partial arrays have room for every row the grid covers, so no
  // address here depends on the sequence's lengths: all loads of up to eight splits are issued
  // together with the load of the node count, one memory round trip, and the running maximum is
  // carried across blocks of eight.  Rows past the end read what nobody wrote and are dropped.
  const size_t block0 = static_cast<size_t>(bg) * a.splits * a.rows_pad;
  const size_t base = block0 + rho;
  const size_t in_block = (static_cast<size_t>(slab) * a.rows_pad + rho) * 8 + 4 * h;
  float M = kNegInfF;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float den = 0.f;
  for (int s0 = 0; s0 < a.splits; s0 += 8) {
    float ms[8], ls[8];
    bf16x4 vs[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int s = s0 + u;
      ms[u] = kNegInfF;
      ls[u] = 0.f;
      vs[u] = bf16x4{0, 0, 0, 0};
      if (s < a.splits) {   // uniform
        const size_t pr = base + static_cast<size_t>(s) * a.rows_pad;
        ms[u] = a.part_m[pr];
        ls[u] = a.part_l[pr];
        vs[u] = *reinterpret_cast<const bf16x4*>(a.part_o + (block0 + static_cast<size_t>(s) * a.rows_pad) * DH + in_block);
      }
    }
    float Mb = M;
#pragma unroll
    for (int u = 0; u < 8; ++u) Mb = fmaxf(Mb, ms[u]);
    if (Mb == kNegInfF) continue;              // nothing but empty splits so far
    const float keep = __builtin_amdgcn_exp2f(M - Mb);   // 0 on the first block that holds anything
    M = Mb;
    den *= keep;
    acc.x *= keep; acc.y *= keep; acc.z *= keep; acc.w *= keep;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float w = ms[u] == kNegInfF ? 0.f : __builtin_amdgcn_exp2f(ms[u] - M) * ls[u];   // an empty split: weight 0
      den += w;
      acc.x += w * static_cast<float>(vs[u][0]); acc.y += w * static_cast<float>(vs[u][1]);
      acc.z += w * static_cast<float>(vs[u][2]); acc.w += w * static_cast<float>(vs[u][3]);
    }
  }
  if (blockIdx.x * RPW >= rows) return;  // the whole workgroup is past the end
  const bool valid = rho < rows;
  const float inv = 1.f / den;
  bf16x4 v;
  v[0] = static_cast<__bf16>(acc.x * inv);
  v[1] = static_cast<__bf16>(acc.y * inv);
  v[2] = static_cast<__bf16>(acc.z * inv);
  v[3] = static_cast<__bf16>(acc.w * inv);
  s_out[r][c] = v;
  if (a.out_lse && c == 0 && valid) {
    const int node = rho / a.G;
    const size_t orow = (static_cast<size_t>(b) * a.N_pad + node) * a.Hq + g * a.G + (rho - node * a.G);
    a.out_lse[orow] = (M + __builtin_amdgcn_logf(den)) * 0.6931471805599453f;
  }
  __syncthreads();
  const int r2 = t / QPR;
  const int c2 = t - r2 * QPR;
  const int rho2 = blockIdx.x * RPW + r2;
  if (rho2 < rows) {
    const int node = rho2 / a.G;
    const size_t orow = (static_cast<size_t>(b) * a.N_pad + node) * a.Hq + g * a.G + (rho2 - node * a.G);
    *reinterpret_cast<bf16x4*>(a.out + orow * DH + 4 * c2) = s_out[r2][c2];
  }
}

template <int DH, int NW>
hipError_t launch_one(const AttnArgs& a_in, hipStream_t s) {
  AttnArgs a = a_in;
  a.row_tiles = (a.N_pad * a.G + 32 * NW - 1) / (32 * NW);
  a.total_items = a.row_tiles * a.splits * a.B * a.Hkv;
  auto kern = tree_attention_kernel<DH, NW>;
  // (initialisation of a function-local static is thread-safe: two host threads making their
  // first call together set the attribute once)
  static const hipError_t attr_result = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, Smem<DH>::BYTES);
  if (attr_result != hipSuccess) return attr_result;
  hipLaunchKernelGGL(kern, dim3(8 * ((a.total_items + 7) / 8)), dim3(64 * NW), Smem<DH>::BYTES, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.splits > 1) {
    const int threads = a.N_pad * a.G * (DH / 4);
    hipLaunchKernelGGL(tree_attention_combine_kernel<DH>, dim3((threads + kThreads - 1) / kThreads, a.B * a.Hkv),
                       dim3(kThreads), 0, s, a);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace

// Launch plan: rows per workgroup and the number of KV splits.  A workgroup is 4 wavefronts
// (128 packed rows, two workgroups per compute unit) or, when a (sequence, KV head) has at
// least 512 packed rows, 8 wavefronts (256 rows, one per compute unit): the same 8 wavefronts
// per compute unit, but a K/V tile is loaded once for 256 rows instead of twice.  Either way
// the grid aims at filling 256 compute units; but a split must keep enough key tiles to
// amortise its fixed work (query load, first tile, the partial result it writes and the
// merge reads back).
#ifndef TALON_TUNING
constexpr int tuned_int(const char*, int dflt) { return dflt; }
#endif

int attention_waves(int rows) {
  const int forced = tuned_int("TALON_ATTN_WAVES", 0);   // tuning builds: 4 or 8
  if (forced == 4 || forced == 8) return forced;
  return rows >= 512 ? 8 : 4;
}

void attention_plan(int B, int N_pad, int Hq, int Hkv, int Dh, int max_prefix_len, int* splits,
                    int* tiles_per_split, int* rows_pad) {
  (void)Dh;
  const int min_tiles = tuned_int("TALON_ATTN_MIN_TILES", 4);   // key tiles a split must keep
  const int G = Hq / Hkv;
  const int rows = N_pad * G;
  const int waves = attention_waves(rows);
  const int mt = 32 * waves;
  const int row_tiles = (rows + mt - 1) / mt;
  const int tiles = (max_prefix_len + kKeyTile - 1) / kKeyTile + N_pad / kKeyTile;
  const long long base = static_cast<long long>(B) * Hkv * row_tiles;
  const long long slots = waves == 8 ? 256 : 512;
  long long want = (slots + base - 1) / base;
  const long long cap = tiles / min_tiles > 1 ? tiles / min_tiles : 1;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  const int tps = static_cast<int>((tiles + want - 1) / want);
  *tiles_per_split = tps;
  *splits = (tiles + tps - 1) / tps;
  *rows_pad = row_tiles * mt;
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t s) {
  const bool wide = attention_waves(a.N_pad * a.G) == 8;
  if (a.Dh == 128) return wide ? launch_one<128, 8>(a, s) : launch_one<128, 4>(a, s);
  return wide ? launch_one<64, 8>(a, s) : launch_one<64, 4>(a, s);
}

}  // namespace talon
