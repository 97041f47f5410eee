// Tree attention (App. B "Tree Attention"; mask of Fig. 5(b)): every tree node attends to
// the whole prefix KV cache plus the tree keys on its own root-to-node path.
//
// Dense contraction on bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulation, fp32 online
// softmax in base-2 units.
//
// Tiling.  The G = Hq/Hkv query heads that share a KV head are packed with the tree nodes
// into one row dimension (row = node * G + head-in-group), so one K/V tile read from HBM
// feeds G * n query rows.  A workgroup (4 wavefronts) owns 128*RB packed rows of one
// (sequence, KV head) and a contiguous range of 64-key tiles (split-KV); each wavefront
// owns RB blocks of 32 rows.  K and V tiles are staged through LDS (double buffered, one
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
#include "device_utils.h"
#include "talon_internal.h"

namespace talon {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef short short4v __attribute__((ext_vector_type(4)));

constexpr int kKeyTile = 64;
constexpr float kNegInfF = -__builtin_huge_valf();

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

template <int DH>
struct Smem {
  static constexpr int KSTR = DH + 8;    // 16 bytes of padding per key row (conflict-free 16-byte reads)
  static constexpr int VSTR = DH + 32;   // 64 bytes of padding per key row (conflict-free transpose reads)
  static constexpr int K_ELEMS = kKeyTile * KSTR;
  static constexpr int V_ELEMS = kKeyTile * VSTR;
  static constexpr int STAGE_ELEMS = K_ELEMS + V_ELEMS;
  static constexpr int BYTES = 2 * STAGE_ELEMS * 2;
};

template <int DH, int RB>
__global__ __launch_bounds__(kThreads) void tree_attention_kernel(AttnArgs a) {
  using SM = Smem<DH>;
  constexpr int DSTEPS = DH / 16;   // MFMA steps over the head dimension for S^T
  constexpr int DB = DH / 32;       // 32-row blocks of O^T
  constexpr int CPR = DH / 8;       // 16-byte pieces per key row
  constexpr int NLD = kKeyTile * CPR / kThreads;  // pieces per thread per tile and tensor
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int h = lane >> 5;

  const int split = blockIdx.x;
  const int bg = blockIdx.z;
  const int b = bg / a.Hkv;
  const int g = bg - b * a.Hkv;
  const int G = a.G;
  const int n = a.n_nodes[b];
  int L = a.prefix_len[b];
  L = L < 0 ? 0 : (L > a.max_prefix_len ? a.max_prefix_len : L);
  const int rows = n * G;
  const int row0 = blockIdx.y * (128 * RB);
  if (row0 >= rows) return;

  const int nPT = (L + kKeyTile - 1) / kKeyTile;
  const int nTT = (n + kKeyTile - 1) / kKeyTile;
  const int T = nPT + nTT;
  const int t_begin = split * a.tiles_per_split;
  const int t_end = (t_begin + a.tiles_per_split < T) ? t_begin + a.tiles_per_split : T;
  const int words = a.N_pad / 64;

  // ---- this lane's queries (one per row block) and their Q^T operands
  const int wrow0 = row0 + wave * 32 * RB;
  bf16x8 bq[RB][DSTEPS];
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
    const uint16_t* qp = a.q + orow_rb[rb] * DH + 8 * h;
#pragma unroll
    for (int ds = 0; ds < DSTEPS; ++ds) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (valid) v = *reinterpret_cast<const uint4*>(qp + 16 * ds);
      bq[rb][ds] = as_bf16x8(v);
    }
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

  uint4 kreg[NLD], vreg[NLD];
  auto load_tile = [&](int t) {
    const bool is_prefix = t < nPT;
    const int key0 = (is_prefix ? t : t - nPT) * kKeyTile;
    const int limit = is_prefix ? L : n;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int p = i * kThreads + tid;
      const int key = key0 + p / CPR;
      const int c = p % CPR;
      uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
      if (key < limit) {
        const size_t off = is_prefix ? static_cast<size_t>(key) * a.kv_stride_t : static_cast<size_t>(key) * tree_stride;
        const uint16_t* ks = (is_prefix ? kp_base : kt_base) + off + c * 8;
        const uint16_t* vs = (is_prefix ? vp_base : vt_base) + off + c * 8;
        kv = *reinterpret_cast<const uint4*>(ks);
        vv = *reinterpret_cast<const uint4*>(vs);
      }
      kreg[i] = kv;
      vreg[i] = vv;
    }
  };
  auto store_tile = [&](int buf) {
    uint16_t* sK = smem + buf * SM::STAGE_ELEMS;
    uint16_t* sV = sK + SM::K_ELEMS;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int p = i * kThreads + tid;
      const int key = p / CPR;
      const int c = p % CPR;
      *reinterpret_cast<uint4*>(sK + key * SM::KSTR + c * 8) = kreg[i];
      *reinterpret_cast<uint4*>(sV + key * SM::VSTR + c * 8) = vreg[i];
    }
  };

  const float c2 = a.scale_log2e;

  if (t_begin < t_end) {
    load_tile(t_begin);
    store_tile(0);
  }
  __syncthreads();

  int buf = 0;
  for (int t = t_begin; t < t_end; ++t) {
    const bool have_next = t + 1 < t_end;
    if (have_next) load_tile(t + 1);

    const uint16_t* sK = smem + buf * SM::STAGE_ELEMS;
    const uint16_t* sV = sK + SM::K_ELEMS;

    // ---- S^T = K . Q^T for the 64 keys of the tile
    floatx16 s[2][RB];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][rb][r] = 0.f;
      const uint16_t* krow = sK + (32 * kb + l32) * SM::KSTR + 8 * h;
#pragma unroll
      for (int ds = 0; ds < DSTEPS; ++ds) {
        const bf16x8 ak = as_bf16x8(*reinterpret_cast<const uint4*>(krow + 16 * ds));
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          s[kb][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, bq[rb][ds], s[kb][rb], 0, 0, 0);
      }
    }

    // ---- mask: ancestor bits on tree tiles, length bound on the ragged prefix tile
    const bool is_prefix = t < nPT;
    const int key0 = (is_prefix ? t : t - nPT) * kKeyTile;
    const bool full = is_prefix && key0 + kKeyTile <= L;
    if (!full) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        unsigned long long allow;
        if (is_prefix) allow = (1ull << (L - key0)) - 1ull;
        else allow = valid_rb[rb] ? a.mask[(static_cast<size_t>(b) * a.N_pad + node_rb[rb]) * words + (t - nPT)] : 0ull;
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
    }

    // ---- online softmax (base 2), per query = per lane pair (lane, lane ^ 32)
    bf16x8 pb[2][2][RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float mx = kNegInfF;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][rb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run[rb], mx * c2);
      const float m_safe = m_new == kNegInfF ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[rb] - m_safe);
      m_run[rb] = m_new;
      float sum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
          bf16x8 pk;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][rb][8 * sp + e], c2, -m_safe));
            sum += p;
            pk[e] = static_cast<__bf16>(p);
          }
          pb[kb][sp][rb] = pk;
        }
      }
      l_run[rb] = l_run[rb] * alpha + sum;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][rb][r] *= alpha;
    }

    // ---- O^T += V^T . P^T
    {
      const int i16 = lane & 15;
      const int dhblk = (lane >> 4) & 1;
      const uint16_t* vbase = sV + (4 * h + (i16 >> 2)) * SM::VSTR + 16 * dhblk + 4 * (i16 & 3);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const uint16_t* vp = vbase + (32 * kb + 16 * sp) * SM::VSTR + 32 * db;
            const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) short4v*)(vp));
            const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) short4v*)(vp + 8 * SM::VSTR));
            typedef short short8v __attribute__((ext_vector_type(8)));
            const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            const bf16x8 av = __builtin_bit_cast(bf16x8, both);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
              o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pb[kb][sp][rb], o[db][rb], 0, 0, 0);
          }
        }
      }
    }

    if (have_next) store_tile(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // ---- epilogue
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const float l_tot = l_run[rb] + __shfl_xor(l_run[rb], 32);
    if (!valid_rb[rb]) continue;
    if (a.splits == 1) {
      const float inv = 1.f / l_tot;
      uint16_t* op = a.out + orow_rb[rb] * DH;
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
      if (a.out_lse && h == 0) a.out_lse[orow_rb[rb]] = (m_run[rb] + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    } else {
      const int rho = wrow0 + 32 * rb + l32;
      const size_t prow = (static_cast<size_t>(bg) * a.splits + split) * a.rows_pad + rho;
      float* po = a.part_o + prow * DH;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          float4 v = make_float4(o[db][rb][4 * q4], o[db][rb][4 * q4 + 1], o[db][rb][4 * q4 + 2], o[db][rb][4 * q4 + 3]);
          *reinterpret_cast<float4*>(po + 32 * db + 8 * q4 + 4 * h) = v;
        }
      }
      if (h == 0) {
        a.part_m[prow] = m_run[rb];
        a.part_l[prow] = l_tot;
      }
    }
  }
}

// Merge of the split-KV partial results: out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// One thread per (packed row, 4 head-dim values).
template <int DH>
__global__ __launch_bounds__(kThreads) void tree_attention_combine_kernel(AttnArgs a) {
  constexpr int QPR = DH / 4;
  const int bg = blockIdx.y;
  const int b = bg / a.Hkv;
  const int g = bg - b * a.Hkv;
  const int rows = a.n_nodes[b] * a.G;
  const int idx = blockIdx.x * kThreads + threadIdx.x;
  const int rho = idx / QPR;
  const int c = idx - rho * QPR;
  if (rho >= rows) return;
  int L = a.prefix_len[b];
  L = L < 0 ? 0 : (L > a.max_prefix_len ? a.max_prefix_len : L);
  const int T = (L + kKeyTile - 1) / kKeyTile + (a.n_nodes[b] + kKeyTile - 1) / kKeyTile;
  int ns = (T + a.tiles_per_split - 1) / a.tiles_per_split;  // splits that held at least one tile
  ns = ns < a.splits ? ns : a.splits;
  const size_t base = static_cast<size_t>(bg) * a.splits * a.rows_pad + rho;
  float M = kNegInfF;
  for (int s = 0; s < ns; ++s) M = fmaxf(M, a.part_m[base + static_cast<size_t>(s) * a.rows_pad]);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float den = 0.f;
  for (int s = 0; s < ns; ++s) {
    const size_t pr = base + static_cast<size_t>(s) * a.rows_pad;
    const float ms = a.part_m[pr];
    if (ms == kNegInfF) continue;
    const float w = __builtin_amdgcn_exp2f(ms - M);
    den += w * a.part_l[pr];
    const float4 v = *reinterpret_cast<const float4*>(a.part_o + pr * DH + 4 * c);
    acc.x += w * v.x; acc.y += w * v.y; acc.z += w * v.z; acc.w += w * v.w;
  }
  const float inv = 1.f / den;
  const int node = rho / a.G;
  const int j = rho - node * a.G;
  const size_t orow = (static_cast<size_t>(b) * a.N_pad + node) * a.Hq + g * a.G + j;
  bf16x4 v;
  v[0] = static_cast<__bf16>(acc.x * inv);
  v[1] = static_cast<__bf16>(acc.y * inv);
  v[2] = static_cast<__bf16>(acc.z * inv);
  v[3] = static_cast<__bf16>(acc.w * inv);
  *reinterpret_cast<bf16x4*>(a.out + orow * DH + 4 * c) = v;
  if (a.out_lse && c == 0) a.out_lse[orow] = (M + __builtin_amdgcn_logf(den)) * 0.6931471805599453f;
}

template <int DH, int RB>
hipError_t launch_one(const AttnArgs& a, hipStream_t s) {
  const int row_tiles = (a.N_pad * a.G + 128 * RB - 1) / (128 * RB);
  auto kern = tree_attention_kernel<DH, RB>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       Smem<DH>::BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(a.splits, row_tiles, a.B * a.Hkv), dim3(kThreads), Smem<DH>::BYTES, s, a);
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

// Launch plan: rows per workgroup (128 or 256) and the number of KV splits, chosen so that
// the grid holds at least two workgroups per compute unit when the problem allows it.
void attention_plan(int B, int N_pad, int Hq, int Hkv, int Dh, int max_prefix_len, int* splits,
                    int* tiles_per_split, int* rows_pad) {
  (void)Dh;
  const int G = Hq / Hkv;
  const int rows = N_pad * G;
  const int rb = 1;
  const int mt = 128 * rb;
  const int row_tiles = (rows + mt - 1) / mt;
  const int tiles = (max_prefix_len + kKeyTile - 1) / kKeyTile + N_pad / kKeyTile;
  const long long base = static_cast<long long>(B) * Hkv * row_tiles;
  long long want = (512 + base - 1) / base;
  if (want < 1) want = 1;
  if (want > tiles) want = tiles;
  const int tps = static_cast<int>((tiles + want - 1) / want);
  *tiles_per_split = tps;
  *splits = (tiles + tps - 1) / tps;
  *rows_pad = row_tiles * mt;
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t s) {
  if (a.Dh == 128) return launch_one<128, 1>(a, s);
  return launch_one<64, 1>(a, s);
}

}  // namespace talon
