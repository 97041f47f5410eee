// C ABI of libtalon: argument validation and kernel launches.  Everything that can be
// checked on the host is checked before the first launch, so a failed call enqueues nothing.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "talon_internal.h"
#ifdef TALON_TUNING
#include "tuning.h"
#endif

#include <atomic>
#include <mutex>
#include <vector>

namespace talon {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return TALON_OK;
  set_error("%s: %s", what, hipGetErrorString(e));
  return TALON_ERR_RUNTIME;
}

namespace {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int check_state(const talon_tree_state* st) {
  if (!st) { set_error("tree state is NULL"); return TALON_ERR_INVALID_ARG; }
  if (st->B < 1 || st->B > TALON_B_MAX) { set_error("B=%d outside [1, %d]", st->B, TALON_B_MAX); return TALON_ERR_INVALID_ARG; }
  if (st->N < 1 || st->N > TALON_N_MAX) { set_error("N=%d outside [1, %d]", st->N, TALON_N_MAX); return TALON_ERR_INVALID_ARG; }
  if (st->N_pad < st->N || st->N_pad % 64 != 0 || st->N_pad > TALON_N_MAX) {
    set_error("N_pad=%d must be a multiple of 64 with N <= N_pad <= %d", st->N_pad, TALON_N_MAX);
    return TALON_ERR_INVALID_ARG;
  }
  const void* ptrs[] = {st->token, st->parent, st->depth, st->prob, st->logp, st->n_nodes,
                        st->frontier_begin, st->frontier_count, st->depth_cur, st->status};
  for (const void* p : ptrs) {
    if (!p) { set_error("tree state holds a NULL pointer"); return TALON_ERR_INVALID_ARG; }
    if (reinterpret_cast<uintptr_t>(p) & 7u) { set_error("tree state pointer is not 8-byte aligned"); return TALON_ERR_INVALID_ARG; }
  }
  return TALON_OK;
}

struct ExpandLayout {
  size_t off_max, off_sum, off_keys, off_ticket, off_seq_ticket, off_desc, off_exit, total;
  int chunks;
};

int expand_layout(int B, int N_pad, int vocab, int k, int dtype, ExpandLayout* L) {
  if (dtype != TALON_DTYPE_F32 && dtype != TALON_DTYPE_BF16) { set_error("dtype %d not supported", dtype); return TALON_ERR_UNSUPPORTED; }
  if (B < 1 || B > TALON_B_MAX || N_pad < 64 || N_pad > TALON_N_MAX || N_pad % 64) { set_error("bad B=%d or N_pad=%d", B, N_pad); return TALON_ERR_INVALID_ARG; }
  if (vocab < 1) { set_error("vocab=%d must be >= 1", vocab); return TALON_ERR_INVALID_ARG; }
  if (k < 1 || k > TALON_K_MAX) { set_error("k=%d outside [1, %d]", k, TALON_K_MAX); return TALON_ERR_INVALID_ARG; }
  const int ce = expand_chunk_elems(dtype);
  const long long chunks = (static_cast<long long>(vocab) + ce - 1) / ce;
  if (chunks * k > kMergeCap) {
    set_error("vocab=%d with k=%d needs %lld chunk partials per row; at most %d are supported", vocab, k, chunks * k, kMergeCap);
    return TALON_ERR_UNSUPPORTED;
  }
  const size_t rows = static_cast<size_t>(B) * N_pad;
  L->chunks = static_cast<int>(chunks);
  L->off_ticket = 0;
  L->off_seq_ticket = align_up(rows * sizeof(int32_t), 256);
  L->off_desc = L->off_seq_ticket + align_up(static_cast<size_t>(B) * sizeof(int32_t), 256);
  L->off_exit = L->off_desc + align_up(static_cast<size_t>(N_pad) * B * sizeof(uint64_t), 256);
  L->off_max = L->off_exit + align_up(static_cast<size_t>(kExitWords + 1) * sizeof(uint32_t), 256);   // + the cap_hit word
  L->off_sum = L->off_max + align_up(rows * chunks * sizeof(float), 256);
  L->off_keys = L->off_sum + align_up(rows * chunks * sizeof(double), 256);
  L->total = L->off_keys + align_up(rows * chunks * k * sizeof(uint64_t), 256);
  return TALON_OK;
}

int check_expand_args(const void* logits, int dtype, int64_t row_stride, int64_t seq_stride, int row_mode,
                      const talon_tree_state* st, int32_t vocab, int32_t k, const void* cand_token,
                      const void* cand_logit, const void* cand_prob, const void* cand_edge_logp,
                      const void* row_max, const void* row_lse, void* workspace, size_t workspace_bytes,
                      ExpandLayout* L) {
  int rc = check_state(st);
  if (rc) return rc;
  rc = expand_layout(st->B, st->N_pad, vocab, k, dtype, L);
  if (rc) return rc;
  const void* ptrs[] = {logits, cand_token, cand_logit, cand_prob, cand_edge_logp, row_max, row_lse, workspace};
  for (const void* p : ptrs) {
    if (!p) { set_error("NULL pointer argument"); return TALON_ERR_INVALID_ARG; }
    if (!aligned16(p)) { set_error("pointer argument is not 16-byte aligned"); return TALON_ERR_INVALID_ARG; }
  }
  const int epv = dtype == TALON_DTYPE_F32 ? 4 : 8;
  if (row_stride < vocab || row_stride % epv) { set_error("row_stride=%lld must be >= vocab and a multiple of %d elements", (long long)row_stride, epv); return TALON_ERR_INVALID_ARG; }
  if (seq_stride < 0 || seq_stride % epv || (st->B > 1 && seq_stride < row_stride)) { set_error("seq_stride=%lld invalid", (long long)seq_stride); return TALON_ERR_INVALID_ARG; }
  if (row_mode != TALON_ROWS_BY_NODE && row_mode != TALON_ROWS_BY_FRONTIER) { set_error("row_mode=%d unknown", row_mode); return TALON_ERR_INVALID_ARG; }
  if (workspace_bytes < L->total) { set_error("workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, L->total); return TALON_ERR_WORKSPACE; }
  return TALON_OK;
}

int check_select_args(const talon_tree_state* st, int32_t k, const void* cand_token, const void* cand_prob,
                      const void* cand_edge_logp, float mu, int32_t K_init, int32_t init_layers, int32_t max_depth) {
  int rc = check_state(st);
  if (rc) return rc;
  if (k < 1 || k > TALON_K_MAX) { set_error("k=%d outside [1, %d]", k, TALON_K_MAX); return TALON_ERR_INVALID_ARG; }
  if (!(mu > 0.f && mu <= 1.f)) { set_error("mu=%g outside (0, 1]", (double)mu); return TALON_ERR_INVALID_ARG; }
  if (K_init < 1) { set_error("K_init=%d must be >= 1", K_init); return TALON_ERR_INVALID_ARG; }
  if (init_layers < 0) { set_error("init_layers=%d must be >= 0", init_layers); return TALON_ERR_INVALID_ARG; }
  if (max_depth < 1) { set_error("max_depth=%d must be >= 1", max_depth); return TALON_ERR_INVALID_ARG; }
  if (!cand_token || !cand_prob || !cand_edge_logp) { set_error("NULL candidate pointer"); return TALON_ERR_INVALID_ARG; }
  if (static_cast<long long>(st->N - 1) * k > 4096) {
    set_error("(N-1)*k = %lld candidates per layer; the selection holds at most 4096", static_cast<long long>(st->N - 1) * k);
    return TALON_ERR_UNSUPPORTED;
  }
  return TALON_OK;
}

// Launch heuristics.  Tuning builds (-DTALON_TUNING) can override them from the environment;
// the default build compiles the constants in.
#ifndef TALON_TUNING
constexpr int tuned_int(const char*, int dflt) { return dflt; }
#endif
// (row, chunk) items a scan launch aims for when it cuts rows into chunks (from a sweep over c2, c3, c5)
int expand_target_items() { return tuned_int("TALON_EXPAND_TARGET_ITEMS", 512); }

ExpandArgs make_expand_args(const void* logits, int64_t row_stride, int64_t seq_stride, int row_mode,
                            const talon_tree_state* st, int32_t vocab, int32_t k, int32_t* cand_token,
                            float* cand_logit, float* cand_prob, double* cand_edge_logp, float* row_max,
                            double* row_lse, void* workspace, const ExpandLayout& L) {
  ExpandArgs a;
  a.logits = logits; a.row_stride = row_stride; a.seq_stride = seq_stride; a.row_mode = row_mode;
  a.B = st->B; a.N_pad = st->N_pad; a.vocab = vocab; a.k = k; a.chunks = L.chunks;
  a.target_items = expand_target_items();
  a.frontier_begin = st->frontier_begin; a.frontier_count = st->frontier_count; a.status = st->status;
  a.cand_token = cand_token; a.cand_logit = cand_logit; a.cand_prob = cand_prob;
  a.cand_edge_logp = cand_edge_logp; a.row_max = row_max; a.row_lse = row_lse;
  char* w = static_cast<char*>(workspace);
  a.ticket = reinterpret_cast<int32_t*>(w + L.off_ticket);
  a.seq_ticket = reinterpret_cast<int32_t*>(w + L.off_seq_ticket);
  a.desc = reinterpret_cast<unsigned long long*>(w + L.off_desc);
  a.exit_ticket = reinterpret_cast<uint32_t*>(w + L.off_exit);
  a.layers = 0;
  a.root_token = nullptr;
  a.launch_idx = 0;
  a.layers = 0;
  a.spin_ticks = 0;
  a.tree_mask = nullptr;
  a.run_if = nullptr;
  memset(&a.sel, 0, sizeof(a.sel));
  a.part_max = reinterpret_cast<float*>(w + L.off_max);
  a.part_sum = reinterpret_cast<double*>(w + L.off_sum);
  a.part_keys = reinterpret_cast<unsigned long long*>(w + L.off_keys);
  return a;
}

// Workgroups for the scan of layer `layer` (-1: unknown): one per (row, chunk) item of the
// widest frontier that layer can have, capped at the number of workgroups resident at once.  Layer 0 has the root only; every later frontier is bounded by k children
// per parent, by K_init on top-K layers and by the budget left after one node per earlier layer.
int expand_grid(const talon_tree_state* st, int chunks, int layer, int k, int K_init, int init_layers) {
  long long f = st->N > 1 ? st->N - 1 : 1;
  if (layer >= 0) {
    long long w = 1;
    for (int d = 1; d <= layer; ++d) {
      w *= k;
      if (d - 1 < init_layers && w > K_init) w = K_init;
      const long long left = st->N - d;
      if (w > left) w = left;
      if (w < 1) w = 1;
    }
    f = w;
  }
  long long items = static_cast<long long>(st->B) * f * chunks;
  if (items > 1024) items = 1024;   // 4 resident workgroups per compute unit; more only costs dispatch time
  if (items < 1) items = 1;
  return static_cast<int>(items);
}

// Workspace of talon_target_argmax: the scan's workspace for k = 1, then the stand-in frontier
// {begin, count, status}[B] and the scan outputs nobody asked for.
struct VerifyLayout {
  ExpandLayout scan;
  size_t off_begin, off_count, off_status, off_logit, off_prob, off_edge, off_max, off_lse, total;
};

int verify_layout(int B, int N_pad, int vocab, int dtype, VerifyLayout* V) {
  int rc = expand_layout(B, N_pad, vocab, 1, dtype, &V->scan);
  if (rc) return rc;
  const size_t rows = static_cast<size_t>(B) * N_pad;
  size_t o = V->scan.total;
  V->off_begin = o;  o += align_up(B * sizeof(int32_t), 256);
  V->off_count = o;  o += align_up(B * sizeof(int32_t), 256);
  V->off_status = o; o += align_up(B * sizeof(uint32_t), 256);
  V->off_logit = o;  o += align_up(rows * sizeof(float), 256);
  V->off_prob = o;   o += align_up(rows * sizeof(float), 256);
  V->off_edge = o;   o += align_up(rows * sizeof(double), 256);
  V->off_max = o;    o += align_up(rows * sizeof(float), 256);
  V->off_lse = o;    o += align_up(rows * sizeof(double), 256);
  V->total = o;
  return TALON_OK;
}

// Workspace of talon_expand_literal: the scan's workspace and its outputs (laid out for the
// most candidates per row the call ever asks the scan for) and the survivors of every
// frontier row.
constexpr int kLiteralScanK = 16;
struct LiteralLayout {
  ExpandLayout scan;
  int k_max;   // candidates per row the layout has room for: kLiteralScanK, or 1 for very wide rows
  size_t off_token, off_logit, off_prob, off_edge, off_max, off_lse, off_count, off_keys, off_part_count, off_part_keys, part_keys_per_seq, total;
  // Trees of at most 64 nodes: a row can never get more than N - 1 <= 63 children, so a per-row
  // cap of N - 1 is no cap at all and the capped single-launch loop builds the uncapped tree.
  // Its workspace and candidate arrays (for k = 63) lie over the same bytes as the layout above.
  bool capped_loop_fits;
  size_t c_workspace, c_token, c_logit, c_prob, c_edge, c_max, c_lse, c_saved;
};
constexpr int kCappedLoopK = 63;
// The loop is first tried with this per-row cap, which is far cheaper to rank than N - 1: the tree
// is the uncapped one unless a selection kept the last candidate of a row (SelectArgs::cap_hit).
constexpr int kCappedLoopTryK = 32;

int literal_layout(int B, int N_pad, int vocab, int dtype, LiteralLayout* V) {
  int rc = expand_layout(B, N_pad, vocab, 1, dtype, &V->scan);
  if (rc) return rc;
  V->k_max = 1;
  const int ce = expand_chunk_elems(dtype);
  if ((static_cast<long long>(vocab) + ce - 1) / ce * kLiteralScanK <= kMergeCap) {
    V->k_max = kLiteralScanK;
    if ((rc = expand_layout(B, N_pad, vocab, kLiteralScanK, dtype, &V->scan))) return rc;
  }
  const size_t rows = static_cast<size_t>(B) * N_pad;
  const size_t cands = rows * V->k_max;
  size_t o = V->scan.total;
  V->off_token = o; o += align_up(cands * sizeof(int32_t), 256);
  V->off_logit = o; o += align_up(cands * sizeof(float), 256);
  V->off_prob = o;  o += align_up(cands * sizeof(float), 256);
  V->off_edge = o;  o += align_up(cands * sizeof(double), 256);
  V->off_max = o;   o += align_up(rows * sizeof(float), 256);
  V->off_lse = o;   o += align_up(rows * sizeof(double), 256);
  V->off_count = o; o += align_up(rows * sizeof(int32_t), 256);
  V->off_keys = o;  o += align_up(rows * kLiteralRowCap * sizeof(uint64_t), 256);
  V->off_part_count = o; o += align_up(rows * kLiteralChunks * sizeof(int32_t), 256);
  // parts of rows: a layer's rows times the nodes it may take never exceed (N / 2)^2
  V->part_keys_per_seq = static_cast<size_t>(kLiteralChunks) * (N_pad / 2) * (N_pad / 2);
  V->off_part_keys = o;  o += align_up(static_cast<size_t>(B) * V->part_keys_per_seq * sizeof(uint64_t), 256);
  V->total = o;
  V->capped_loop_fits = false;
  ExpandLayout C;
  if (N_pad == 64 && expand_layout(B, N_pad, vocab, kCappedLoopK, dtype, &C) == TALON_OK) {
    V->capped_loop_fits = true;
    const size_t cc = rows * kCappedLoopK;
    size_t c = C.total;
    V->c_workspace = C.total;
    V->c_token = c; c += align_up(cc * sizeof(int32_t), 256);
    V->c_logit = c; c += align_up(cc * sizeof(float), 256);
    V->c_prob = c;  c += align_up(cc * sizeof(float), 256);
    V->c_edge = c;  c += align_up(cc * sizeof(double), 256);
    V->c_max = c;   c += align_up(rows * sizeof(float), 256);
    V->c_lse = c;   c += align_up(rows * sizeof(double), 256);
    V->c_saved = c; c += align_up(static_cast<size_t>(5) * B * sizeof(int32_t), 256);
    V->total = c > V->total ? c : V->total;
  }
  return TALON_OK;
}

}  // namespace
}  // namespace talon

using namespace talon;

// ---- scratch of the entry point that takes no workspace (talon_tree_attention_static).
// One array per GPU, part of the library's code object: it exists from the moment the library
// is loaded on a device until the process ends.  In host code the array's name is only a
// handle: its device address is looked up once per device and that address is what kernels get.
constexpr size_t kStaticScratchBytes = static_cast<size_t>(32) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (looked up on the first call per device).
int static_scratch_address(void** out) {
  int dev = -1;
  int rc = check_hip(hipGetDevice(&dev), "hipGetDevice");
  if (rc) return rc;
  if (dev < 0 || dev >= kMaxDevices) { set_error("device index %d outside [0, %d)", dev, kMaxDevices); return TALON_ERR_UNSUPPORTED; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    rc = check_hip(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
    if (rc) return rc;
    if (!p) { set_error("hipGetSymbolAddress returned a null address"); return TALON_ERR_RUNTIME; }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return TALON_OK;
}
}  // namespace

extern "C" {

const char* talon_last_error_string(void) { return g_err; }

int talon_tree_init(const talon_tree_state* st, const int32_t* root_token, void* stream) {
  int rc = check_state(st);
  if (rc) return rc;
  if (!root_token) { set_error("root_token is NULL"); return TALON_ERR_INVALID_ARG; }
  return check_hip(launch_tree_init(*st, root_token, static_cast<hipStream_t>(stream)), "tree_init launch");
}

size_t talon_expand_workspace_bytes(int32_t B, int32_t N_pad, int32_t vocab, int32_t k, int dtype) {
  ExpandLayout L;
  if (expand_layout(B, N_pad, vocab, k, dtype, &L)) return 0;
  return L.total;
}

int talon_expand_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace || !aligned16(workspace)) { set_error("workspace is NULL or not 16-byte aligned"); return TALON_ERR_INVALID_ARG; }
  if (workspace_bytes % 4) { set_error("workspace_bytes must be a multiple of 4"); return TALON_ERR_INVALID_ARG; }
  return check_hip(launch_fill_zero(workspace, workspace_bytes, static_cast<hipStream_t>(stream)), "workspace fill launch");
}

int talon_expand_layer(const void* logits, int dtype, int64_t row_stride, int64_t seq_stride, int row_mode,
                       int32_t layer, const talon_tree_state* st, int32_t vocab, int32_t k, int32_t* cand_token,
                       float* cand_logit, float* cand_prob, double* cand_edge_logp, float* row_max,
                       double* row_lse, void* workspace, size_t workspace_bytes, void* stream) {
  ExpandLayout L;
  int rc = check_expand_args(logits, dtype, row_stride, seq_stride, row_mode, st, vocab, k, cand_token, cand_logit,
                             cand_prob, cand_edge_logp, row_max, row_lse, workspace, workspace_bytes, &L);
  if (rc) return rc;
  const ExpandArgs a = make_expand_args(logits, row_stride, seq_stride, row_mode, st, vocab, k, cand_token,
                                        cand_logit, cand_prob, cand_edge_logp, row_max, row_lse, workspace, L);
  return check_hip(launch_expand(a, dtype, expand_grid(st, L.chunks, layer < 0 ? -1 : layer, k, k, 0), false, static_cast<hipStream_t>(stream)), "expand launch");
}

int talon_select_budget(const talon_tree_state* st, int32_t k, const int32_t* cand_token, const float* cand_prob,
                        const double* cand_edge_logp, float mu, int32_t K_init, int32_t init_layers,
                        int32_t max_depth, void* stream) {
  int rc = check_select_args(st, k, cand_token, cand_prob, cand_edge_logp, mu, K_init, init_layers, max_depth);
  if (rc) return rc;
  SelectArgs a;
  a.st = *st; a.k = k; a.cand_token = cand_token; a.cand_prob = cand_prob; a.cand_edge_logp = cand_edge_logp;
  a.log_mu = log(static_cast<double>(mu)); a.K_init = K_init; a.init_layers = init_layers; a.max_depth = max_depth;
  a.cap_hit = nullptr;
  return check_hip(launch_select(a, static_cast<hipStream_t>(stream)), "select launch");
}

namespace {

// Measurement hook state: pairs of events recorded around each fused scan launch.
struct ScanProfile {
  bool enabled = false;
  std::vector<hipEvent_t> events;   // pool, two per launch
  size_t used = 0;
};
ScanProfile g_profile;

hipError_t profile_record(hipStream_t s) {
  if (g_profile.used == g_profile.events.size()) {
    hipEvent_t e;
    hipError_t err = hipEventCreate(&e);
    if (err != hipSuccess) return err;
    g_profile.events.push_back(e);
  }
  return hipEventRecord(g_profile.events[g_profile.used++], s);
}

// Fused launches of `layers` consecutive layers starting from the public tree state.
// Resident workgroups of the single-launch kernel, per element type, queried once.
int tree_grid_limit(int dtype) {
  static std::atomic<int> cached[2] = {{-1}, {-1}};
  std::atomic<int>& c = cached[dtype == TALON_DTYPE_F32 ? 0 : 1];
  int v = c.load(std::memory_order_relaxed);
  if (v < 0) {
    v = expand_tree_max_grid(dtype);
    c.store(v, std::memory_order_relaxed);
  }
  return v;
}

// Bound of the wait between two layers of the single-launch kernel, in ticks of the 100 MHz
// wall clock (default 0.2 s; talon_set_spin_limit_us changes it).
std::atomic<long long> g_spin_limit_us{200000};
unsigned long long spin_limit_ticks() {
  const long long us = g_spin_limit_us.load(std::memory_order_relaxed);
  return static_cast<unsigned long long>(us < 0 ? 0 : us) * 100ull;
}

// A single launch that is one of a pair (talon_expand_literal): the first runs with a small
// per-row cap, saves the per-sequence state it starts from and raises a flag if the cap may have
// mattered; the second runs with the full cap from the saved state, and only if the flag is up.
struct Speculation {
  uint32_t* cap_hit;        // first launch: raised by its selections
  const uint32_t* run_if;   // second launch: the same word
  int32_t* saved;           // [5][B]
};

int run_fused_layers(bool single_launch, const int32_t* root_token, uint64_t* mask, const void* logits, int dtype, int64_t row_stride, int64_t seq_stride, int row_mode,
                     int first_layer, int layers, const talon_tree_state* st, int32_t vocab, int32_t k, float mu,
                     int32_t K_init, int32_t init_layers, int32_t max_depth, int32_t* cand_token, float* cand_logit,
                     float* cand_prob, double* cand_edge_logp, float* row_max, double* row_lse, void* workspace,
                     size_t workspace_bytes, void* stream, const Speculation* spec = nullptr) {
  ExpandLayout L;
  int rc = check_expand_args(logits, dtype, row_stride, seq_stride, row_mode, st, vocab, k, cand_token, cand_logit,
                             cand_prob, cand_edge_logp, row_max, row_lse, workspace, workspace_bytes, &L);
  if (rc) return rc;
  rc = check_select_args(st, k, cand_token, cand_prob, cand_edge_logp, mu, K_init, init_layers, max_depth);
  if (rc) return rc;
  ExpandArgs ea = make_expand_args(logits, row_stride, seq_stride, row_mode, st, vocab, k, cand_token,
                                   cand_logit, cand_prob, cand_edge_logp, row_max, row_lse, workspace, L);
  SelectArgs sa;
  sa.st = *st; sa.k = k; sa.cand_token = cand_token; sa.cand_prob = cand_prob; sa.cand_edge_logp = cand_edge_logp;
  sa.log_mu = log(static_cast<double>(mu)); sa.K_init = K_init; sa.init_layers = init_layers; sa.max_depth = max_depth;
  sa.cap_hit = spec ? spec->cap_hit : nullptr;
  ea.sel = sa;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (layers <= 0) {   // N = 1: the tree is its root
    if (root_token && (rc = check_hip(launch_tree_init(*st, root_token, s), "tree_init launch"))) return rc;
    if (mask) return check_hip(launch_mask(*st, mask, s), "mask launch");
    return TALON_OK;
  }
  ea.spin_ticks = spin_limit_ticks();
  if (!single_launch) {
    ea.spin_ticks = 200000000ull;   // two seconds of the 100 MHz clock: this wait always ends (see below), the bound is a safety net
    // One layer, one launch.  Its workgroups read the frontier from the public tree state and
    // its selections rewrite that state, so a selection waits until every workgroup of the
    // grid has read it (two counters in the workspace, back at zero when the launch ends).
    ea.launch_idx = 0;
    if (g_profile.enabled && (rc = check_hip(profile_record(s), "profile event"))) return rc;
    rc = check_hip(launch_expand(ea, dtype, expand_grid(st, L.chunks, first_layer, k, K_init, init_layers), true, s), "expand launch");
    if (rc) return rc;
    if (g_profile.enabled && (rc = check_hip(profile_record(s), "profile event"))) return rc;
    return TALON_OK;
  }
  // The single launch starts fresh trees itself and leaves its counters clean; when it continues
  // trees, its first frontier comes from a snapshot of the public tree state made by a small
  // launch of its own (layer i of the loop reads descriptor i).
  const bool starts_trees = root_token != nullptr;   // talon_build_tree only: first layer 0
  if (starts_trees) {
    ea.root_token = root_token;
  } else {
    FusedInitArgs fi;
    fi.mode = !spec ? kInitPlain : (spec->run_if ? kInitRestoreIf : kInitSave);
    fi.saved = spec ? spec->saved : nullptr;
    fi.flag = spec ? spec->run_if : nullptr;
    fi.clear = spec && !spec->run_if ? ea.exit_ticket : nullptr;
    if ((rc = check_hip(launch_fused_init(*st, ea, fi, s), "fused init launch"))) return rc;
  }
  ea.run_if = spec ? spec->run_if : nullptr;
  // One launch walks all layers.  Its grid is the widest layer's, capped by what the device
  // holds at once (the kernel's workgroups wait for each other between layers).
  int grid = 1;
  for (int d = 0; d < layers; ++d) {
    const int g = expand_grid(st, L.chunks, first_layer + d, k, K_init, init_layers);
    grid = g > grid ? g : grid;
  }
  const int resident = tree_grid_limit(dtype);
  if (resident < 1) { set_error("occupancy query for the single-launch kernel failed"); return TALON_ERR_RUNTIME; }
  grid = grid < resident ? grid : resident;
  if (grid > 0xFFFF) grid = 0xFFFF;   // the exit ticket counts workgroups in 16 bits
  ea.layers = layers;
  ea.tree_mask = mask;
  if (g_profile.enabled && (rc = check_hip(profile_record(s), "profile event"))) return rc;
  rc = check_hip(launch_expand_tree(ea, dtype, grid, s), "expand tree launch");
  if (rc) return rc;
  if (g_profile.enabled && (rc = check_hip(profile_record(s), "profile event"))) return rc;
  return TALON_OK;
}

}  // namespace

int talon_expand_select_layer(const void* logits, int dtype, int64_t row_stride, int64_t seq_stride, int row_mode,
                              int32_t layer, const talon_tree_state* st, int32_t vocab, int32_t k, float mu,
                              int32_t K_init, int32_t init_layers, int32_t max_depth, int32_t* cand_token,
                              float* cand_logit, float* cand_prob, double* cand_edge_logp, float* row_max,
                              double* row_lse, void* workspace, size_t workspace_bytes, void* stream) {
  return run_fused_layers(false, nullptr, nullptr, logits, dtype, row_stride, seq_stride, row_mode, layer, 1, st, vocab, k, mu, K_init,
                          init_layers, max_depth, cand_token, cand_logit, cand_prob, cand_edge_logp, row_max,
                          row_lse, workspace, workspace_bytes, stream);
}

int talon_expand_tree(const void* logits, int dtype, int64_t row_stride, int64_t seq_stride, int row_mode,
                      const talon_tree_state* st, int32_t vocab, int32_t k, float mu, int32_t K_init,
                      int32_t init_layers, int32_t max_depth, int32_t* cand_token, float* cand_logit,
                      float* cand_prob, double* cand_edge_logp, float* row_max, double* row_lse,
                      void* workspace, size_t workspace_bytes, void* stream) {
  // a tree of N nodes has at most N-1 layers: later iterations could not add anything.
  // One launch for the whole loop: the scan runs each sequence's budget selection in its tail
  // and the grid moves on to the next layer when every selection of a layer is done.
  int layers = 0;
  if (st && max_depth > 0) layers = max_depth < st->N - 1 ? max_depth : (st->N > 1 ? st->N - 1 : 0);
  return run_fused_layers(true, nullptr, nullptr, logits, dtype, row_stride, seq_stride, row_mode, 0, layers, st, vocab, k, mu, K_init,
                          init_layers, max_depth, cand_token, cand_logit, cand_prob, cand_edge_logp, row_max,
                          row_lse, workspace, workspace_bytes, stream);
}

int talon_build_tree(const int32_t* root_token, const void* logits, int dtype, int64_t row_stride, int64_t seq_stride,
                     int row_mode, const talon_tree_state* st, int32_t vocab, int32_t k, float mu, int32_t K_init,
                     int32_t init_layers, int32_t max_depth, int32_t* cand_token, float* cand_logit, float* cand_prob,
                     double* cand_edge_logp, float* row_max, double* row_lse, uint64_t* mask, void* workspace,
                     size_t workspace_bytes, void* stream) {
  if (!root_token) { set_error("root_token is NULL"); return TALON_ERR_INVALID_ARG; }
  if (mask && (reinterpret_cast<uintptr_t>(mask) & 7u)) { set_error("mask is not 8-byte aligned"); return TALON_ERR_INVALID_ARG; }
  int layers = 0;
  if (st && max_depth > 0) layers = max_depth < st->N - 1 ? max_depth : (st->N > 1 ? st->N - 1 : 0);
  return run_fused_layers(true, root_token, mask, logits, dtype, row_stride, seq_stride, row_mode, 0, layers, st, vocab,
                          k, mu, K_init, init_layers, max_depth, cand_token, cand_logit, cand_prob, cand_edge_logp,
                          row_max, row_lse, workspace, workspace_bytes, stream);
}

int talon_build_tree_checked(const int32_t* root_token, const void* logits, int dtype, int64_t row_stride,
                             int64_t seq_stride, int row_mode, const talon_tree_state* st, int32_t vocab, int32_t k,
                             float mu, int32_t K_init, int32_t init_layers, int32_t max_depth, int32_t* cand_token,
                             float* cand_logit, float* cand_prob, double* cand_edge_logp, float* row_max,
                             double* row_lse, uint64_t* mask, void* workspace, size_t workspace_bytes, void* stream,
                             int32_t* fell_back) {
  if (fell_back) *fell_back = 0;
  int rc = talon_build_tree(root_token, logits, dtype, row_stride, seq_stride, row_mode, st, vocab, k, mu, K_init,
                            init_layers, max_depth, cand_token, cand_logit, cand_prob, cand_edge_logp, row_max, row_lse,
                            mask, workspace, workspace_bytes, stream);
  if (rc) return rc;
  // the outcome of the single launch: did any workgroup give up its wait between two layers?
  hipStream_t s = static_cast<hipStream_t>(stream);
  std::vector<uint32_t> status(static_cast<size_t>(st->B));
  rc = check_hip(hipMemcpyAsync(status.data(), st->status, status.size() * sizeof(uint32_t), hipMemcpyDeviceToHost, s),
                 "status copy");
  if (rc) return rc;
  rc = check_hip(hipStreamSynchronize(s), "stream synchronize");
  if (rc) return rc;
  bool aborted = false;
  for (uint32_t v : status) aborted = aborted || (v & TALON_STATUS_ABORTED) != 0;
  if (!aborted) return TALON_OK;
  // The launch that gave up has put the workspace back in order (its last workgroup clears
  // every ticket and descriptor): build the same trees again, one launch per layer, which
  // needs no two workgroups to be resident together.
  if (fell_back) *fell_back = 1;
  rc = talon_tree_init(st, root_token, stream);
  if (rc) return rc;
  const int layers = max_depth < st->N - 1 ? max_depth : st->N - 1;
  for (int d = 0; d < layers; ++d) {
    rc = talon_expand_select_layer(logits, dtype, row_stride, seq_stride, row_mode, d, st, vocab, k, mu, K_init, init_layers,
                                   max_depth, cand_token, cand_logit, cand_prob, cand_edge_logp, row_max, row_lse,
                                   workspace, workspace_bytes, stream);
    if (rc) return rc;
  }
  if (mask) rc = talon_build_tree_mask(st, mask, stream);
  return rc;
}

size_t talon_literal_workspace_bytes(int32_t B, int32_t N_pad, int32_t vocab, int dtype) {
  LiteralLayout V;
  if (literal_layout(B, N_pad, vocab, dtype, &V)) return 0;
  return V.total;
}

int talon_expand_literal(const void* logits, int dtype, int64_t row_stride, int64_t seq_stride, int row_mode,
                         int32_t layers, const talon_tree_state* st, int32_t vocab, float mu, int32_t K_init,
                         int32_t init_layers, int32_t max_depth, void* workspace, size_t workspace_bytes,
                         void* stream) {
  int rc = check_state(st);
  if (rc) return rc;
  LiteralLayout V;
  rc = literal_layout(st->B, st->N_pad, vocab, dtype, &V);
  if (rc) return rc;
  char* w = static_cast<char*>(workspace);
  ExpandLayout L;
  // The scan ranks the 16 best tokens of every row where the workspace has room for them: on
  // top-K layers with K_init <= 16 they are the row's survivors, and on gated layers they settle
  // every row of which fewer than 16 tokens pass the gate; other rows are read a second time.
  const int k_scan = V.k_max;
  // the scan's own checks (pointers, alignment, strides), its outputs in the workspace
  rc = check_expand_args(logits, dtype, row_stride, seq_stride, row_mode, st, vocab, k_scan, w ? w + V.off_token : nullptr,
                         w ? w + V.off_logit : nullptr, w ? w + V.off_prob : nullptr, w ? w + V.off_edge : nullptr,
                         w ? w + V.off_max : nullptr, w ? w + V.off_lse : nullptr, workspace, workspace_bytes, &L);
  if (rc) return rc;
  if (workspace_bytes < V.total) {
    set_error("workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, V.total);
    return TALON_ERR_WORKSPACE;
  }
  if (!(mu > 0.f && mu <= 1.f)) { set_error("mu=%g outside (0, 1]", (double)mu); return TALON_ERR_INVALID_ARG; }
  if (K_init < 1) { set_error("K_init=%d must be >= 1", K_init); return TALON_ERR_INVALID_ARG; }
  if (init_layers < 0) { set_error("init_layers=%d must be >= 0", init_layers); return TALON_ERR_INVALID_ARG; }
  if (max_depth < 1) { set_error("max_depth=%d must be >= 1", max_depth); return TALON_ERR_INVALID_ARG; }
  if (layers < 1) { set_error("layers=%d must be >= 1", layers); return TALON_ERR_INVALID_ARG; }
  if (V.capped_loop_fits && st->N >= 2) {
    // At most 64 nodes: with a per-row cap of N - 1 (the whole row, if the vocabulary is smaller)
    // no row is ever cut short, so the capped loop in its single launch builds the same tree
    // (Alg. 2 with the pool as printed; a row's children enter in rank order, so a child
    // beyond rank N - 1 could only be chosen after N - 1 siblings, which the budget forbids).
    // The same argument bounds K_init.
    const int k = st->N - 1 < vocab ? st->N - 1 : vocab;
    const int most_layers = layers < st->N - 1 ? layers : st->N - 1;
    ExpandLayout C;
    rc = expand_layout(st->B, st->N_pad, vocab, k, dtype, &C);
    if (rc) return rc;
    auto run = [&](int kk, const Speculation* spec) {
      return run_fused_layers(true, nullptr, nullptr, logits, dtype, row_stride, seq_stride, row_mode, 0, most_layers, st, vocab, kk,
                              mu, K_init < kk ? K_init : kk, init_layers, max_depth, reinterpret_cast<int32_t*>(w + V.c_token),
                              reinterpret_cast<float*>(w + V.c_logit), reinterpret_cast<float*>(w + V.c_prob),
                              reinterpret_cast<double*>(w + V.c_edge), reinterpret_cast<float*>(w + V.c_max),
                              reinterpret_cast<double*>(w + V.c_lse), workspace, V.c_workspace, stream, spec);
    };
    // (the start of a single launch that continues trees zeroes row tickets, sequence tickets and
    // descriptors; the other counters are zeroed here, or by the start of the first launch below)
    if (k <= kCappedLoopTryK) {
      rc = check_hip(launch_fill_zero(w + C.off_exit, C.off_max - C.off_exit, static_cast<hipStream_t>(stream)), "counter fill launch");
      if (rc) return rc;
      return run(k, nullptr);
    }
    // Ranking N - 1 candidates per row costs about twice what 32 cost, and trees whose rows get
    // that many children are rare.  So the loop runs with a cap of 32 first, from a saved copy
    // of the per-sequence state, and its selections say whether any of them kept the 32nd
    // candidate of a row.  If none did, the cap never cut a row short and the tree is the one of
    // the uncapped pool: a selection that wants more than 32 tokens of a row wants its 32 best
    // too, the last of them included.  Otherwise a second launch, which every workgroup leaves
    // at once when the flag is down, builds the trees again from the saved state with the full
    // cap.  (The flag word lies behind the exit tickets; the first launch's start zeroes all of them.)
    uint32_t* flag = reinterpret_cast<uint32_t*>(w + C.off_exit) + kCapHitWord;
    Speculation first = {flag, nullptr, reinterpret_cast<int32_t*>(w + V.c_saved)};
    Speculation second = {nullptr, flag, reinterpret_cast<int32_t*>(w + V.c_saved)};
    if ((rc = run(kCappedLoopTryK, &first))) return rc;
    return run(k, &second);
  }
  L = V.scan;   // offsets of the roomier layout; the scan strides its partial keys by k_scan
  const ExpandArgs ea = make_expand_args(logits, row_stride, seq_stride, row_mode, st, vocab, k_scan,
                                         reinterpret_cast<int32_t*>(w + V.off_token), reinterpret_cast<float*>(w + V.off_logit),
                                         reinterpret_cast<float*>(w + V.off_prob), reinterpret_cast<double*>(w + V.off_edge),
                                         reinterpret_cast<float*>(w + V.off_max), reinterpret_cast<double*>(w + V.off_lse),
                                         workspace, L);
  LiteralArgs la;
  la.logits = logits; la.row_stride = row_stride; la.seq_stride = seq_stride; la.row_mode = row_mode; la.vocab = vocab;
  la.st = *st; la.log_mu = log(static_cast<double>(mu)); la.K_init = K_init; la.init_layers = init_layers;
  la.max_depth = max_depth;
  la.k_scan = k_scan;
  la.scan_token = reinterpret_cast<const int32_t*>(w + V.off_token);
  la.top_logit = reinterpret_cast<const float*>(w + V.off_logit);
  la.row_lse = reinterpret_cast<const double*>(w + V.off_lse);
  la.row_count = reinterpret_cast<int32_t*>(w + V.off_count);
  la.row_key = reinterpret_cast<unsigned long long*>(w + V.off_keys);
  la.part_key = reinterpret_cast<unsigned long long*>(w + V.off_part_keys);
  la.part_keys_per_seq = V.part_keys_per_seq;
  la.part_count = reinterpret_cast<int32_t*>(w + V.off_part_count);
  la.row_ticket = ea.ticket;        // the scan's row tickets: zero whenever the scan is not running
  hipStream_t s = static_cast<hipStream_t>(stream);
  // the scan's row tickets start at zero and every launch leaves them so
  rc = check_hip(launch_fill_zero(w + L.off_ticket, L.off_max - L.off_ticket, s), "ticket fill launch");
  if (rc) return rc;
  // a tree of N nodes has at most N - 1 layers; a layer of finished sequences costs three empty launches
  const int most = st->N > 1 ? st->N - 1 : 0;
  const int run = layers < most ? layers : most;
  for (int d = 0; d < run; ++d) {
    rc = check_hip(launch_expand(ea, dtype, expand_grid(st, L.chunks, -1, k_scan, k_scan, 0), false, s), "scan launch");
    if (rc) return rc;
    rc = check_hip(launch_literal_layer(la, dtype, s), "literal layer launch");
    if (rc) return rc;
  }
  return TALON_OK;
}

int talon_set_spin_limit_us(int64_t microseconds) {
  if (microseconds < 0) { set_error("spin limit of %lld us is negative", (long long)microseconds); return TALON_ERR_INVALID_ARG; }
  g_spin_limit_us.store(microseconds, std::memory_order_relaxed);
  return TALON_OK;
}

int talon_profile_scan_launches(int enable) {
  g_profile.enabled = enable != 0;
  g_profile.used = 0;
  return TALON_OK;
}

int talon_profile_read(float* durations_us, int32_t capacity, int32_t* n_launches) {
  if (!n_launches || (capacity > 0 && !durations_us) || capacity < 0) {
    set_error("talon_profile_read: null output or negative capacity");
    return TALON_ERR_INVALID_ARG;
  }
  const size_t pairs = g_profile.used / 2;
  *n_launches = static_cast<int32_t>(pairs);
  const size_t n = pairs < static_cast<size_t>(capacity) ? pairs : static_cast<size_t>(capacity);
  for (size_t i = 0; i < n; ++i) {
    int rc = check_hip(hipEventSynchronize(g_profile.events[2 * i + 1]), "profile event synchronize");
    if (rc) return rc;
    float ms = 0.f;
    rc = check_hip(hipEventElapsedTime(&ms, g_profile.events[2 * i], g_profile.events[2 * i + 1]), "profile elapsed time");
    if (rc) return rc;
    durations_us[i] = ms * 1000.f;
  }
  g_profile.used = 0;
  return TALON_OK;
}

int talon_prune_tree(const talon_tree_state* st, int32_t n_keep, int32_t* kept_ids, void* stream) {
  int rc = check_state(st);
  if (rc) return rc;
  if (n_keep < 1 || n_keep > st->N_pad) { set_error("n_keep=%d outside [1, N_pad=%d]", n_keep, st->N_pad); return TALON_ERR_INVALID_ARG; }
  if (!kept_ids) { set_error("kept_ids is NULL"); return TALON_ERR_INVALID_ARG; }
  return check_hip(launch_prune(*st, n_keep, kept_ids, static_cast<hipStream_t>(stream)), "prune launch");
}

size_t talon_verify_workspace_bytes(int32_t B, int32_t N_pad, int32_t vocab, int dtype) {
  VerifyLayout V;
  if (verify_layout(B, N_pad, vocab, dtype, &V)) return 0;
  return V.total;
}

int talon_target_argmax(const void* logits, int dtype, int64_t row_stride, int64_t seq_stride,
                        const talon_tree_state* st, int32_t vocab, int32_t* target_token, float* target_prob,
                        uint32_t* scan_status, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_state(st);
  if (rc) return rc;
  VerifyLayout V;
  rc = verify_layout(st->B, st->N_pad, vocab, dtype, &V);
  if (rc) return rc;
  if (!scan_status) { set_error("scan_status is NULL"); return TALON_ERR_INVALID_ARG; }
  char* w = static_cast<char*>(workspace);
  ExpandLayout L;
  // the scan's own checks (pointers, alignment, strides), with the unused outputs in the workspace
  float* prob = target_prob ? target_prob : (w ? reinterpret_cast<float*>(w + V.off_prob) : nullptr);
  rc = check_expand_args(logits, dtype, row_stride, seq_stride, TALON_ROWS_BY_NODE, st, vocab, 1, target_token,
                         w ? w + V.off_logit : nullptr, prob, w ? w + V.off_edge : nullptr, w ? w + V.off_max : nullptr,
                         w ? w + V.off_lse : nullptr, workspace, workspace_bytes, &L);
  if (rc) return rc;
  if (workspace_bytes < V.total) {
    set_error("workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, V.total);
    return TALON_ERR_WORKSPACE;
  }
  ExpandArgs a = make_expand_args(logits, row_stride, seq_stride, TALON_ROWS_BY_NODE, st, vocab, 1, target_token,
                                  reinterpret_cast<float*>(w + V.off_logit), prob,
                                  reinterpret_cast<double*>(w + V.off_edge), reinterpret_cast<float*>(w + V.off_max),
                                  reinterpret_cast<double*>(w + V.off_lse), workspace, L);
  int32_t* begin = reinterpret_cast<int32_t*>(w + V.off_begin);
  int32_t* count = reinterpret_cast<int32_t*>(w + V.off_count);
  a.frontier_begin = begin; a.frontier_count = count; a.status = scan_status;
  hipStream_t s = static_cast<hipStream_t>(stream);
  rc = check_hip(launch_all_nodes_frontier(*st, begin, count, scan_status, a.ticket, s), "frontier launch");
  if (rc) return rc;
  // every node of every tree is a row: N rows per sequence at most
  long long items = static_cast<long long>(st->B) * st->N * L.chunks;
  const int grid = static_cast<int>(items > 1024 ? 1024 : (items < 1 ? 1 : items));
  return check_hip(launch_expand(a, dtype, grid, false, s), "target scan launch");
}

int talon_greedy_accept(const talon_tree_state* st, const int32_t* target_token, const uint32_t* scan_status,
                        int32_t* path, int32_t* accept_len, int32_t* bonus_token, void* stream) {
  int rc = check_state(st);
  if (rc) return rc;
  if (!target_token || !scan_status || !path || !accept_len || !bonus_token) {
    set_error("talon_greedy_accept: NULL pointer argument");
    return TALON_ERR_INVALID_ARG;
  }
  return check_hip(launch_accept(*st, target_token, scan_status, path, accept_len, bonus_token,
                                 static_cast<hipStream_t>(stream)), "accept launch");
}

int talon_compact_kv(const void* k_tree, const void* v_tree, const int32_t* path, const int32_t* accept_len,
                     const int32_t* prefix_len, int32_t* new_prefix_len, void* k_prefix, void* v_prefix, int32_t B,
                     int32_t N_pad, int32_t Hkv, int32_t Dh, int32_t prefix_capacity, int64_t kv_stride_b,
                     int64_t kv_stride_t, int64_t kv_stride_h, void* stream) {
  const void* ptrs[] = {k_tree, v_tree, path, accept_len, prefix_len, new_prefix_len, k_prefix, v_prefix};
  for (const void* p : ptrs)
    if (!p) { set_error("talon_compact_kv: NULL pointer argument"); return TALON_ERR_INVALID_ARG; }
  if (!aligned16(k_tree) || !aligned16(v_tree) || !aligned16(k_prefix) || !aligned16(v_prefix)) {
    set_error("talon_compact_kv: K/V pointers must be 16-byte aligned");
    return TALON_ERR_INVALID_ARG;
  }
  if (B < 1 || B > TALON_B_MAX || N_pad < 64 || N_pad > TALON_N_MAX || N_pad % 64) { set_error("bad B=%d or N_pad=%d", B, N_pad); return TALON_ERR_INVALID_ARG; }
  if (Hkv < 1 || Dh < 8 || Dh % 8) { set_error("Hkv=%d, Dh=%d: Dh must be a positive multiple of 8", Hkv, Dh); return TALON_ERR_INVALID_ARG; }
  if (prefix_capacity < 1) { set_error("prefix_capacity=%d must be >= 1", prefix_capacity); return TALON_ERR_INVALID_ARG; }
  if (kv_stride_t % 8 || kv_stride_h % 8 || kv_stride_b % 8 || kv_stride_h < Dh) {
    set_error("talon_compact_kv: KV strides must be multiples of 8 elements with a contiguous Dh run");
    return TALON_ERR_INVALID_ARG;
  }
  return check_hip(launch_compact_kv(static_cast<const uint16_t*>(k_tree), static_cast<const uint16_t*>(v_tree), path,
                                     accept_len, prefix_len, new_prefix_len, static_cast<uint16_t*>(k_prefix),
                                     static_cast<uint16_t*>(v_prefix), B, N_pad, Hkv, Dh, prefix_capacity, kv_stride_b,
                                     kv_stride_t, kv_stride_h, static_cast<hipStream_t>(stream)), "compact launch");
}

int talon_probe_read(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf || !sink || bytes < 16 || (reinterpret_cast<uintptr_t>(buf) & 15u)) {
    set_error("talon_probe_read: needs a 16-byte aligned device buffer of at least 16 bytes and a 4-byte device sink");
    return TALON_ERR_INVALID_ARG;
  }
  return check_hip(launch_read_probe(buf, bytes, sink, static_cast<hipStream_t>(stream)), "read probe launch");
}

int talon_probe_mfma(int32_t workgroups, int32_t iters, void* sink, double* flops, void* stream) {
  if (!sink || workgroups < 1 || workgroups > 65536 || iters < 1) {
    set_error("talon_probe_mfma: workgroups in [1, 65536], iters >= 1 and a 4-byte device sink are required");
    return TALON_ERR_INVALID_ARG;
  }
  // 4 wavefronts per workgroup, 4 MFMA 32x32x16 per iteration, 2*32*32*16 FLOP each
  if (flops) *flops = static_cast<double>(workgroups) * 4.0 * iters * 4.0 * 32768.0;
  return check_hip(launch_mfma_probe(workgroups, iters, sink, static_cast<hipStream_t>(stream)), "mfma probe launch");
}

int talon_probe_issue(int32_t mode, int32_t waves, int32_t iters, uint64_t* cycles, void* sink, void* stream) {
  if (!cycles || !sink || mode < 0 || mode > 4 || (waves != 4 && waves != 8) || iters < 1 ||
      (reinterpret_cast<uintptr_t>(cycles) & 7u)) {
    set_error("talon_probe_issue: mode in [0, 4], waves 4 or 8, iters >= 1, 8 device words for the cycles and a 4-byte device sink are required");
    return TALON_ERR_INVALID_ARG;
  }
  return check_hip(launch_issue_probe(mode, waves, iters, cycles, sink, static_cast<hipStream_t>(stream)), "issue probe launch");
}

int talon_probe_tile_loads(const void* window, size_t window_bytes, int32_t loads, int32_t with_mfma, int32_t waves,
                           int32_t iters, uint64_t* cycles, void* sink, void* stream) {
  if (!window || !cycles || !sink || (loads != 4 && loads != 8) || (waves != 4 && waves != 8) || iters < 1 ||
      window_bytes < (static_cast<size_t>(256) << 16) || (reinterpret_cast<uintptr_t>(window) & 15u) ||
      (reinterpret_cast<uintptr_t>(cycles) & 7u)) {
    set_error("talon_probe_tile_loads: a 16-byte aligned window of at least 16 MiB, loads 4 or 8, waves 4 or 8, iters >= 1, "
              "2048 device words for the cycles and a 4-byte device sink are required");
    return TALON_ERR_INVALID_ARG;
  }
  return check_hip(launch_tile_load_probe(loads, with_mfma != 0, waves, iters, window, cycles, sink, static_cast<hipStream_t>(stream)),
                   "tile load probe launch");
}

int talon_build_tree_mask(const talon_tree_state* st, uint64_t* mask, void* stream) {
  int rc = check_state(st);
  if (rc) return rc;
  if (!mask || (reinterpret_cast<uintptr_t>(mask) & 7u)) { set_error("mask is NULL or misaligned"); return TALON_ERR_INVALID_ARG; }
  return check_hip(launch_mask(*st, mask, static_cast<hipStream_t>(stream)), "mask launch");
}

static int attention_layout(int32_t B, int32_t N_pad, int32_t Hq, int32_t Hkv, int32_t Dh, int32_t max_prefix_len,
                            int* splits, int* tps, int* rows_pad, size_t* off_m, size_t* off_l, size_t* total) {
  if (B < 1 || B > TALON_B_MAX) { set_error("B=%d outside [1, %d]", B, TALON_B_MAX); return TALON_ERR_INVALID_ARG; }
  if (N_pad < 64 || N_pad > TALON_N_MAX || N_pad % 64) { set_error("N_pad=%d must be a multiple of 64 in [64, %d]", N_pad, TALON_N_MAX); return TALON_ERR_INVALID_ARG; }
  if (Hq < 1 || Hkv < 1 || max_prefix_len < 0) { set_error("Hq, Hkv must be >= 1 and max_prefix_len >= 0"); return TALON_ERR_INVALID_ARG; }
  if (Dh != 64 && Dh != 128) { set_error("Dh=%d not supported (64 or 128)", Dh); return TALON_ERR_UNSUPPORTED; }
  if (Hq % Hkv) { set_error("Hq=%d is not a multiple of Hkv=%d", Hq, Hkv); return TALON_ERR_UNSUPPORTED; }
  if (Hq / Hkv > 16) { set_error("Hq/Hkv=%d above 16 is not supported", Hq / Hkv); return TALON_ERR_UNSUPPORTED; }
  attention_plan(B, N_pad, Hq, Hkv, Dh, max_prefix_len, splits, tps, rows_pad);
  const size_t prow = static_cast<size_t>(B) * Hkv * (*splits) * (*rows_pad);
  *off_m = prow * Dh * sizeof(uint16_t);   // bf16 partial outputs, then fp32 maxima and denominators
  *off_l = *off_m + prow * sizeof(float);
  *total = *off_l + prow * sizeof(float);
  if (*splits == 1) *total = 256;  // nothing is staged, keep a token size
  return TALON_OK;
}

size_t talon_tree_attention_workspace_bytes(int32_t B, int32_t N_pad, int32_t Hq, int32_t Hkv, int32_t Dh,
                                            int32_t max_prefix_len) {
  int splits, tps, rows_pad;
  size_t off_m, off_l, total;
  if (attention_layout(B, N_pad, Hq, Hkv, Dh, max_prefix_len, &splits, &tps, &rows_pad, &off_m, &off_l, &total)) return 0;
  return total;
}

static int tree_attention_call(const void* q, const void* k_prefix, const void* v_prefix, const void* k_tree,
                               const void* v_tree, const uint64_t* mask, const int32_t* n_nodes,
                               const int32_t* prefix_len, int32_t B, int32_t N_pad, int32_t Hq, int32_t Hkv, int32_t Dh,
                               int32_t max_prefix_len, int64_t kv_stride_b, int64_t kv_stride_t, int64_t kv_stride_h,
                               float scale, void* out, float* out_lse, void* workspace, size_t workspace_bytes,
                               bool static_scratch, void* stream) {
  AttnArgs a;
  size_t off_m, off_l, total;
  int rc = attention_layout(B, N_pad, Hq, Hkv, Dh, max_prefix_len, &a.splits, &a.tiles_per_split, &a.rows_pad, &off_m,
                            &off_l, &total);
  if (rc) return rc;
  const void* ptrs[] = {q, k_tree, v_tree, mask, out};
  for (const void* p : ptrs) {
    if (!p) { set_error("NULL pointer argument"); return TALON_ERR_INVALID_ARG; }
    if (!aligned16(p)) { set_error("pointer argument is not 16-byte aligned"); return TALON_ERR_INVALID_ARG; }
  }
  if (!n_nodes || !prefix_len) { set_error("n_nodes / prefix_len is NULL"); return TALON_ERR_INVALID_ARG; }
  if (max_prefix_len > 0) {
    if (!k_prefix || !v_prefix) { set_error("prefix K/V is NULL"); return TALON_ERR_INVALID_ARG; }
    if (!aligned16(k_prefix) || !aligned16(v_prefix)) { set_error("prefix K/V is not 16-byte aligned"); return TALON_ERR_INVALID_ARG; }
    if (kv_stride_t < Dh || kv_stride_h < Dh || kv_stride_b < 0 || kv_stride_t % 8 || kv_stride_h % 8 || kv_stride_b % 8) {
      set_error("prefix K/V strides must be >= Dh and multiples of 8 elements");
      return TALON_ERR_INVALID_ARG;
    }
    if (kv_stride_t > (1ll << 24)) {   // a tile's 64 rows are addressed with 32-bit byte offsets
      set_error("prefix K/V token stride of %lld elements is above 2^24", (long long)kv_stride_t);
      return TALON_ERR_UNSUPPORTED;
    }
  }
  if (out_lse && (reinterpret_cast<uintptr_t>(out_lse) & 3u)) { set_error("out_lse is misaligned"); return TALON_ERR_INVALID_ARG; }
  if (!(scale >= 0.f) || isinf(scale)) { set_error("scale=%g must be finite and >= 0 (0 selects 1/sqrt(Dh))", (double)scale); return TALON_ERR_INVALID_ARG; }
  if (static_scratch) {
    // the split-KV partial results go to the library's own device array: size first (a host
    // check), then the array's address on the current device
    if (a.splits > 1 && total > kStaticScratchBytes) {
      set_error("this shape needs %zu bytes of split-KV scratch; the call without a workspace holds at most %zu "
                "(use talon_tree_attention with a caller-provided workspace)", total, kStaticScratchBytes);
      return TALON_ERR_WORKSPACE;
    }
    if ((rc = static_scratch_address(&workspace))) return rc;
    workspace_bytes = kStaticScratchBytes;
  }
  if (a.splits > 1) {
    if (!workspace || !aligned16(workspace)) { set_error("workspace is NULL or not 16-byte aligned"); return TALON_ERR_INVALID_ARG; }
    if (workspace_bytes < total) { set_error("workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, total); return TALON_ERR_WORKSPACE; }
  }
  a.q = static_cast<const uint16_t*>(q);
  a.k_prefix = static_cast<const uint16_t*>(k_prefix);
  a.v_prefix = static_cast<const uint16_t*>(v_prefix);
  a.k_tree = static_cast<const uint16_t*>(k_tree);
  a.v_tree = static_cast<const uint16_t*>(v_tree);
  a.mask = mask; a.n_nodes = n_nodes; a.prefix_len = prefix_len;
  a.B = B; a.N_pad = N_pad; a.Hq = Hq; a.Hkv = Hkv; a.G = Hq / Hkv; a.Dh = Dh; a.max_prefix_len = max_prefix_len;
  a.kv_stride_b = kv_stride_b; a.kv_stride_t = kv_stride_t; a.kv_stride_h = kv_stride_h;
  const float sc = scale == 0.f ? 1.f / sqrtf(static_cast<float>(Dh)) : scale;
  a.scale_log2e = sc * 1.4426950408889634f;
  a.out = static_cast<uint16_t*>(out);
  a.out_lse = out_lse;
  char* w = static_cast<char*>(workspace);
  a.part_o = reinterpret_cast<uint16_t*>(w);
  a.part_m = reinterpret_cast<float*>(w + off_m);
  a.part_l = reinterpret_cast<float*>(w + off_l);
  return check_hip(launch_attention(a, static_cast<hipStream_t>(stream)), "tree attention launch");
}

int talon_tree_attention(const void* q, const void* k_prefix, const void* v_prefix, const void* k_tree,
                         const void* v_tree, const uint64_t* mask, const int32_t* n_nodes,
                         const int32_t* prefix_len, int32_t B, int32_t N_pad, int32_t Hq, int32_t Hkv, int32_t Dh,
                         int32_t max_prefix_len, int64_t kv_stride_b, int64_t kv_stride_t, int64_t kv_stride_h,
                         float scale, void* out, float* out_lse, void* workspace, size_t workspace_bytes,
                         void* stream) {
  return tree_attention_call(q, k_prefix, v_prefix, k_tree, v_tree, mask, n_nodes, prefix_len, B, N_pad, Hq, Hkv, Dh,
                             max_prefix_len, kv_stride_b, kv_stride_t, kv_stride_h, scale, out, out_lse, workspace,
                             workspace_bytes, false, stream);
}

size_t talon_static_scratch_bytes(void) { return kStaticScratchBytes; }

int talon_static_scratch_init(void) {
  void* p = nullptr;
  return static_scratch_address(&p);
}

int talon_tree_attention_static(const void* q, const void* k_prefix, const void* v_prefix, const void* k_tree,
                                const void* v_tree, const uint64_t* mask, const int32_t* n_nodes,
                                const int32_t* prefix_len, int32_t B, int32_t N_pad, int32_t Hq, int32_t Hkv,
                                int32_t Dh, int32_t max_prefix_len, int64_t kv_stride_b, int64_t kv_stride_t,
                                int64_t kv_stride_h, float scale, void* out, float* out_lse, void* stream) {
  return tree_attention_call(q, k_prefix, v_prefix, k_tree, v_tree, mask, n_nodes, prefix_len, B, N_pad, Hq, Hkv, Dh,
                             max_prefix_len, kv_stride_b, kv_stride_t, kv_stride_h, scale, out, out_lse, nullptr, 0,
                             true, stream);
}

}  // extern "C"
