// Internal declarations shared by the translation units of libtalon (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "talon.h"

namespace talon {

constexpr int kThreads = 256;       // every kernel here runs 4 wavefronts per workgroup
constexpr int kScanTiles = 4;       // 16-byte vectors per thread per vocab chunk
constexpr int kChunkBytes = kThreads * kScanTiles * 16;  // 16 KiB of a logits row per workgroup pass
constexpr int kMergeCap = 2048;     // chunks * k keys one row merge stages in LDS
constexpr uint32_t kDoneMask = TALON_STATUS_DONE_BUDGET | TALON_STATUS_DONE_DEPTH | TALON_STATUS_ABORTED;

void set_error(const char* fmt, ...);
int check_hip(hipError_t e, const char* what);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct SelectArgs {
  talon_tree_state st;
  int k;
  const int32_t* cand_token;
  const float* cand_prob;
  const double* cand_edge_logp;
  double log_mu;
  int K_init, init_layers, max_depth;
  // Optional: set to 1 when a selection keeps the last (k-th) candidate of a row, i.e. when the
  // per-row cap may have cut the pool of Alg. 2 short.  While it stays 0 the tree is the one the
  // uncapped pool gives: a selection that wants more than k tokens of a row also wants the row's
  // k best, all of which the capped pool holds.
  uint32_t* cap_hit;
};

// Workgroups leave the single-launch kernel through a two-level ticket (one counter for all
// of them would serialise several hundred atomics on one address at the end of the launch).
// Measured over 8 to 255 groups on grids of 300 to 700 workgroups: 128 is the fastest; fewer
// groups lengthen the first level, more lengthen the second.
constexpr int kExitGroups = 128;
// Words of the exit-ticket array: the groups' count, one count per group, and two counters of the
// launches of one layer (workgroups that have read the frontier; selections that have finished).
constexpr int kStartedWord = kExitGroups + 1;
constexpr int kSelectedWord = kExitGroups + 2;
constexpr int kExitWords = kExitGroups + 3;
// One more word behind them, which no launch clears: the cap_hit flag of a speculative run.
constexpr int kCapHitWord = kExitWords;
constexpr unsigned long long kDescReady = 1ull << 63;

struct ExpandArgs {
  const void* logits;
  int64_t row_stride, seq_stride;
  int row_mode;
  int B, N_pad, vocab, k;
  int chunks;            // 16 KiB blocks per row = most chunks a row is ever cut into
  int target_items;      // (row, chunk) items a launch aims for when it cuts rows into chunks
  const int32_t* frontier_begin;
  const int32_t* frontier_count;
  uint32_t* status;
  int32_t* cand_token;
  float* cand_logit;
  float* cand_prob;
  double* cand_edge_logp;
  float* row_max;
  double* row_lse;
  float* part_max;       // [rows][chunks]
  double* part_sum;      // [rows][chunks]
  unsigned long long* part_keys;  // [rows][chunks][k]
  int32_t* ticket;       // [rows]
  // Fused modes (the scan runs the budget selection of a sequence in its tail, when the last
  // row of that sequence's frontier has been written): selection parameters, the index of
  // this launch in the loop, per-sequence row tickets and per-layer frontier descriptors
  // [N_pad][B], one 8-byte word each: begin in the low half, count and kDescReady in the
  // high half.  In the single launch, layer i reads desc[i] (desc[0] is copied from the public
  // tree state, or known when the launch starts the trees itself) and its selections write
  // desc[i+1], so a workgroup that is late still sees the frontier of its own layer.  A launch
  // of one layer reads the public tree state instead and holds its selections back until every
  // workgroup has done so (kStartedWord).
  SelectArgs sel;
  int launch_idx;
  int32_t* seq_ticket;   // [B]
  unsigned long long* desc;
  // Single-launch mode: one grid walks all layers.  A descriptor is stored once everything
  // its selection wrote has been performed, with kDescReady set; a workgroup enters layer i
  // when every desc[i][b] is ready (it polls them; the wait is bounded by spin_ticks of the
  // 100 MHz wall clock).  Descriptors of layers >= 1 are zero between launches.
  // The launch leaves its workspace as it found it: every workgroup takes an exit ticket
  // when it has finished with tickets and descriptors and the last one clears them.  With
  // root_token set the launch also starts the trees itself (Alg. 2 line 1): layer 0 is the
  // root row of every sequence, and the workgroup that writes that row initialises the
  // sequence's state first.
  int layers;
  uint32_t* exit_ticket; // [kExitWords] workgroups that have left, counted per group, then the groups; see kStartedWord
  unsigned long long spin_ticks;
  uint64_t* tree_mask;   // optional: ancestor masks written at the end of the single launch
  const int32_t* root_token;   // optional [B]
  const uint32_t* run_if;      // optional: the single launch does nothing unless this word is non-zero
};

// Start of a single launch that continues trees: what it does with the five per-sequence words
// of the tree state (nodes, frontier begin and count, depth, status) besides reading them.
constexpr int kInitPlain = 0;     // nothing
constexpr int kInitSave = 1;      // copy them to `saved` [5][B] first
constexpr int kInitRestoreIf = 2; // if *flag is non-zero: put them back from `saved`, then start; else do nothing
struct FusedInitArgs {
  int mode;
  int32_t* saved;
  const uint32_t* flag;
  uint32_t* clear;   // optional: kExitWords + 1 words (exit tickets, layer counters, cap_hit) set to zero with kInitSave
};

// Uncapped ("paper-literal") layer of Alg. 2: the pool of a parent is its whole row.
#ifndef TALON_LITERAL_CHUNKS
#define TALON_LITERAL_CHUNKS 8
#endif
constexpr int kLiteralChunks = TALON_LITERAL_CHUNKS;     // parts a row is streamed in at most (their survivors, 8 * 255 keys, are merged in LDS)
constexpr int kLiteralRowCap = 256;   // survivors of one row that can still be chosen: at most N - 1 <= 255
struct LiteralPlan {   // what a layer does for one sequence
  double thr;          // gate threshold on the path score, log(mu) + anchor (-inf on top-K layers)
  int32_t active, F, fb, n, d, limit;
  uint32_t status;
  int32_t pad;
};
struct LiteralArgs {
  const void* logits;
  int64_t row_stride, seq_stride;
  int row_mode, vocab;
  talon_tree_state st;
  double log_mu;
  int K_init, init_layers, max_depth;
  int k_scan;                      // candidates per row the scan ranks (K_init on top-K layers, else 1)
  const int32_t* scan_token;       // [B*N_pad][k_scan] the scan's candidates ...
  const float* top_logit;          // [B*N_pad][k_scan] ... and their logits; the first is the row's largest
  const double* row_lse;           // [B*N_pad]
  int32_t* row_count;              // [B*N_pad] survivors kept of a row
  unsigned long long* row_key;     // [B*N_pad][kLiteralRowCap] their keys (sortable logit << 32 | ~token)
  // A row of a sequence with few rows is streamed in up to kLiteralChunks parts by as many
  // workgroups: part c of frontier row j of a layer that takes at most `limit` nodes leaves its
  // survivors at part_key[b * part_keys_per_seq + (j * parts + c) * limit] (rows * limit never
  // exceeds (N / 2)^2) and their number in part_count.
  unsigned long long* part_key;
  size_t part_keys_per_seq;
  int32_t* part_count;             // [B*N_pad][kLiteralChunks]
  int32_t* row_ticket;             // [B*N_pad] parts of a row that have finished; zero between launches
};

struct AttnArgs {
  const uint16_t* q;
  const uint16_t* k_prefix;
  const uint16_t* v_prefix;
  const uint16_t* k_tree;
  const uint16_t* v_tree;
  const uint64_t* mask;
  const int32_t* n_nodes;
  const int32_t* prefix_len;
  int B, N_pad, Hq, Hkv, G, Dh;
  int max_prefix_len;
  int64_t kv_stride_b, kv_stride_t, kv_stride_h;
  float scale_log2e;     // scale * log2(e): scores are kept in base-2 units
  uint16_t* out;
  float* out_lse;
  int splits;            // KV splits per (sequence, kv head, row tile)
  int tiles_per_split;   // key tiles of kAttnKeyTile per split
  uint16_t* part_o;      // [B][Hkv][splits][Dh/8][rows_pad][8] bf16: each split's output, normalised by its own denominator
  float* part_m;         // [B][Hkv][splits][rows_pad]      running max (base-2 units)
  float* part_l;         // [B][Hkv][splits][rows_pad]      running denominator
  int rows_pad;          // N_pad * G rounded up to the row tile
  int row_tiles;         // row tiles per (sequence, KV head)
  int total_items;       // row_tiles * splits * B * Hkv work items of the main kernel
};

// launchers (each checks nothing: arguments were validated by the ABI layer)
hipError_t launch_tree_init(const talon_tree_state& st, const int32_t* root_token, hipStream_t s);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
hipError_t launch_prune(const talon_tree_state& st, int n_keep, int32_t* kept_ids, hipStream_t s);
hipError_t launch_all_nodes_frontier(const talon_tree_state& st, int32_t* begin, int32_t* count, uint32_t* status,
                                     int32_t* ticket, hipStream_t s);
hipError_t launch_accept(const talon_tree_state& st, const int32_t* target_token, const uint32_t* scan_status,
                         int32_t* path, int32_t* accept_len, int32_t* bonus_token, hipStream_t s);
hipError_t launch_compact_kv(const uint16_t* k_tree, const uint16_t* v_tree, const int32_t* path, const int32_t* accept_len,
                             const int32_t* prefix_len, int32_t* new_prefix_len, uint16_t* k_prefix, uint16_t* v_prefix,
                             int B, int N_pad, int Hkv, int Dh, int capacity, int64_t sb, int64_t st_, int64_t sh,
                             hipStream_t s);
hipError_t launch_read_probe(const void* buf, size_t bytes, void* sink, hipStream_t s);
hipError_t launch_mfma_probe(int workgroups, int iters, void* sink, hipStream_t s);
hipError_t launch_issue_probe(int mode, int waves, int iters, void* cycles, void* sink, hipStream_t s);
hipError_t launch_tile_load_probe(int loads, bool with_mfma, int waves, int iters, const void* window, void* cycles, void* sink, hipStream_t s);
hipError_t launch_fused_init(const talon_tree_state& st, const ExpandArgs& a, const FusedInitArgs& f, hipStream_t s);
hipError_t launch_expand_tree(const ExpandArgs& a, int dtype, int grid, hipStream_t s);
int expand_tree_max_grid(int dtype);
hipError_t launch_expand(const ExpandArgs& a, int dtype, int grid, bool fused, hipStream_t s);
hipError_t launch_select(const SelectArgs& a, hipStream_t s);
hipError_t launch_mask(const talon_tree_state& st, uint64_t* mask, hipStream_t s);
hipError_t launch_literal_layer(const LiteralArgs& a, int dtype, hipStream_t s);
hipError_t launch_attention(const AttnArgs& a, hipStream_t s);

int expand_chunk_elems(int dtype);
void attention_plan(int B, int N_pad, int Hq, int Hkv, int Dh, int max_prefix_len, int* splits,
                    int* tiles_per_split, int* rows_pad);

}  // namespace talon
