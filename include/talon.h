/*
 * talon.h - C ABI of the MI355X (gfx950) hot path of one Talon speculative-decoding step:
 * budget-driven adaptive draft-tree expansion and tree-attention verification
 * (arXiv 2601.07353, Sec. 5 and App. A/B).
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless it is marked "host".  The caller owns every
 *     buffer and the library allocates no device memory.  State it keeps between calls, all of
 *     it host-side and per process: the measurement hook's HIP events (created on demand while
 *     the hook is enabled), the wait bound of talon_set_spin_limit_us, two cached launch facts
 *     (how many workgroups of the single-launch kernel the device holds at once; that the
 *     attention kernel's LDS size has been raised), and the device address of the scratch
 *     array of talon_tree_attention_static.  None of it depends on the arguments of a call.
 *   - Calls only enqueue work on `stream` (a hipStream_t passed as void*; NULL = the null
 *     stream) and return at once.  Nothing synchronises with the host.
 *   - Every call returns TALON_OK or a negative TALON_ERR_* code; all argument checks run on
 *     the host before anything is launched, so a failed call has enqueued nothing.
 *     talon_last_error_string() gives the reason (thread-local, host pointer).
 *   - Problems only the device can see (a NaN logit, a row with no finite maximum) set
 *     TALON_STATUS_BAD_ROW in status[b] and stop that sequence; they are not host errors.
 *   - Device pointers must be 16-byte aligned.
 *
 * Notation (paper): B sequences, V vocabulary, K top-K width, N node budget (root counted,
 * Alg. 2 starts from T = {x_t}), mu gate threshold, P_d frontier of layer d, S_d candidate
 * pool, p(u) path confidence (Eq. 2).
 */
#ifndef TALON_H_
#define TALON_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TALON_OK 0
#define TALON_ERR_INVALID_ARG (-1)
#define TALON_ERR_UNSUPPORTED (-2)
#define TALON_ERR_WORKSPACE (-3)
#define TALON_ERR_RUNTIME (-4)

#define TALON_DTYPE_F32 0
#define TALON_DTYPE_BF16 1

/* limits */
#define TALON_K_MAX 64     /* per-row candidate cap k; the selection also needs (N-1)*k <= 4096 */
#define TALON_N_MAX 256    /* node budget N (root included)                     */
#define TALON_B_MAX 256    /* sequences per call                                */

/* status[b] bits */
#define TALON_STATUS_DONE_BUDGET 1u /* |T| reached N (Alg. 2 loop condition false)    */
#define TALON_STATUS_DONE_DEPTH 2u  /* max_depth layers built before the budget ran out */
#define TALON_STATUS_BAD_ROW 4u     /* NaN / +inf logit or a row with no finite maximum */
#define TALON_STATUS_ABORTED 8u     /* talon_expand_tree gave up waiting between two layers */

/* logits row addressing for talon_expand_layer */
#define TALON_ROWS_BY_NODE 0     /* row of node i of sequence b = i                        */
#define TALON_ROWS_BY_FRONTIER 1 /* row = i - frontier_begin[b] (dense draft-forward batch) */

/*
 * Token tree T of Alg. 2 in structure-of-arrays form, one slab of N_pad entries per
 * sequence (N_pad = N rounded up to a multiple of 64).  Node 0 is the root x_t.  Node ids
 * are layer-major; inside a layer they are ordered (parent id ascending, in-row rank
 * ascending), so the frontier P_d is always the contiguous id range
 * [frontier_begin, frontier_begin + frontier_count).
 */
typedef struct talon_tree_state {
  int32_t B, N, N_pad;
  int32_t* token;          /* [B][N_pad] token id of the node                            */
  int32_t* parent;         /* [B][N_pad] parent node id; root: -1                         */
  int32_t* depth;          /* [B][N_pad] root: 0; child = parent + 1                      */
  float* prob;             /* [B][N_pad] edge probability P(token | path); root: 1        */
  double* logp;            /* [B][N_pad] log path confidence log p(v) (Eq. 2); root: 0    */
  int32_t* n_nodes;        /* [B] |T|                                                     */
  int32_t* frontier_begin; /* [B] first node id of the last layer built                   */
  int32_t* frontier_count; /* [B] size of that layer                                      */
  int32_t* depth_cur;      /* [B] number of layers built (d of Alg. 2)                    */
  uint32_t* status;        /* [B] TALON_STATUS_* bits                                     */
} talon_tree_state;

/* Reason for the last non-OK return on this thread (host string, never NULL). */
const char* talon_last_error_string(void);

/*
 * Alg. 2 line 1: T = {x_t}, P_0 = {x_t}, p(x_t) = 1, d = 0 for every sequence.
 * root_token [B] (device).  Entries of the per-node arrays beyond node 0 are not touched.
 */
int talon_tree_init(const talon_tree_state* st, const int32_t* root_token, void* stream);

/*
 * Scratch for talon_expand_layer.  Size it once for the largest call; before the first
 * use (and never again) clear it with talon_expand_workspace_init.
 */
size_t talon_expand_workspace_bytes(int32_t B, int32_t N_pad, int32_t vocab, int32_t k, int dtype);
int talon_expand_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/*
 * Candidate pool S_d of one layer (Eq. 3; Alg. 2 "gather" loop), restricted to the k best
 * tokens of every parent.  For every frontier node v of every unfinished sequence: one
 * pass over its logits row gives the softmax statistics (P(.|x<=v) is the softmax of the
 * row) and the k largest logits ordered (logit descending, token id ascending).
 *
 *   logits      row-major rows of `vocab` elements (f32 or bf16), row_stride elements
 *               between rows of a sequence, seq_stride elements between sequences.
 *               Each row is read exactly once.  -inf entries are allowed (probability 0).
 *   row_mode    which row node i reads (TALON_ROWS_BY_NODE / _BY_FRONTIER).
 *   layer       depth d of the layer being expanded if the caller knows it (all sequences
 *               at the same depth), else -1.  Only sizes the launch: layer d of a tree has a
 *               bounded frontier, so fewer workgroups are started; results do not depend on it.
 *   outputs, all indexed by [b][node id][rank], only rows of frontier nodes are written:
 *     cand_token     [B][N_pad][k] int32   token ids; -1 where vocab < k
 *     cand_logit     [B][N_pad][k] float   their logits (exact input values)
 *     cand_prob      [B][N_pad][k] float   P(w | x<=v) = exp(logit - lse)
 *     cand_edge_logp [B][N_pad][k] double  logit - lse (log of the above, unrounded)
 *     row_max        [B][N_pad]    float   max logit of the row
 *     row_lse        [B][N_pad]    double  log-sum-exp of the row
 *   A row whose lse is not finite sets TALON_STATUS_BAD_ROW for its sequence.
 *   Errors: INVALID_ARG (null/unaligned pointer, k not in [1, TALON_K_MAX], vocab < 1,
 *   strides too small or not a multiple of 16 bytes), UNSUPPORTED (dtype, vocab beyond
 *   what one merge supports), WORKSPACE (too small).
 */
int talon_expand_layer(const void* logits, int dtype, int64_t row_stride, int64_t seq_stride,
                       int row_mode, int32_t layer, const talon_tree_state* st, int32_t vocab,
                       int32_t k, int32_t* cand_token, float* cand_logit, float* cand_prob,
                       double* cand_edge_logp, float* row_max, double* row_lse,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Hybrid allocation of the remaining budget (Sec. 5.2; Alg. 2 "Hybrid Expansion Strategy"
 * and "Budget Check"), one layer, every unfinished sequence:
 *   score(u) = logp[v] + cand_edge_logp[v][rank]                 (log of Eq. 2 / Sec. 5.2.1)
 *   layer < init_layers : P_{d+1} = Top-K_init of the pool        (Eq. 5)
 *   otherwise           : m_d = max score;  keep score >= log(mu) + m_d   (Eq. 4)
 *   if more than R = N - |T| remain, keep the R best               (budget check)
 * Ties: (score descending, parent id ascending, rank ascending).  The kept candidates are
 * appended to the tree in (parent, rank) order; n_nodes, frontier_*, depth_cur and status
 * are advanced.  A sequence stops with DONE_BUDGET when |T| = N, or with DONE_DEPTH when
 * depth_cur reaches max_depth first.
 *   Errors: INVALID_ARG (mu outside (0,1], K_init < 1, init_layers < 0, max_depth < 1,
 *   k outside [1, TALON_K_MAX], N > TALON_N_MAX, null pointers).
 */
int talon_select_budget(const talon_tree_state* st, int32_t k, const int32_t* cand_token,
                        const float* cand_prob, const double* cand_edge_logp, float mu,
                        int32_t K_init, int32_t init_layers, int32_t max_depth, void* stream);

/*
 * One iteration of the while-loop of Alg. 2 in a single launch: the vocabulary scan of
 * talon_expand_layer with the budget selection of talon_select_budget run in its tail, per
 * sequence, by the workgroup that writes the last row of that sequence's frontier.  Same
 * results as the two calls in a row; arguments and errors as theirs.  `workspace` must have
 * been initialised by talon_expand_workspace_init (once: every launch leaves it as it found it).
 * The selections rewrite the tree state that every workgroup of the launch reads when it
 * starts, so a selection holds back until all of them have read it; the other workgroups
 * never wait, so this ends whatever else runs on the device (no need for the whole grid to be
 * resident).  Should it not end within two seconds (a workspace that was never initialised),
 * the sequence is marked TALON_STATUS_ABORTED and left as it was.
 */
int talon_expand_select_layer(const void* logits, int dtype, int64_t row_stride, int64_t seq_stride,
                              int row_mode, int32_t layer, const talon_tree_state* st, int32_t vocab,
                              int32_t k, float mu, int32_t K_init, int32_t init_layers,
                              int32_t max_depth, int32_t* cand_token, float* cand_logit,
                              float* cand_prob, double* cand_edge_logp, float* row_max,
                              double* row_lse, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The whole while-loop of Alg. 2 in one call and one scan launch: the grid walks up to
 * min(max_depth, N-1) layers, each as talon_expand_select_layer runs it, and moves on to the
 * next layer when every selection of a layer is done; it ends at the first layer with no
 * frontier.  The workgroups wait for each other between layers, so the grid is limited to
 * what the device holds at once; the wait is bounded, and a launch whose wait runs out
 * (it never should) marks every sequence TALON_STATUS_ABORTED and ends.  Arguments as in the
 * calls above; `workspace` initialised by talon_expand_workspace_init.
 */
int talon_expand_tree(const void* logits, int dtype, int64_t row_stride, int64_t seq_stride,
                      int row_mode, const talon_tree_state* st, int32_t vocab, int32_t k,
                      float mu, int32_t K_init, int32_t init_layers, int32_t max_depth,
                      int32_t* cand_token, float* cand_logit, float* cand_prob,
                      double* cand_edge_logp, float* row_max, double* row_lse,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * Bound of the wait between two layers inside talon_expand_tree / talon_build_tree, in
 * microseconds (default 200000).  A launch whose workgroups cannot all be resident (the device
 * is shared with other work) ends after this long with TALON_STATUS_ABORTED on every sequence
 * instead of hanging; the caller then re-runs the step layer by layer with
 * talon_tree_init + talon_expand_select_layer on the same workspace.  0 makes every wait give
 * up at once (used by tests of that path).  Process-wide; applies to calls made afterwards.
 */
int talon_set_spin_limit_us(int64_t microseconds);

/*
 * Alg. 2 from its first line to its last, and the tree's attention mask, in one launch:
 * T = {x_t} as talon_tree_init sets it (root_token: device, [B]), the whole loop as
 * talon_expand_tree runs it, and, if `mask` is not NULL, the ancestor mask of
 * talon_build_tree_mask written by the same launch once every sequence is complete.
 * Same results as the three calls in a row; arguments and errors as theirs.  `workspace`
 * must have been initialised by talon_expand_workspace_init (once: every launch leaves it
 * as it found it).
 */
int talon_build_tree(const int32_t* root_token, const void* logits, int dtype, int64_t row_stride,
                     int64_t seq_stride, int row_mode, const talon_tree_state* st, int32_t vocab,
                     int32_t k, float mu, int32_t K_init, int32_t init_layers, int32_t max_depth,
                     int32_t* cand_token, float* cand_logit, float* cand_prob,
                     double* cand_edge_logp, float* row_max, double* row_lse, uint64_t* mask,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * talon_build_tree with the recovery from a launch that gave up (TALON_STATUS_ABORTED: the
 * device could not hold the whole grid at once, e.g. because other work was running on it).
 * Runs talon_build_tree, WAITS for `stream` (the only call of this library that synchronises
 * with the host: not for use under graph capture), reads status[b] and, if any sequence is
 * marked ABORTED, builds the same trees again on the same buffers and workspace with one launch
 * per layer: talon_tree_init, min(max_depth, N-1) x talon_expand_select_layer, and the mask.
 * The result is the tree talon_build_tree builds.  *fell_back (host, optional) is set to 1 if
 * the layer-by-layer path ran, else 0.  Arguments and errors as talon_build_tree, plus
 * TALON_ERR_RUNTIME if the copy or the wait fails.
 */
int talon_build_tree_checked(const int32_t* root_token, const void* logits, int dtype,
                             int64_t row_stride, int64_t seq_stride, int row_mode,
                             const talon_tree_state* st, int32_t vocab, int32_t k, float mu,
                             int32_t K_init, int32_t init_layers, int32_t max_depth,
                             int32_t* cand_token, float* cand_logit, float* cand_prob,
                             double* cand_edge_logp, float* row_max, double* row_lse,
                             uint64_t* mask, void* workspace, size_t workspace_bytes, void* stream,
                             int32_t* fell_back);

/*
 * Alg. 2 with the candidate pool exactly as the listing writes it (Sec. 5.2, "Hybrid Expansion
 * Strategy" and "Budget Check"): S_d holds every token of every frontier row, with no per-row
 * cap, for any budget N <= TALON_N_MAX.  The calls above cap a row at k <= TALON_K_MAX
 * candidates, which gives the same tree whenever k >= N - |T|; this is the general, slower
 * form: per layer one vocabulary scan for the row statistics and the 16 best tokens of every
 * row, then per frontier row the tokens that pass the gate (at most the remaining budget of
 * them; rows of which fewer than 16 pass are settled by the scan, the others are read again,
 * with a radix select over the row when more pass than can be taken), then per sequence the
 * budget check over what the rows kept.
 * Runs `layers` >= 1 layers from the tree state as it stands (1: one layer between two draft
 * passes; >= max_depth: the whole loop); sequences that are finished are skipped.  Same tree
 * state, node order, ties and status bits as talon_expand_select_layer; no candidate
 * arrays are written.
 * Trees of at most 64 nodes (N_pad = 64) take a shortcut where the workspace allows it: a row can
 * get at most N - 1 <= 63 children, so the capped loop with k = N - 1 cuts nothing and builds
 * the same tree in one launch (the launch talon_expand_tree makes).  When N - 1 > 32 that loop
 * first runs with k = 32, which is much cheaper to rank, and its selections record whether any
 * of them kept the 32nd candidate of a row; if none did, no row was cut short and the tree
 * stands.  Otherwise a second launch (enqueued with the first, left at once by every workgroup
 * when it is not needed) rebuilds the layers of this call from the state the call started
 * from, with k = N - 1.  With `layers` > 1 these launches' workgroups wait for each other
 * between layers and can give up as described at talon_build_tree (TALON_STATUS_ABORTED on
 * every sequence); calls with `layers` = 1 never wait.
 *   `workspace`: talon_literal_workspace_bytes bytes of device memory, no initialisation
 *   needed; it must not be shared with a call running at the same time.
 *   Errors: as talon_expand_layer and talon_select_budget (k does not apply).
 */
size_t talon_literal_workspace_bytes(int32_t B, int32_t N_pad, int32_t vocab, int dtype);
int talon_expand_literal(const void* logits, int dtype, int64_t row_stride, int64_t seq_stride,
                         int row_mode, int32_t layers, const talon_tree_state* st, int32_t vocab,
                         float mu, int32_t K_init, int32_t init_layers, int32_t max_depth,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement hook (no counterpart in the paper).  While enabled, talon_expand_tree and
 * talon_expand_select_layer record a HIP event on the launch stream before and after every
 * fused scan launch; talon_profile_read waits for them, writes the first `capacity`
 * durations in microseconds (launch order) to the host array `durations_us`, stores the
 * number of launches recorded since the last read in *n_launches and starts over.  Not to
 * be enabled while a stream is being captured into a graph.  Not thread-safe.
 */
int talon_profile_scan_launches(int enable);
int talon_profile_read(float* durations_us, int32_t capacity, int32_t* n_launches);

/*
 * Static tree construction (Alg. 1, the baseline the paper compares with) on the same
 * kernels: call talon_build_tree with init_layers = max_depth = D + 1, K_init = K and a tree
 * state of N = 1 + K*(D+1) nodes (every layer keeps the K best of the K x K pool), then
 * talon_prune_tree, Alg. 1's "final pruning to budget N": the n_keep nodes of highest path
 * confidence are kept (ties: lower node id), compacted in place in their old order, parents
 * re-indexed; n_nodes is updated, the frontier is emptied and DONE_BUDGET is set.
 * kept_ids [B][N_pad] (device) receives the old id of every kept node, -1 beyond.  The mask
 * and attention calls then work on the pruned tree.  Errors: INVALID_ARG.
 */
int talon_prune_tree(const talon_tree_state* st, int32_t n_keep, int32_t* kept_ids, void* stream);

/*
 * Verification outcome at temperature 0 (App. B "Token-Tree Verification", step (2): the
 * longest valid prefix; Sec. 2: "accepting the longest matched prefix").  Three calls.
 *
 * talon_target_argmax: the target model's greedy token after every node of every tree.
 *   logits: device, target logits, row i of sequence b at (b*seq_stride + i*row_stride)
 *   elements (same layout rules as talon_expand_layer, rows by node).  Outputs, device:
 *   target_token [B][N_pad] int32 (largest logit, lowest id among equals; rows >= n_nodes
 *   untouched), target_prob [B][N_pad] float (softmax probability of that token; may be
 *   NULL), scan_status [B] uint32 (TALON_STATUS_BAD_ROW if a row of the sequence held a NaN
 *   or +inf).  One pass of the vocabulary scan with k = 1 over n_nodes rows per sequence.
 *   `workspace`: talon_verify_workspace_bytes bytes of device memory, no initialisation
 *   needed.  Errors as talon_expand_layer.
 *
 * talon_greedy_accept: starting at the root, the child whose drafted token equals the
 *   target's token at the current node is accepted and becomes the current node, until no
 *   child matches.  Outputs, device: path [B][N_pad] int32 (accepted node ids from the root
 *   on, path[b][0] = 0, -1 beyond), accept_len [B] (accepted drafted tokens; the root is not
 *   counted), bonus_token [B] (the target's token after the last accepted node).  A sequence
 *   whose scan_status has BAD_ROW gets that bit in st->status; its outputs are then not
 *   meaningful.
 *
 * talon_compact_kv: the keys and values of the accept_len[b] + 1 nodes on the path (tree
 *   K/V [B][N_pad][Hkv][Dh] bf16) are copied to positions prefix_len[b] + j of the prefix
 *   cache (strided as in talon_tree_attention), new_prefix_len[b] = prefix_len[b] +
 *   accept_len[b] + 1.  Rows that would land at or beyond prefix_capacity are not written and
 *   new_prefix_len is clamped to prefix_capacity.  The caller owns all buffers.
 *   Errors: INVALID_ARG (NULL or misaligned pointers, Dh not a multiple of 8, strides).
 */
size_t talon_verify_workspace_bytes(int32_t B, int32_t N_pad, int32_t vocab, int dtype);
int talon_target_argmax(const void* logits, int dtype, int64_t row_stride, int64_t seq_stride,
                        const talon_tree_state* st, int32_t vocab, int32_t* target_token,
                        float* target_prob, uint32_t* scan_status, void* workspace,
                        size_t workspace_bytes, void* stream);
int talon_greedy_accept(const talon_tree_state* st, const int32_t* target_token,
                        const uint32_t* scan_status, int32_t* path, int32_t* accept_len,
                        int32_t* bonus_token, void* stream);
int talon_compact_kv(const void* k_tree, const void* v_tree, const int32_t* path,
                     const int32_t* accept_len, const int32_t* prefix_len, int32_t* new_prefix_len,
                     void* k_prefix, void* v_prefix, int32_t B, int32_t N_pad, int32_t Hkv,
                     int32_t Dh, int32_t prefix_capacity, int64_t kv_stride_b, int64_t kv_stride_t,
                     int64_t kv_stride_h, void* stream);

/*
 * Attainable-rate probes (no counterpart in the paper), for a second denominator beside the
 * published peaks.  talon_probe_read streams `bytes` of the device buffer `buf` (16-byte
 * aligned) through the vector units once and writes nothing; talon_probe_mfma runs, on
 * `workgroups` workgroups of 4 wavefronts, `iters` rounds of 4 independent
 * v_mfma_f32_32x32x16_bf16 on register operands and stores the FLOP count of the launch in
 * *flops (host, optional).  `sink` is a 4-byte device word that is never actually written.
 * The caller times the launches.  Errors: INVALID_ARG.
 */
int talon_probe_read(const void* buf, size_t bytes, void* sink, void* stream);
int talon_probe_mfma(int32_t workgroups, int32_t iters, void* sink, double* flops, void* stream);

/*
 * Two probes of what a tree-attention step is made of, in cycles of the shader clock (no
 * counterpart in the paper; they back the analysis of that kernel).
 * talon_probe_issue: one workgroup of `waves` (4 or 8: one or two per SIMD) wavefronts; each
 * runs `iters` rounds of instruction mix `mode` (0: 32 independent exp2; 1: 32 independent
 * fma; 2: 16 v_mfma_f32_32x32x16_bf16 over four accumulators; 3: the same over one; 4: 16
 * matrix instructions with 32 (fma, exp2) pairs between them) and stores its cycle count in
 * cycles[wavefront] (device, 8 words).
 * talon_probe_tile_loads: 256 workgroups of `waves` wavefronts; per round every wavefront issues
 * `loads` (4 or 8) direct-to-LDS loads of 1 KB from its workgroup's 64 KB of `window` (device,
 * at least 16 MiB, 16-byte aligned; the windows stay in the L2), with sixteen matrix
 * instructions around them if `with_mfma`, and waits for them; cycles[workgroup * 8 +
 * wavefront] (device, 2048 words) gets the cycles of all `iters` rounds.
 * `sink` as above.  Errors: INVALID_ARG.
 */
int talon_probe_issue(int32_t mode, int32_t waves, int32_t iters, uint64_t* cycles, void* sink, void* stream);
int talon_probe_tile_loads(const void* window, size_t window_bytes, int32_t loads, int32_t with_mfma,
                           int32_t waves, int32_t iters, uint64_t* cycles, void* sink, void* stream);

/*
 * Tree attention mask (Fig. 5(b); App. B): bit j of row i is set iff node j is node i or
 * one of its ancestors, the root included.
 *   mask [B][N_pad][N_pad/64] uint64, bit j of row i = word j/64, bit j%64.
 *   Rows of node ids >= n_nodes[b] and all padding bits are written as zero.
 */
int talon_build_tree_mask(const talon_tree_state* st, uint64_t* mask, void* stream);

/*
 * Scratch for talon_tree_attention (split-KV partial results).  max_prefix_len is the
 * largest prefix length any call will pass.
 */
size_t talon_tree_attention_workspace_bytes(int32_t B, int32_t N_pad, int32_t Hq, int32_t Hkv,
                                            int32_t Dh, int32_t max_prefix_len);

/*
 * One attention layer of the verification forward (App. B): tree node i of sequence b,
 * query head h, attends to the prefix keys 0..prefix_len[b]-1 and to the tree keys j whose
 * mask bit (i, j) is set; KV head = h / (Hq/Hkv).
 *   out[b][i][h][:] = sum_j softmax_j(scale * q[b][i][h] . k_j) v_j
 *
 *   q, k_tree, v_tree  bf16 [B][N_pad][Hq|Hkv][Dh], dense
 *   k_prefix, v_prefix bf16, element (b, t, g, :) at b*kv_stride_b + t*kv_stride_t +
 *                      g*kv_stride_h (strides in elements; the Dh run is contiguous)
 *   mask               as written by talon_build_tree_mask
 *   n_nodes [B], prefix_len [B] int32 (device); prefix_len[b] <= max_prefix_len (host bound
 *                      used to size the launch)
 *   scale              0 means 1/sqrt(Dh)
 *   out                bf16 [B][N_pad][Hq][Dh]; rows of node ids >= n_nodes[b] are untouched
 *   out_lse            optional (NULL to skip) float [B][N_pad][Hq]: natural-log softmax
 *                      denominator of the scaled scores
 *   Arithmetic: bf16 MFMA with fp32 accumulation, fp32 online softmax, probabilities
 *   rounded to bf16 before the P.V product, output rounded to bf16.
 *   Errors: INVALID_ARG, UNSUPPORTED (Dh != 64 and != 128, Hq % Hkv != 0, Hq/Hkv > 16),
 *   WORKSPACE.
 */
int talon_tree_attention(const void* q, const void* k_prefix, const void* v_prefix,
                         const void* k_tree, const void* v_tree, const uint64_t* mask,
                         const int32_t* n_nodes, const int32_t* prefix_len, int32_t B,
                         int32_t N_pad, int32_t Hq, int32_t Hkv, int32_t Dh,
                         int32_t max_prefix_len, int64_t kv_stride_b, int64_t kv_stride_t,
                         int64_t kv_stride_h, float scale, void* out, float* out_lse,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * talon_tree_attention for callers that cannot allocate device memory or pass a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * same call, the same kernels and the same results, with the split-KV partial results kept in
 * a device array that is part of the library itself (talon_static_scratch_bytes() = 32 MiB per
 * GPU, held from the moment the library is loaded on that GPU until the process ends).  The
 * call allocates nothing and frees nothing.
 *   - Shapes whose partial results need more than that (talon_tree_attention_workspace_bytes
 *     says how much) are refused with TALON_ERR_WORKSPACE; nothing is launched then.
 *   - The array's device address is looked up on the first call on a device;
 *     talon_static_scratch_init() does the same lookup ahead of time (call it once per device,
 *     with that device current, before capturing a graph).
 *   - Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two host threads) race and give wrong results.  Calls on one stream are safe.
 *     Nothing in the array has to be zero: a call never reads what an earlier one left.
 * Arguments and all other errors: as talon_tree_attention.
 */
size_t talon_static_scratch_bytes(void);
int talon_static_scratch_init(void);
int talon_tree_attention_static(const void* q, const void* k_prefix, const void* v_prefix,
                                const void* k_tree, const void* v_tree, const uint64_t* mask,
                                const int32_t* n_nodes, const int32_t* prefix_len, int32_t B,
                                int32_t N_pad, int32_t Hq, int32_t Hkv, int32_t Dh,
                                int32_t max_prefix_len, int64_t kv_stride_b, int64_t kv_stride_t,
                                int64_t kv_stride_h, float scale, void* out, float* out_lse,
                                void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TALON_H_ */
