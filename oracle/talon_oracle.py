"""CPU oracle for the Talon draft-tree expansion and tree-attention verification.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Plain, slow, float64 numpy written from
the paper (arXiv 2601.07353).  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may import this file; the GPU library shares no
code with it and never calls it.

What each function follows:
  softmax_stats        the draft model's next-token distribution P(.|x<=v) is the
                       softmax of its logits (Sec. 3.2, "next-token distributions")
  row_candidates       Top-K of one parent's distribution (Eq. 5; Alg. 2 "Robust Init")
  expand_layer         candidate pool S_d with path scores p(u) = p(v) * P(w|x<=v)
                       (Eq. 3 and the sentence after it; Alg. 2 "Gather" loop)
  select_budget        hybrid strategy: Top-K at d < init_layers (Eq. 5), else anchor
                       m_d = max p(u) and gate p(u) >= mu * m_d (Eq. 4), then the
                       budget check Top-(N-|T|) (Sec. 5.2.1 last sentence; Alg. 2
                       "Budget Check")
  build_tree           the while |T| < N loop of Alg. 2
  build_tree_mask      each tree token sees its root-to-node path (Fig. 5(b), App. B)
  tree_attention       one attention layer under that mask plus the whole prefix
                       (App. B "Tree Attention")
  target_argmax        the target model's greedy token after each tree node (temperature 0)
  greedy_accept        verification at temperature 0: the longest root path on which every
                       drafted token is the target's own choice ("accepting the longest
                       matched prefix", Sec. 2; App. B step (2), "selecting the optimal
                       valid prefix"); the token after it comes from the target
  compact_kv           the accepted tokens' keys and values join the prefix cache
  build_static_tree    the static baseline the paper compares with (Alg. 1): every layer keeps
                       the K best of the K x K pool, D + 1 layers, then the N best nodes overall
  prune_top_n          Alg. 1's last step, "final pruning to budget N"

Readings taken where the paper is silent (each also listed in the design notes):
  * per-row candidate cap `cap`: the pool of a parent is its `cap` best tokens.
    cap = V is the pool exactly as Alg. 2 writes it; any cap >= N - |T| gives the
    same tree (a global top-R never takes more than R children of one parent and
    the gate keeps an upper set).
  * N counts the root (Alg. 2 starts from T = {x_t} and loops while |T| < N).
  * Dmax: optional cap on the number of layers (not in the paper; safety bound).
  * ties: inside a row (logit desc, token id asc); across the pool
    (score desc, parent node id asc, in-row rank asc).
  * node ids: layer-major; inside a layer (parent id asc, in-row rank asc).
  * scores are compared in the log domain: log p(u) = log p(v) + (logit_w - lse_v),
    gate log p(u) >= log mu + log m_d.  Monotone-equivalent to Eq. 4.
  * P(w|x<=v) is the softmax over the full row (no renormalisation over the cap).
  * mask: ancestor-or-self, root included; every node also sees the whole prefix.
  * attention scale 1/sqrt(Dh) unless given.

Pins (tests/test_oracle_pins.py): scipy logsumexp/softmax, a full Python sort,
brute-force enumeration of every admissible layer and tree on tiny instances,
closed-form special cases (mu = 1 chain, mu -> 0 plain top-R, star tree, one-hot
and constant rows), a hand-worked example in tests/golden/, parent-walk masks,
and per-path causal attention through torch's scaled_dot_product_attention.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Callable, List, Optional

import numpy as np


# --------------------------------------------------------------------------
# a1 / a2: per-row softmax statistics and ranked candidates
# --------------------------------------------------------------------------
def softmax_stats(row: np.ndarray):
    """max and log-sum-exp of one logits row (float64)."""
    row = np.asarray(row, dtype=np.float64)
    if np.isnan(row).any():
        raise ValueError("NaN logit")
    mx = float(np.max(row))
    if not math.isfinite(mx):
        raise ValueError("row has no finite maximum")
    lse = mx + math.log(float(np.sum(np.exp(row - mx))))
    return mx, lse


def row_candidates(row: np.ndarray, cap: int) -> np.ndarray:
    """Token ids of the `cap` largest logits, ordered (logit desc, token id asc)."""
    row = np.asarray(row, dtype=np.float64)
    V = row.shape[0]
    order = np.lexsort((np.arange(V), -row))  # primary key last: -logit, then token id
    return order[: min(cap, V)].astype(np.int64)


@dataclass
class RowResult:
    node: int                 # parent node id v
    row_max: float
    row_lse: float
    token: np.ndarray         # [c] candidate token ids
    logit: np.ndarray         # [c] their logits
    edge_logp: np.ndarray     # [c] logit - lse  = log P(w | x<=v)
    prob: np.ndarray          # [c] P(w | x<=v)
    score: np.ndarray         # [c] log p(u) = log p(v) + edge_logp


def expand_layer(frontier: List[int], logp: List[float],
                 row_of: Callable[[int], np.ndarray], cap: int) -> List[RowResult]:
    """Candidate pool of one layer: for each parent v its `cap` best (v, w) with scores."""
    out = []
    for v in frontier:
        row = np.asarray(row_of(v), dtype=np.float64)
        mx, lse = softmax_stats(row)
        tok = row_candidates(row, cap)
        lg = row[tok]
        edge = lg - lse
        out.append(RowResult(node=v, row_max=mx, row_lse=lse, token=tok, logit=lg,
                             edge_logp=edge, prob=np.exp(edge), score=logp[v] + edge))
    return out


# --------------------------------------------------------------------------
# a3 / a4: hybrid allocation of the remaining budget
# --------------------------------------------------------------------------
@dataclass
class Selection:
    kept: list                 # [(parent, rank)] in (parent asc, rank asc) order
    anchor: float              # m_d in the log domain (max score of the pool)
    n_pass: int                # candidates that passed the gate (or pool size at init)
    cut: bool                  # True when the budget check trimmed the layer
    margin: float              # smallest cross-parent score gap that decided anything


def _cross_parent_margin(kept, dropped):
    """Smallest score gap between a kept and a dropped candidate of different parents.

    Candidates of one parent are ordered by their logits alone, which every
    arithmetic reproduces exactly, so only cross-parent pairs can be decided
    differently by an implementation whose log-sum-exp is rounded differently.
    """
    if not kept or not dropped:
        return math.inf
    lo = min(s for s, _, _ in kept)
    hi = max(s for s, _, _ in dropped)
    if lo - hi > 1.0:
        return lo - hi
    best = math.inf
    for sk, pk, _ in kept:
        if sk - hi > best:
            continue
        for sd, pd, _ in dropped:
            if pk != pd:
                best = min(best, abs(sk - sd))
    return best


def select_budget(pool: List[RowResult], layer: int, R: int, K: int, mu: float,
                  init_layers: int = 1) -> Selection:
    """Choose the next layer P_{d+1} from the pool S_d.

    layer < init_layers : Top-K of the pool by path score (Eq. 5).
    otherwise           : keep score >= log(mu) + anchor (Eq. 4).
    Then, if more than R = N - |T| candidates remain, keep the R best (budget check).
    """
    cands = []  # (score, parent, rank)
    for r in pool:
        for j in range(len(r.token)):
            cands.append((float(r.score[j]), r.node, j))
    ordered = sorted(cands, key=lambda u: (-u[0], u[1], u[2]))
    anchor = ordered[0][0]
    margin = math.inf
    if layer < init_layers:
        survivors = ordered[:K]
        gate_dropped = ordered[K:]
        margin = min(margin, _cross_parent_margin(survivors, gate_dropped))
    else:
        thr = math.log(mu) + anchor
        survivors = [u for u in ordered if u[0] >= thr]
        gate_dropped = [u for u in ordered if not (u[0] >= thr)]
        for u in ordered:
            if u[0] != anchor and math.isfinite(u[0]):
                margin = min(margin, abs(u[0] - thr))
    n_pass = len(survivors)
    cut = n_pass > R
    if cut:
        margin = min(margin, _cross_parent_margin(survivors[:R], survivors[R:]))
        survivors = survivors[:R]
    kept = sorted([(p, j) for _, p, j in survivors])
    return Selection(kept=kept, anchor=anchor, n_pass=n_pass, cut=cut, margin=margin)


# --------------------------------------------------------------------------
# a5: Alg. 2, the budget-driven loop
# --------------------------------------------------------------------------
@dataclass
class Tree:
    token: List[int] = field(default_factory=list)
    parent: List[int] = field(default_factory=list)
    depth: List[int] = field(default_factory=list)
    prob: List[float] = field(default_factory=list)    # edge probability; root = 1
    logp: List[float] = field(default_factory=list)    # log path confidence; root = 0
    layers: List[range] = field(default_factory=list)  # node-id range of each layer
    pools: List[List[RowResult]] = field(default_factory=list)
    selections: List[Selection] = field(default_factory=list)
    exit_reason: str = ""                              # "budget" | "depth"
    margin: float = math.inf

    @property
    def n(self) -> int:
        return len(self.token)

    def confidence(self) -> np.ndarray:
        return np.exp(np.asarray(self.logp, dtype=np.float64))


def build_tree(row_of: Callable[[int], np.ndarray], root_token: int, N: int, K: int,
               mu: float, cap: Optional[int] = None, Dmax: Optional[int] = None,
               init_layers: int = 1) -> Tree:
    """Alg. 2: grow the draft tree layer by layer until |T| = N (or Dmax layers).

    row_of(i) returns the draft logits row for node id i (the row the draft model
    emits when node i is the last token of its path).
    """
    if not (0.0 < mu <= 1.0):
        raise ValueError("mu must lie in (0, 1]")
    cap = K if cap is None else cap
    t = Tree(token=[root_token], parent=[-1], depth=[0], prob=[1.0], logp=[0.0])
    t.layers.append(range(0, 1))
    frontier = [0]
    d = 0
    while t.n < N and (Dmax is None or d < Dmax):
        pool = expand_layer(frontier, t.logp, row_of, cap)
        sel = select_budget(pool, d, N - t.n, K, mu, init_layers)
        by_node = {r.node: r for r in pool}
        begin = t.n
        for (v, j) in sel.kept:
            r = by_node[v]
            t.token.append(int(r.token[j]))
            t.parent.append(v)
            t.depth.append(t.depth[v] + 1)
            t.prob.append(float(r.prob[j]))
            t.logp.append(float(r.score[j]))
        t.layers.append(range(begin, t.n))
        t.pools.append(pool)
        t.selections.append(sel)
        t.margin = min(t.margin, sel.margin)
        frontier = list(range(begin, t.n))
        d += 1
    t.exit_reason = "budget" if t.n >= N else "depth"
    return t


# --------------------------------------------------------------------------
# a6: tree attention mask
# --------------------------------------------------------------------------
def build_tree_mask(parent: List[int]) -> np.ndarray:
    """Boolean [n][n]: entry (i, j) is True iff j is i or an ancestor of i."""
    n = len(parent)
    m = np.zeros((n, n), dtype=bool)
    for i in range(n):
        if parent[i] >= 0:
            m[i] = m[parent[i]]
        m[i, i] = True
    return m


def mask_to_words(mask: np.ndarray, N_pad: int) -> np.ndarray:
    """Pack a boolean [n][n] mask into uint64 words [N_pad][N_pad/64], bit j of word j//64."""
    n = mask.shape[0]
    words = np.zeros((N_pad, N_pad // 64), dtype=np.uint64)
    for i in range(n):
        for j in range(n):
            if mask[i, j]:
                words[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
    return words


# --------------------------------------------------------------------------
# a7: tree attention
# --------------------------------------------------------------------------
def tree_attention(q: np.ndarray, k_prefix: np.ndarray, v_prefix: np.ndarray,
                   k_tree: np.ndarray, v_tree: np.ndarray, mask: np.ndarray,
                   scale: Optional[float] = None, nodes=None, heads=None):
    """Attention of every tree node over the prefix plus the tree keys its mask allows.

    q [n][Hq][Dh], k_prefix/v_prefix [L][Hkv][Dh], k_tree/v_tree [n][Hkv][Dh] (float64),
    mask boolean [n][n].  Query head h reads KV head h // (Hq // Hkv).
    Returns (out [n][Hq][Dh], lse [n][Hq]); `nodes` / `heads` restrict the work to
    a subset (other entries stay NaN).
    """
    n, Hq, Dh = q.shape
    Hkv = k_prefix.shape[1]
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(Dh) if scale is None else scale
    out = np.full((n, Hq, Dh), np.nan)
    lse = np.full((n, Hq), np.nan)
    for i in (range(n) if nodes is None else nodes):
        vis = np.nonzero(mask[i])[0]
        for g in range(Hkv):
            group = [h for h in range(g * G, (g + 1) * G) if heads is None or h in heads]
            if not group:
                continue
            keys = np.concatenate([k_prefix[:, g, :], k_tree[vis, g, :]], axis=0)
            vals = np.concatenate([v_prefix[:, g, :], v_tree[vis, g, :]], axis=0)
            for h in group:
                s = (keys @ q[i, h]) * scale
                mx = np.max(s)
                e = np.exp(s - mx)
                z = np.sum(e)
                out[i, h] = (e / z) @ vals
                lse[i, h] = mx + math.log(z)
    return out, lse


# --------------------------------------------------------------------------
# verification outcome at temperature 0 (greedy): acceptance walk and cache update
# --------------------------------------------------------------------------
def target_argmax(row: np.ndarray) -> int:
    """Greedy token of one target-logits row: the largest logit, lowest id among equals
    (-0.0 equals +0.0)."""
    x = np.asarray(row, dtype=np.float64) + 0.0
    return int(np.argmax(x))   # numpy returns the first (lowest-id) maximum


def greedy_accept(token: List[int], parent: List[int], target_token: List[int]):
    """Longest accepted path of a draft tree at temperature 0.

    token[i], parent[i]: the tree (node 0 is the root, the last verified token);
    target_token[i]: the target's greedy token after node i.  Starting at the root, the
    child whose drafted token equals the target's token at the current node is accepted and
    becomes the current node; the walk stops where no child matches.  Returns
    (path, bonus): the accepted node ids from the root on (the root is always on it), and the
    target's token after the last accepted node (the token this step emits on top).
    """
    n = len(token)
    path = [0]
    cur = 0
    while True:
        want = target_token[cur]
        nxt = [c for c in range(n) if parent[c] == cur and token[c] == want]
        if not nxt:
            break
        cur = nxt[0]          # siblings carry distinct tokens: at most one can match
        path.append(cur)
    return path, int(target_token[cur])


def compact_kv(cache: np.ndarray, tree: np.ndarray, path: List[int], prefix_len: int) -> int:
    """Append the rows of `tree` [n][...] on the accepted path to `cache` [cap][...] at
    positions prefix_len, prefix_len + 1, ... (in place); returns the new prefix length."""
    for j, node in enumerate(path):
        cache[prefix_len + j] = tree[node]
    return prefix_len + len(path)


# --------------------------------------------------------------------------
# Alg. 1: the static (EAGLE-style) tree, as a second workload for the same kernels
# --------------------------------------------------------------------------
@dataclass
class PrunedTree:
    token: List[int]
    parent: List[int]          # re-indexed
    depth: List[int]
    prob: List[float]
    logp: List[float]
    kept: List[int]            # ids the nodes had before pruning, ascending
    margin: float              # smallest gap between a kept and a dropped node of different parents

    @property
    def n(self) -> int:
        return len(self.token)


def prune_top_n(tree: Tree, N: int) -> PrunedTree:
    """T <- Top-N(T by p(u)) (Alg. 1, last step).  Order: (path confidence descending, node
    id ascending); a node's confidence never exceeds its parent's and the parent has the
    smaller id, so the kept set is closed under "parent of".  Kept nodes keep their relative
    order and are renumbered 0..N-1."""
    n = tree.n
    order = sorted(range(n), key=lambda i: (-tree.logp[i], i))
    kept = sorted(order[:N])
    dropped = order[N:]
    margin = math.inf
    for i in kept:
        for j in dropped:
            if tree.parent[i] != tree.parent[j]:
                margin = min(margin, abs(tree.logp[i] - tree.logp[j]))
    new_id = {old: new for new, old in enumerate(kept)}
    return PrunedTree(token=[tree.token[i] for i in kept],
                      parent=[-1 if tree.parent[i] < 0 else new_id[tree.parent[i]] for i in kept],
                      depth=[tree.depth[i] for i in kept], prob=[tree.prob[i] for i in kept],
                      logp=[tree.logp[i] for i in kept], kept=kept, margin=margin)


def build_static_tree(row_of: Callable[[int], np.ndarray], root_token: int, D: int, K: int, N: int):
    """Alg. 1: for d = 0..D every parent proposes its K best tokens, the K best of the pool (by
    path confidence) become the next parents and join the tree; at the end the N best nodes
    of the tree are kept.  Returns (the tree before pruning, the pruned tree).  row_of(i) is
    the draft row of node i in the numbering before pruning."""
    full = build_tree(row_of, root_token, N=1 + K * (D + 1), K=K, mu=1.0, cap=K, Dmax=D + 1,
                      init_layers=D + 1)
    return full, prune_top_n(full, N)
