"""Pins for the CPU oracle: every check here compares the oracle with something
other than itself: a library routine, a closed form, a hand-worked example, or
brute-force enumeration written independently in the probability domain."""
import itertools
import json
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import talon_oracle as O
from workloads import CONFIGS, bf16_bits_to_f64, f32_to_bf16_bits, logits_row, storage_to_f64, zipf_row

HERE = os.path.dirname(os.path.abspath(__file__))


def rows_from_probs(rows_prob):
    return {int(k): np.log(np.asarray(v, dtype=np.float64)) for k, v in rows_prob.items()}


def random_rows(rng, n_rows, V, beta_lo=0.5, beta_hi=4.0):
    return {i: rng.normal(size=V) * rng.uniform(beta_lo, beta_hi) for i in range(n_rows)}


# ---------------------------------------------------------------- softmax / lse
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_softmax_stats_vs_scipy(seed):
    rng = np.random.default_rng(seed)
    row = rng.normal(size=5000) * rng.uniform(0.5, 8.0)
    mx, lse = O.softmax_stats(row)
    assert mx == row.max()
    assert abs(lse - scipy.special.logsumexp(row)) < 1e-12
    p = np.exp(row - lse)
    assert abs(p.sum() - 1.0) < 1e-12
    np.testing.assert_allclose(p, scipy.special.softmax(row), rtol=1e-12, atol=0)


def test_softmax_stats_shift_invariance_and_large_logits():
    row = np.array([1000.0, 999.0, 998.0])
    _, lse = O.softmax_stats(row)
    assert abs(lse - (1000.0 + math.log(1 + math.exp(-1) + math.exp(-2)))) < 1e-12
    _, lse0 = O.softmax_stats(row - 1000.0)
    assert abs((lse - 1000.0) - lse0) < 1e-12


def test_softmax_stats_uniform_closed_form():
    _, lse = O.softmax_stats(np.full(1024, 3.25))
    assert abs(lse - (3.25 + math.log(1024))) < 1e-12


# ---------------------------------------------------------------- row top-k + ties
@pytest.mark.parametrize("seed", [0, 1])
def test_row_candidates_vs_python_sort(seed):
    rng = np.random.default_rng(seed)
    row = np.round(rng.normal(size=300) * 2.0, 1)  # coarse grid: many ties
    want = sorted(range(300), key=lambda w: (-row[w], w))
    for k in (1, 2, 7, 300, 999):
        got = O.row_candidates(row, k)
        assert list(got) == want[: min(k, 300)]


def test_row_candidates_all_equal_and_signed_zero():
    assert list(O.row_candidates(np.zeros(50), 5)) == [0, 1, 2, 3, 4]
    row = np.array([-0.0, 0.0, -1.0, 0.0, -0.0])
    assert list(O.row_candidates(row, 4)) == [0, 1, 3, 4]  # -0.0 == +0.0: id order


def test_row_candidates_vs_torch_topk_no_ties():
    rng = np.random.default_rng(5)
    row = rng.normal(size=4096)
    got = O.row_candidates(row, 16)
    want = torch.topk(torch.from_numpy(row), 16).indices.numpy()
    assert list(got) == list(want)


def test_row_candidates_bf16_zipf_ties_ascending_ids():
    x = bf16_bits_to_f64(f32_to_bf16_bits(zipf_row(5000, 1.2, 7, 3)))
    got = O.row_candidates(x, 400)
    vals = x[got]
    assert np.all(np.diff(vals) <= 0)
    for a, b in zip(range(399), range(1, 400)):
        if vals[a] == vals[b]:
            assert got[a] < got[b]
    assert len(np.unique(vals)) < 400  # the rounded tail really has ties


# ---------------------------------------------------------------- hand-worked example
@pytest.mark.parametrize("case,N", [("N6", 6), ("N5", 5)])
def test_worked_example(case, N):
    g = json.load(open(os.path.join(HERE, "golden", "worked_example.json")))
    rows = rows_from_probs(g["rows_prob"])
    t = O.build_tree(lambda i: rows[i], g["root_token"], N=N, K=g["K"], mu=g["mu"], cap=g["cap"])
    e = g["expected"][case]
    assert t.token == e["token"]
    assert t.parent == e["parent"]
    assert t.depth == e["depth"]
    np.testing.assert_allclose(t.confidence(), e["confidence"], rtol=1e-12)
    m = O.build_tree_mask(t.parent)
    for i, row in enumerate(e["mask_rows"]):
        assert list(np.nonzero(m[i])[0]) == row
    assert t.exit_reason == "budget"


# ---------------------------------------------------------------- brute force: one layer
def brute_force_layer(cands_p, R, mu, init, K):
    """cands_p: list of path probabilities (distinct).  Returns the index set the rule fixes:
    among all subsets A with |A| <= limit whose members all pass the gate and whose size is
    maximal, the one with the largest total probability."""
    n = len(cands_p)
    if init:
        passing = list(range(n))
        limit = min(K, R)
    else:
        m = max(cands_p)
        passing = [i for i in range(n) if cands_p[i] >= mu * m]
        limit = R
    size = min(limit, len(passing))
    best, best_sum = None, -1.0
    for A in itertools.combinations(passing, size):
        s = sum(cands_p[i] for i in A)
        if s > best_sum:
            best, best_sum = set(A), s
    return best


@pytest.mark.parametrize("seed", range(12))
def test_select_budget_vs_bruteforce_layer(seed):
    rng = np.random.default_rng(100 + seed)
    V, cap = 5, 3
    F = int(rng.integers(1, 4))
    parents = list(range(10, 10 + F))
    logp = {v: math.log(rng.uniform(0.05, 1.0)) for v in parents}
    rows = {v: rng.normal(size=V) * rng.uniform(0.5, 3.0) for v in parents}
    mu = float(rng.choice([0.03, 0.2, 0.6, 1.0]))
    R = int(rng.integers(1, 8))
    K = int(rng.integers(1, 4))
    for init in (False, True):
        pool = O.expand_layer(parents, logp, lambda v: rows[v], cap)
        sel = O.select_budget(pool, 0 if init else 1, R, K, mu, init_layers=1)
        # independent scoring in the probability domain
        flat = []
        for v in parents:
            p = scipy.special.softmax(rows[v])
            top = sorted(range(V), key=lambda w: (-p[w], w))[:cap]
            for j, w in enumerate(top):
                flat.append(((v, j), math.exp(logp[v]) * p[w]))
        want = brute_force_layer([x[1] for x in flat], R, mu, init, K)
        got = {i for i, (key, _) in enumerate(flat) if key in set(sel.kept)}
        assert got == want


# ---------------------------------------------------------------- decision margin
def _random_layer(rng):
    """A random pool: F parents with path confidences and rows close enough together that
    cross-parent comparisons are tight."""
    V = int(rng.integers(4, 9))
    cap = int(rng.integers(1, V + 1))
    F = int(rng.integers(1, 6))
    parents = list(range(20, 20 + F))
    logp = {v: math.log(rng.uniform(0.2, 1.0)) for v in parents}
    spread = float(rng.choice([0.05, 0.5, 3.0]))
    rows = {v: rng.normal(size=V) * spread for v in parents}
    return parents, logp, rows, cap


@pytest.mark.parametrize("seed", range(40))
def test_margin_is_the_all_pairs_minimum(seed):
    """The margin the oracle reports (and the test harness selects seeds by) against its
    definition written out: over every (kept, dropped) pair of candidates of DIFFERENT parents
    the smallest score gap at the top-K / budget cut, and over every candidate other than the
    anchor the distance to the gate threshold.  The oracle's own routine prunes and exits early;
    this one looks at all pairs."""
    rng = np.random.default_rng(7000 + seed)
    parents, logp, rows, cap = _random_layer(rng)
    mu = float(rng.choice([0.03, 0.3, 0.8, 1.0]))
    R = int(rng.integers(1, 12))
    K = int(rng.integers(1, 6))
    for layer in (0, 1):
        pool = O.expand_layer(parents, logp, lambda v: rows[v], cap)
        sel = O.select_budget(pool, layer, R, K, mu, init_layers=1)
        cands = [(float(r.score[j]), r.node, j) for r in pool for j in range(len(r.token))]
        ordered = sorted(cands, key=lambda u: (-u[0], u[1], u[2]))

        def all_pairs(kept, dropped):
            gaps = [abs(a[0] - b[0]) for a in kept for b in dropped if a[1] != b[1]]
            return min(gaps) if gaps else math.inf

        want = math.inf
        if layer == 0:
            survivors = ordered[:K]
            want = min(want, all_pairs(survivors, ordered[K:]))
        else:
            anchor = ordered[0][0]
            thr = math.log(mu) + anchor
            survivors = [u for u in ordered if u[0] >= thr]
            for u in ordered:
                if u[0] != anchor:
                    want = min(want, abs(u[0] - thr))
        if len(survivors) > R:
            want = min(want, all_pairs(survivors[:R], survivors[R:]))
        # the routine may answer early with the gap between the lowest kept and the highest
        # dropped score when that gap exceeds 1: a lower bound of the all-pairs minimum
        if sel.margin > 1.0 and want > 1.0:
            assert sel.margin <= want
        else:
            assert sel.margin == want, (layer, sel.margin, want)


@pytest.mark.parametrize("seed", range(40))
def test_margin_means_what_the_harness_needs(seed):
    """What the margin promises: if every row's log-sum-exp is off by less than half the margin
    (each row by its own amount, as another arithmetic's rounding would be), the layer keeps
    exactly the same candidates.  (That the margin is not smaller than it has to be is the
    equality with the all-pairs minimum above.)"""
    rng = np.random.default_rng(9000 + seed)
    parents, logp, rows, cap = _random_layer(rng)
    mu = float(rng.choice([0.03, 0.3, 0.8]))
    R = int(rng.integers(1, 12))
    K = int(rng.integers(1, 6))
    for layer in (0, 1):
        pool = O.expand_layer(parents, logp, lambda v: rows[v], cap)
        sel = O.select_budget(pool, layer, R, K, mu, init_layers=1)
        if not math.isfinite(sel.margin) or sel.margin < 1e-9:
            continue
        for trial in range(10):
            shift = {v: rng.uniform(-0.49, 0.49) * min(sel.margin, 10.0) for v in parents}
            moved = [O.RowResult(node=r.node, row_max=r.row_max, row_lse=r.row_lse - shift[r.node], token=r.token,
                                 logit=r.logit, edge_logp=r.edge_logp + shift[r.node], prob=r.prob,
                                 score=r.score + shift[r.node]) for r in pool]
            assert O.select_budget(moved, layer, R, K, mu, init_layers=1).kept == sel.kept


# ---------------------------------------------------------------- brute force: whole tree
def enumerate_trees(V, max_nodes, max_depth):
    """Every prefix-closed set of token paths (tuples) with <= max_nodes paths, depth <= max_depth."""
    all_paths = []
    for d in range(1, max_depth + 1):
        all_paths += list(itertools.product(range(V), repeat=d))
    out = []

    def rec(start, chosen):
        out.append(frozenset(chosen))
        if len(chosen) == max_nodes:
            return
        for idx in range(start, len(all_paths)):
            p = all_paths[idx]
            if len(p) == 1 or p[:-1] in chosen:
                chosen.add(p)
                rec(idx + 1, chosen)
                chosen.discard(p)

    rec(0, set())
    return out


def path_prob(path, row_for_path):
    p = 1.0
    for d in range(len(path)):
        p *= row_for_path(path[:d])[path[d]]
    return p


def admissible(tree_paths, V, N, K, mu, Dmax, row_for_path):
    """Declarative check of Alg. 2 with the uncapped pool S_d = P_d x V (probability domain)."""
    layers = {}
    for p in tree_paths:
        layers.setdefault(len(p), set()).add(p)
    depth = max(layers) if layers else 0
    if sorted(layers) != list(range(1, depth + 1)):
        return False
    total = 1
    parents = {()}
    for d in range(0, depth + 1):
        if total >= N or d >= Dmax:
            return d == depth  # must have stopped exactly here
        if d == depth:
            return False  # budget and depth left but the tree stopped
        pool = {v + (w,): path_prob(v + (w,), row_for_path) for v in parents for w in range(V)}
        R = N - total
        if d == 0:
            ranked = sorted(pool, key=lambda u: -pool[u])
            passing = set(ranked[:K])
        else:
            m = max(pool.values())
            passing = {u for u in pool if pool[u] >= mu * m}
        layer = layers[d + 1]
        if not layer <= passing:
            return False
        if len(passing) <= R:
            if layer != passing:
                return False
        else:
            if len(layer) != R:
                return False
            if min(pool[u] for u in layer) < max(pool[u] for u in passing - layer):
                return False
        total += len(layer)
        parents = layer
    return True


@pytest.mark.parametrize("seed", range(6))
def test_build_tree_vs_bruteforce_enumeration(seed):
    rng = np.random.default_rng(200 + seed)
    V, N, K, Dmax = 3, 6, 2, 3
    mu = float(rng.choice([0.05, 0.3, 0.7]))
    cache = {}

    def row_for_path(path):
        if path not in cache:
            cache[path] = scipy.special.softmax(rng.normal(size=V) * rng.uniform(0.5, 3.0))
        return cache[path]

    trees = enumerate_trees(V, N - 1, Dmax)
    ok = [t for t in trees if admissible(t, V, N, K, mu, Dmax, row_for_path)]
    assert len(ok) == 1
    # the oracle addresses rows by node id: give it the row of that node's path
    node_path = {0: ()}

    class Rows:
        def __init__(self):
            self.tree = None

    def run(cap):
        # node ids are assigned during construction; resolve paths lazily via a closure on t
        paths = {0: ()}
        state = {"t": None}

        def row_of(i):
            return np.log(row_for_path(paths[i]))

        # build layer by layer so that paths of new nodes are known before their rows are read
        t = O.Tree(token=[-1], parent=[-1], depth=[0], prob=[1.0], logp=[0.0])
        frontier, d = [0], 0
        while t.n < N and d < Dmax:
            pool = O.expand_layer(frontier, t.logp, row_of, cap)
            sel = O.select_budget(pool, d, N - t.n, K, mu, 1)
            by = {r.node: r for r in pool}
            begin = t.n
            for v, j in sel.kept:
                paths[t.n] = paths[v] + (int(by[v].token[j]),)
                t.token.append(int(by[v].token[j])); t.parent.append(v)
                t.depth.append(t.depth[v] + 1); t.prob.append(float(by[v].prob[j]))
                t.logp.append(float(by[v].score[j]))
            frontier = list(range(begin, t.n)); d += 1
        return frozenset(p for p in paths.values() if p)

    assert run(cap=V) == ok[0]          # pool exactly as Alg. 2 writes it
    assert run(cap=N - 1) == ok[0]      # any cap >= remaining budget gives the same tree


def test_build_tree_loop_matches_manual_layering():
    """build_tree is expand_layer + select_budget in a loop: same result as stepping by hand."""
    rng = np.random.default_rng(7)
    rows = random_rows(rng, 40, 64)
    t = O.build_tree(lambda i: rows[i], 3, N=20, K=4, mu=0.1, Dmax=8)
    n, frontier, logp = 1, [0], [0.0]
    parent = [-1]
    for d in range(len(t.layers) - 1):
        pool = O.expand_layer(frontier, logp, lambda i: rows[i], 4)
        sel = O.select_budget(pool, d, 20 - n, 4, 0.1)
        by = {r.node: r for r in pool}
        for v, j in sel.kept:
            parent.append(v); logp.append(float(by[v].score[j]))
        frontier = list(range(n, len(parent))); n = len(parent)
    assert parent == t.parent
    assert logp == t.logp


@pytest.mark.parametrize("seed", range(8))
def test_capped_pool_equals_uncapped_when_cap_covers_budget(seed):
    rng = np.random.default_rng(300 + seed)
    V, N = 40, 14
    rows = random_rows(rng, N, V)
    mu = float(rng.choice([0.01, 0.03, 0.2]))
    full = O.build_tree(lambda i: rows[i], 0, N=N, K=3, mu=mu, cap=V)
    capd = O.build_tree(lambda i: rows[i], 0, N=N, K=3, mu=mu, cap=N - 1)
    assert full.token == capd.token and full.parent == capd.parent
    np.testing.assert_allclose(full.logp, capd.logp, rtol=0, atol=0)


# ---------------------------------------------------------------- special cases -> textbook
def test_mu_one_gives_topk_then_greedy_chain():
    rng = np.random.default_rng(11)
    V, N, K = 200, 12, 4
    rows = random_rows(rng, N, V)
    t = O.build_tree(lambda i: rows[i], 0, N=N, K=K, mu=1.0)
    root_top = list(np.argsort(-rows[0], kind="stable")[:K])
    assert t.token[1:K + 1] == root_top and t.parent[1:K + 1] == [0] * K
    # layer 2: the single best (parent, token) by p(v) * P(w|v); afterwards argmax chain
    p0 = scipy.special.softmax(rows[0])
    best = max(((p0[t.token[v]] * scipy.special.softmax(rows[v]).max(), v) for v in range(1, K + 1)))
    assert t.parent[K + 1] == best[1]
    for i in range(K + 1, N):
        assert t.token[i] == int(np.argmax(rows[t.parent[i]]))
        if i > K + 1:
            assert t.parent[i] == i - 1
    assert max(t.depth) == N - K
    assert t.n == N


def test_mu_tiny_gives_plain_top_R_each_layer():
    rng = np.random.default_rng(12)
    V, N, K = 50, 30, 3
    rows = random_rows(rng, N, V)
    t = O.build_tree(lambda i: rows[i], 0, N=N, K=K, mu=1e-30)
    for d, layer in enumerate(t.layers[1:]):
        parents = list(t.layers[d])
        R = N - layer.start
        scored = []
        for v in parents:
            p = scipy.special.softmax(rows[v])
            top = np.argsort(-p, kind="stable")[:K]
            scored += [(t.confidence()[v] * p[w], v, int(w)) for w in top]
        limit = min(K, R) if d == 0 else min(R, len(scored))
        want = sorted(sorted(scored, key=lambda s: -s[0])[:limit], key=lambda s: (s[1],))
        got = [(t.parent[i], t.token[i]) for i in layer]
        assert sorted(got) == sorted((v, w) for _, v, w in want)


def test_star_tree_when_K_covers_budget():
    rng = np.random.default_rng(13)
    V, N = 500, 9
    rows = random_rows(rng, N, V)
    t = O.build_tree(lambda i: rows[i], 0, N=N, K=N - 1, mu=0.03)
    p = torch.softmax(torch.from_numpy(rows[0]), dim=0)
    top = torch.topk(p, N - 1)
    assert t.token[1:] == top.indices.tolist()
    np.testing.assert_allclose(t.prob[1:], top.values.numpy(), rtol=1e-12)
    assert t.parent[1:] == [0] * (N - 1) and t.depth[1:] == [1] * (N - 1)


def test_k_init_larger_than_budget_takes_remaining():
    rng = np.random.default_rng(14)
    rows = random_rows(rng, 4, 100)
    t = O.build_tree(lambda i: rows[i], 0, N=4, K=10, mu=0.03)
    assert t.n == 4 and t.parent[1:] == [0, 0, 0]
    assert t.token[1:] == list(np.argsort(-rows[0], kind="stable")[:3])


def test_peaked_rows_deep_narrow_and_flat_rows_shallow_wide():
    """The two shapes of Sec. 5.2.1 'Intuition'."""
    V, N, K = 1000, 20, 5
    peaked = np.zeros(V); peaked[123] = 40.0
    t = O.build_tree(lambda i: peaked, 0, N=N, K=K, mu=0.03)
    assert t.n == N and max(t.depth) == N - K  # K init nodes then a chain of the dominant token
    assert all(t.token[i] == 123 for i in range(K + 1, N))
    flat = np.zeros(V)
    t = O.build_tree(lambda i: flat, 0, N=N, K=K, mu=0.03)
    assert t.n == N and max(t.depth) == 2      # budget is spent at the second layer
    assert t.token[1:K + 1] == [0, 1, 2, 3, 4]   # all tied: lowest ids
    # every candidate ties; budget cut keeps (parent asc, rank asc)
    assert t.parent[K + 1:] == [1] * 5 + [2] * 5 + [3] * 4
    assert t.token[K + 1:] == [0, 1, 2, 3, 4] * 2 + [0, 1, 2, 3]


# ---------------------------------------------------------------- structural invariants
@pytest.mark.parametrize("cfg_name,V", [("c1", None), ("c2", 4096), ("c5", 4096)])
def test_tree_invariants_on_workload_rows(cfg_name, V):
    import dataclasses
    cfg = CONFIGS[cfg_name]
    if V is not None:
        cfg = dataclasses.replace(cfg, V=V)
    for b in range(min(cfg.B, 2)):
        rows = {}

        def row_of(i):
            if i not in rows:
                rows[i] = storage_to_f64(logits_row(cfg, cfg.seed, b, i))
            return rows[i]

        t = O.build_tree(row_of, 1, N=cfg.N, K=cfg.K, mu=cfg.mu, Dmax=cfg.Dmax)
        assert t.n <= cfg.N
        assert (t.n == cfg.N) == (t.exit_reason == "budget")
        if t.exit_reason == "depth":
            assert len(t.layers) - 1 == cfg.Dmax
        assert len(t.layers[1]) == min(cfg.K, cfg.N - 1)
        conf = t.confidence()
        for i in range(1, t.n):
            v = t.parent[i]
            assert t.depth[i] == t.depth[v] + 1
            assert v in t.layers[t.depth[i] - 1]
            # path confidence = product of edge probabilities along the path (Eq. 2)
            prod, j = 1.0, i
            while j > 0:
                prod *= t.prob[j]; j = t.parent[j]
            assert abs(conf[i] - prod) <= 1e-12 * prod
            assert conf[i] <= conf[v] * (1 + 1e-15)
            # stored edge prob is the softmax entry of the parent's row
            p = scipy.special.softmax(row_of(v))
            assert abs(t.prob[i] - p[t.token[i]]) <= 1e-12
        for d, (pool, sel) in enumerate(zip(t.pools, t.selections)):
            layer = t.layers[d + 1]
            assert len(layer) >= 1
            kept = set(sel.kept)
            scores = {(r.node, j): r.score[j] for r in pool for j in range(len(r.token))}
            anchor = max(scores.values())
            if d >= 1:
                thr = math.log(cfg.mu) + anchor
                assert all(scores[u] >= thr for u in kept)                 # gate soundness
                assert max(scores, key=lambda u: (scores[u], -u[0], -u[1])) in kept  # anchor kept
                if not sel.cut:
                    assert all((scores[u] >= thr) == (u in kept) for u in scores)  # completeness
            if sel.cut:
                dropped_pass = [scores[u] for u in scores if u not in kept and
                                (d == 0 or scores[u] >= math.log(cfg.mu) + anchor)]
                assert min(scores[u] for u in kept) >= max(dropped_pass)
            # node order inside the layer: (parent asc, rank asc)
            assert [(t.parent[i]) for i in layer] == sorted(t.parent[i] for i in layer)


# ---------------------------------------------------------------- mask
def test_mask_matches_parent_walk():
    rng = np.random.default_rng(21)
    rows = random_rows(rng, 60, 300, 0.5, 8.0)
    t = O.build_tree(lambda i: rows[i], 0, N=60, K=10, mu=0.03, Dmax=12)
    m = O.build_tree_mask(t.parent)
    for i in range(t.n):
        anc, j = set(), i
        while j >= 0:
            anc.add(j); j = t.parent[j]
        assert set(np.nonzero(m[i])[0]) == anc
        assert m[i].sum() == t.depth[i] + 1
    assert np.all(m[:, 0]) and np.all(np.diag(m)) and not np.any(np.triu(m, 1))
    w = O.mask_to_words(m, 64)
    assert w.shape == (64, 1)
    for i in range(t.n):
        assert int(w[i, 0]) == sum(1 << int(j) for j in np.nonzero(m[i])[0])
    assert not w[t.n:].any()


# ---------------------------------------------------------------- tree attention
def sdpa_path_reference(q, kp, vp, kt, vt, parent, i, scale=None):
    """Ordinary causal attention over prefix + root-to-i path, through torch SDPA."""
    path, j = [], i
    while j >= 0:
        path.append(j); j = parent[j]
    path = path[::-1]
    L, Hkv, Dh = kp.shape
    Hq = q.shape[1]
    G = Hq // Hkv
    k_seq = torch.from_numpy(np.concatenate([kp, kt[path]], 0)).permute(1, 0, 2)  # [Hkv][S][Dh]
    v_seq = torch.from_numpy(np.concatenate([vp, vt[path]], 0)).permute(1, 0, 2)
    q_seq = torch.zeros(Hq, L + len(path), Dh, dtype=torch.float64)
    q_seq[:, L:, :] = torch.from_numpy(q[path]).permute(1, 0, 2)
    k_rep = k_seq.repeat_interleave(G, dim=0)
    v_rep = v_seq.repeat_interleave(G, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(
        q_seq[None], k_rep[None], v_rep[None], is_causal=True, scale=scale)[0]
    return o[:, -1, :].numpy()  # [Hq][Dh] for node i


def small_attention_case(seed, n_parent, Hq=4, Hkv=2, Dh=16, L=24):
    rng = np.random.default_rng(seed)
    n = len(n_parent)
    q = rng.normal(size=(n, Hq, Dh)); kt = rng.normal(size=(n, Hkv, Dh)); vt = rng.normal(size=(n, Hkv, Dh))
    kp = rng.normal(size=(L, Hkv, Dh)); vp = rng.normal(size=(L, Hkv, Dh))
    return q, kp, vp, kt, vt


def test_tree_attention_equals_per_path_causal_attention():
    parent = [-1, 0, 0, 1, 1, 2, 3, 3, 6, 8]
    q, kp, vp, kt, vt = small_attention_case(31, parent)
    out, lse = O.tree_attention(q, kp, vp, kt, vt, O.build_tree_mask(parent))
    for i in range(len(parent)):
        ref = sdpa_path_reference(q, kp, vp, kt, vt, parent, i)
        np.testing.assert_allclose(out[i], ref, rtol=1e-10, atol=1e-12)


def test_tree_attention_chain_equals_plain_causal_attention():
    n = 7
    parent = [-1] + list(range(n - 1))
    q, kp, vp, kt, vt = small_attention_case(32, parent, Hq=4, Hkv=4)
    out, lse = O.tree_attention(q, kp, vp, kt, vt, O.build_tree_mask(parent), scale=0.3)
    L = kp.shape[0]
    k_all = torch.from_numpy(np.concatenate([kp, kt], 0)).permute(1, 0, 2)[None]
    v_all = torch.from_numpy(np.concatenate([vp, vt], 0)).permute(1, 0, 2)[None]
    qq = torch.zeros(1, 4, L + n, q.shape[2], dtype=torch.float64)
    qq[0, :, L:, :] = torch.from_numpy(q).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(qq, k_all, v_all, is_causal=True, scale=0.3)
    np.testing.assert_allclose(out, ref[0, :, L:, :].permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)
    # lse: log of the softmax denominator
    s = (torch.einsum("hd,hsd->hs", torch.from_numpy(q[n - 1]), k_all[0]) * 0.3)
    np.testing.assert_allclose(lse[n - 1], torch.logsumexp(s, dim=1).numpy(), rtol=1e-12)


def test_tree_attention_star_leaves_see_prefix_root_self_only():
    n = 6
    parent = [-1] + [0] * (n - 1)
    q, kp, vp, kt, vt = small_attention_case(33, parent)
    out, _ = O.tree_attention(q, kp, vp, kt, vt, O.build_tree_mask(parent))
    # changing a sibling's K/V must not change a leaf's output; changing the root's must
    kt2, vt2 = kt.copy(), vt.copy()
    kt2[2] += 5.0; vt2[2] -= 3.0
    out2, _ = O.tree_attention(q, kp, vp, kt2, vt2, O.build_tree_mask(parent))
    for i in (1, 3, 4, 5):
        np.testing.assert_array_equal(out[i], out2[i])
    assert np.abs(out[2] - out2[2]).max() > 1e-3
    kt3 = kt.copy(); kt3[0] += 5.0
    out3, _ = O.tree_attention(q, kp, vp, kt3, vt, O.build_tree_mask(parent))
    assert all(np.abs(out[i] - out3[i]).max() > 1e-6 for i in range(n))


def test_tree_attention_permutation_of_siblings_permutes_outputs():
    parent = [-1, 0, 0, 0, 1, 2]
    q, kp, vp, kt, vt = small_attention_case(34, parent)
    out, _ = O.tree_attention(q, kp, vp, kt, vt, O.build_tree_mask(parent))
    perm = [0, 2, 1, 3, 5, 4]            # swap nodes 1<->2 and their children 4<->5
    parent_p = [-1, 0, 0, 0, 1, 2]
    out_p, _ = O.tree_attention(q[perm], kp, vp, kt[perm], vt[perm], O.build_tree_mask(parent_p))
    np.testing.assert_allclose(out_p, out[perm], rtol=1e-12, atol=1e-14)


def test_tree_attention_no_prefix_root_returns_own_value():
    parent = [-1, 0]
    q, kp, vp, kt, vt = small_attention_case(35, parent, L=0)
    out, lse = O.tree_attention(q, kp, vp, kt, vt, O.build_tree_mask(parent))
    G = q.shape[1] // kt.shape[1]
    for h in range(q.shape[1]):
        np.testing.assert_allclose(out[0, h], vt[0, h // G], rtol=1e-14)


# ---------------------------------------------------------------- input generators
def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(41)
    x = (rng.normal(size=100000) * 10 ** rng.uniform(-3, 3, size=100000)).astype(np.float32)
    bits = f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, want)
    back = bf16_bits_to_f64(bits)
    np.testing.assert_array_equal(back, torch.from_numpy(x).to(torch.bfloat16).double().numpy())


def test_logits_rows_are_pure_functions_of_their_key():
    cfg = CONFIGS["c1"]
    a = logits_row(cfg, 5, 0, 3); b = logits_row(cfg, 5, 0, 3)
    np.testing.assert_array_equal(a, b)
    assert not np.array_equal(a, logits_row(cfg, 5, 0, 4))
    assert not np.array_equal(a, logits_row(cfg, 6, 0, 3))
    assert a.dtype == np.float32 and a.shape == (1024,)


# ---------------------------------------------------------------- greedy verification (T = 0)
def test_target_argmax_matches_torch_and_tie_rule():
    rng = np.random.default_rng(51)
    for _ in range(20):
        row = rng.normal(size=777)
        assert O.target_argmax(row) == int(torch.argmax(torch.from_numpy(row)))
    assert O.target_argmax(np.array([1.0, 3.0, 3.0, 2.0, 3.0])) == 1          # lowest id among equals
    assert O.target_argmax(np.array([-1.0, -0.0, 0.0, -2.0])) == 1            # -0.0 ties with +0.0
    assert O.target_argmax(np.array([-np.inf, -np.inf, -5.0])) == 2
    # the greedy token is the first of the row's ranked candidates
    row = rng.normal(size=500); row[100] = row[400] = row.max() + 1.0
    assert O.target_argmax(row) == int(O.row_candidates(row, 1)[0]) == 100


def _valid_nodes_by_definition(token, parent, target_token):
    """Every node whose whole root path was drafted as the target would have chosen."""
    def ok(i):
        return i == 0 or (token[i] == target_token[parent[i]] and ok(parent[i]))
    return [i for i in range(len(token)) if ok(i)]


def random_tree(rng, n, vocab, fan=3):
    token, parent = [int(rng.integers(vocab))], [-1]
    while len(token) < n:
        p = int(rng.integers(len(token)))
        used = {token[c] for c in range(len(token)) if parent[c] == p}
        if len(used) >= min(fan, vocab):
            continue
        t = int(rng.integers(vocab))
        if t in used:
            continue
        token.append(t); parent.append(p)
    return token, parent


def test_greedy_accept_equals_the_set_definition_on_random_trees():
    rng = np.random.default_rng(52)
    lengths = []
    for trial in range(300):
        n = int(rng.integers(1, 30)); vocab = int(rng.integers(2, 5))
        token, parent = random_tree(rng, n, vocab)
        target = [int(rng.integers(vocab)) for _ in range(n)]
        path, bonus = O.greedy_accept(token, parent, target)
        valid = _valid_nodes_by_definition(token, parent, target)
        # the valid nodes form one chain from the root, and the walk returns exactly it
        assert sorted(path) == sorted(valid)
        assert path[0] == 0 and all(parent[path[j + 1]] == path[j] for j in range(len(path) - 1))
        # maximal: no child of the last accepted node carries the target's token; bonus is that token
        last = path[-1]
        assert bonus == target[last]
        assert not any(parent[c] == last and token[c] == bonus for c in range(n))
        lengths.append(len(path))
    assert max(lengths) >= 4 and min(lengths) == 1      # the cases are not all trivial


def test_greedy_accept_closed_forms():
    # a chain drafted exactly as the target decodes: everything is accepted
    n = 9
    token = [50] + list(range(1, n)); parent = [-1] + list(range(n - 1))
    target = [token[i + 1] for i in range(n - 1)] + [77]
    assert O.greedy_accept(token, parent, target) == (list(range(n)), 77)
    # one wrong draft token at depth d cuts the chain there
    for d in range(1, n):
        t2 = list(token); t2[d] = 999
        path, bonus = O.greedy_accept(t2, parent, target)
        assert path == list(range(d)) and bonus == target[d - 1]
    # a star: the target's first token picks one leaf or none
    token = [5, 10, 11, 12, 13]; parent = [-1, 0, 0, 0, 0]
    assert O.greedy_accept(token, parent, [12, 1, 2, 3, 4]) == ([0, 3], 3)
    assert O.greedy_accept(token, parent, [14, 1, 2, 3, 4]) == ([0], 14)
    # a tree with only the root
    assert O.greedy_accept([3], [-1], [8]) == ([0], 8)


def test_greedy_accept_hand_worked_cases():
    g = json.load(open(os.path.join(HERE, "golden", "accept_example.json")))
    for case in g["cases"]:
        path, bonus = O.greedy_accept(g["token"], g["parent"], case["target_token"])
        assert path == case["path"] and bonus == case["bonus"], case["why"]


def test_compact_kv_is_a_gather_appended_to_the_cache():
    rng = np.random.default_rng(53)
    L, cap, n = 7, 20, 10
    cache = rng.normal(size=(cap, 2, 4)); tree = rng.normal(size=(n, 2, 4))
    before = cache.copy()
    path = [0, 2, 5, 9]
    new_len = O.compact_kv(cache, tree, path, L)
    assert new_len == L + 4
    np.testing.assert_array_equal(cache[:L], before[:L])
    np.testing.assert_array_equal(cache[L:new_len], tree[np.array(path)])
    np.testing.assert_array_equal(cache[new_len:], before[new_len:])


# ---------------------------------------------------------------- Alg. 1, the static tree
def alg1_literal(rows_prob_of_path, D, K, N):
    """Alg. 1 written out on paths (tuples of tokens) in the probability domain, independent of
    the oracle's layer functions.  rows_prob_of_path(path) -> probability row after that path."""
    tree = [((), 1.0)]                       # (path, p); the root is the empty path
    parents = [((), 1.0)]
    for d in range(D + 1):
        pool = []
        for pi, (path, p) in enumerate(parents):
            row = rows_prob_of_path(path)
            best = sorted(range(len(row)), key=lambda w: (-row[w], w))[:K]
            pool += [(p * row[w], pi, r, path + (w,)) for r, w in enumerate(best)]
        chosen = sorted(pool, key=lambda c: (-c[0], c[1], c[2]))[:K]
        chosen = sorted(chosen, key=lambda c: (c[1], c[2]))          # node order: (parent, rank)
        parents = [(c[3], c[0]) for c in chosen]
        tree += parents
    order = sorted(range(len(tree)), key=lambda i: (-tree[i][1], i))[:N]
    return [tree[i] for i in sorted(order)]


@pytest.mark.parametrize("seed", range(6))
def test_static_tree_vs_literal_alg1(seed):
    rng = np.random.default_rng(600 + seed)
    V, K, D = 5, int(rng.integers(2, 4)), int(rng.integers(1, 4))
    N = int(rng.integers(2, 1 + K * (D + 1) + 1))
    table = {}

    def prob_row(path):
        if path not in table:
            p = rng.dirichlet(np.ones(V) * 0.7)
            table[path] = p
        return table[path]

    want = alg1_literal(prob_row, D, K, N)
    # the oracle is driven by node ids: keep the path of every node as it is created, layer by
    # layer through the oracle's own layer functions
    paths = {0: ()}

    def row_of_lazy(i):
        return np.log(prob_row(paths[i]))

    t = O.Tree(token=[0], parent=[-1], depth=[0], prob=[1.0], logp=[0.0])
    frontier = [0]
    t.layers.append(range(0, 1))
    for d in range(D + 1):
        pool = O.expand_layer(frontier, t.logp, row_of_lazy, K)
        sel = O.select_budget(pool, d, 10 ** 6, K, 1.0, D + 1)
        by_node = {r.node: r for r in pool}
        begin = t.n
        for (v, j) in sel.kept:
            r = by_node[v]
            paths[t.n] = paths[v] + (int(r.token[j]),)
            t.token.append(int(r.token[j])); t.parent.append(v); t.depth.append(t.depth[v] + 1)
            t.prob.append(float(r.prob[j])); t.logp.append(float(r.score[j]))
        frontier = list(range(begin, t.n))
    pruned = O.prune_top_n(t, N)
    got = [(paths[i], math.exp(t.logp[i])) for i in pruned.kept]
    assert [g[0] for g in got] == [w[0] for w in want]
    np.testing.assert_allclose([g[1] for g in got], [w[1] for w in want], rtol=1e-12)
    # and the one-call form builds the same tree (same layer functions, same arguments)
    full, pruned2 = O.build_static_tree(lambda i: np.log(prob_row(paths[i])), 0, D, K, N)
    assert full.token == t.token and full.parent == t.parent
    assert pruned2.kept == pruned.kept and pruned2.parent == pruned.parent


def test_prune_top_n_properties_and_closed_forms():
    rng = np.random.default_rng(61)
    for _ in range(100):
        n = int(rng.integers(1, 40))
        token, parent = random_tree(rng, n, 50, fan=4)
        logp = [0.0] * n
        for i in range(1, n):
            logp[i] = logp[parent[i]] - float(rng.exponential(1.0))
        depth = [0] * n
        for i in range(1, n):
            depth[i] = depth[parent[i]] + 1
        t = O.Tree(token=token, parent=parent, depth=depth, prob=[1.0] * n, logp=logp)
        N = int(rng.integers(1, n + 1))
        p = O.prune_top_n(t, N)
        assert p.n == N and p.kept == sorted(p.kept) and p.kept[0] == 0
        kept = set(p.kept)
        assert all(parent[i] in kept for i in p.kept if i > 0)                 # closed under "parent of"
        worst_kept = min(logp[i] for i in p.kept)
        assert all(logp[j] <= worst_kept for j in range(n) if j not in kept)   # nothing better was dropped
        for new, old in enumerate(p.kept):                                       # renumbering is consistent
            assert p.token[new] == token[old] and p.depth[new] == depth[old]
            assert (p.parent[new] == -1) if old == 0 else (p.kept[p.parent[new]] == parent[old])
    # a chain keeps its first N nodes; equal confidences keep the lower ids
    chain = O.Tree(token=list(range(6)), parent=[-1, 0, 1, 2, 3, 4], depth=list(range(6)), prob=[1.0] * 6,
                   logp=[0.0, -1.0, -2.0, -3.0, -4.0, -5.0])
    assert O.prune_top_n(chain, 4).kept == [0, 1, 2, 3]
    star = O.Tree(token=[9, 1, 2, 3, 4], parent=[-1, 0, 0, 0, 0], depth=[0, 1, 1, 1, 1], prob=[1.0] * 5,
                  logp=[0.0, -1.0, -1.0, -1.0, -1.0])
    assert O.prune_top_n(star, 3).kept == [0, 1, 2]


def test_static_tree_shape():
    # every layer of Alg. 1 adds exactly K nodes (the pool has K*K >= K candidates)
    rng = np.random.default_rng(62)
    rows = {}

    def row_of(i):
        if i not in rows:
            rows[i] = rng.normal(size=64) * 2.0
        return rows[i]

    full, pruned = O.build_static_tree(row_of, 3, D=4, K=3, N=10)
    assert full.n == 1 + 3 * 5 and [len(r) for r in full.layers] == [1, 3, 3, 3, 3, 3]
    assert pruned.n == 10
