"""Alg. 2 with the candidate pool as the listing writes it (every token of every frontier row)
through talon_expand_literal, against the oracle.

The oracle runs with a per-row cap of N - 1: a layer never takes more than N - |T| <= N - 1
nodes, so that pool gives the uncapped tree (tests/test_oracle_pins.py checks that equivalence
against the full-vocabulary pool by brute force).  Seeds are admissible for that pool (every
cross-parent decision leaves a margin above the harness tolerance); topology, tokens, depths,
counters, status bits and the mask are then compared bit for bit, probabilities to 1e-5."""
import dataclasses

import numpy as np
import pytest

from tests import harness as H
from workloads import CONFIGS

pytestmark = pytest.mark.gpu

CASES = {
    # fp32 rows so flat that one parent receives more than 64 children: beyond the capped path
    "flat-f32-n200": dataclasses.replace(CONFIGS["c1"], name="literal-flat", V=4099, N=200, Dmax=8, K=4,
                                         recipe=("gauss", 0.3, 0.5)),
    # tiny fp32 shape, ragged vocabulary, K_init larger than the per-row cap of the fast path's config
    "tiny-f32": dataclasses.replace(CONFIGS["c1"], name="literal-tiny", V=1021, N=16, K=3),
    # Qwen3-8B-shaped rows, N = 128: one low-temperature and one high-temperature sequence
    "qwen-bf16-n128": dataclasses.replace(CONFIGS["c3"], name="literal-c3", B=2,
                                          recipe=(("gauss", 6.0, 8.0), ("gauss", 0.5, 1.0))),
    # the stress recipe (Zipf-peaked and near-uniform rows), N = 256, three sequences
    "zipf-bf16-n256": dataclasses.replace(CONFIGS["c5"], name="literal-n256", B=3, V=32003),
}


def _case(cfg, init_layers=1, layer_by_layer=False):
    cap = cfg.N - 1
    seeds, trees = [], []
    for b in range(cfg.B):
        s, _ = H.find_admissible_seed(cfg, b, cfg.seed + 100 * b, cap=cap, init_layers=init_layers)
        seeds.append(s)
    pool = H.build_pool(cfg, seeds)
    roots = H.root_tokens(cfg)
    from oracle import talon_oracle as O
    masks = []
    for b in range(cfg.B):
        t = H.oracle_tree(cfg, pool[b], roots[b], init_layers=init_layers, cap=cap)
        trees.append(t)
        masks.append(O.build_tree_mask(t.parent))
    for roomy in ((False, True) if cfg.N_pad == 64 else (False,)):
        gpu = H.run_gpu_literal(cfg, pool, cfg.K, init_layers=init_layers, layer_by_layer=layer_by_layer, roomy_state=roomy)
        H.compare_tree(cfg, gpu, trees, check_rows=False)
        H.compare_mask(cfg, gpu, masks)
    return trees


@pytest.mark.parametrize("name", list(CASES))
def test_uncapped_pool_matches_the_oracle(name):
    trees = _case(CASES[name])
    fan = max(int(np.bincount(np.asarray(t.parent[1:]), minlength=t.n).max()) for t in trees)
    print(name, "largest fan-out", fan, "nodes", [t.n for t in trees])
    if name == "flat-f32-n200":
        assert fan > 64   # the case the capped path cannot build


def test_one_layer_per_call_and_two_top_k_layers():
    _case(CASES["qwen-bf16-n128"], init_layers=2, layer_by_layer=True)
    _case(CASES["tiny-f32"], init_layers=0, layer_by_layer=True)


@pytest.mark.parametrize("layer_by_layer", [False, True])
def test_small_trees_whose_rows_get_more_than_32_children(layer_by_layer):
    """Trees of at most 64 nodes are first built with a per-row cap of 32 and, when a selection
    kept the 32nd candidate of a row, again from the saved state with the cap N - 1.  Three
    sequences in one call: peaked rows (largest fan-out 5), flat rows where one parent gets 31
    children (the last count the first build may keep) and flat rows where one gets 36 (the
    second build, which then redoes all three).  With one call per layer the wide layer is the
    second call, so the state the second build goes back to is not the root's."""
    cfg = dataclasses.replace(CONFIGS["c1"], name="literal-wide-n60", B=3, V=4099, N=60, Dmax=8, K=2, mu=0.1,
                              recipe=(("gauss", 6.0, 8.0), ("gauss", 0.3, 0.5), ("gauss", 2.0, 2.5)))
    trees = _case(cfg, layer_by_layer=layer_by_layer)
    fans = [int(np.bincount(np.asarray(t.parent[1:]), minlength=t.n).max()) for t in trees]
    print("largest fan-out per sequence", fans, "nodes", [t.n for t in trees])
    assert fans[0] < 31 and fans[1] == 31 and fans[2] > 32
    # the same recipes one sequence at a time (other rows: fan-outs 5, 45, 38): a call whose first build stands, two whose second runs
    for b in range(3):
        one = dataclasses.replace(cfg, name="literal-wide-n60-%d" % b, B=1, recipe=cfg.recipe[b], seed=cfg.seed + 100 * b)
        _case(one, layer_by_layer=layer_by_layer)


@pytest.mark.parametrize("dtype,V", [("f32", 40001), ("bf16", 70001)])
def test_rows_streamed_in_parts(dtype, V):
    """A layer of a few rows leaves compute units idle, and its rows are streamed in parts by
    several workgroups (four here: two rows per sequence, at least 2048 vectors per part).
    Second layer of the three sequences: rows of which every token passes the gate (every part
    cuts to the limit of 197, the merge selects among 4 x 197 survivors); rows of which 320-380
    pass (f32: no part overflows, the merge selects) or about 60 (bf16: the merge copies); rows
    that the scan's 16 best settle (nothing is streamed)."""
    cfg = dataclasses.replace(CONFIGS["c1"], name="literal-parts", B=3, V=V, logits_dtype=dtype, N=200, Dmax=6, K=2, mu=0.05,
                              recipe=(("gauss", 0.05, 0.1), ("gauss", 1.6, 1.9), ("gauss", 6.0, 8.0)))
    trees = _case(cfg)
    fans = [int(np.bincount(np.asarray(t.parent[1:]), minlength=t.n).max()) for t in trees]
    print("largest fan-out per sequence", fans, "nodes", [t.n for t in trees])
    assert fans[0] > 190 and fans[1] >= 64 and fans[2] < 16
    _case(cfg, layer_by_layer=True)


def test_capped_path_agrees_where_its_cap_suffices():
    """N = 60, k = 59: the fast path's tree is the uncapped tree, so both entry points must
    produce the same arrays, bit for bit (probabilities included: same arithmetic)."""
    cfg = dataclasses.replace(CONFIGS["c2"], name="c2-cap59", K=59, V=32003)
    seeds = [H.find_admissible_seed(cfg, 0, cfg.seed, K_init=10)[0]]
    pool = H.build_pool(cfg, seeds)
    fast = H.run_gpu_step(cfg, seeds=seeds, pool=pool, with_attention=False, K_init=10)
    lit = H.run_gpu_literal(cfg, pool, 10)
    n = int(fast["n_nodes"][0])
    assert int(lit["n_nodes"][0]) == n
    for name in ("token", "parent", "depth", "prob", "logp"):
        np.testing.assert_array_equal(lit[name][0, :n], fast[name][0, :n], err_msg=name)
    for name in ("status", "depth_cur", "frontier_begin", "frontier_count"):
        assert int(lit[name][0]) == int(fast[name][0]), name
    np.testing.assert_array_equal(lit["mask"][0], fast["mask"][0])


# ----------------------------------------------------------------------------- degenerate rows
def _compare_pool(cfg, make_pool, need_margin=True, **kw):
    """make_pool(attempt) -> pool.  With need_margin the first pool that leaves every cross-parent
    decision a margin is used (the test fails if none of 16 does); otherwise make_pool(0)."""
    from oracle import talon_oracle as O
    roots = H.root_tokens(cfg)
    if need_margin:
        pool, trees = H.admissible_pool(cfg, make_pool, cap=max(cfg.N - 1, 1), **kw)
    else:
        pool = make_pool(0)
        trees = [H.oracle_tree(cfg, pool[b], roots[b], cap=max(cfg.N - 1, 1), **kw) for b in range(cfg.B)]
    # trees of at most 64 nodes: once through the call's shortcut, once kept on the general path
    for roomy in ((False, True) if cfg.N_pad == 64 else (False,)):
        gpu = H.run_gpu_literal(cfg, pool, cfg.K, roomy_state=roomy, **kw)
        H.compare_tree(cfg, gpu, trees, check_rows=False)
        H.compare_mask(cfg, gpu, [O.build_tree_mask(t.parent) for t in trees])
    return gpu, trees


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_constant_rows_every_candidate_ties(dtype):
    """Every logit equal: all scores of a layer tie exactly, in any arithmetic.  The order
    (parent ascending, token ascending) must decide: the first child of the root receives the
    whole remaining budget, 114 children with tokens 0..113."""
    from tests.test_gpu_parity import custom_pool, small
    cfg = small(name="lit-const", V=20011, logits_dtype=dtype, K=5, N=120, Dmax=6)
    pool = custom_pool(cfg, lambda b, i: np.full(cfg.V, 1.5))
    gpu, _ = _compare_pool(cfg, lambda attempt: pool, need_margin=False)
    assert list(gpu["token"][0, 1:6]) == [0, 1, 2, 3, 4]
    assert list(gpu["parent"][0, 6:120]) == [1] * 114
    assert list(gpu["token"][0, 6:120]) == list(range(114))


def test_two_valued_rows_cut_inside_a_run_of_equal_logits():
    """Rows with two distinct values: the budget cut falls inside a long run of equal logits of
    one parent, after whole runs of its siblings."""
    from tests.test_gpu_parity import custom_pool, small
    cfg = small(name="lit-two", V=9001, logits_dtype="f32", K=3, N=150, Dmax=6, mu=0.5)

    def make_pool(attempt):
        def fill(b, i):
            x = np.full(cfg.V, 0.0)
            x[(7 * i) % 50::50] = 2.0 + (0.01 + 0.001 * attempt) * i   # 181 high entries, their level depends on the node
            return x
        return custom_pool(cfg, fill)

    _compare_pool(cfg, make_pool)


def test_sorted_rows_and_neg_inf_entries():
    from tests.test_gpu_parity import custom_pool, small
    cfg = small(name="lit-sorted", V=17003, logits_dtype="f32", K=8, N=90, Dmax=8)

    def make_pool(attempt):
        rng = np.random.default_rng(5 + attempt)

        def fill(b, i):
            if i % 3 == 0:
                return np.linspace(-3, 3, cfg.V) * (1 + 0.1 * i)
            if i % 3 == 1:
                return np.linspace(4, -4, cfg.V) * (1 + 0.05 * i)
            x = np.full(cfg.V, -np.inf)
            idx = rng.choice(cfg.V, size=5, replace=False)
            x[idx] = rng.normal(size=5)
            return x

        return custom_pool(cfg, fill)

    _compare_pool(cfg, make_pool)


def test_vocab_smaller_than_the_first_layer():
    from tests.test_gpu_parity import small
    cfg = small(name="lit-tinyv", V=8, logits_dtype="f32", K=12, N=40, Dmax=4, mu=1e-30)
    _compare_pool(cfg, lambda attempt: H.build_pool(cfg, [cfg.seed + attempt]))


def test_nan_row_sets_status_and_stops_sequence():
    from tests.test_gpu_parity import small
    cfg = small(name="lit-nan", V=5000, logits_dtype="f32", K=3, N=20, Dmax=6, B=2)
    seeds = [H.find_admissible_seed(cfg, 0, cfg.seed, cap=cfg.N - 1)[0], cfg.seed]
    pool = H.build_pool(cfg, seeds)
    pool[1, 2, 1234] = np.nan
    t = H.oracle_tree(cfg, pool[0], H.root_tokens(cfg)[0], cap=cfg.N - 1)
    assert t.margin > H.MARGIN_TOL
    for roomy in (False, True):      # the shortcut for small trees, then the general path
        gpu = H.run_gpu_literal(cfg, pool, cfg.K, roomy_state=roomy)
        assert int(gpu["status"][1]) & 4
        assert int(gpu["n_nodes"][1]) == 1 + cfg.K          # stopped after the layer that read the bad row
        assert int(gpu["frontier_count"][1]) == 0
        H.compare_tree(cfg, {k: v[:1] for k, v in gpu.items()}, [t], check_rows=False)


def test_budget_of_one_and_two():
    from tests.test_gpu_parity import small
    for N in (1, 2):
        cfg = small(name="lit-n%d" % N, V=2048, logits_dtype="bf16", K=4, N=N, Dmax=4)
        _compare_pool(cfg, lambda attempt: H.build_pool(cfg, [cfg.seed]), need_margin=False)


# ----------------------------------------------------------------------------- full sizes
def _full_size(cfg_name, oracle_seqs):
    """All sequences of a benchmark configuration through the uncapped call; the oracle builds the
    stated sequences in full, every sequence is checked for the properties any tree must have."""
    from oracle import talon_oracle as O
    from tests.test_gpu_full_size import structural_checks
    cfg = CONFIGS[cfg_name]
    cap = cfg.N - 1
    seeds = [cfg.seed] * cfg.B
    trees = {}
    for b in oracle_seqs:
        seeds[b], trees[b] = H.find_admissible_seed(cfg, b, cfg.seed, cap=cap)
    print("case", cfg.name, "uncapped, seeds", seeds, "oracle sequences", oracle_seqs, flush=True)
    pool = H.build_pool(cfg, seeds)
    gpu = H.run_gpu_literal(cfg, pool, cfg.K)
    for b in range(cfg.B):
        structural_checks(cfg, gpu, b)
    for b in oracle_seqs:
        t = trees[b]
        assert t.margin > H.MARGIN_TOL
        H.compare_tree(cfg, {k: v[b:b + 1] for k, v in gpu.items()}, [t], check_rows=False)
        np.testing.assert_array_equal(gpu["mask"][b], O.mask_to_words(O.build_tree_mask(t.parent), cfg.N_pad))


def test_c3_qwen3_8b_x4_full_size_uncapped():
    _full_size("c3", [0, 1, 2, 3])


def test_c5_stress_full_size_uncapped():
    _full_size("c5", list(range(16)))


def test_repeated_calls_on_one_workspace_agree():
    """Survivors are collected in whatever order the lanes claim their slots; the tree must not
    depend on it, nor on what an earlier call left in the workspace (a different, larger shape
    first, then the same call twenty times)."""
    import torch
    import paper_2601_07353_amd as T
    big = CASES["zipf-bf16-n256"]
    cfg = CASES["qwen-bf16-n128"]
    dt = T.TALON_DTYPE_BF16
    ws = T.make_literal_workspace(big.B, big.N_pad, big.V, dt)
    assert ws.numel() >= T.load_library().talon_literal_workspace_bytes(cfg.B, cfg.N_pad, cfg.V, dt)

    def run(c, pool_dev):
        st = T.TreeState(c.B, c.N)
        T.talon_tree_init(st, torch.from_numpy(H.root_tokens(c)).cuda())
        T.talon_expand_literal(pool_dev, st, c.Dmax, c.mu, c.K, 1, c.Dmax, ws)
        torch.cuda.synchronize()
        n = st.n_nodes.cpu().numpy()
        return [n] + [getattr(st, f).cpu().numpy() for f in ("token", "parent", "depth", "prob", "logp", "status")]

    run(big, H.to_device_logits(H.build_pool(big, [big.seed] * big.B)))
    dev = H.to_device_logits(H.build_pool(cfg, [cfg.seed, cfg.seed + 100]))
    first = run(cfg, dev)
    assert all(int(v) == cfg.N for v in first[0])
    for _ in range(20):
        again = run(cfg, dev)
        for x, y in zip(first, again):
            n = first[0]
            if x.ndim == 2:
                for b in range(cfg.B):
                    np.testing.assert_array_equal(x[b, :n[b]], y[b, :n[b]])
            else:
                np.testing.assert_array_equal(x, y)


def test_random_small_configurations():
    """Thirty seeded random shapes (vocabulary 8 to 60001, both logit types, N 2-256, K_init 1-19
    -- above 16 the top-K layers take the streaming route too --, 1-3 sequences, 0-2 top-K layers,
    four thresholds and recipes, depth cap from 1), alternately in one call and one call per
    layer.  Configurations whose oracle tree leaves no margin are skipped; most must run."""
    from oracle import talon_oracle as O
    from workloads import WorkloadConfig
    rng = np.random.default_rng(20260107)
    ran = 0
    for it in range(30):
        dtype = str(rng.choice(["f32", "bf16"]))
        V = int(rng.choice([8, 63, 500, 4099, 20000, 60001]))
        N = int(rng.integers(2, 257))
        K = int(rng.integers(1, 20))
        B = int(rng.integers(1, 4))
        init_layers = int(rng.integers(0, 3))
        mu = float(rng.choice([0.3, 0.03, 0.003, 1e-6]))
        rec = [("gauss", 0.5, 4.0), ("gauss", 0.05, 0.3), ("gauss", 4.0, 8.0), ("zipf_mix", 1.2, 0.05)][int(rng.integers(0, 4))]
        Dmax = int(rng.integers(1, 10))
        if B * ((N + 63) // 64 * 64) * V > 60e6:
            V = 4099
        cfg = WorkloadConfig("literal-random-%d" % it, B=B, V=V, logits_dtype=dtype, K=K, N=N, Dmax=Dmax, mu=mu,
                             Hq=4, Hkv=4, Dh=64, L=16, recipe=rec, seed=1000 + it)
        pool = H.build_pool(cfg, [cfg.seed + 7 * b for b in range(B)])
        roots = H.root_tokens(cfg)
        trees = [H.oracle_tree(cfg, pool[b], roots[b], init_layers=init_layers, cap=max(N - 1, 1)) for b in range(B)]
        if min(t.margin for t in trees) <= H.MARGIN_TOL:
            continue
        print("case", it, dtype, "V", V, "N", N, "K", K, "B", B, "init", init_layers, "mu", mu, rec, "Dmax", Dmax, flush=True)
        for roomy in ((False, True) if cfg.N_pad == 64 else (False,)):
            gpu = H.run_gpu_literal(cfg, pool, K, init_layers=init_layers, layer_by_layer=bool(it % 2), roomy_state=roomy)
            H.compare_tree(cfg, gpu, trees, check_rows=False)
            H.compare_mask(cfg, gpu, [O.build_tree_mask(t.parent) for t in trees])
        ran += 1
    assert ran >= 24


def test_dense_frontier_batches_with_padded_rows():
    """The layout a serving loop has: after every layer the draft model's logits exist for the
    new frontier only, as a dense batch [B][frontier rows][padded row] (TALON_ROWS_BY_FRONTIER,
    row stride larger than the vocabulary, values in the padding that would win any maximum).
    One uncapped call per layer on a freshly gathered batch must build the oracle's tree."""
    import torch
    import paper_2601_07353_amd as T
    from tests.test_gpu_parity import small
    cfg = small(name="literal-dense", V=20011, logits_dtype="bf16", K=6, N=150, Dmax=9, B=3,
                recipe=(("gauss", 4.0, 8.0), ("gauss", 0.5, 1.0), ("gauss", 2.0, 6.0)))
    cap = cfg.N - 1
    seeds = [H.find_admissible_seed(cfg, b, cfg.seed + 100 * b, cap=cap)[0] for b in range(cfg.B)]
    pool = H.build_pool(cfg, seeds)
    roots = H.root_tokens(cfg)
    trees = [H.oracle_tree(cfg, pool[b], roots[b], cap=cap) for b in range(cfg.B)]
    pool_dev = H.to_device_logits(pool)                      # [B][N_pad][V], only used to gather from
    stride = (cfg.V + 8 + 63) // 64 * 64
    st = T.TreeState(cfg.B, cfg.N)
    ws = T.make_literal_workspace(cfg.B, st.N_pad, cfg.V, T.TALON_DTYPE_BF16)
    T.talon_tree_init(st, torch.from_numpy(roots).cuda())
    for _ in range(cfg.Dmax):
        begin = st.frontier_begin.cpu().numpy()
        count = st.frontier_count.cpu().numpy()
        done = (st.status.cpu().numpy() & 3) != 0
        if done.all():
            break
        fmax = max(1, int(count.max()))
        dense = torch.full((cfg.B, fmax, stride), 30000.0, dtype=torch.bfloat16, device="cuda")
        for b in range(cfg.B):
            if not done[b]:
                dense[b, :count[b], :cfg.V] = pool_dev[b, begin[b]:begin[b] + count[b]]
        T.talon_expand_literal(dense, st, 1, cfg.mu, cfg.K, 1, cfg.Dmax, ws, row_mode=T.TALON_ROWS_BY_FRONTIER,
                               vocab=cfg.V)
        torch.cuda.synchronize()
    n = st.n_nodes.cpu().numpy()
    for b, t in enumerate(trees):
        assert int(n[b]) == t.n
        np.testing.assert_array_equal(st.token[b, :t.n].cpu().numpy(), np.asarray(t.token, dtype=np.int32))
        np.testing.assert_array_equal(st.parent[b, :t.n].cpu().numpy(), np.asarray(t.parent, dtype=np.int32))
        np.testing.assert_allclose(np.exp(st.logp[b, :t.n].cpu().numpy()), t.confidence(), rtol=H.PROB_RTOL, atol=0)
    assert max(int(np.bincount(np.asarray(t.parent[1:])).max()) for t in trees) > cfg.K
