"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded synthetic inputs.  Topology, token ids, masks: bit-exact.  Probabilities and path
confidences: 1e-5 relative.  Tree attention: 2e-2 absolute (bf16 inputs, fp64 oracle)."""
import dataclasses

import numpy as np
import pytest

from tests import harness as H
from workloads import CONFIGS, WorkloadConfig, f32_to_bf16_bits

pytestmark = pytest.mark.gpu


def admissible_seeds(cfg):
    return [H.find_admissible_seed(cfg, b, cfg.seed)[0] for b in range(cfg.B)]


def small(name="t", **kw):
    base = dict(name=name, B=1, V=1024, logits_dtype="f32", K=2, N=16, Dmax=6, mu=0.03, Hq=4, Hkv=4, Dh=64,
                L=128, recipe=("gauss", 0.5, 4.0))
    base.update(kw)
    return WorkloadConfig(**base)


def step_and_compare(cfg, seeds=None, **kw):
    seeds = admissible_seeds(cfg) if seeds is None else seeds
    print("case", cfg.name, "seeds", seeds, flush=True)
    pool = H.build_pool(cfg, seeds)
    gpu = H.run_gpu_step(cfg, seeds, pool=pool, **kw)
    okw = {k: v for k, v in kw.items() if k in ("init_layers", "mu", "K_init", "with_attention")}
    ref = H.run_oracle_step(cfg, seeds, pool=pool, **okw)
    return H.compare_step(cfg, gpu, ref), gpu, ref


# ----------------------------------------------------------------------------- whole steps
def test_c1_tiny_step():
    worst, gpu, ref = step_and_compare(CONFIGS["c1"])
    assert ref["trees"][0].n == 16


@pytest.mark.parametrize("mode", ["split", "fused", "tree"])
def test_c1_layerwise_entry_points_match_single_call(mode):
    cfg = CONFIGS["c1"]
    seeds = admissible_seeds(cfg)
    a = H.run_gpu_step(cfg, seeds, with_attention=False, layerwise=mode)
    b = H.run_gpu_step(cfg, seeds, with_attention=False, layerwise=False)
    for key in ("token", "parent", "depth", "n_nodes", "status", "mask", "prob", "logp"):
        np.testing.assert_array_equal(a[key], b[key])


def test_tree_launch_gives_up_cleanly_when_the_wait_is_cut_short():
    """The single-launch loop bounds its wait between layers.  With the bound forced to zero from
    the host, a workgroup either finds the layer already complete or gives up: the launch must
    end, and every sequence is then either expanded exactly as usual or marked ABORTED."""
    import torch
    import paper_2601_07353_amd as T
    cfg = small(name="abort", V=40000, logits_dtype="bf16", K=8, N=100, Dmax=12, B=3,
                recipe=(("gauss", 6.0, 8.0), ("gauss", 0.5, 1.0), ("gauss", 2.0, 8.0)))
    seeds = admissible_seeds(cfg)
    pool = H.build_pool(cfg, seeds)
    ref = H.run_gpu_step(cfg, seeds, pool=pool, with_attention=False)
    T.talon_set_spin_limit_us(0)
    try:
        got = H.run_gpu_step(cfg, seeds, pool=pool, with_attention=False)
        torch.cuda.synchronize()
    finally:
        T.talon_set_spin_limit_us(200000)
    aborted = (got["status"] & T.TALON_STATUS_ABORTED) != 0
    assert aborted.all() or not aborted.any()
    if not aborted.any():
        for key in ("token", "parent", "depth", "n_nodes", "status"):
            np.testing.assert_array_equal(got[key], ref[key])
    else:
        assert np.all(got["n_nodes"] >= 1) and np.all(got["n_nodes"] <= cfg.N)
    again = H.run_gpu_step(cfg, seeds, pool=pool, with_attention=False)
    for key in ("token", "parent", "depth", "n_nodes", "status"):
        np.testing.assert_array_equal(again[key], ref[key])


def test_a_launch_that_gives_up_is_rebuilt_layer_by_layer():
    """The recovery a caller needs when the single launch cannot keep its whole grid resident:
    talon_build_tree_checked sees TALON_STATUS_ABORTED (forced here from the host: wait bound zero, so
    every kernel still ends normally) and builds the trees again with one launch per layer on the same
    workspace.  The result must be the oracle's tree, and the workspace must serve the next plain call."""
    import torch
    import paper_2601_07353_amd as T
    cfg = small(name="fallback", V=40000, logits_dtype="bf16", K=8, N=100, Dmax=12, B=3,
                recipe=(("gauss", 6.0, 8.0), ("gauss", 0.5, 1.0), ("gauss", 2.0, 8.0)))
    seeds = admissible_seeds(cfg)
    pool = H.build_pool(cfg, seeds)
    ref = H.run_oracle_step(cfg, seeds, pool=pool, with_attention=False)
    pool_dev = H.to_device_logits(pool)
    st = T.TreeState(cfg.B, cfg.N)
    cand = T.Candidates(cfg.B, st.N_pad, cfg.K)
    ws = T.make_expand_workspace(cfg.B, st.N_pad, cfg.V, cfg.K, T.TALON_DTYPE_BF16)
    roots = torch.from_numpy(H.root_tokens(cfg)).cuda()
    mask = torch.full((cfg.B, st.N_pad, st.N_pad // 64), -1, dtype=torch.int64, device="cuda")

    def snapshot():
        torch.cuda.synchronize()
        return {"token": st.token.cpu().numpy(), "parent": st.parent.cpu().numpy(), "depth": st.depth.cpu().numpy(),
                "prob": st.prob.cpu().numpy(), "logp": st.logp.cpu().numpy(), "n_nodes": st.n_nodes.cpu().numpy(),
                "status": st.status.cpu().numpy(), "depth_cur": st.depth_cur.cpu().numpy(),
                "frontier_begin": st.frontier_begin.cpu().numpy(), "frontier_count": st.frontier_count.cpu().numpy(),
                "mask": mask.cpu().numpy().view(np.uint64)}

    assert T.talon_build_tree_checked(roots, pool_dev, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, mask=mask) is False
    H.compare_tree(cfg, snapshot(), ref["trees"], check_rows=False)
    T.talon_set_spin_limit_us(0)
    try:
        fell = T.talon_build_tree_checked(roots, pool_dev, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, mask=mask)
    finally:
        T.talon_set_spin_limit_us(200000)
    assert fell is True          # a workgroup that leaves layer 0 finds layer 1 not yet selected and gives up
    got = snapshot()
    H.compare_tree(cfg, got, ref["trees"], check_rows=False)
    H.compare_mask(cfg, got, ref["mask"])
    T.talon_build_tree(roots, pool_dev, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, mask=mask)
    got = snapshot()
    H.compare_tree(cfg, got, ref["trees"], check_rows=False)
    H.compare_mask(cfg, got, ref["mask"])


def _expand_on(cfg, pool_dev, st, cand, ws, mask, roots):
    import torch
    import paper_2601_07353_amd as T
    T.talon_build_tree(roots, pool_dev, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, mask=mask)
    torch.cuda.synchronize()
    n = [int(x) for x in st.n_nodes.cpu()]
    return {"n": n, "status": st.status.cpu().numpy().copy(),
            "token": [st.token[b, :k].cpu().numpy().copy() for b, k in enumerate(n)],
            "parent": [st.parent[b, :k].cpu().numpy().copy() for b, k in enumerate(n)],
            "logp": [st.logp[b, :k].cpu().numpy().copy() for b, k in enumerate(n)],
            "mask": [mask[b, :k].cpu().numpy().copy() for b, k in enumerate(n)]}


def _same_trees(a, b):
    assert a["n"] == b["n"]
    np.testing.assert_array_equal(a["status"], b["status"])
    for key in ("token", "parent", "logp", "mask"):
        for x, y in zip(a[key], b[key]):
            np.testing.assert_array_equal(x, y)


def test_one_workspace_serves_call_after_call():
    """talon_build_tree leaves its workspace as it found it: the same workspace, tree state and
    output buffers serve 40 calls that alternate between two inputs, then a launch that is
    made to give up (wait bound forced to zero from the host), then the two inputs again;
    every complete call must give exactly what a call on a fresh workspace gives."""
    import torch
    import paper_2601_07353_amd as T
    cfg = small(name="reuse", V=40000, logits_dtype="bf16", K=8, N=100, Dmax=12, B=3,
                recipe=(("gauss", 6.0, 8.0), ("gauss", 0.5, 1.0), ("gauss", 2.0, 8.0)))
    seeds_a = admissible_seeds(cfg)
    seeds_b = admissible_seeds(dataclasses.replace(cfg, seed=cfg.seed + 77))
    pools = [H.to_device_logits(H.build_pool(cfg, seeds_a)), H.to_device_logits(H.build_pool(cfg, seeds_b))]
    roots = torch.from_numpy(H.root_tokens(cfg)).cuda()

    def fresh():
        st = T.TreeState(cfg.B, cfg.N)
        return (st, T.Candidates(cfg.B, st.N_pad, cfg.K),
                T.make_expand_workspace(cfg.B, st.N_pad, cfg.V, cfg.K, T.TALON_DTYPE_BF16),
                torch.full((cfg.B, st.N_pad, st.N_pad // 64), -1, dtype=torch.int64, device="cuda"))

    want = []
    for p in pools:
        st, cand, ws, mask = fresh()
        want.append(_expand_on(cfg, p, st, cand, ws, mask, roots))
    assert want[0]["token"][0].tolist() != want[1]["token"][0].tolist()
    st, cand, ws, mask = fresh()
    for i in range(40):
        _same_trees(_expand_on(cfg, pools[i % 2], st, cand, ws, mask, roots), want[i % 2])
    T.talon_set_spin_limit_us(0)
    try:
        cut = _expand_on(cfg, pools[0], st, cand, ws, mask, roots)
    finally:
        T.talon_set_spin_limit_us(200000)
    aborted = (cut["status"] & T.TALON_STATUS_ABORTED) != 0
    assert aborted.all() or not aborted.any()
    for i in range(6):
        _same_trees(_expand_on(cfg, pools[i % 2], st, cand, ws, mask, roots), want[i % 2])


def test_launch_forms_share_one_workspace():
    """All four launch forms (whole tree in one launch, continued tree in one launch, one fused
    launch per layer, scan and selection as separate launches) take turns on ONE workspace and
    tree state, on two inputs: none may leave anything behind that another one trips over."""
    import torch
    import paper_2601_07353_amd as T
    cfg = small(name="forms", V=40000, logits_dtype="bf16", K=8, N=100, Dmax=12, B=3,
                recipe=(("gauss", 6.0, 8.0), ("gauss", 0.5, 1.0), ("gauss", 2.0, 8.0)))
    seeds_a = admissible_seeds(cfg)
    seeds_b = admissible_seeds(dataclasses.replace(cfg, seed=cfg.seed + 77))
    pools = [H.to_device_logits(H.build_pool(cfg, seeds_a)), H.to_device_logits(H.build_pool(cfg, seeds_b))]
    roots = torch.from_numpy(H.root_tokens(cfg)).cuda()
    st = T.TreeState(cfg.B, cfg.N)
    cand = T.Candidates(cfg.B, st.N_pad, cfg.K)
    ws = T.make_expand_workspace(cfg.B, st.N_pad, cfg.V, cfg.K, T.TALON_DTYPE_BF16)
    mask = torch.full((cfg.B, st.N_pad, st.N_pad // 64), -1, dtype=torch.int64, device="cuda")

    def snapshot():
        torch.cuda.synchronize()
        n = [int(x) for x in st.n_nodes.cpu()]
        return {"n": n, "status": st.status.cpu().numpy().copy(),
                "token": [st.token[b, :k].cpu().numpy().copy() for b, k in enumerate(n)],
                "parent": [st.parent[b, :k].cpu().numpy().copy() for b, k in enumerate(n)],
                "logp": [st.logp[b, :k].cpu().numpy().copy() for b, k in enumerate(n)]}

    def same(a, b):
        # The launch forms cut rows into chunks by different rules (a layer at a time: from all
        # frontier rows of the layer; the single launch: per sequence), so a row's log-sum-exp is
        # summed in a different order and path confidences agree to rounding, not bit for bit.
        assert a["n"] == b["n"]
        np.testing.assert_array_equal(a["status"], b["status"])
        for key in ("token", "parent"):
            for x, y in zip(a[key], b[key]):
                np.testing.assert_array_equal(x, y)
        for x, y in zip(a["logp"], b["logp"]):
            np.testing.assert_allclose(x, y, rtol=0, atol=2 * H.LSE_ATOL * 24)   # one rounding per layer on the path

    def whole(p):
        T.talon_build_tree(roots, p, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, mask=mask)

    def continued(p):
        T.talon_tree_init(st, roots)
        T.talon_expand_tree(p, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws)

    def per_layer(p):
        T.talon_tree_init(st, roots)
        for d in range(cfg.Dmax):
            T.talon_expand_select_layer(p, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, layer=d)

    def split(p):
        T.talon_tree_init(st, roots)
        for d in range(cfg.Dmax):
            T.talon_expand_layer(p, st, cfg.K, cand, ws, layer=d)
            T.talon_select_budget(st, cfg.K, cand, cfg.mu, cfg.K, 1, cfg.Dmax)

    want = []
    for p in pools:
        whole(p)
        want.append(snapshot())
    order = [(whole, 0), (per_layer, 1), (whole, 0), (continued, 1), (split, 0), (whole, 1), (continued, 0),
             (per_layer, 0), (whole, 1), (split, 1), (continued, 1), (whole, 0)]
    for form, which in order:
        form(pools[which])
        same(snapshot(), want[which])


def test_captured_steps_replay_like_eager_ones():
    """A serving loop captures its step once and replays it.  Two graphs over ONE workspace and tree
    state (one launch per layer + mask; the whole tree in one launch) are replayed in turns, with
    the logits buffer they read rewritten, eager launches of the other forms and synchronisations
    between the replays: every replay must give the tree and mask the eager launch gives, so the
    counters the launches share (row tickets, the two per-layer counts, exit tickets) have to be
    back at zero after every replay, not only after the first."""
    import torch
    import paper_2601_07353_amd as T
    cfg = small(name="replay", V=40000, logits_dtype="bf16", K=8, N=100, Dmax=12, B=3,
                recipe=(("gauss", 6.0, 8.0), ("gauss", 0.5, 1.0), ("gauss", 2.0, 8.0)))
    seeds = [admissible_seeds(dataclasses.replace(cfg, seed=cfg.seed + 31 * i)) for i in range(3)]
    pools = [H.to_device_logits(H.build_pool(cfg, s)) for s in seeds]
    live = torch.empty_like(pools[0])          # the buffer the captured launches read
    roots = torch.from_numpy(H.root_tokens(cfg)).cuda()
    st = T.TreeState(cfg.B, cfg.N)
    cand = T.Candidates(cfg.B, st.N_pad, cfg.K)
    ws = T.make_expand_workspace(cfg.B, st.N_pad, cfg.V, cfg.K, T.TALON_DTYPE_BF16)
    mask = torch.zeros((cfg.B, st.N_pad, st.N_pad // 64), dtype=torch.int64, device="cuda")

    def snapshot():
        torch.cuda.synchronize()
        n = [int(x) for x in st.n_nodes.cpu()]
        return {"n": n, "status": st.status.cpu().numpy().copy(),
                "token": [st.token[b, :k].cpu().numpy().copy() for b, k in enumerate(n)],
                "parent": [st.parent[b, :k].cpu().numpy().copy() for b, k in enumerate(n)],
                "mask": [mask[b, :k].cpu().numpy().copy() for b, k in enumerate(n)]}

    def same(a, b):
        assert a["n"] == b["n"]
        np.testing.assert_array_equal(a["status"], b["status"])
        for key in ("token", "parent", "mask"):
            for x, y in zip(a[key], b[key]):
                np.testing.assert_array_equal(x, y)

    def per_layer(p):
        T.talon_tree_init(st, roots)
        for d in range(cfg.Dmax):
            T.talon_expand_select_layer(p, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, layer=d)
        T.talon_build_tree_mask(st, mask)

    def whole(p):
        T.talon_build_tree(roots, p, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, mask=mask)

    want = []
    for p in pools:
        per_layer(p)
        want.append(snapshot())
    assert want[0]["token"][0].tolist() != want[1]["token"][0].tolist()

    graphs = {}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):             # one eager pass on the capture stream first
        live.copy_(pools[0])
        per_layer(live)
        whole(live)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for name, form in (("per_layer", per_layer), ("whole", whole)):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            form(live)
        graphs[name] = g

    order = [("per_layer", 1), ("per_layer", 2), ("whole", 0), ("per_layer", 0), ("whole", 1), ("per_layer", 1),
             ("per_layer", 2), ("whole", 2), ("per_layer", 0)]
    for i, (name, which) in enumerate(order):
        live.copy_(pools[which])
        mask.fill_(-1)
        graphs[name].replay()
        same(snapshot(), want[which])
        other = (which + 1) % 3               # eager work of the other form on the same workspace in between
        (whole if name == "per_layer" else per_layer)(pools[other])
        same(snapshot(), want[other])
        if i % 3 == 2:
            torch.cuda.synchronize()
            (live.float().sum() + st.logp.sum()).item()   # library work of the program's own between replays


@pytest.mark.parametrize("fused", [True, False])
def test_dense_frontier_batches_with_padded_rows(fused):
    """The layout a serving loop has: after every layer the draft model's logits exist for the
    new frontier only, as a dense batch [B][frontier rows][padded row] (TALON_ROWS_BY_FRONTIER,
    row stride larger than the vocabulary, garbage in the padding).  One call per layer on a
    freshly gathered batch must build the tree the oracle builds."""
    import torch
    import paper_2601_07353_amd as T
    cfg = small(name="dense", V=20011, logits_dtype="bf16", K=6, N=70, Dmax=9, B=3,
                recipe=(("gauss", 4.0, 8.0), ("gauss", 0.5, 1.0), ("gauss", 2.0, 6.0)))
    seeds = admissible_seeds(cfg)
    pool = H.build_pool(cfg, seeds)
    ref = H.run_oracle_step(cfg, seeds, pool=pool, with_attention=False)
    pool_dev = H.to_device_logits(pool)                      # [B][N_pad][V], only used to gather from
    stride = (cfg.V + 8 + 63) // 64 * 64                     # padded rows
    st = T.TreeState(cfg.B, cfg.N)
    cand = T.Candidates(cfg.B, st.N_pad, cfg.K)
    ws = T.make_expand_workspace(cfg.B, st.N_pad, cfg.V, cfg.K, T.TALON_DTYPE_BF16)
    T.talon_tree_init(st, torch.from_numpy(H.root_tokens(cfg)).cuda())
    for d in range(cfg.Dmax):
        begin = st.frontier_begin.cpu().numpy()
        count = st.frontier_count.cpu().numpy()
        done = (st.status.cpu().numpy() & 3) != 0
        if done.all():
            break
        fmax = max(1, int(count.max()))
        dense = torch.full((cfg.B, fmax, stride), 30000.0, dtype=torch.bfloat16, device="cuda")   # padding would win any max
        for b in range(cfg.B):
            if not done[b]:
                dense[b, :count[b], :cfg.V] = pool_dev[b, begin[b]:begin[b] + count[b]]
        if fused:
            T.talon_expand_select_layer(dense, st, cfg.K, cfg.mu, cfg.K, 1, cfg.Dmax, cand, ws, layer=d,
                                        row_mode=T.TALON_ROWS_BY_FRONTIER, vocab=cfg.V)
        else:
            T.talon_expand_layer(dense, st, cfg.K, cand, ws, row_mode=T.TALON_ROWS_BY_FRONTIER, layer=d, vocab=cfg.V)
            T.talon_select_budget(st, cfg.K, cand, cfg.mu, cfg.K, 1, cfg.Dmax)
        torch.cuda.synchronize()
    n = st.n_nodes.cpu().numpy()
    for b, t in enumerate(ref["trees"]):
        assert int(n[b]) == t.n
        np.testing.assert_array_equal(st.token[b, :t.n].cpu().numpy(), np.asarray(t.token, dtype=np.int32))
        np.testing.assert_array_equal(st.parent[b, :t.n].cpu().numpy(), np.asarray(t.parent, dtype=np.int32))
        np.testing.assert_allclose(np.exp(st.logp[b, :t.n].cpu().numpy()), t.confidence(), rtol=H.PROB_RTOL, atol=0)


@pytest.mark.parametrize("mode", ["split", "fused", "tree"])
def test_layerwise_entry_points_against_oracle(mode):
    """The per-layer entry points (scan and selection as two launches, or as one) on a batch
    of three sequences with different logit recipes, several chunks per row."""
    cfg = small(name="layerwise-" + mode, V=40000, logits_dtype="bf16", K=8, N=130, Dmax=20, B=3, Hq=8, Hkv=2,
                Dh=128, L=200, recipe=(("gauss", 6.0, 8.0), ("gauss", 0.5, 1.0), ("zipf_mix", 1.2, 0.05)))
    step_and_compare(cfg, with_attention=False, layerwise=mode)


def test_repeated_calls_agree_on_every_row():
    """The same call 200 times, each on a freshly cleared workspace: every row's softmax
    statistics, every candidate and every tree must come out the same each time, and equal to
    the oracle's.  (A chunk's partial results must have been performed before the ticket that
    announces them: a ticket that overtakes them shows up here as a row whose log-sum-exp
    misses one chunk, once in some tens of calls.)"""
    import torch
    cfg = small(name="repeat", V=40000, logits_dtype="bf16", K=8, N=130, Dmax=20, B=3, Hq=8, Hkv=2, Dh=128, L=200,
                recipe=(("gauss", 6.0, 8.0), ("gauss", 0.5, 1.0), ("zipf_mix", 1.2, 0.05)))
    seeds = admissible_seeds(cfg)
    pool = H.build_pool(cfg, seeds)
    ref = H.run_oracle_step(cfg, seeds, pool=pool, with_attention=False)
    pool_dev = H.to_device_logits(pool)
    first = None
    for rep in range(200):
        st, cand, _, mask = H.run_gpu_expand(cfg, pool_dev)
        got = {"row_lse": cand.row_lse, "row_max": cand.row_max, "cand_token": cand.token, "token": st.token,
               "parent": st.parent, "n_nodes": st.n_nodes, "mask": mask}
        n = [int(x) for x in st.n_nodes.cpu()]
        assert n == [t.n for t in ref["trees"]], (rep, n)
        rows = [(b, r.node) for b, t in enumerate(ref["trees"]) for pl in t.pools for r in pl]
        bi = torch.tensor([b for b, _ in rows], device="cuda"); ni = torch.tensor([i for _, i in rows], device="cuda")
        snap = {"row_lse": got["row_lse"][bi, ni].clone(), "row_max": got["row_max"][bi, ni].clone(),
                "cand_token": got["cand_token"][bi, ni].clone(),
                "token": torch.cat([got["token"][b, :k] for b, k in enumerate(n)]),
                "parent": torch.cat([got["parent"][b, :k] for b, k in enumerate(n)]),
                "mask": torch.cat([got["mask"][b, :k].reshape(-1) for b, k in enumerate(n)])}
        if first is None:
            first = snap
            want = np.array([r.row_lse for t in ref["trees"] for pl in t.pools for r in pl])
            assert np.abs(snap["row_lse"].cpu().numpy() - want).max() <= H.LSE_ATOL
        else:
            for key, v in snap.items():
                assert torch.equal(v, first[key]), (rep, key)


def test_c2_llama3_8b_step_full_size():
    worst, gpu, ref = step_and_compare(CONFIGS["c2"])
    print("c2 attention worst abs err", worst)


@pytest.mark.parametrize("kw", [
    dict(V=1000, logits_dtype="bf16", K=5, N=40, Dmax=10),        # bf16 row with a ragged 8-vector tail? (1000 % 8 == 0)
    dict(V=1003, logits_dtype="f32", K=4, N=33, Dmax=9),           # ragged f32 tail, N not a multiple of 64
    dict(V=20011, logits_dtype="bf16", K=16, N=100, Dmax=12, recipe=("gauss", 0.5, 8.0)),   # 3 chunks, ragged
    dict(V=9001, logits_dtype="f32", K=7, N=64, Dmax=16, recipe=("gauss", 2.0, 8.0)),       # 3 f32 chunks
    dict(V=40000, logits_dtype="bf16", K=8, N=130, Dmax=20, B=3, Hq=8, Hkv=2, Dh=128, L=200,
         recipe=(("gauss", 6.0, 8.0), ("gauss", 0.5, 1.0), ("zipf_mix", 1.2, 0.05))),
    dict(V=32000, logits_dtype="bf16", K=10, N=256, Dmax=24, B=2, Hq=8, Hkv=8, Dh=64, L=70,
         recipe=("zipf_mix", 1.2, 0.05)),
])
def test_small_variants(kw):
    cfg = small(name="variant", **kw)
    step_and_compare(cfg)


@pytest.mark.parametrize("mu", [0.01, 0.04, 1.0, 1e-30])
def test_mu_sweep(mu):
    cfg = small(name="mu", V=4096, logits_dtype="bf16", K=6, N=48, Dmax=48, mu=mu)
    step_and_compare(cfg, with_attention=False)


@pytest.mark.parametrize("init_layers,K_init", [(0, 4), (2, 4), (3, 2), (1, 9)])
def test_init_layer_variants(init_layers, K_init):
    cfg = small(name="init", V=4096, logits_dtype="bf16", K=6, N=40, Dmax=12)
    seeds = [H.find_admissible_seed(cfg, 0, cfg.seed + 3, init_layers=init_layers, K_init=K_init)[0]]
    pool = H.build_pool(cfg, seeds)
    gpu = H.run_gpu_step(cfg, seeds, pool=pool, with_attention=False, init_layers=init_layers, K_init=K_init)
    ref = H.run_oracle_step(cfg, seeds, pool=pool, with_attention=False, init_layers=init_layers, K_init=K_init)
    assert ref["trees"][0].margin > H.MARGIN_TOL
    H.compare_step(cfg, gpu, ref)


# ----------------------------------------------------------------------------- degenerate rows
def custom_pool(cfg, fill):
    dt = np.float32 if cfg.logits_dtype == "f32" else np.uint16
    pool = np.zeros((cfg.B, cfg.N_pad, cfg.V), dtype=dt)
    for b in range(cfg.B):
        for i in range(cfg.N):
            x = fill(b, i).astype(np.float32)
            pool[b, i] = x if cfg.logits_dtype == "f32" else f32_to_bf16_bits(x)
    return pool


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_constant_rows_all_ties(dtype):
    """Every logit equal: every candidate ties, lowest token ids win, budget spent at layer 2."""
    cfg = small(name="const", V=20000, logits_dtype=dtype, K=5, N=20, Dmax=6)
    pool = custom_pool(cfg, lambda b, i: np.full(cfg.V, 1.5))
    gpu = H.run_gpu_step(cfg, pool=pool, with_attention=False)
    ref = H.run_oracle_step(cfg, pool=pool, with_attention=False)
    H.compare_step(cfg, gpu, ref)
    assert list(gpu["token"][0, 1:6]) == [0, 1, 2, 3, 4]


def test_one_hot_rows_deep_chain():
    cfg = small(name="onehot", V=30000, logits_dtype="bf16", K=4, N=24, Dmax=64)

    def fill(b, i):
        x = np.zeros(cfg.V); x[(977 * (i + 1)) % cfg.V] = 40.0
        return x

    pool = custom_pool(cfg, fill)
    gpu = H.run_gpu_step(cfg, pool=pool, with_attention=False)
    ref = H.run_oracle_step(cfg, pool=pool, with_attention=False)
    H.compare_step(cfg, gpu, ref)
    assert gpu["depth"][0, :24].max() == 24 - 4


def test_sorted_rows_and_neg_inf_entries():
    """Monotone rows (all of a chunk's best logits sit in one lane) and rows that are mostly -inf."""
    cfg = small(name="sorted", V=17000, logits_dtype="f32", K=8, N=30, Dmax=8)

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

    pool, _ = H.admissible_pool(cfg, make_pool, cap=cfg.K)
    gpu = H.run_gpu_step(cfg, pool=pool, with_attention=False)
    ref = H.run_oracle_step(cfg, pool=pool, with_attention=False)
    H.compare_step(cfg, gpu, ref)


def test_vocab_smaller_than_k():
    cfg = small(name="tinyv", V=8, logits_dtype="f32", K=12, N=14, Dmax=4, mu=1e-30)
    seeds = admissible_seeds(cfg)
    pool = H.build_pool(cfg, seeds)
    gpu = H.run_gpu_step(cfg, seeds, pool=pool, with_attention=False)
    ref = H.run_oracle_step(cfg, seeds, pool=pool, with_attention=False)
    assert min(t.margin for t in ref["trees"]) > H.MARGIN_TOL
    H.compare_step(cfg, gpu, ref)
    assert (gpu["cand_token"][0, 0, 8:] == -1).all()


def test_nan_row_sets_status_and_stops_sequence():
    cfg = small(name="nan", V=5000, logits_dtype="f32", K=3, N=20, Dmax=6, B=2)
    seeds = [H.find_admissible_seed(cfg, 0, cfg.seed)[0], cfg.seed]
    pool = H.build_pool(cfg, seeds)
    pool[1, 2, 1234] = np.nan
    gpu = H.run_gpu_step(cfg, seeds, pool=pool, with_attention=False)
    ref = H.run_oracle_step(dataclasses.replace(cfg, B=1), seeds[:1], pool=pool[:1], with_attention=False)
    assert int(gpu["status"][1]) & 4
    assert int(gpu["n_nodes"][1]) == 1 + cfg.K          # stopped after the layer that read the bad row
    assert int(gpu["frontier_count"][1]) == 0
    assert ref["trees"][0].margin > H.MARGIN_TOL
    H.compare_tree(cfg, {k: v[:1] for k, v in gpu.items()}, ref["trees"])


def test_budget_of_one_and_two():
    for N in (1, 2):
        cfg = small(name="n%d" % N, V=2048, logits_dtype="bf16", K=4, N=N, Dmax=4)
        gpu = H.run_gpu_step(cfg, [cfg.seed], with_attention=False)
        ref = H.run_oracle_step(cfg, [cfg.seed], with_attention=False)
        H.compare_step(cfg, gpu, ref)


def test_maximum_batch_of_256_sequences():
    """B at the library's limit: 256 tiny sequences in one call (prefix over sequences, item
    map and the per-sequence tickets at their largest)."""
    cfg = small(name="b256", B=256, V=520, logits_dtype="bf16", K=3, N=9, Dmax=5, Hq=4, Hkv=4, Dh=64, L=16,
                recipe=("gauss", 1.0, 4.0))
    step_and_compare(cfg)


def test_integer_outputs_are_reproducible_run_to_run():
    cfg = small(name="repro", V=50000, logits_dtype="bf16", K=10, N=60, Dmax=12, B=2, recipe=("gauss", 0.5, 8.0))
    seeds = [cfg.seed, cfg.seed]
    pool = H.build_pool(cfg, seeds)
    a = H.run_gpu_step(cfg, seeds, pool=pool, with_attention=False)
    for _ in range(3):
        b = H.run_gpu_step(cfg, seeds, pool=pool, with_attention=False)
        for key in ("token", "parent", "depth", "n_nodes", "mask", "cand_token", "row_lse", "logp"):
            np.testing.assert_array_equal(a[key], b[key])


# ----------------------------------------------------------------------------- attention only
def attention_case(B, n_list, Hq, Hkv, Dh, L_list, seed, parents=None):
    """Random trees (random parent pointers) straight into mask + attention, ragged prefix lengths."""
    import torch
    import paper_2601_07353_amd as T
    from oracle import talon_oracle as O
    rng = np.random.default_rng(seed)
    N = max(n_list)
    N_pad = (N + 63) // 64 * 64
    Lmax = max(L_list)
    st = T.TreeState(B, N)
    parent = np.full((B, N_pad), -1, dtype=np.int32)
    for b in range(B):
        for i in range(1, n_list[b]):
            parent[b, i] = rng.integers(0, i) if parents is None else parents[b][i]
    st.parent.copy_(torch.from_numpy(parent))
    st.n_nodes.copy_(torch.tensor(n_list, dtype=torch.int32))
    mask = torch.zeros(B, N_pad, N_pad // 64, dtype=torch.int64, device="cuda")
    T.talon_build_tree_mask(st, mask)

    def bits(shape):
        return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))

    q, kt, vt = bits((B, N_pad, Hq, Dh)), bits((B, N_pad, Hkv, Dh)), bits((B, N_pad, Hkv, Dh))
    kp, vp = bits((B, max(Lmax, 1), Hkv, Dh)), bits((B, max(Lmax, 1), Hkv, Dh))
    out = torch.zeros(B, N_pad, Hq, Dh, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(B, N_pad, Hq, dtype=torch.float32, device="cuda")
    nb = T.talon_tree_attention_workspace_bytes(B, N_pad, Hq, Hkv, Dh, Lmax)
    ws = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
    plen = torch.tensor(L_list, dtype=torch.int32, device="cuda")
    T.talon_tree_attention(H.bf16_to_device(q), H.bf16_to_device(kp), H.bf16_to_device(vp), H.bf16_to_device(kt),
                           H.bf16_to_device(vt), mask, st.n_nodes, plen, Lmax, out, lse, ws)
    torch.cuda.synchronize()
    got, got_lse = out.float().cpu().numpy(), lse.cpu().numpy()
    gmask = mask.cpu().numpy().view(np.uint64)
    worst = 0.0
    for b in range(B):
        n, L = n_list[b], L_list[b]
        m = O.build_tree_mask(list(parent[b, :n]))
        np.testing.assert_array_equal(gmask[b], O.mask_to_words(m, N_pad))
        f = H.bf16_bits_to_f64
        want, wlse = O.tree_attention(f(q[b, :n]), f(kp[b, :L]), f(vp[b, :L]), f(kt[b, :n]), f(vt[b, :n]), m)
        err, _ = H.check_attention_rows(got[b, :n], got_lse[b, :n], want, wlse, L + m.sum(axis=1), (b,))
        worst = max(worst, err)
        assert not got[b, n:].any()
    return worst


@pytest.mark.parametrize("B,n_list,Hq,Hkv,Dh,L_list", [
    (1, [16], 4, 4, 64, [128]),
    (2, [60, 37], 8, 2, 128, [300, 77]),        # GQA 4, ragged prefix lengths, ragged tiles
    (1, [1], 4, 2, 64, [0]),                    # root only, empty prefix: output = own value
    (3, [200, 130, 256], 4, 1, 128, [64, 1, 1000]),   # several tree tiles, G = 4
    (1, [100], 16, 1, 64, [513]),               # G = 16
    (2, [64, 65], 6, 2, 128, [4096, 63]),       # G = 3 (rows of a node straddle row blocks)
])
def test_tree_attention_random_trees(B, n_list, Hq, Hkv, Dh, L_list):
    worst = attention_case(B, n_list, Hq, Hkv, Dh, L_list, seed=123)
    print("worst abs err", worst)


def test_tree_attention_chain_and_star():
    n = 50
    attention_case(1, [n], 8, 4, 128, [100], seed=5, parents=[[-1] + list(range(n - 1))])
    attention_case(1, [n], 8, 4, 128, [100], seed=6, parents=[[-1] + [0] * (n - 1)])


def test_tree_attention_strided_prefix_view():
    """Prefix K/V given as a strided view of a larger cache (extra heads and tokens)."""
    import torch
    import paper_2601_07353_amd as T
    from oracle import talon_oracle as O
    rng = np.random.default_rng(9)
    B, n, Hq, Hkv, Dh, L = 2, 20, 4, 2, 64, 150
    N_pad = 64
    st = T.TreeState(B, n)
    parent = np.full((B, N_pad), -1, dtype=np.int32)
    for b in range(B):
        for i in range(1, n):
            parent[b, i] = rng.integers(0, i)
    st.parent.copy_(torch.from_numpy(parent)); st.n_nodes.fill_(n)
    mask = torch.zeros(B, N_pad, 1, dtype=torch.int64, device="cuda")
    T.talon_build_tree_mask(st, mask)
    bits = lambda shape: f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))
    q, kt, vt = bits((B, N_pad, Hq, Dh)), bits((B, N_pad, Hkv, Dh)), bits((B, N_pad, Hkv, Dh))
    cache_k, cache_v = bits((B, 2 * L, Hkv + 3, Dh)), bits((B, 2 * L, Hkv + 3, Dh))
    dk, dv = H.bf16_to_device(cache_k), H.bf16_to_device(cache_v)
    kp, vp = dk[:, 10:10 + L, 1:1 + Hkv, :], dv[:, 10:10 + L, 1:1 + Hkv, :]
    out = torch.zeros(B, N_pad, Hq, Dh, dtype=torch.bfloat16, device="cuda")
    nb = T.talon_tree_attention_workspace_bytes(B, N_pad, Hq, Hkv, Dh, L)
    ws = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
    plen = torch.full((B,), L, dtype=torch.int32, device="cuda")
    T.talon_tree_attention(H.bf16_to_device(q), kp, vp, H.bf16_to_device(kt), H.bf16_to_device(vt), mask,
                           st.n_nodes, plen, L, out, None, ws)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    f = H.bf16_bits_to_f64
    for b in range(B):
        m = O.build_tree_mask(list(parent[b, :n]))
        want, _ = O.tree_attention(f(q[b, :n]), f(cache_k[b, 10:10 + L, 1:1 + Hkv]), f(cache_v[b, 10:10 + L, 1:1 + Hkv]),
                                   f(kt[b, :n]), f(vt[b, :n]), m)
        H.check_attention_rows(got[b, :n], None, want, None, L + m.sum(axis=1), (b,))


# ----------------------------------------------------------------------------- long candidate lists
def _seeds_for_kinit(cfg, K_init):
    from workloads import logits_row
    roots = H.root_tokens(cfg)
    seeds = []
    for b in range(cfg.B):
        for s in range(cfg.seed, cfg.seed + 64):
            rows = {}

            class Lazy:
                def __getitem__(self, i):
                    if i not in rows:
                        rows[i] = logits_row(cfg, s, b, i)
                    return rows[i]

            t = H.oracle_tree(cfg, Lazy(), roots[b], K_init=K_init)
            if t.margin > H.MARGIN_TOL:
                seeds.append(s)
                break
        else:
            raise RuntimeError("no admissible seed")
    return seeds


@pytest.mark.parametrize("kw", [
    dict(V=5000, logits_dtype="f32", K=40, N=33, Dmax=10),                                    # cap 40 >= N - 1
    dict(V=40000, logits_dtype="bf16", K=64, N=60, Dmax=12, B=2, Hq=8, Hkv=2, Dh=128, L=100,
         recipe=(("gauss", 0.5, 1.0), ("gauss", 2.0, 6.0))),                                   # flat and peaked rows
])
def test_per_row_cap_up_to_64(kw):
    """Candidate lists longer than 16 per row (the long-list merge paths), first layer Top-10."""
    cfg = small(name="cap64", **kw)
    seeds = _seeds_for_kinit(cfg, 10)
    step_and_compare(cfg, seeds=seeds, K_init=10, with_attention=False)


def test_c2_shape_uncapped_gate_is_the_paper_literal_tree():
    """Alg. 2 pools every token of every parent.  With a per-row cap of 64 >= N - 1 = 59 the capped
    pool gives exactly that tree: the GPU (k = 64) is compared with the oracle run on the full
    vocabulary (cap = V), Llama-3-8B shape, Top-10 first layer."""
    import dataclasses
    from oracle import talon_oracle as O
    from workloads import logits_row, storage_to_f64
    cfg = dataclasses.replace(CONFIGS["c2"], name="c2-cap64", K=64)
    seeds = _seeds_for_kinit(cfg, 10)
    worst, gpu, ref = step_and_compare(cfg, seeds=seeds, K_init=10, with_attention=False)
    rows = {}

    def row_of(i):
        if i not in rows:
            rows[i] = storage_to_f64(logits_row(cfg, seeds[0], 0, i))
        return rows[i]

    full = O.build_tree(row_of, int(H.root_tokens(cfg)[0]), N=cfg.N, K=10, mu=float(np.float32(cfg.mu)), cap=cfg.V,
                        Dmax=cfg.Dmax, init_layers=1)
    n = full.n
    assert int(gpu["n_nodes"][0]) == n
    np.testing.assert_array_equal(gpu["token"][0, :n], np.asarray(full.token, dtype=np.int32))
    np.testing.assert_array_equal(gpu["parent"][0, :n], np.asarray(full.parent, dtype=np.int32))
    fan = np.bincount(np.asarray(full.parent[1:]), minlength=n)
    print("c2 shape, uncapped gate: largest fan-out", int(fan.max()), "depths", np.bincount(full.depth).tolist())
