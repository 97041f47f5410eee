"""Test harness: runs one expand+verify step through the HIP library and through the CPU
oracle on the same seeded inputs, and compares them.  Test infrastructure only."""
from __future__ import annotations

import math

import numpy as np

from workloads import (WorkloadConfig, attention_inputs, bf16_bits_to_f64, bf16_to_device, build_pool,  # noqa: F401
                       logits_row, root_tokens, storage_to_f64, to_device_logits)

MARGIN_TOL = 1e-4   # smallest cross-parent score gap a seed must leave (log units)
PROB_RTOL = 1e-5    # probabilities and path confidences, relative
ATTN_ATOL = 2e-2    # tree-attention outputs, absolute (bf16 inputs, fp64 oracle): the stated bound
LSE_ATOL = 2e-6     # row log-sum-exp, absolute
# Beside the stated bound, one tied to the signal, so that at long prefixes (outputs of a few
# hundredths) a lost tree key or a wrong mask bit cannot hide below 2e-2.  The kernel rounds the
# softmax weights to bf16 before the P.V product and the result to bf16:
#   output rounding      <= 2^-8 |out|   (half a unit in the last of 8 significant bits)
#   weight rounding      each weight off by a relative delta_j, |delta_j| <= 2^-8, independent:
#                        error = sum_j p_j delta_j v_j, standard deviation about
#                        2^-8 / sqrt(3) * sqrt(sum_j p_j^2) for unit-variance values; with
#                        N(0,1) scores sum_j p_j^2 is about e / keys, i.e. 3.7e-3 / sqrt(keys);
#                        six standard deviations (millions of elements are compared)
ATTN_OUT_RTOL = 2.0 ** -8
ATTN_KEYS_ATOL = 2.2e-2      # divided by sqrt(number of keys the row attends to)
ATTN_LSE_ATOL = 2e-5         # fp32 scores and denominators against fp64 (observed worst 1.6e-6)


def seeds_for(cfg: WorkloadConfig, seeds=None):
    if seeds is None:
        return [cfg.seed] * cfg.B
    if isinstance(seeds, int):
        return [seeds] * cfg.B
    return list(seeds)


# --------------------------------------------------------------------------- oracle side
def oracle_tree(cfg: WorkloadConfig, pool_b: np.ndarray, root: int, init_layers: int = 1, mu=None, K_init=None,
                cap=None):
    from oracle import talon_oracle as O
    cache = {}

    def row_of(i):
        if i not in cache:
            cache[i] = storage_to_f64(pool_b[i])
        return cache[i]

    mu = float(np.float32(cfg.mu if mu is None else mu))  # the ABI takes mu as a float
    K_init = cfg.K if K_init is None else K_init
    return O.build_tree(row_of, int(root), N=cfg.N, K=K_init, mu=mu, cap=cfg.K if cap is None else cap, Dmax=cfg.Dmax,
                        init_layers=init_layers)


def find_admissible_seed(cfg: WorkloadConfig, b: int, base_seed: int, tol: float = MARGIN_TOL, max_tries: int = 64,
                         **tree_kw):
    """First seed >= base_seed whose oracle tree for sequence b leaves every cross-parent
    decision a margin > tol, so that an fp32 log-sum-exp cannot change the topology."""
    roots = root_tokens(cfg)
    for s in range(base_seed, base_seed + max_tries):
        rows = {}

        class Lazy:
            def __getitem__(self, i):
                if i not in rows:
                    rows[i] = logits_row(cfg, s, b, i)
                return rows[i]

        t = oracle_tree(cfg, Lazy(), roots[b], **tree_kw)
        if t.margin > tol:
            return s, t
    raise RuntimeError("no admissible seed found for %s sequence %d" % (cfg.name, b))


def admissible_pool(cfg: WorkloadConfig, make_pool, tries: int = 16, **tree_kw):
    """First of make_pool(0), make_pool(1), ... whose oracle trees all leave every cross-parent
    decision a margin > MARGIN_TOL.  Returns (pool, trees); fails the test if none qualifies, so
    a case can never go untested in silence."""
    roots = root_tokens(cfg)
    for attempt in range(tries):
        pool = make_pool(attempt)
        trees = [oracle_tree(cfg, pool[b], roots[b], **tree_kw) for b in range(cfg.B)]
        if min(t.margin for t in trees) > MARGIN_TOL:
            return pool, trees
    raise AssertionError("no admissible pool among %d tries for %s" % (tries, cfg.name))


def run_oracle_step(cfg: WorkloadConfig, seeds=None, pool=None, attn=None, attn_nodes=None, attn_heads=None,
                    with_attention=True, init_layers=1, mu=None, K_init=None):
    from oracle import talon_oracle as O
    seeds = seeds_for(cfg, seeds)
    pool = build_pool(cfg, seeds) if pool is None else pool
    roots = root_tokens(cfg)
    res = {"trees": [], "mask": [], "attn_out": [], "attn_lse": []}
    for b in range(cfg.B):
        t = oracle_tree(cfg, pool[b], roots[b], init_layers, mu, K_init)
        m = O.build_tree_mask(t.parent)
        res["trees"].append(t)
        res["mask"].append(m)
        if with_attention:
            x = attention_inputs(cfg, seeds[b], b) if attn is None else attn[b]
            n = t.n
            out, lse = O.tree_attention(bf16_bits_to_f64(x["q"][:n]), bf16_bits_to_f64(x["k_prefix"]),
                                        bf16_bits_to_f64(x["v_prefix"]), bf16_bits_to_f64(x["k_tree"][:n]),
                                        bf16_bits_to_f64(x["v_tree"][:n]), m, nodes=attn_nodes, heads=attn_heads)
            res["attn_out"].append(out)
            res["attn_lse"].append(lse)
    return res


# --------------------------------------------------------------------------- GPU side
def run_gpu_expand(cfg: WorkloadConfig, pool_dev, init_layers=1, mu=None, K_init=None, layerwise=False):
    """Whole expansion loop on the GPU.  Default: talon_build_tree (init, loop and mask in two
    launches; the mask is returned).  layerwise="tree": talon_tree_init + talon_expand_tree;
    "fused": one talon_expand_select_layer per layer; True / "split": talon_expand_layer +
    talon_select_budget per layer.  Those three return no mask."""
    import torch
    import paper_2601_07353_amd as T
    st = T.TreeState(cfg.B, cfg.N)
    cand = T.Candidates(cfg.B, st.N_pad, cfg.K)
    dt = T.TALON_DTYPE_F32 if cfg.logits_dtype == "f32" else T.TALON_DTYPE_BF16
    ws = T.make_expand_workspace(cfg.B, st.N_pad, cfg.V, cfg.K, dt)
    roots = torch.from_numpy(root_tokens(cfg)).cuda()
    mu = cfg.mu if mu is None else mu
    K_init = cfg.K if K_init is None else K_init
    mask = None
    if layerwise == "fused":
        T.talon_tree_init(st, roots)
        for d in range(cfg.Dmax):
            T.talon_expand_select_layer(pool_dev, st, cfg.K, mu, K_init, init_layers, cfg.Dmax, cand, ws,
                                        layer=d if d % 2 == 0 else -1)
    elif layerwise == "tree":
        T.talon_tree_init(st, roots)
        T.talon_expand_tree(pool_dev, st, cfg.K, mu, K_init, init_layers, cfg.Dmax, cand, ws)
    elif layerwise:
        T.talon_tree_init(st, roots)
        for d in range(cfg.Dmax):
            T.talon_expand_layer(pool_dev, st, cfg.K, cand, ws, layer=d if d % 2 == 0 else -1)
            T.talon_select_budget(st, cfg.K, cand, mu, K_init, init_layers, cfg.Dmax)
    else:
        mask = torch.full((cfg.B, st.N_pad, st.N_pad // 64), -1, dtype=torch.int64, device="cuda")
        T.talon_build_tree(roots, pool_dev, st, cfg.K, mu, K_init, init_layers, cfg.Dmax, cand, ws, mask=mask)
    torch.cuda.synchronize()
    return st, cand, ws, mask


def run_gpu_literal(cfg: WorkloadConfig, pool: np.ndarray, K_init: int, init_layers: int = 1, mu=None,
                    layer_by_layer: bool = False, row_mode_frontier: bool = False, roomy_state: bool = False):
    """Alg. 2 with the uncapped pool through talon_expand_literal: talon_tree_init, the loop (one
    call, or one call per layer), talon_build_tree_mask.  Trees of at most 64 nodes take the call's
    shortcut through the capped loop; with roomy_state the tree state is padded to 128 nodes, which
    keeps such a tree on the general path (results are cut back to cfg.N_pad columns)."""
    import torch
    import paper_2601_07353_amd as T
    pool_dev = to_device_logits(pool)
    st = T.TreeState(cfg.B, cfg.N, N_pad=max(128, cfg.N_pad) if roomy_state else None)
    dt = T.TALON_DTYPE_F32 if cfg.logits_dtype == "f32" else T.TALON_DTYPE_BF16
    ws = T.make_literal_workspace(cfg.B, st.N_pad, cfg.V, dt)
    ws.fill_(0xA5)   # the call must not depend on what the workspace holds
    roots = torch.from_numpy(root_tokens(cfg)).cuda()
    mu = cfg.mu if mu is None else mu
    T.talon_tree_init(st, roots)
    if layer_by_layer:
        for _ in range(cfg.Dmax):
            T.talon_expand_literal(pool_dev, st, 1, mu, K_init, init_layers, cfg.Dmax, ws)
    else:
        T.talon_expand_literal(pool_dev, st, cfg.Dmax, mu, K_init, init_layers, cfg.Dmax, ws)
    mask = torch.zeros(cfg.B, st.N_pad, st.N_pad // 64, dtype=torch.int64, device="cuda")
    T.talon_build_tree_mask(st, mask)
    torch.cuda.synchronize()
    P, W = cfg.N_pad, cfg.N_pad // 64
    words = mask.cpu().numpy().view(np.uint64)
    assert not words[:, P:].any() and not words[:, :, W:].any()      # nothing beyond the tree's own padding
    cut = lambda t: t.cpu().numpy()[:, :P]
    return {
        "token": cut(st.token), "parent": cut(st.parent), "depth": cut(st.depth),
        "prob": cut(st.prob), "logp": cut(st.logp), "n_nodes": st.n_nodes.cpu().numpy(),
        "status": st.status.cpu().numpy(), "depth_cur": st.depth_cur.cpu().numpy(),
        "frontier_begin": st.frontier_begin.cpu().numpy(), "frontier_count": st.frontier_count.cpu().numpy(),
        "mask": np.ascontiguousarray(words[:, :P, :W]),
    }


def run_gpu_step(cfg: WorkloadConfig, seeds=None, pool=None, attn=None, with_attention=True, init_layers=1,
                 mu=None, K_init=None, layerwise=False):
    import torch
    import paper_2601_07353_amd as T
    seeds = seeds_for(cfg, seeds)
    pool = build_pool(cfg, seeds) if pool is None else pool
    pool_dev = to_device_logits(pool)
    st, cand, _, mask = run_gpu_expand(cfg, pool_dev, init_layers, mu, K_init, layerwise)
    if mask is None:
        mask = torch.zeros(cfg.B, st.N_pad, st.N_pad // 64, dtype=torch.int64, device="cuda")
        T.talon_build_tree_mask(st, mask)
    res = {
        "token": st.token.cpu().numpy(), "parent": st.parent.cpu().numpy(), "depth": st.depth.cpu().numpy(),
        "prob": st.prob.cpu().numpy(), "logp": st.logp.cpu().numpy(), "n_nodes": st.n_nodes.cpu().numpy(),
        "status": st.status.cpu().numpy(), "depth_cur": st.depth_cur.cpu().numpy(),
        "frontier_begin": st.frontier_begin.cpu().numpy(), "frontier_count": st.frontier_count.cpu().numpy(),
        "mask": mask.cpu().numpy().view(np.uint64),
        "cand_token": cand.token.cpu().numpy(), "cand_logit": cand.logit.cpu().numpy(),
        "cand_prob": cand.prob.cpu().numpy(), "cand_edge_logp": cand.edge_logp.cpu().numpy(),
        "row_max": cand.row_max.cpu().numpy(), "row_lse": cand.row_lse.cpu().numpy(),
    }
    if with_attention:
        xs = [attention_inputs(cfg, seeds[b], b) for b in range(cfg.B)] if attn is None else attn
        q = bf16_to_device(np.stack([x["q"] for x in xs]))
        kp = bf16_to_device(np.stack([x["k_prefix"] for x in xs]))
        vp = bf16_to_device(np.stack([x["v_prefix"] for x in xs]))
        kt = bf16_to_device(np.stack([x["k_tree"] for x in xs]))
        vt = bf16_to_device(np.stack([x["v_tree"] for x in xs]))
        L = kp.shape[1]
        plen = torch.full((cfg.B,), L, dtype=torch.int32, device="cuda")
        out = torch.zeros(cfg.B, st.N_pad, cfg.Hq, cfg.Dh, dtype=torch.bfloat16, device="cuda")
        lse = torch.zeros(cfg.B, st.N_pad, cfg.Hq, dtype=torch.float32, device="cuda")
        nb = T.talon_tree_attention_workspace_bytes(cfg.B, st.N_pad, cfg.Hq, cfg.Hkv, cfg.Dh, L)
        ws = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
        T.talon_tree_attention(q, kp, vp, kt, vt, mask, st.n_nodes, plen, L, out, lse, ws)
        torch.cuda.synchronize()
        res["attn_out"] = out.float().cpu().numpy()
        res["attn_lse"] = lse.cpu().numpy()
        res["prefix_len"] = np.full(cfg.B, L, dtype=np.int64)
    return res


# --------------------------------------------------------------------------- comparison
def compare_tree(cfg: WorkloadConfig, gpu: dict, trees, check_rows=True):
    """Topology, tokens and counters bit-exact; probabilities and confidences to PROB_RTOL."""
    for b, t in enumerate(trees):
        n = t.n
        assert int(gpu["n_nodes"][b]) == n, (b, int(gpu["n_nodes"][b]), n)
        np.testing.assert_array_equal(gpu["token"][b, :n], np.asarray(t.token, dtype=np.int32))
        np.testing.assert_array_equal(gpu["parent"][b, :n], np.asarray(t.parent, dtype=np.int32))
        np.testing.assert_array_equal(gpu["depth"][b, :n], np.asarray(t.depth, dtype=np.int32))
        np.testing.assert_allclose(gpu["prob"][b, :n], np.asarray(t.prob), rtol=PROB_RTOL, atol=0)
        np.testing.assert_allclose(np.exp(gpu["logp"][b, :n]), t.confidence(), rtol=PROB_RTOL, atol=0)
        want_status = 1 if t.exit_reason == "budget" else 2
        assert int(gpu["status"][b]) == want_status, (b, int(gpu["status"][b]), want_status)
        assert int(gpu["depth_cur"][b]) == len(t.layers) - 1
        last = t.layers[-1]
        assert int(gpu["frontier_begin"][b]) == last.start and int(gpu["frontier_count"][b]) == len(last)
        if check_rows:
            for pool in t.pools:
                for r in pool:
                    c = len(r.token)
                    np.testing.assert_array_equal(gpu["cand_token"][b, r.node, :c], r.token.astype(np.int32))
                    np.testing.assert_array_equal(gpu["cand_logit"][b, r.node, :c], r.logit.astype(np.float32))
                    assert float(gpu["row_max"][b, r.node]) == r.row_max
                    assert abs(float(gpu["row_lse"][b, r.node]) - r.row_lse) <= LSE_ATOL
                    np.testing.assert_allclose(gpu["cand_prob"][b, r.node, :c], r.prob, rtol=PROB_RTOL, atol=1e-37)
                    np.testing.assert_allclose(gpu["cand_edge_logp"][b, r.node, :c], r.edge_logp, rtol=0, atol=LSE_ATOL)


def compare_mask(cfg: WorkloadConfig, gpu: dict, masks):
    from oracle import talon_oracle as O
    for b, m in enumerate(masks):
        np.testing.assert_array_equal(gpu["mask"][b], O.mask_to_words(m, cfg.N_pad))


def check_attention_rows(got_out, got_lse, want_out, want_lse, keys, where=()):
    """Rows [n][Hq][Dh] of one sequence against the oracle's (NaN = not computed, skipped).
    `keys`: keys each node attends to (a number, or one per node).  Two bounds on every element:
    the stated 2e-2 absolute, and the signal-tied one derived above.  Returns the worst output
    and LSE errors."""
    sel = ~np.isnan(want_out)
    assert sel.any(), where
    err = np.abs(got_out - np.where(sel, want_out, 0.0))
    err = np.where(sel, err, 0.0)
    worst = float(err.max())
    assert worst <= ATTN_ATOL, (where, worst)
    keys = np.broadcast_to(np.asarray(keys, dtype=np.float64), want_out.shape[:1])
    tol = ATTN_OUT_RTOL * np.abs(np.where(sel, want_out, 0.0)) + (ATTN_KEYS_ATOL / np.sqrt(keys))[:, None, None]
    bad = err > tol
    assert not bad.any(), (where, "signal-tied bound", float((err / tol).max()), np.argwhere(bad)[:4].tolist())
    worst_lse = 0.0
    if got_lse is not None:
        sl = ~np.isnan(want_lse)
        worst_lse = float(np.abs(got_lse[sl] - want_lse[sl]).max())
        assert worst_lse <= ATTN_LSE_ATOL, (where, worst_lse)
    return worst, worst_lse


def compare_attention(cfg: WorkloadConfig, gpu: dict, ref: dict):
    worst = 0.0
    for b in range(cfg.B):
        want = ref["attn_out"][b]
        n = want.shape[0]
        keys = int(gpu["prefix_len"][b]) + ref["mask"][b].sum(axis=1)
        w, _ = check_attention_rows(gpu["attn_out"][b, :n], gpu["attn_lse"][b, :n], want, ref["attn_lse"][b], keys, (b,))
        worst = max(worst, w)
        # rows beyond n_nodes must be untouched (the harness pre-fills the output with zeros)
        assert not gpu["attn_out"][b, n:].any()
    return worst


def compare_step(cfg: WorkloadConfig, gpu: dict, ref: dict, check_rows=True):
    compare_tree(cfg, gpu, ref["trees"], check_rows)
    compare_mask(cfg, gpu, ref["mask"])
    if "attn_out" in gpu and ref["attn_out"]:
        return compare_attention(cfg, gpu, ref)
    return None


# --------------------------------------------------------------------------- greedy verification
def run_gpu_verify(cfg: WorkloadConfig, st, target_pool: np.ndarray, attn, capacity=None):
    """Target argmax over every tree node, acceptance walk, cache compaction, through the C ABI.
    `st`: the device tree state after expansion; `attn`: per-sequence attention inputs (their
    prefix and tree K/V are the cache and the tree's keys/values)."""
    import torch
    import paper_2601_07353_amd as T
    dev = to_device_logits(target_pool)
    dt = T.TALON_DTYPE_F32 if cfg.logits_dtype == "f32" else T.TALON_DTYPE_BF16
    ws = T.make_verify_workspace(cfg.B, st.N_pad, cfg.V, dt)
    tgt = torch.full((cfg.B, st.N_pad), -7, dtype=torch.int32, device="cuda")
    prob = torch.zeros(cfg.B, st.N_pad, dtype=torch.float32, device="cuda")
    sstat = torch.zeros(cfg.B, dtype=torch.int32, device="cuda")
    path = torch.full((cfg.B, st.N_pad), -9, dtype=torch.int32, device="cuda")
    alen = torch.full((cfg.B,), -9, dtype=torch.int32, device="cuda")
    bonus = torch.full((cfg.B,), -9, dtype=torch.int32, device="cuda")
    T.talon_target_argmax(dev, st, tgt, prob, sstat, ws)
    T.talon_greedy_accept(st, tgt, sstat, path, alen, bonus)
    capacity = cfg.L + st.N_pad if capacity is None else capacity
    kp = np.zeros((cfg.B, capacity, cfg.Hkv, cfg.Dh), dtype=np.uint16)
    vp = np.zeros_like(kp)
    keep = min(cfg.L, capacity)
    for b in range(cfg.B):
        kp[b, :keep] = attn[b]["k_prefix"][:keep]
        vp[b, :keep] = attn[b]["v_prefix"][:keep]
    kp_d, vp_d = bf16_to_device(kp), bf16_to_device(vp)
    kt_d = bf16_to_device(np.stack([x["k_tree"] for x in attn]))
    vt_d = bf16_to_device(np.stack([x["v_tree"] for x in attn]))
    plen = torch.full((cfg.B,), keep, dtype=torch.int32, device="cuda")
    new_plen = torch.full((cfg.B,), -9, dtype=torch.int32, device="cuda")
    T.talon_compact_kv(kt_d, vt_d, path, alen, plen, new_plen, kp_d, vp_d)
    torch.cuda.synchronize()
    return {"target_token": tgt.cpu().numpy(), "target_prob": prob.cpu().numpy(), "scan_status": sstat.cpu().numpy(),
            "path": path.cpu().numpy(), "accept_len": alen.cpu().numpy(), "bonus": bonus.cpu().numpy(),
            "new_prefix_len": new_plen.cpu().numpy(), "prefix_len": keep,
            "k_cache": kp_d.view(torch.int16).cpu().numpy().view(np.uint16),
            "v_cache": vp_d.view(torch.int16).cpu().numpy().view(np.uint16),
            "k_cache_before": kp, "v_cache_before": vp}


def compare_verify(cfg: WorkloadConfig, gpu: dict, b: int, token, parent, target_rows_f64, attn_b):
    """One sequence of run_gpu_verify against the oracle's greedy verification."""
    from oracle import talon_oracle as O
    n = len(token)
    want_tok = [O.target_argmax(target_rows_f64[i]) for i in range(n)]
    np.testing.assert_array_equal(gpu["target_token"][b, :n], np.asarray(want_tok, dtype=np.int32))
    assert np.all(gpu["target_token"][b, n:] == -7)                      # rows beyond the tree untouched
    for i in range(n):
        _, lse = O.softmax_stats(target_rows_f64[i])
        want_p = math.exp(target_rows_f64[i][want_tok[i]] - lse)
        assert abs(float(gpu["target_prob"][b, i]) - want_p) <= PROB_RTOL * want_p + 1e-30, (b, i)
    path, bonus = O.greedy_accept(list(token), list(parent), want_tok)
    assert int(gpu["accept_len"][b]) == len(path) - 1
    np.testing.assert_array_equal(gpu["path"][b, :len(path)], np.asarray(path, dtype=np.int32))
    assert np.all(gpu["path"][b, len(path):] == -1)
    assert int(gpu["bonus"][b]) == bonus
    L = gpu["prefix_len"]
    cap = gpu["k_cache"].shape[1]
    for name, tree in (("k_cache", attn_b["k_tree"]), ("v_cache", attn_b["v_tree"])):
        want = gpu[name + "_before"][b].copy()
        fit = [p for j, p in enumerate(path) if L + j < cap]
        new_len = O.compact_kv(want, tree, fit, L)
        np.testing.assert_array_equal(gpu[name][b], want)                 # bit-exact, untouched elsewhere
    assert int(gpu["new_prefix_len"][b]) == new_len == min(L + len(path), cap)
    return len(path) - 1
