"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (one talon_build_tree call: init, loop and mask; one talon_tree_attention call).

Expansion: every sequence of every configuration is built by the oracle and compared bit for bit
(c5: all sixteen trees).  Tree attention: every (node, head) pair at c3 and c4; at c5, where the
oracle's fp64 loops would take minutes, a stated sample: all nodes x 2 heads x 2 sequences plus
256 random (sequence, head, node) triples.  Every output also goes through the properties that
hold at any size."""
import numpy as np
import pytest

from tests import harness as H
from workloads import CONFIGS, attention_inputs, bf16_bits_to_f64

pytestmark = pytest.mark.gpu


def structural_checks(cfg, gpu, b):
    """Properties every tree must have, whatever the inputs (Alg. 2; Fig. 5(b))."""
    n = int(gpu["n_nodes"][b])
    assert 1 <= n <= cfg.N
    status = int(gpu["status"][b])
    assert status in (1, 2)
    assert (n == cfg.N) == (status == 1)              # the budget is met exactly unless depth-capped
    parent, depth = gpu["parent"][b, :n], gpu["depth"][b, :n]
    assert parent[0] == -1 and depth[0] == 0
    assert np.all(parent[1:] >= 0) and np.all(parent[1:] < np.arange(1, n))
    assert np.all(depth[1:] == depth[parent[1:]] + 1)
    assert np.all(np.diff(depth) >= 0)                # node ids are layer-major
    assert np.all(np.diff(parent[1:]) >= 0)           # inside a layer: parent ascending
    assert int((depth == 1).sum()) == min(cfg.K, cfg.N - 1)
    assert depth.max() <= cfg.Dmax
    # path confidence = product of edge probabilities (Eq. 2), child <= parent
    logp, prob = gpu["logp"][b, :n], gpu["prob"][b, :n].astype(np.float64)
    np.testing.assert_allclose(np.exp(logp[1:]), np.exp(logp[parent[1:]]) * prob[1:], rtol=2e-6)
    assert np.all(logp[1:] <= logp[parent[1:]] + 1e-12)
    # mask: popcount = depth + 1, bit of the node itself and of the root, parent's row is a subset
    words = gpu["mask"][b]
    pop = np.array([sum(bin(int(w)).count("1") for w in words[i]) for i in range(n)])
    assert np.all(pop == depth + 1)
    for i in range(1, n):
        assert (int(words[i, i // 64]) >> (i % 64)) & 1 and int(words[i, 0]) & 1
        own = np.zeros_like(words[i]); own[i // 64] = np.uint64(1) << np.uint64(i % 64)
        np.testing.assert_array_equal(words[i], words[parent[i]] | own)
    assert not words[n:].any()


class Decoded:
    """fp64 copies of one sequence's attention inputs (decoded once, used for many oracle calls)."""

    def __init__(self, x, n):
        self.q = bf16_bits_to_f64(x["q"][:n])
        self.kp, self.vp = bf16_bits_to_f64(x["k_prefix"]), bf16_bits_to_f64(x["v_prefix"])
        self.kt, self.vt = bf16_bits_to_f64(x["k_tree"][:n]), bf16_bits_to_f64(x["v_tree"][:n])


def attention_check(cfg, gpu, b, mask, dec, nodes=None, heads=None):
    """Oracle attention of sequence b on the given nodes and heads (None: all of them) against the
    GPU's rows, through the harness's bounds.  Returns (worst output error, worst LSE error)."""
    from oracle import talon_oracle as O
    out, lse = O.tree_attention(dec.q, dec.kp, dec.vp, dec.kt, dec.vt, mask, nodes=nodes, heads=heads)
    n = out.shape[0]
    return H.check_attention_rows(gpu["attn_out"][b, :n], gpu["attn_lse"][b, :n], out, lse,
                                  cfg.L + mask.sum(axis=1), (b,))


def run_config(cfg_name):
    """GPU step on admissible seeds for every sequence; every tree and mask against the oracle."""
    from oracle import talon_oracle as O
    cfg = CONFIGS[cfg_name]
    found = [H.find_admissible_seed(cfg, b, cfg.seed) for b in range(cfg.B)]
    seeds = [s for s, _ in found]
    trees = [t for _, t in found]
    print("case", cfg.name, "seeds", seeds, flush=True)
    pool = H.build_pool(cfg, seeds)
    attn = [attention_inputs(cfg, seeds[b], b) for b in range(cfg.B)]
    gpu = H.run_gpu_step(cfg, seeds, pool=pool, attn=attn)
    masks = []
    for b in range(cfg.B):
        structural_checks(cfg, gpu, b)
        assert trees[b].margin > H.MARGIN_TOL
        H.compare_tree(cfg, {k: v[b:b + 1] for k, v in gpu.items()}, [trees[b]])
        masks.append(O.build_tree_mask(trees[b].parent))
        np.testing.assert_array_equal(gpu["mask"][b], O.mask_to_words(masks[b], cfg.N_pad))
        # rows of nodes beyond n_nodes are untouched
        assert not gpu["attn_out"][b, int(gpu["n_nodes"][b]):].any()
    return cfg, gpu, trees, masks, attn, pool


def run_full(cfg_name):
    cfg, gpu, trees, masks, attn, _ = run_config(cfg_name)
    worst = (0.0, 0.0)
    for b in range(cfg.B):
        w = attention_check(cfg, gpu, b, masks[b], Decoded(attn[b], trees[b].n))
        worst = (max(worst[0], w[0]), max(worst[1], w[1]))
    print(cfg.name, "attention over all (node, head) pairs: worst abs err", worst[0], "worst LSE err", worst[1], flush=True)


def test_c3_qwen3_8b_x4_full_size():
    run_full("c3")


def test_c4_70b_shaped_full_size():
    run_full("c4")


@pytest.fixture(scope="module")
def c5_run():
    return run_config("c5")     # sixteen trees and masks against the oracle


def test_c5_stress_full_size_all_trees(c5_run):
    cfg, gpu, trees, _, _, _ = c5_run
    assert len(trees) == 16 and all(t.n == int(gpu["n_nodes"][b]) for b, t in enumerate(trees))


def test_c5_stress_per_layer_launches(c5_run):
    """The same sixteen trees through one fused launch per layer (talon_expand_select_layer).  At
    this size a launch has more workgroups than the device starts at once: every workgroup must
    still see the frontier the launch began with, so a selection may rewrite the tree state only
    when every workgroup of the grid has read it."""
    cfg, _, trees, masks, _, pool = c5_run
    gpu = H.run_gpu_step(cfg, pool=pool, with_attention=False, layerwise="fused")
    H.compare_tree(cfg, gpu, trees, check_rows=False)
    H.compare_mask(cfg, gpu, masks)


def test_c5_stress_full_size_attention_sample(c5_run):
    """All nodes x heads {2, 29} x sequences {3, 12}, then 256 random (sequence, head, node) triples."""
    cfg, gpu, trees, masks, attn, _ = c5_run
    worst = [0.0, 0.0]

    def note(w):
        worst[0], worst[1] = max(worst[0], w[0]), max(worst[1], w[1])

    for b in (3, 12):
        note(attention_check(cfg, gpu, b, masks[b], Decoded(attn[b], trees[b].n), heads=[2, 29]))
    rng = np.random.default_rng(20260107)
    triples = [(int(rng.integers(cfg.B)), int(rng.integers(cfg.Hq)), 0) for _ in range(256)]
    triples = sorted((b, h, int(rng.integers(trees[b].n))) for b, h, _ in triples)
    dec, dec_b = None, -1
    for b, h, i in triples:
        if b != dec_b:
            dec, dec_b = Decoded(attn[b], trees[b].n), b
        note(attention_check(cfg, gpu, b, masks[b], dec, nodes=[i], heads=[h]))
    print(cfg.name, "sampled attention worst abs err", worst[0], "worst LSE err", worst[1], flush=True)
