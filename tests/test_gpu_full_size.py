"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (one talon_build_tree call: init, loop and mask; one talon_tree_attention call).

Where the oracle cannot finish the whole configuration in seconds, it checks a stated sample
(some sequences in full for the expansion, sampled (node, head) pairs for attention) and the
remaining outputs are checked through properties that hold at any size."""
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


def sampled_attention_check(cfg, gpu, b, tree, mask, x, nodes, heads):
    from oracle import talon_oracle as O
    n = tree.n
    out, lse = O.tree_attention(bf16_bits_to_f64(x["q"][:n]), bf16_bits_to_f64(x["k_prefix"]),
                                bf16_bits_to_f64(x["v_prefix"]), bf16_bits_to_f64(x["k_tree"][:n]),
                                bf16_bits_to_f64(x["v_tree"][:n]), mask, nodes=nodes, heads=heads)
    worst = 0.0
    for i in nodes:
        for h in heads:
            err = float(np.abs(gpu["attn_out"][b, i, h] - out[i, h]).max())
            worst = max(worst, err)
            assert err <= H.ATTN_ATOL, (b, i, h, err)
            assert abs(float(gpu["attn_lse"][b, i, h]) - lse[i, h]) <= 2e-3
    return worst


def spread(n, count):
    return sorted(set([0, n - 1] + [int(v) for v in np.linspace(0, n - 1, count)]))


def run_full(cfg_name, oracle_seqs, n_nodes_sample, heads):
    from oracle import talon_oracle as O
    cfg = CONFIGS[cfg_name]
    seeds = [cfg.seed] * cfg.B
    for b in oracle_seqs:
        seeds[b] = H.find_admissible_seed(cfg, b, cfg.seed)[0]
    print("case", cfg.name, "seeds", seeds, "oracle sequences", oracle_seqs, flush=True)
    pool = H.build_pool(cfg, seeds)
    attn = [attention_inputs(cfg, seeds[b], b) for b in range(cfg.B)]
    gpu = H.run_gpu_step(cfg, seeds, pool=pool, attn=attn)
    roots = H.root_tokens(cfg)
    for b in range(cfg.B):
        structural_checks(cfg, gpu, b)
    worst = 0.0
    for b in oracle_seqs:
        t = H.oracle_tree(cfg, pool[b], roots[b])
        assert t.margin > H.MARGIN_TOL
        sub = {k: v[b:b + 1] for k, v in gpu.items()}
        H.compare_tree(cfg, sub, [t])
        m = O.build_tree_mask(t.parent)
        np.testing.assert_array_equal(gpu["mask"][b], O.mask_to_words(m, cfg.N_pad))
        worst = max(worst, sampled_attention_check(cfg, gpu, b, t, m, attn[b], spread(t.n, n_nodes_sample), heads))
    # rows of nodes beyond n_nodes are untouched in every sequence
    for b in range(cfg.B):
        assert not gpu["attn_out"][b, int(gpu["n_nodes"][b]):].any()
    print(cfg.name, "sampled attention worst abs err", worst, flush=True)


def test_c3_qwen3_8b_x4_full_size():
    run_full("c3", oracle_seqs=[0, 1, 2, 3], n_nodes_sample=8, heads=[0, 5, 17, 31])


def test_c4_70b_shaped_full_size():
    run_full("c4", oracle_seqs=[0], n_nodes_sample=8, heads=[0, 7, 8, 33, 63])


def test_c5_stress_full_size():
    run_full("c5", oracle_seqs=[3, 12], n_nodes_sample=5, heads=[2, 29])
