"""Whole steps on randomly drawn small configurations, against the oracle: vocabulary sizes
from 8 to 60000 (ragged tails, fewer logits than k), both logit types, k from 1 to 16, budgets
from 2 to 139, depth caps from 1, batches of 1 to 5, 0 to 3 top-K-initialised layers, four
thresholds, four logit recipes, prefix lengths from 0, both head dimensions, grouped heads.
Each configuration runs through talon_build_tree and through one fused launch per layer."""
import numpy as np
import pytest

from tests import harness as H
from workloads import WorkloadConfig

pytestmark = pytest.mark.gpu

RECIPES = [("gauss", 0.5, 4.0), ("gauss", 4.0, 8.0), ("zipf_mix", 1.2, 0.05), ("gauss", 0.2, 0.6)]


def draw(rng, case):
    dtype = str(rng.choice(["bf16", "f32"]))
    V = int(rng.choice([int(rng.integers(8, 300)), int(rng.integers(300, 5000)), int(rng.integers(5000, 60000))]))
    if dtype == "bf16" and rng.random() < 0.5:
        V = max(8, V // 8 * 8)
    K = int(rng.integers(1, 17))
    N = int(rng.integers(2, 140))
    G, Hkv = int(rng.choice([1, 2, 4])), int(rng.choice([1, 2]))
    cfg = WorkloadConfig(name="random%d" % case, B=int(rng.choice([1, 1, 2, 3, 5])), V=V, logits_dtype=dtype, K=K, N=N,
                         Dmax=int(rng.integers(1, 14)), mu=float(rng.choice([0.03, 0.003, 0.2, 0.5])), Hq=G * Hkv,
                         Hkv=Hkv, Dh=int(rng.choice([64, 128])), L=int(rng.choice([0, int(rng.integers(1, 300))])),
                         recipe=RECIPES[int(rng.integers(0, 4))], seed=1000 + case)
    return cfg, int(rng.choice([0, 1, 1, 2, 3]))


def test_random_configurations_against_oracle():
    rng = np.random.default_rng(20260107)
    checked = 0
    for case in range(48):
        cfg, init_layers = draw(rng, case)
        try:
            seeds = [H.find_admissible_seed(cfg, b, cfg.seed)[0] for b in range(cfg.B)]
        except RuntimeError:
            continue   # no seed leaves a safe margin at this shape
        pool = H.build_pool(cfg, seeds)
        ref = H.run_oracle_step(cfg, seeds, pool=pool, init_layers=init_layers)
        if min(t.margin for t in ref["trees"]) <= H.MARGIN_TOL:
            continue   # a cross-parent decision closer than fp32 log-sum-exp can settle
        print("case", case, cfg, "init_layers", init_layers, flush=True)
        for form in (False, "fused"):
            gpu = H.run_gpu_step(cfg, seeds, pool=pool, init_layers=init_layers, layerwise=form)
            H.compare_step(cfg, gpu, ref)
        checked += 1
    assert checked >= 40


def test_no_prefix_at_all():
    """prefix_len = 0 and no prefix tensors: every node attends to its own root path only."""
    cfg = WorkloadConfig(name="noprefix", B=2, V=3000, logits_dtype="bf16", K=6, N=40, Dmax=8, mu=0.03, Hq=4, Hkv=2,
                         Dh=128, L=0, recipe=("gauss", 0.5, 4.0), seed=77)
    seeds = [H.find_admissible_seed(cfg, b, cfg.seed)[0] for b in range(cfg.B)]
    pool = H.build_pool(cfg, seeds)
    ref = H.run_oracle_step(cfg, seeds, pool=pool)
    gpu = H.run_gpu_step(cfg, seeds, pool=pool)
    H.compare_step(cfg, gpu, ref)
