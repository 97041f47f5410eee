"""GPU parity of the greedy (temperature 0) verification outcome: target argmax per tree node,
acceptance walk, cache compaction, through the C ABI, against the CPU oracle.  Everything here
is integer or byte work (bit-exact) except the probability of the target's token (1e-5
relative)."""
import dataclasses

import numpy as np
import pytest

from tests import harness as H
from tests.test_gpu_parity import admissible_seeds, small
from workloads import CONFIGS, attention_inputs, storage_to_f64, target_logits_row

pytestmark = pytest.mark.gpu


def verify_case(cfg, seqs=None, capacity=None, noise=0.25):
    import torch
    seeds = admissible_seeds(cfg)
    print("case", cfg.name, "seeds", seeds, flush=True)
    pool = H.build_pool(cfg, seeds)
    st, _, _, _ = H.run_gpu_expand(cfg, H.to_device_logits(pool))
    n = st.n_nodes.cpu().numpy()
    token, parent = st.token.cpu().numpy(), st.parent.cpu().numpy()
    seqs = range(cfg.B) if seqs is None else seqs
    dt = np.float32 if cfg.logits_dtype == "f32" else np.uint16
    tpool = np.zeros((cfg.B, cfg.N_pad, cfg.V), dtype=dt)
    for b in seqs:
        for i in range(int(n[b])):
            tpool[b, i] = target_logits_row(cfg, seeds[b], b, i, noise)
    attn = [attention_inputs(cfg, seeds[b], b) for b in range(cfg.B)]
    gpu = H.run_gpu_verify(cfg, st, tpool, attn, capacity)
    assert not gpu["scan_status"].any()
    lens = []
    for b in seqs:
        rows = [storage_to_f64(tpool[b, i]) for i in range(int(n[b]))]
        lens.append(H.compare_verify(cfg, gpu, b, token[b, :n[b]], parent[b, :n[b]], rows, attn[b]))
    print(cfg.name, "accepted lengths", lens, flush=True)
    return lens, gpu


def test_c1_tiny_verify():
    verify_case(CONFIGS["c1"])


def test_verify_batch_of_three_bf16():
    cfg = small(name="verify3", V=40000, logits_dtype="bf16", K=8, N=130, Dmax=20, B=3, Hq=8, Hkv=2, Dh=128, L=200,
                recipe=(("gauss", 6.0, 8.0), ("gauss", 0.5, 1.0), ("zipf_mix", 1.2, 0.05)))
    lens, _ = verify_case(cfg)


def test_verify_ragged_f32_rows_and_low_noise_accepts_deep():
    cfg = small(name="verify-f32", V=1003, logits_dtype="f32", K=4, N=33, Dmax=9, Hq=4, Hkv=4, Dh=64, L=64)
    lens, _ = verify_case(cfg, noise=0.02)
    assert max(lens) >= 2       # the target nearly copies the draft: several tokens are accepted


def test_verify_capacity_clamp():
    cfg = small(name="verify-cap", V=4096, logits_dtype="bf16", K=6, N=48, Dmax=12, Hq=4, Hkv=2, Dh=64, L=32)
    lens, gpu = verify_case(cfg, capacity=cfg.L + 1, noise=0.02)   # room for the root's row only
    assert int(gpu["new_prefix_len"][0]) == cfg.L + 1


def test_c2_llama3_8b_verify_full_size():
    verify_case(CONFIGS["c2"])


def test_c3_qwen3_8b_x4_verify_full_size():
    verify_case(CONFIGS["c3"])


def test_nan_target_row_is_reported():
    import torch
    import paper_2601_07353_amd as T
    cfg = small(name="verify-nan", V=2048, logits_dtype="f32", K=3, N=12, Dmax=6, B=2, Hq=4, Hkv=4, Dh=64, L=32)
    seeds = admissible_seeds(cfg)
    pool = H.build_pool(cfg, seeds)
    st, _, _, _ = H.run_gpu_expand(cfg, H.to_device_logits(pool))
    tpool = pool.copy()
    tpool[1, 2, 77] = np.nan                      # one bad target row in sequence 1
    attn = [attention_inputs(cfg, seeds[b], b) for b in range(cfg.B)]
    gpu = H.run_gpu_verify(cfg, st, tpool, attn)
    assert int(gpu["scan_status"][0]) == 0 and int(gpu["scan_status"][1]) & T.TALON_STATUS_BAD_ROW
    status = st.status.cpu().numpy()
    assert not (int(status[0]) & T.TALON_STATUS_BAD_ROW) and int(status[1]) & T.TALON_STATUS_BAD_ROW
    # the clean sequence is unaffected: the target equals the draft, so greedy decoding follows the draft's best child
    n0 = int(st.n_nodes[0])
    rows = [storage_to_f64(tpool[0, i]) for i in range(n0)]
    H.compare_verify(cfg, gpu, 0, st.token[0, :n0].cpu().numpy(), st.parent[0, :n0].cpu().numpy(), rows, attn[0])
