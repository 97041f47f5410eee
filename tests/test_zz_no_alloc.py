"""talon_tree_attention_static (the call that takes no workspace: split-KV partial results in the
library's own device array) against talon_tree_attention on the same inputs: same kernels, same
launch plan, so the outputs must agree bit for bit.  Two calls in a row, the second on a smaller
input, so that nothing the first left in the array may matter."""
import numpy as np
import pytest

from workloads import bf16_to_device, f32_to_bf16_bits

pytestmark = pytest.mark.gpu


def _case(rng, B, n_list, Hq, Hkv, Dh, L_list):
    import torch
    import paper_2601_07353_amd as T
    N = max(n_list)
    N_pad = (N + 63) // 64 * 64
    Lmax = max(L_list)
    st = T.TreeState(B, N)
    parent = np.full((B, N_pad), -1, dtype=np.int32)
    for b in range(B):
        for i in range(1, n_list[b]):
            parent[b, i] = rng.integers(0, i)
    st.parent.copy_(torch.from_numpy(parent))
    st.n_nodes.copy_(torch.tensor(n_list, dtype=torch.int32))
    mask = torch.zeros(B, N_pad, N_pad // 64, dtype=torch.int64, device="cuda")
    T.talon_build_tree_mask(st, mask)

    def dev(shape):
        return bf16_to_device(f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32)))

    q, kt, vt = dev((B, N_pad, Hq, Dh)), dev((B, N_pad, Hkv, Dh)), dev((B, N_pad, Hkv, Dh))
    kp, vp = dev((B, Lmax, Hkv, Dh)), dev((B, Lmax, Hkv, Dh))
    plen = torch.tensor(L_list, dtype=torch.int32, device="cuda")
    nb = T.talon_tree_attention_workspace_bytes(B, N_pad, Hq, Hkv, Dh, Lmax)
    assert 256 < nb <= T.talon_static_scratch_bytes(), nb          # split-KV in use, and it fits
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    want = torch.full((B, N_pad, Hq, Dh), 7.0, dtype=torch.bfloat16, device="cuda")
    want_lse = torch.full((B, N_pad, Hq), 7.0, dtype=torch.float32, device="cuda")
    T.talon_tree_attention(q, kp, vp, kt, vt, mask, st.n_nodes, plen, Lmax, want, want_lse, ws)
    got = torch.full_like(want, 7.0)
    got_lse = torch.full_like(want_lse, 7.0)
    T.talon_tree_attention_static(q, kp, vp, kt, vt, mask, st.n_nodes, plen, Lmax, got, got_lse)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    assert torch.equal(got_lse, want_lse)
    # something was computed at all: row 0 of every sequence differs from the fill value
    assert (got[:, 0].float() != 7.0).any()


def test_static_scratch_attention_matches_the_workspace_call_twice_in_a_row():
    import paper_2601_07353_amd as T
    T.talon_static_scratch_init()
    rng = np.random.default_rng(20260107)
    _case(rng, 1, [60], 32, 8, 128, [2048])            # the Llama-3-8B-shaped call: 7 splits, 3.8 MB of partials
    _case(rng, 2, [37, 20], 8, 2, 64, [700, 333])      # smaller, ragged, other head size: same array


def test_static_scratch_refuses_what_does_not_fit():
    """Host-side check: a shape whose partial results need a little more than the array holds (the launch plan
    keeps them near twice the chip's workgroup slots, so few shapes do); nothing is launched."""
    import torch
    import paper_2601_07353_amd as T
    B, N_pad, Hq, Hkv, Dh, L = 21, 192, 16, 8, 128, 8192
    assert T.talon_tree_attention_workspace_bytes(B, N_pad, Hq, Hkv, Dh, L) > T.talon_static_scratch_bytes()
    z = lambda *shape: torch.zeros(*shape, dtype=torch.bfloat16, device="cuda")
    n = torch.ones(B, dtype=torch.int32, device="cuda")
    plen = torch.full((B,), L, dtype=torch.int32, device="cuda")
    mask = torch.zeros(B, N_pad, N_pad // 64, dtype=torch.int64, device="cuda")
    with pytest.raises(T.TalonError) as e:
        T.talon_tree_attention_static(z(B, N_pad, Hq, Dh), z(B, L, Hkv, Dh), z(B, L, Hkv, Dh), z(B, N_pad, Hkv, Dh),
                                      z(B, N_pad, Hkv, Dh), mask, n, plen, L, z(B, N_pad, Hq, Dh))
    assert e.value.code == T.TALON_ERR_WORKSPACE
