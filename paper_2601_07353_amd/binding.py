"""ctypes binding of libtalon.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA tensors used purely as device buffers; every step of the path runs
in the library's HIP kernels.  There is no CPU fallback: if the library is missing, or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "lib", "libtalon.so")

TALON_OK = 0
TALON_ERR_INVALID_ARG = -1
TALON_ERR_UNSUPPORTED = -2
TALON_ERR_WORKSPACE = -3
TALON_ERR_RUNTIME = -4
TALON_DTYPE_F32 = 0
TALON_DTYPE_BF16 = 1
TALON_K_MAX = 64
TALON_N_MAX = 256
TALON_B_MAX = 256
TALON_STATUS_DONE_BUDGET = 1
TALON_STATUS_DONE_DEPTH = 2
TALON_STATUS_BAD_ROW = 4
TALON_STATUS_ABORTED = 8
TALON_ROWS_BY_NODE = 0
TALON_ROWS_BY_FRONTIER = 1

EXPORTS = [
    "talon_last_error_string", "talon_tree_init", "talon_expand_workspace_bytes",
    "talon_expand_workspace_init", "talon_expand_layer", "talon_select_budget", "talon_expand_select_layer",
    "talon_expand_tree", "talon_build_tree", "talon_build_tree_checked", "talon_set_spin_limit_us", "talon_profile_scan_launches", "talon_profile_read", "talon_probe_read", "talon_probe_mfma", "talon_probe_issue", "talon_probe_tile_loads", "talon_verify_workspace_bytes", "talon_target_argmax",
    "talon_literal_workspace_bytes", "talon_expand_literal",
    "talon_greedy_accept", "talon_compact_kv", "talon_prune_tree",
    "talon_build_tree_mask", "talon_tree_attention_workspace_bytes", "talon_tree_attention",
    "talon_static_scratch_bytes", "talon_static_scratch_init", "talon_tree_attention_static",
]


class TalonError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("talon error %d: %s" % (code, message))
        self.code = code


class _CTreeState(Structure):
    _fields_ = [("B", c_int32), ("N", c_int32), ("N_pad", c_int32),
                ("token", c_void_p), ("parent", c_void_p), ("depth", c_void_p),
                ("prob", c_void_p), ("logp", c_void_p), ("n_nodes", c_void_p),
                ("frontier_begin", c_void_p), ("frontier_count", c_void_p),
                ("depth_cur", c_void_p), ("status", c_void_p)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libtalon.so (built in-tree by paper_2601_07353_amd.build); never falls back."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libtalon.so is not built (%s): run `python -m paper_2601_07353_amd.build` "
                           "or __graft_entry__.build()" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    P = c_void_p
    lib.talon_last_error_string.restype = c_char_p
    lib.talon_last_error_string.argtypes = []
    lib.talon_tree_init.argtypes = [POINTER(_CTreeState), P, P]
    lib.talon_expand_workspace_bytes.restype = c_size_t
    lib.talon_expand_workspace_bytes.argtypes = [c_int32, c_int32, c_int32, c_int32, c_int]
    lib.talon_expand_workspace_init.argtypes = [P, c_size_t, P]
    lib.talon_expand_layer.argtypes = [P, c_int, c_int64, c_int64, c_int, c_int32, POINTER(_CTreeState), c_int32,
                                       c_int32, P, P, P, P, P, P, P, c_size_t, P]
    lib.talon_select_budget.argtypes = [POINTER(_CTreeState), c_int32, P, P, P, c_float, c_int32, c_int32, c_int32, P]
    lib.talon_expand_tree.argtypes = [P, c_int, c_int64, c_int64, c_int, POINTER(_CTreeState), c_int32, c_int32,
                                      c_float, c_int32, c_int32, c_int32, P, P, P, P, P, P, P, c_size_t, P]
    lib.talon_expand_select_layer.argtypes = [P, c_int, c_int64, c_int64, c_int, c_int32, POINTER(_CTreeState),
                                              c_int32, c_int32, c_float, c_int32, c_int32, c_int32, P, P, P, P, P, P,
                                              P, c_size_t, P]
    lib.talon_build_tree.argtypes = [P, P, c_int, c_int64, c_int64, c_int, POINTER(_CTreeState), c_int32, c_int32,
                                     c_float, c_int32, c_int32, c_int32, P, P, P, P, P, P, P, P, c_size_t, P]
    lib.talon_build_tree_checked.argtypes = lib.talon_build_tree.argtypes + [POINTER(c_int32)]
    lib.talon_set_spin_limit_us.argtypes = [c_int64]
    lib.talon_profile_scan_launches.argtypes = [c_int]
    lib.talon_profile_read.argtypes = [POINTER(c_float), c_int32, POINTER(c_int32)]
    lib.talon_literal_workspace_bytes.restype = c_size_t
    lib.talon_literal_workspace_bytes.argtypes = [c_int32, c_int32, c_int32, c_int]
    lib.talon_expand_literal.argtypes = [P, c_int, c_int64, c_int64, c_int, c_int32, POINTER(_CTreeState), c_int32,
                                         c_float, c_int32, c_int32, c_int32, P, c_size_t, P]
    lib.talon_verify_workspace_bytes.restype = c_size_t
    lib.talon_verify_workspace_bytes.argtypes = [c_int32, c_int32, c_int32, c_int]
    lib.talon_target_argmax.argtypes = [P, c_int, c_int64, c_int64, POINTER(_CTreeState), c_int32, P, P, P, P, c_size_t, P]
    lib.talon_greedy_accept.argtypes = [POINTER(_CTreeState), P, P, P, P, P, P]
    lib.talon_compact_kv.argtypes = [P, P, P, P, P, P, P, P, c_int32, c_int32, c_int32, c_int32, c_int32, c_int64,
                                     c_int64, c_int64, P]
    lib.talon_prune_tree.argtypes = [POINTER(_CTreeState), c_int32, P, P]
    lib.talon_probe_read.argtypes = [P, c_size_t, P, P]
    lib.talon_probe_mfma.argtypes = [c_int32, c_int32, P, POINTER(c_double), P]
    lib.talon_probe_issue.argtypes = [c_int32, c_int32, c_int32, P, P, P]
    lib.talon_probe_tile_loads.argtypes = [P, c_size_t, c_int32, c_int32, c_int32, c_int32, P, P, P]
    lib.talon_build_tree_mask.argtypes = [POINTER(_CTreeState), P, P]
    lib.talon_tree_attention_workspace_bytes.restype = c_size_t
    lib.talon_tree_attention_workspace_bytes.argtypes = [c_int32] * 6
    lib.talon_tree_attention.argtypes = [P, P, P, P, P, P, P, P, c_int32, c_int32, c_int32, c_int32, c_int32, c_int32,
                                         c_int64, c_int64, c_int64, c_float, P, P, P, c_size_t, P]
    lib.talon_static_scratch_bytes.restype = c_size_t
    lib.talon_static_scratch_bytes.argtypes = []
    lib.talon_static_scratch_init.argtypes = []
    lib.talon_tree_attention_static.argtypes = [P, P, P, P, P, P, P, P, c_int32, c_int32, c_int32, c_int32, c_int32,
                                                c_int32, c_int64, c_int64, c_int64, c_float, P, P, P]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if fn.restype is c_int:
            fn.restype = c_int
    _lib = lib
    return lib


def _check(rc: int):
    if rc != TALON_OK:
        raise TalonError(rc, load_library().talon_last_error_string().decode())


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


class TreeState:
    """Device buffers of the token tree T (structure of arrays) plus the C struct that names them."""

    def __init__(self, B: int, N: int, device="cuda", N_pad: int | None = None):
        self.B, self.N = B, N
        self.N_pad = (N + 63) // 64 * 64 if N_pad is None else N_pad   # a multiple of 64, at least N
        i32 = dict(dtype=torch.int32, device=device)
        self.token = torch.zeros(B, self.N_pad, **i32)
        self.parent = torch.full((B, self.N_pad), -1, **i32)
        self.depth = torch.zeros(B, self.N_pad, **i32)
        self.prob = torch.zeros(B, self.N_pad, dtype=torch.float32, device=device)
        self.logp = torch.zeros(B, self.N_pad, dtype=torch.float64, device=device)
        self.n_nodes = torch.zeros(B, **i32)
        self.frontier_begin = torch.zeros(B, **i32)
        self.frontier_count = torch.zeros(B, **i32)
        self.depth_cur = torch.zeros(B, **i32)
        self.status = torch.zeros(B, **i32)
        self.c = _CTreeState(B, N, self.N_pad, *[t.data_ptr() for t in (
            self.token, self.parent, self.depth, self.prob, self.logp, self.n_nodes,
            self.frontier_begin, self.frontier_count, self.depth_cur, self.status)])


class Candidates:
    """Device buffers for the per-row outputs of talon_expand_layer."""

    def __init__(self, B: int, N_pad: int, k: int, device="cuda"):
        self.k = k
        self.token = torch.full((B, N_pad, k), -1, dtype=torch.int32, device=device)
        self.logit = torch.zeros(B, N_pad, k, dtype=torch.float32, device=device)
        self.prob = torch.zeros(B, N_pad, k, dtype=torch.float32, device=device)
        self.edge_logp = torch.zeros(B, N_pad, k, dtype=torch.float64, device=device)
        self.row_max = torch.zeros(B, N_pad, dtype=torch.float32, device=device)
        self.row_lse = torch.zeros(B, N_pad, dtype=torch.float64, device=device)


def _logits_meta(logits: torch.Tensor):
    if logits.dtype == torch.float32:
        dt = TALON_DTYPE_F32
    elif logits.dtype == torch.bfloat16:
        dt = TALON_DTYPE_BF16
    else:
        raise TalonError(TALON_ERR_UNSUPPORTED, "logits dtype %s" % logits.dtype)
    if logits.dim() != 3 or logits.stride(2) != 1:
        raise TalonError(TALON_ERR_INVALID_ARG, "logits must be [B][rows][V] with contiguous rows")
    return dt, logits.stride(1), logits.stride(0), logits.shape[2]


def talon_tree_init(st: TreeState, root_token: torch.Tensor, stream=None):
    _check(load_library().talon_tree_init(ctypes.byref(st.c), _ptr(root_token), _stream(stream)))


def talon_expand_workspace_bytes(B, N_pad, vocab, k, dtype) -> int:
    return load_library().talon_expand_workspace_bytes(B, N_pad, vocab, k, dtype)


def talon_expand_workspace_init(workspace: torch.Tensor, stream=None):
    _check(load_library().talon_expand_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                                      _stream(stream)))


def make_expand_workspace(B, N_pad, vocab, k, dtype, device="cuda") -> torch.Tensor:
    nbytes = talon_expand_workspace_bytes(B, N_pad, vocab, k, dtype)
    if nbytes == 0:
        raise TalonError(TALON_ERR_UNSUPPORTED, load_library().talon_last_error_string().decode())
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    talon_expand_workspace_init(ws)
    return ws


def talon_expand_layer(logits, st: TreeState, k, cand: Candidates, workspace, row_mode=TALON_ROWS_BY_NODE,
                       layer=-1, vocab=None, stream=None):
    dt, row_stride, seq_stride, V = _logits_meta(logits)
    _check(load_library().talon_expand_layer(
        _ptr(logits), dt, row_stride, seq_stride, row_mode, layer, ctypes.byref(st.c),
        V if vocab is None else vocab, k,
        _ptr(cand.token), _ptr(cand.logit), _ptr(cand.prob), _ptr(cand.edge_logp), _ptr(cand.row_max),
        _ptr(cand.row_lse), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def talon_select_budget(st: TreeState, k, cand: Candidates, mu, K_init, init_layers, max_depth, stream=None):
    _check(load_library().talon_select_budget(
        ctypes.byref(st.c), k, _ptr(cand.token), _ptr(cand.prob), _ptr(cand.edge_logp), c_float(mu), K_init,
        init_layers, max_depth, _stream(stream)))


def talon_expand_tree(logits, st: TreeState, k, mu, K_init, init_layers, max_depth, cand: Candidates, workspace,
                      row_mode=TALON_ROWS_BY_NODE, vocab=None, stream=None):
    dt, row_stride, seq_stride, V = _logits_meta(logits)
    _check(load_library().talon_expand_tree(
        _ptr(logits), dt, row_stride, seq_stride, row_mode, ctypes.byref(st.c), V if vocab is None else vocab, k,
        c_float(mu), K_init, init_layers, max_depth, _ptr(cand.token), _ptr(cand.logit), _ptr(cand.prob),
        _ptr(cand.edge_logp), _ptr(cand.row_max), _ptr(cand.row_lse), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def talon_expand_select_layer(logits, st: TreeState, k, mu, K_init, init_layers, max_depth, cand: Candidates,
                              workspace, layer=-1, row_mode=TALON_ROWS_BY_NODE, vocab=None, stream=None):
    dt, row_stride, seq_stride, V = _logits_meta(logits)
    _check(load_library().talon_expand_select_layer(
        _ptr(logits), dt, row_stride, seq_stride, row_mode, layer, ctypes.byref(st.c), V if vocab is None else vocab,
        k, c_float(mu), K_init, init_layers, max_depth, _ptr(cand.token), _ptr(cand.logit), _ptr(cand.prob),
        _ptr(cand.edge_logp), _ptr(cand.row_max), _ptr(cand.row_lse), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def talon_build_tree(root_token, logits, st: TreeState, k, mu, K_init, init_layers, max_depth, cand: Candidates,
                     workspace, mask=None, row_mode=TALON_ROWS_BY_NODE, vocab=None, stream=None):
    dt, row_stride, seq_stride, V = _logits_meta(logits)
    _check(load_library().talon_build_tree(
        _ptr(root_token), _ptr(logits), dt, row_stride, seq_stride, row_mode, ctypes.byref(st.c),
        V if vocab is None else vocab, k, c_float(mu), K_init, init_layers, max_depth, _ptr(cand.token),
        _ptr(cand.logit), _ptr(cand.prob), _ptr(cand.edge_logp), _ptr(cand.row_max), _ptr(cand.row_lse), _ptr(mask),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def talon_build_tree_checked(root_token, logits, st: TreeState, k, mu, K_init, init_layers, max_depth,
                             cand: Candidates, workspace, mask=None, row_mode=TALON_ROWS_BY_NODE, vocab=None,
                             stream=None) -> bool:
    """talon_build_tree, then the layer-by-layer rebuild if the launch gave up.  Waits for the stream.
    Returns whether the layer-by-layer path ran."""
    dt, row_stride, seq_stride, V = _logits_meta(logits)
    fell = c_int32(0)
    _check(load_library().talon_build_tree_checked(
        _ptr(root_token), _ptr(logits), dt, row_stride, seq_stride, row_mode, ctypes.byref(st.c),
        V if vocab is None else vocab, k, c_float(mu), K_init, init_layers, max_depth, _ptr(cand.token),
        _ptr(cand.logit), _ptr(cand.prob), _ptr(cand.edge_logp), _ptr(cand.row_max), _ptr(cand.row_lse), _ptr(mask),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream), ctypes.byref(fell)))
    return bool(fell.value)


def talon_set_spin_limit_us(microseconds: int):
    _check(load_library().talon_set_spin_limit_us(microseconds))


def talon_profile_scan_launches(enable: bool):
    _check(load_library().talon_profile_scan_launches(1 if enable else 0))


def talon_profile_read(capacity: int):
    """Durations (microseconds, launch order) of the fused scan launches recorded since the last read."""
    buf = (c_float * max(capacity, 1))()
    n = c_int32(0)
    _check(load_library().talon_profile_read(buf, capacity, ctypes.byref(n)))
    return [float(buf[i]) for i in range(min(n.value, capacity))], n.value


def talon_probe_read(buf: torch.Tensor, sink: torch.Tensor, stream=None):
    _check(load_library().talon_probe_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream(stream)))


def talon_probe_mfma(workgroups: int, iters: int, sink: torch.Tensor, stream=None) -> float:
    """Launches the MFMA probe; returns the FLOPs of the launch."""
    fl = c_double(0.0)
    _check(load_library().talon_probe_mfma(workgroups, iters, _ptr(sink), ctypes.byref(fl), _stream(stream)))
    return fl.value


def talon_probe_issue(mode: int, waves: int, iters: int, cycles: torch.Tensor, sink: torch.Tensor, stream=None):
    """cycles: 8 int64 on the device, one per wavefront."""
    _check(load_library().talon_probe_issue(mode, waves, iters, _ptr(cycles), _ptr(sink), _stream(stream)))


def talon_probe_tile_loads(window: torch.Tensor, loads: int, with_mfma: bool, waves: int, iters: int,
                           cycles: torch.Tensor, sink: torch.Tensor, stream=None):
    """window: at least 16 MiB on the device; cycles: 2048 int64 on the device, [workgroup][wavefront]."""
    _check(load_library().talon_probe_tile_loads(_ptr(window), window.numel() * window.element_size(), loads,
                                                 1 if with_mfma else 0, waves, iters, _ptr(cycles), _ptr(sink),
                                                 _stream(stream)))


def talon_build_tree_mask(st: TreeState, mask: torch.Tensor, stream=None):
    _check(load_library().talon_build_tree_mask(ctypes.byref(st.c), _ptr(mask), _stream(stream)))


def talon_tree_attention_workspace_bytes(B, N_pad, Hq, Hkv, Dh, max_prefix_len) -> int:
    return load_library().talon_tree_attention_workspace_bytes(B, N_pad, Hq, Hkv, Dh, max_prefix_len)


def talon_static_scratch_bytes() -> int:
    return load_library().talon_static_scratch_bytes()


def talon_static_scratch_init():
    _check(load_library().talon_static_scratch_init())


def talon_tree_attention_static(q, k_prefix, v_prefix, k_tree, v_tree, mask, n_nodes, prefix_len, max_prefix_len, out,
                                out_lse=None, scale=0.0, stream=None):
    """talon_tree_attention without a workspace argument (the library's own scratch array)."""
    return talon_tree_attention(q, k_prefix, v_prefix, k_tree, v_tree, mask, n_nodes, prefix_len, max_prefix_len,
                                out, out_lse, None, scale, stream, _static=True)


def talon_tree_attention(q, k_prefix, v_prefix, k_tree, v_tree, mask, n_nodes, prefix_len, max_prefix_len, out,
                         out_lse=None, workspace=None, scale=0.0, stream=None, _static=False):
    """q/k_tree/v_tree [B][N_pad][H][Dh] bf16 dense; k_prefix/v_prefix [B][L][Hkv][Dh] views (any strides
    with a contiguous Dh run); mask [B][N_pad][N_pad/64] int64."""
    B, N_pad, Hq, Dh = q.shape
    Hkv = k_tree.shape[2]
    for t in (q, k_tree, v_tree, out, mask):
        if not t.is_contiguous():
            raise TalonError(TALON_ERR_INVALID_ARG, "q, k_tree, v_tree, mask and out must be contiguous")
    if max_prefix_len == 0 or (k_prefix is not None and k_prefix.numel() == 0):
        k_prefix = v_prefix = None     # no prefix: the tree attends to itself only
    if k_prefix is not None:
        if k_prefix.stride() != v_prefix.stride() or k_prefix.stride(3) != 1:
            raise TalonError(TALON_ERR_INVALID_ARG, "k_prefix and v_prefix must share strides, Dh contiguous")
        sb, st_, sh = k_prefix.stride(0), k_prefix.stride(1), k_prefix.stride(2)
    else:
        sb = st_ = sh = Dh
    if _static:
        _check(load_library().talon_tree_attention_static(
            _ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_tree), _ptr(v_tree), _ptr(mask), _ptr(n_nodes),
            _ptr(prefix_len), B, N_pad, Hq, Hkv, Dh, max_prefix_len, sb, st_, sh, c_float(scale), _ptr(out),
            _ptr(out_lse), _stream(stream)))
        return
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().talon_tree_attention(
        _ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_tree), _ptr(v_tree), _ptr(mask), _ptr(n_nodes),
        _ptr(prefix_len), B, N_pad, Hq, Hkv, Dh, max_prefix_len, sb, st_, sh, c_float(scale), _ptr(out),
        _ptr(out_lse), _ptr(workspace), ws_bytes, _stream(stream)))


def make_literal_workspace(B, N_pad, vocab, dtype) -> torch.Tensor:
    nb = load_library().talon_literal_workspace_bytes(B, N_pad, vocab, dtype)
    if nb == 0:
        raise TalonError(TALON_ERR_INVALID_ARG, load_library().talon_last_error_string().decode())
    return torch.empty(nb, dtype=torch.uint8, device="cuda")


def talon_expand_literal(logits, st: TreeState, layers, mu, K_init, init_layers, max_depth, workspace,
                         row_mode=TALON_ROWS_BY_NODE, vocab=None, stream=None):
    dt, row_stride, seq_stride, V = _logits_meta(logits)
    _check(load_library().talon_expand_literal(
        _ptr(logits), dt, row_stride, seq_stride, row_mode, layers, ctypes.byref(st.c), V if vocab is None else vocab,
        c_float(mu), K_init, init_layers, max_depth, _ptr(workspace), workspace.numel() * workspace.element_size(),
        _stream(stream)))


def make_verify_workspace(B, N_pad, vocab, dtype) -> torch.Tensor:
    nb = load_library().talon_verify_workspace_bytes(B, N_pad, vocab, dtype)
    if nb == 0:
        raise TalonError(TALON_ERR_INVALID_ARG, load_library().talon_last_error_string().decode())
    return torch.empty(nb, dtype=torch.uint8, device="cuda")


def talon_target_argmax(logits, st: TreeState, target_token, target_prob, scan_status, workspace, vocab=None,
                        stream=None):
    dt, row_stride, seq_stride, V = _logits_meta(logits)
    _check(load_library().talon_target_argmax(
        _ptr(logits), dt, row_stride, seq_stride, ctypes.byref(st.c), V if vocab is None else vocab,
        _ptr(target_token), _ptr(target_prob), _ptr(scan_status), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def talon_greedy_accept(st: TreeState, target_token, scan_status, path, accept_len, bonus_token, stream=None):
    _check(load_library().talon_greedy_accept(ctypes.byref(st.c), _ptr(target_token), _ptr(scan_status), _ptr(path),
                                              _ptr(accept_len), _ptr(bonus_token), _stream(stream)))


def talon_compact_kv(k_tree, v_tree, path, accept_len, prefix_len, new_prefix_len, k_prefix, v_prefix, stream=None):
    """k_tree/v_tree [B][N_pad][Hkv][Dh] bf16 dense; k_prefix/v_prefix [B][capacity][Hkv][Dh] views sharing
    strides, Dh contiguous."""
    B, N_pad, Hkv, Dh = k_tree.shape
    if k_prefix.stride() != v_prefix.stride() or k_prefix.stride(3) != 1:
        raise TalonError(TALON_ERR_INVALID_ARG, "k_prefix and v_prefix must share strides, Dh contiguous")
    _check(load_library().talon_compact_kv(
        _ptr(k_tree), _ptr(v_tree), _ptr(path), _ptr(accept_len), _ptr(prefix_len), _ptr(new_prefix_len),
        _ptr(k_prefix), _ptr(v_prefix), B, N_pad, Hkv, Dh, k_prefix.shape[1], k_prefix.stride(0), k_prefix.stride(1),
        k_prefix.stride(2), _stream(stream)))


def talon_prune_tree(st: TreeState, n_keep: int, kept_ids, stream=None):
    _check(load_library().talon_prune_tree(ctypes.byref(st.c), n_keep, _ptr(kept_ids), _stream(stream)))
