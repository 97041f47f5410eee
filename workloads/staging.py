"""Input staging: whole logits pools on the host, and host arrays moved to device buffers.

Nothing here is part of the method: it lays out input bytes (the rows of `generators`) the way
the library's calls expect them, for the tests and the benchmark alike.
"""
from __future__ import annotations

import numpy as np

from .configs import WorkloadConfig
from .generators import logits_row


def build_pool(cfg: WorkloadConfig, seeds) -> np.ndarray:
    """Pool [B][N_pad][V] of stored rows: row (b, i) is the draft row of node i of sequence b,
    generated from seeds[b]; rows of ids >= N stay zero."""
    dt = np.float32 if cfg.logits_dtype == "f32" else np.uint16
    pool = np.zeros((cfg.B, cfg.N_pad, cfg.V), dtype=dt)
    for b in range(cfg.B):
        for i in range(cfg.N):
            pool[b, i] = logits_row(cfg, seeds[b], b, i)
    return pool


def root_tokens(cfg: WorkloadConfig) -> np.ndarray:
    """Token id of the root x_t of every sequence (any id serves: the expansion never reads it)."""
    return (np.arange(cfg.B, dtype=np.int32) * 7 + 11) % cfg.V


def to_device_logits(pool: np.ndarray):
    """Pool on the device, rows padded to a multiple of 8 elements (the library wants 16-byte row
    strides); the returned view keeps the true vocabulary width."""
    import torch
    V = pool.shape[2]
    V_pad = (V + 7) // 8 * 8
    if V_pad != V:
        padded = np.zeros(pool.shape[:2] + (V_pad,), dtype=pool.dtype)
        padded[:, :, :V] = pool
        pool = padded
    if pool.dtype == np.uint16:
        dev = torch.from_numpy(pool.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        dev = torch.from_numpy(pool).cuda()
    return dev[:, :, :V]


def bf16_to_device(bits: np.ndarray):
    """uint16 bf16 bit patterns -> a torch.bfloat16 device tensor of the same shape."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)
