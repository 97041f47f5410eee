"""Counter-based seeded generators for logits rows and Q/K/V tensors.

Every logits row is a pure function of (seed, config, sequence b, node id), so
any row can be regenerated anywhere, and the row a tree node reads does not
depend on how the tree was built.  bf16 data is carried as raw uint16 bit
patterns (numpy has no bf16); `storage_to_f64` decodes them exactly.

Nothing here is part of the method: these are input bytes only.
"""
from __future__ import annotations

import math

import numpy as np

from .configs import WorkloadConfig

_TAG_LOGITS = 0x10
_TAG_Q = 0x21
_TAG_KP = 0x22
_TAG_VP = 0x23
_TAG_KT = 0x24
_TAG_VT = 0x25
_TAG_TARGET = 0x31


def _rng(seed: int, tag: int, b: int, i: int) -> np.random.Generator:
    """Philox stream keyed by (seed, tag, b, i): independent per key."""
    key = np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF),
                    np.uint64(((tag & 0xFF) << 56) | ((b & 0xFFFFFF) << 32) | (i & 0xFFFFFFFF))],
                   dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if np.any(nan):
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact decode of bf16 bit patterns to float64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def storage_to_f64(x: np.ndarray) -> np.ndarray:
    """Exact upcast of a stored array (uint16 = bf16 bits, float32) to float64."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f64(x)
    return x.astype(np.float64)


def _store(x32: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    if dtype == "f32":
        return np.ascontiguousarray(x32, dtype=np.float32)
    raise ValueError(dtype)


def zipf_row(V: int, alpha: float, a: int, c: int) -> np.ndarray:
    """Zipf logits: logit(w) = -alpha * ln(rank(w)), rank(w) = 1 + ((a*w + c) mod V).

    With gcd(a, V) = 1 the map w -> rank is a bijection, so the row is a
    permuted Zipf distribution P(r) ~ r^-alpha (the paper's micro-benchmark
    recipe, App. E.6).  Returned as float32 before storage rounding.
    """
    assert math.gcd(a, V) == 1
    w = np.arange(V, dtype=np.int64)
    rank = 1 + (a * w + c) % V
    return (-alpha * np.log(rank.astype(np.float64))).astype(np.float32)


def _zipf_keyed(g: np.random.Generator, V: int, alpha: float) -> np.ndarray:
    """Zipf row with a per-row permutation and a per-row exponent within 2% of `alpha`.

    Rows with exactly the same exponent are permutations of one another: they share one
    log-sum-exp and one set of top logits, so candidates of different parents tie exactly in
    real arithmetic and no finite-precision implementation can reproduce the order of those
    ties.  The small jitter keeps the Zipf shape and makes every comparison a real one.
    """
    while True:
        a = int(g.integers(1, V))
        if math.gcd(a, V) == 1:
            break
    c = int(g.integers(0, V))
    return zipf_row(V, alpha * (1.0 + 0.02 * g.uniform(-1.0, 1.0)), a, c)


def _recipe_for(cfg: WorkloadConfig, b: int):
    r = cfg.recipe
    if isinstance(r[0], tuple):
        return r[b % len(r)]
    return r


def logits_row(cfg: WorkloadConfig, seed: int, b: int, node: int) -> np.ndarray:
    """Logits row the draft model would emit for node `node` of sequence `b`.

    Returns the stored row: float32[V] or uint16[V] (bf16 bits).
    """
    g = _rng(seed, _TAG_LOGITS, b, node)
    rec = _recipe_for(cfg, b)
    if rec[0] == "gauss":
        beta = g.uniform(rec[1], rec[2])
        x = g.standard_normal(cfg.V, dtype=np.float32) * np.float32(beta)
    elif rec[0] == "zipf_mix":
        if node % 2 == 0:
            x = _zipf_keyed(g, cfg.V, rec[1])
        else:
            x = g.standard_normal(cfg.V, dtype=np.float32) * np.float32(rec[2])
    elif rec[0] == "zipf":
        x = _zipf_keyed(g, cfg.V, rec[1])
    else:
        raise ValueError(rec)
    return _store(x, cfg.logits_dtype)


def target_logits_row(cfg: WorkloadConfig, seed: int, b: int, node: int, noise: float = 0.25) -> np.ndarray:
    """Logits row the *target* model would emit at node `node` of sequence `b`: the draft's
    stored row plus independent Gaussian noise of `noise` times the row's standard deviation,
    so that the target mostly, but not always, agrees with the draft's best token (a stand-in
    for a real drafter/target pair).  Stored in the config's logits type."""
    draft = storage_to_f64(logits_row(cfg, seed, b, node)).astype(np.float32)
    g = _rng(seed, _TAG_TARGET, b, node)
    sd = np.float32(draft[np.isfinite(draft)].std()) if np.isfinite(draft).any() else np.float32(1.0)
    x = draft + g.standard_normal(cfg.V, dtype=np.float32) * np.float32(noise) * sd
    return _store(x, cfg.logits_dtype)


def target_logits_pool(cfg: WorkloadConfig, seed, noise: float = 0.25) -> np.ndarray:
    """Pool [B][N_pad][V] of target rows; `seed` is one seed or one per sequence."""
    seeds = [seed] * cfg.B if np.isscalar(seed) else list(seed)
    dt = np.float32 if cfg.logits_dtype == "f32" else np.uint16
    pool = np.zeros((cfg.B, cfg.N_pad, cfg.V), dtype=dt)
    for b in range(cfg.B):
        for i in range(cfg.N):
            pool[b, i] = target_logits_row(cfg, seeds[b], b, i, noise)
    return pool


def logits_pool(cfg: WorkloadConfig, seed: int, nodes=None) -> np.ndarray:
    """Pool [B][N_pad][V] of stored rows; row (b, i) feeds node i of sequence b.

    `nodes` limits generation to node ids < nodes (others stay zero); the
    default fills every row a tree can ever read (ids < N).
    """
    n_fill = cfg.N if nodes is None else nodes
    dt = np.float32 if cfg.logits_dtype == "f32" else np.uint16
    pool = np.zeros((cfg.B, cfg.N_pad, cfg.V), dtype=dt)
    for b in range(cfg.B):
        for i in range(n_fill):
            pool[b, i] = logits_row(cfg, seed, b, i)
    return pool


def _normal_bf16(seed: int, tag: int, b: int, shape) -> np.ndarray:
    g = _rng(seed, tag, b, 0)
    return f32_to_bf16_bits(g.standard_normal(shape, dtype=np.float32))


def attention_inputs(cfg: WorkloadConfig, seed: int, b: int, L: int | None = None):
    """bf16 N(0,1) tensors for sequence b, as uint16 bit patterns.

    Returns dict with q [N_pad][Hq][Dh], k_prefix/v_prefix [L][Hkv][Dh],
    k_tree/v_tree [N_pad][Hkv][Dh].
    """
    L = cfg.L if L is None else L
    return {
        "q": _normal_bf16(seed, _TAG_Q, b, (cfg.N_pad, cfg.Hq, cfg.Dh)),
        "k_prefix": _normal_bf16(seed, _TAG_KP, b, (L, cfg.Hkv, cfg.Dh)),
        "v_prefix": _normal_bf16(seed, _TAG_VP, b, (L, cfg.Hkv, cfg.Dh)),
        "k_tree": _normal_bf16(seed, _TAG_KT, b, (cfg.N_pad, cfg.Hkv, cfg.Dh)),
        "v_tree": _normal_bf16(seed, _TAG_VT, b, (cfg.N_pad, cfg.Hkv, cfg.Dh)),
    }
