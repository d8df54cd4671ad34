"""Seeded generator for the synthetic K/V tensors.

Every random stream is keyed by (seed, batch index, layer, head, tensor) through
numpy's SeedSequence, so units can be produced in any order or in parallel and
always come out bit-identical.  Values are drawn in fp64, rounded once to fp32
(round-to-nearest-even) and, for bf16 storage, once more to bf16
(round-to-nearest-even).  bf16 tensors are returned as uint16 bit patterns.

Streams
  [seed, b, l, h, t]   t = 0 for K, 1 for V: everything specific to one tensor
  [seed, b, l, 99]     layer level: outlier fraction, positions, magnitudes
                       (a KV *pair* is the outlier: positions are shared by the
                       layer's heads and by K and V; the added vectors are not)
  [seed, b, 98]        sequence level: (source, destination) duplicate pairs
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Tuple

import numpy as np

from .configs import KVConfig

K_TENSOR, V_TENSOR = 0, 1
_LAYER_STREAM, _SEQ_STREAM = 99, 98


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(key))))


# --------------------------------------------------------------------------- #
# storage-type helpers (pure bit manipulation)
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round-to-nearest-even; finite input."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> float32, exact."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(x64: np.ndarray, dtype: str) -> np.ndarray:
    x32 = x64.astype(np.float32)
    if dtype == "f32":
        return x32
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    raise ValueError(f"unknown storage dtype {dtype!r}")


# --------------------------------------------------------------------------- #
# layer- and sequence-level draws
# --------------------------------------------------------------------------- #
def layer_outlier_positions(cfg: KVConfig, b: int, l: int) -> Tuple[np.ndarray, np.ndarray]:
    """Sorted outlier token positions of layer l and their magnitudes (sigma units)."""
    rng = _rng(cfg.seed, b, l, _LAYER_STREAM)
    if cfg.outlier_frac_range is not None:
        lo, hi = cfg.outlier_frac_range
        frac = float(rng.uniform(lo, hi))
    else:
        frac = cfg.outlier_frac
    n_out = int(round(frac * cfg.n_tokens))
    if cfg.outliers_visual_only and cfg.layout == "blocks":
        lo_t, hi_t = cfg.visual_start, cfg.visual_end
    else:
        lo_t, hi_t = 0, cfg.n_tokens
    n_out = min(n_out, hi_t - lo_t)
    pos = np.sort(lo_t + rng.choice(hi_t - lo_t, size=n_out, replace=False))
    if cfg.outlier_kind == "student":
        mag = cfg.outlier_sigma * np.abs(rng.standard_t(cfg.outlier_nu, size=n_out))
    else:
        mag = np.full(n_out, cfg.outlier_sigma)
    return pos.astype(np.int64), mag


def sequence_duplicates(cfg: KVConfig, b: int) -> Tuple[np.ndarray, np.ndarray]:
    """(src, dst) token pairs: row dst is overwritten by row src in every tensor."""
    n_dup = int(round(cfg.dup_frac * cfg.n_tokens))
    if n_dup == 0:
        e = np.zeros(0, dtype=np.int64)
        return e, e
    rng = _rng(cfg.seed, b, _SEQ_STREAM)
    perm = rng.permutation(cfg.n_tokens)[: 2 * n_dup]
    return perm[:n_dup].astype(np.int64), perm[n_dup:].astype(np.int64)


# --------------------------------------------------------------------------- #
# one tensor
# --------------------------------------------------------------------------- #
def _cos_modes(n: int, n_modes: int) -> np.ndarray:
    t = np.arange(n, dtype=np.float64) + 0.5
    j = np.arange(n_modes, dtype=np.float64)
    return np.cos(np.pi * t[:, None] * j[None, :] / n)            # [n, modes]


def _mode_amplitudes(rng: np.random.Generator, n_modes: int) -> np.ndarray:
    j = np.arange(n_modes, dtype=np.float64)
    return rng.standard_normal(n_modes) * np.sqrt(1.0 / (j + 1.0))  # variance 1/(j+1)


def _tensor(cfg: KVConfig, b: int, l: int, h: int, t: int,
            pos: np.ndarray, mag: np.ndarray) -> np.ndarray:
    n, d, m = cfg.n_tokens, cfg.head_dim, cfg.n_modes
    rng = _rng(cfg.seed, b, l, h, t)
    if cfg.layout == "flat":
        a = _mode_amplitudes(rng, m)
        w = rng.standard_normal((m, d))
        z = rng.standard_normal((n, d))
        x = (_cos_modes(n, m) * a) @ w + cfg.noise_sigma * z
    elif cfg.layout == "blocks":
        nb, bl = cfg.n_blocks, cfg.block_len
        if cfg.drift_delta > 0.0:
            a = _mode_amplitudes(rng, m)
            w_blocks = np.empty((nb, m, d))
            w_blocks[0] = rng.standard_normal((m, d))
            keep = np.sqrt(1.0 - cfg.drift_delta ** 2)
            for k in range(1, nb):
                w_blocks[k] = keep * w_blocks[k - 1] + cfg.drift_delta * rng.standard_normal((m, d))
            a_blocks = np.broadcast_to(a, (nb, m))
        else:
            a_blocks = np.empty((nb, m))
            w_blocks = np.empty((nb, m, d))
            for k in range(nb):
                a_blocks[k] = _mode_amplitudes(rng, m)
                w_blocks[k] = rng.standard_normal((m, d))
        z = rng.standard_normal((n, d))
        x = cfg.text_sigma * z
        basis = _cos_modes(bl, m)
        for k in range(nb):
            s = cfg.visual_start + k * bl
            x[s:s + bl] = (basis * a_blocks[k]) @ w_blocks[k] + cfg.noise_sigma * z[s:s + bl]
    else:
        raise ValueError(f"unknown layout {cfg.layout!r}")
    if pos.size:
        x[pos] += mag[:, None] * rng.standard_normal((pos.size, d))
    return x


def generate_unit(cfg: KVConfig, b: int, l: int, h: int,
                  pos=None, mag=None, dup=None) -> Tuple[np.ndarray, np.ndarray]:
    """K and V of one (sequence, layer, head) unit, shape [N, d], in storage type."""
    if pos is None:
        pos, mag = layer_outlier_positions(cfg, b, l)
    if dup is None:
        dup = sequence_duplicates(cfg, b)
    out = []
    for t in (K_TENSOR, V_TENSOR):
        x = _tensor(cfg, b, l, h, t, pos, mag)
        src, dst = dup
        if src.size:
            x[dst] = x[src]
        out.append(_store(x, cfg.dtype))
    return out[0], out[1]


def generate_sequence(cfg: KVConfig, b: int, workers: int = 1,
                      layers=None) -> Tuple[np.ndarray, np.ndarray]:
    """K and V of sequence b, shape [L', H, N, d] (L' = len(layers) or cfg.layers)."""
    layer_ids = list(range(cfg.layers)) if layers is None else list(layers)
    np_dtype = np.float32 if cfg.dtype == "f32" else np.uint16
    shape = (len(layer_ids), cfg.kv_heads, cfg.n_tokens, cfg.head_dim)
    K = np.empty(shape, dtype=np_dtype)
    V = np.empty(shape, dtype=np_dtype)
    dup = sequence_duplicates(cfg, b)
    per_layer = {l: layer_outlier_positions(cfg, b, l) for l in layer_ids}

    def work(job):
        li, l, h = job
        pos, mag = per_layer[l]
        K[li, h], V[li, h] = generate_unit(cfg, b, l, h, pos, mag, dup)

    jobs = [(li, l, h) for li, l in enumerate(layer_ids) for h in range(cfg.kv_heads)]
    if workers <= 1:
        for j in jobs:
            work(j)
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(work, jobs))
    return K, V


def generate(cfg: KVConfig, workers: int = 1) -> Tuple[np.ndarray, np.ndarray]:
    """All sequences: K and V of shape [B, L, H, N, d]."""
    ks, vs = [], []
    for b in range(cfg.batch):
        k, v = generate_sequence(cfg, b, workers)
        ks.append(k)
        vs.append(v)
    return np.stack(ks), np.stack(vs)
