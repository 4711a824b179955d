"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random numbers and thresholds them; it holds none of the method's
arithmetic (no attention, no layout).  Both the GPU tests/benchmark and the CPU oracle
checks take their inputs from here, so the two sides see identical data.

The paper builds its masks from attention maps averaged over a training set (Eq. (1)) and
a percentile threshold (Eq. (2)).  Neither its datasets nor trained weights are available,
so each configuration below synthesises a "mean attention map" with the structure the paper
reports for such maps -- smooth positional patterns: a band next to the diagonal, an
attention-sink column, separator columns, a jittered alignment band for cross-attention,
rare long-range spikes -- adds noise, and keeps the strongest entries of every head.

Configurations (index = position in the benchmark's config list):
  C1  tiny causal self-attention, fp32           B1  H2  L64   D32   keep 10 % of causal entries
  C2  encoder self-attention (BERT-base shape)   B32 H12 L128  D64   keep 50 %
  C3  autoregressive LM (GPT-2-small shape)      B16 H12 L512  D64   keep 10 % of causal entries
  C4  seq2seq cross-attention                    B32 H8  128x128 D64 keep 50 %
  C5  long-context LM                            B4  H16 L4096 D128  keep 10 % of causal entries
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED = 20120203


@dataclass(frozen=True)
class Config:
    name: str
    index: int          # 1-based, enters the RNG seed
    B: int
    H: int
    Lq: int
    Lk: int
    D: int
    dtype: str          # "f32" or "bf16"
    causal: bool
    keep: float         # fraction of (causal-)valid entries kept per head
    band: int = 0       # band width parameter of the generator
    spike: float = 0.0  # density of long-range spikes


CONFIGS = {
    "C1": Config("C1", 1, 1, 2, 64, 64, 32, "f32", True, 0.10, band=4),
    "C2": Config("C2", 2, 32, 12, 128, 128, 64, "bf16", False, 0.50, band=8),
    "C3": Config("C3", 3, 16, 12, 512, 512, 64, "bf16", True, 0.10, band=32, spike=0.01),
    "C4": Config("C4", 4, 32, 8, 128, 128, 64, "bf16", False, 0.50, band=12),
    "C5": Config("C5", 5, 4, 16, 4096, 4096, 128, "bf16", True, 0.10, band=128, spike=0.001),
}


# A further shape, not one of the five benchmark configurations: a 64-token segment attending to a
# long memory plus itself (the Transformer-XL setting of Section 4.1), for the split forward call.
EXTRA_CONFIGS = {
    "X1": Config("X1", 6, 4, 16, 64, 16384, 128, "bf16", True, 0.10, band=128, spike=0.001),
}


def _keep_top(score: np.ndarray, valid: np.ndarray | None, frac: float) -> np.ndarray:
    """Boolean map that keeps exactly round(frac * #valid) largest valid entries."""
    flat = score.astype(score.dtype, copy=True).ravel()
    if valid is not None:
        flat[~valid.ravel()] = -np.inf
        n_valid = int(valid.sum())
    else:
        n_valid = flat.size
    k = int(round(frac * n_valid))
    keep = np.zeros(flat.size, dtype=bool)
    if k > 0:
        idx = np.argpartition(flat, flat.size - k)[flat.size - k:]
        keep[idx] = True
    return keep.reshape(score.shape)


def head_mask(cfg: Config, h: int) -> np.ndarray:
    """Keep-mask [Lq, Lk] (bool) of head h of configuration cfg."""
    rng = np.random.default_rng([SEED, cfg.index, h])
    Lq, Lk = cfg.Lq, cfg.Lk
    i = np.arange(Lq)[:, None]
    j = np.arange(Lk)[None, :]
    causal_valid = (j <= i + (Lk - Lq)) if cfg.causal else None

    if cfg.name == "C1":
        noise = rng.random((Lq, Lk))
        d = i - j
        score = 1.0 * ((d >= 0) & (d < cfg.band)) + 1.0 * (j == 0) + noise
        keep = _keep_top(score, causal_valid, cfg.keep)
        keep |= (i == j)
    elif cfg.name == "C2":
        noise = rng.lognormal(0.0, 1.0, (Lq, Lk))
        score = 4.0 * (np.abs(i - j) <= cfg.band // 2) + 4.0 * ((j == 0) | (j == Lk - 1)) + noise
        keep = _keep_top(score, None, cfg.keep)
        keep |= (i == j)
    elif cfg.name in ("C3", "C5", "X1"):
        w = np.float32(cfg.band)
        gauss = rng.standard_normal((Lq, Lk), dtype=np.float32)
        spikes = rng.random((Lq, Lk), dtype=np.float32) < np.float32(cfg.spike)
        d = (i + (Lk - Lq) - j).astype(np.float32)           # distance behind the query's own position
        inband = ((d >= 0) & (d < w)).astype(np.float32)
        base = inband * (np.float32(1.0) - d / w)
        with np.errstate(divide="ignore", invalid="ignore"):
            base = base + np.float32(0.1) / (np.float32(1.0) + np.maximum(d, np.float32(0.0)) / w)
        base = base + (j == 0).astype(np.float32)
        score = base * np.exp(np.float32(0.1) * gauss) + np.float32(5.0) * spikes.astype(np.float32)
        del gauss, spikes, base, inband, d
        keep = _keep_top(score, causal_valid, cfg.keep)
        keep |= (j == i + (Lk - Lq))
    elif cfg.name == "C4":
        jitter = rng.integers(-8, 9, Lq)
        noise = rng.lognormal(0.0, 1.0, (Lq, Lk))
        centre = np.clip(np.arange(Lq) * (Lk / Lq) + jitter, 0, Lk - 1).astype(np.int64)[:, None]
        score = 4.0 * (np.abs(j - centre) <= cfg.band // 2) + noise
        keep = _keep_top(score, None, cfg.keep)
        keep |= (j == centre)
    else:
        raise KeyError(cfg.name)
    if cfg.causal:
        keep &= causal_valid
    return keep


def make_mask(cfg: Config, workers: int = 8) -> np.ndarray:
    """uint8 keep-mask [H, Lq, Lk] (1 = kept) for all heads of cfg.

    Heads are independent (each has its own seed), so they are drawn on a small thread pool;
    the result does not depend on the number of workers.
    """
    out = np.empty((cfg.H, cfg.Lq, cfg.Lk), dtype=np.uint8)

    def one(h):
        out[h] = head_mask(cfg, h)

    if cfg.Lq * cfg.Lk < (1 << 20) or workers <= 1:
        for h in range(cfg.H):
            one(h)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(workers, cfg.H)) as pool:
            list(pool.map(one, range(cfg.H)))
    return out


def dense_mask(cfg: Config) -> np.ndarray:
    """All-ones mask of cfg's shape: the paper's p = 0 case (M_p = 0)."""
    return np.ones((cfg.H, cfg.Lq, cfg.Lk), dtype=np.uint8)


def make_qkv(cfg: Config, which: str = "QKV", set_index: int = 0):
    """Standard-normal float32 tensors [B,H,L,D] for the letters in ``which``.

    ``set_index`` selects an independent draw (the benchmark rotates through several sets
    so that no call finds its inputs in cache).
    """
    out = []
    for t, letter in enumerate("QKV"):
        if letter not in which:
            continue
        rng = np.random.default_rng([SEED, cfg.index, 100 + t, set_index])
        L = cfg.Lq if letter == "Q" else cfg.Lk
        out.append(rng.standard_normal((cfg.B, cfg.H, L, cfg.D), dtype=np.float32))
    return out


def make_qk_positional(B: int, H: int, Lq: int, Lk: int, D: int, seed: int,
                       strength: float = 1.0):
    """Queries and keys whose attention concentrates next to the (bottom-right aligned) diagonal,
    as the averaged self-attention patterns in the figure of Section 5.1 do: a sinusoidal
    position code shared by Q and K (query i carries the code of position i + Lk - Lq, key j
    that of position j, one random frequency set per head) plus standard-normal content.
    float32 [B,H,Lq,D], [B,H,Lk,D]."""
    rng = np.random.default_rng([SEED, 777, seed])
    freq = np.exp(rng.uniform(np.log(1e-3), np.log(1.0), size=(H, D // 2)))
    pos = np.arange(Lk, dtype=np.float64)[None, :, None] * freq[:, None, :]        # [H, Lk, D/2]
    code = np.concatenate([np.sin(pos), np.cos(pos)], axis=-1) * strength            # [H, Lk, D]
    Q = rng.standard_normal((B, H, Lq, D)) + code[None, :, Lk - Lq:, :]
    K = rng.standard_normal((B, H, Lk, D)) + code[None]
    return Q.astype(np.float32), K.astype(np.float32)


def make_mean_map(H: int, Lq: int, Lk: int, seed: int) -> np.ndarray:
    """float32 [H,Lq,Lk] stand-in for a layer's mean attention maps: a per-head band that decays
    away from the (bottom-right aligned) diagonal plus a small floor, times uniform noise.
    Rows are not normalised; only the order of the values matters to the threshold."""
    out = np.empty((H, Lq, Lk), dtype=np.float32)
    d = np.abs(np.arange(Lq, dtype=np.float32)[:, None] + np.float32(Lk - Lq)
               - np.arange(Lk, dtype=np.float32)[None, :])
    for h in range(H):
        rng = np.random.default_rng([SEED, 555, seed, h])
        width = np.float32(4.0 * (1 + h % 5))
        noise = rng.random((Lq, Lk), dtype=np.float32) + np.float32(0.05)
        out[h] = (np.exp(-d / width) + np.float32(1e-3)) * noise
    return out


def random_mask(H: int, Lq: int, Lk: int, density: float, seed: int) -> np.ndarray:
    """iid Bernoulli(density) keep-mask: the worst case for tile skipping (the paper's
    random-pruning control uses such patterns)."""
    rng = np.random.default_rng([SEED, 999, seed])
    return (rng.random((H, Lq, Lk)) < density).astype(np.uint8)


def tile_stats(mask_h: np.ndarray, bm: int, bn: int, causal: bool) -> dict:
    """Counts of non-empty BMxBN tiles of one head's mask (plain numpy bookkeeping)."""
    Lq, Lk = mask_h.shape
    nqb, nkb = -(-Lq // bm), -(-Lk // bn)
    pad = np.zeros((nqb * bm, nkb * bn), dtype=bool)
    pad[:Lq, :Lk] = mask_h != 0
    per_tile = pad.reshape(nqb, bm, nkb, bn).sum(axis=(1, 3))
    if causal:
        qi = np.arange(nqb)[:, None] * bm + (bm - 1)
        kj = np.arange(nkb)[None, :] * bn
        valid = kj <= np.minimum(qi, Lq - 1) + (Lk - Lq)
    else:
        valid = np.ones_like(per_tile, dtype=bool)
    return {
        "valid_tiles": int(valid.sum()),
        "nonempty_tiles": int((per_tile > 0).sum()),
        "kept_entries": int(per_tile.sum()),
        "per_tile": per_tile,
    }
