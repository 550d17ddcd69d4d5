"""Seeded synthetic layers (weights W and calibration activations X).

This module only draws random numbers and shapes them; it holds none of the
quantisation method's arithmetic.  Both the CPU oracle's tests and the HIP
path's tests / benchmark read their inputs from here, so the two sides see
the same bytes.

The layers stand in for the public LLaMA linear-layer shapes and for the
paper's calibration set (128 random 2048-token segments, Sec. 4), which are
not available offline.  Activation outlier channels and salient weight
channels are placed in contiguous runs of four at seeded positions, following
the clustered-channel observation of Sec. 3.2.1 and Theorem 1.

Layout conventions (the paper's notation, Sec. 3.1):
  W : (n, m)  n output rows, m input channels, row-major
  X : (m, t)  input channels x tokens, tokens contiguous (so H ~ X X^T)
"""
from __future__ import annotations

import dataclasses
from typing import Iterator, Tuple

import numpy as np

CHUNK_TOKENS = 8192  # X is generated in independent token chunks of this size
RUN = 4              # outlier / salient channels come in runs of this length


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    name: str
    n: int                 # output rows of W
    m: int                 # input channels
    t: int                 # calibration tokens
    beta: int              # group size along the input dimension
    N: int                 # target average bit-width
    w_dtype: str           # "f32" or "f16"
    w_dist: str            # "normal" | "student4"
    w_std: float
    w_salient_frac: float  # fraction of input channels scaled up in W
    w_salient_count: int   # explicit count (overrides the fraction when > 0)
    w_salient_gain: float
    x_dist: str            # "normal" | "lognormal_scale" | "student4"
    x_outlier_frac: float
    x_outlier_count: int
    x_outlier_gain: float
    index: int             # position in the benchmark's config list (seeds)
    percdamp: float = 0.01
    ncand: int = 100
    sqc_lambda: float = 0.1

    @property
    def k(self) -> int:
        return self.m // self.beta

    def seeds(self) -> Tuple[int, int, int]:
        i = self.index
        return 1000 + i, 2000 + i, 3000 + i


CONFIGS = {
    "C1": LayerConfig("C1", 256, 256, 512, 64, 2, "f32", "normal", 0.02,
                      0.0, 4, 10.0, "normal", 0.0, 4, 20.0, 1),
    "C2": LayerConfig("C2", 4096, 4096, 131072, 128, 2, "f16", "normal", 0.02,
                      0.0, 0, 1.0, "lognormal_scale", 0.005, 0, 50.0, 2),
    "C3": LayerConfig("C3", 4096, 11008, 262144, 128, 2, "f16", "student4", 0.02,
                      0.0, 0, 1.0, "student4", 0.01, 0, 100.0, 3),
    "C4": LayerConfig("C4", 13824, 5120, 262144, 128, 3, "f16", "normal", 0.02,
                      0.02, 0, 8.0, "normal", 0.005, 0, 50.0, 4),
    "C5": LayerConfig("C5", 28672, 8192, 262144, 128, 2, "f16", "normal", 0.015,
                      0.01, 0, 10.0, "normal", 0.005, 0, 80.0, 5),
}


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of `cfg` with some sizes replaced (reduced-size parity cases)."""
    return dataclasses.replace(cfg, **kw)


def _channel_runs(rng: np.random.Generator, m: int, count: int) -> np.ndarray:
    """`count` (rounded down to a multiple of RUN) channel indices in runs of RUN."""
    nruns = count // RUN
    if nruns == 0:
        return np.zeros(0, dtype=np.int64)
    starts = rng.choice(m // RUN, size=nruns, replace=False).astype(np.int64) * RUN
    starts.sort()
    return (starts[:, None] + np.arange(RUN)[None, :]).reshape(-1)


def salient_weight_channels(cfg: LayerConfig) -> np.ndarray:
    _, _, spos = cfg.seeds()
    rng = np.random.Generator(np.random.PCG64([spos, 1]))
    count = cfg.w_salient_count or int(cfg.w_salient_frac * cfg.m)
    return _channel_runs(rng, cfg.m, count)


def outlier_activation_channels(cfg: LayerConfig) -> np.ndarray:
    _, _, spos = cfg.seeds()
    rng = np.random.Generator(np.random.PCG64([spos, 2]))
    count = cfg.x_outlier_count or int(cfg.x_outlier_frac * cfg.m)
    return _channel_runs(rng, cfg.m, count)


def _draw(rng: np.random.Generator, dist: str, shape) -> np.ndarray:
    if dist in ("normal", "lognormal_scale"):
        return rng.standard_normal(shape, dtype=np.float32)
    if dist == "student4":
        # Student-t with 4 degrees of freedom has variance 2; rescale to unit variance.
        return (rng.standard_t(4.0, size=shape) / np.sqrt(2.0)).astype(np.float32)
    raise ValueError(dist)


def make_weights(cfg: LayerConfig) -> np.ndarray:
    """W of shape (n, m) in the config's storage dtype (float32 or float16)."""
    sw, _, _ = cfg.seeds()
    rng = np.random.Generator(np.random.PCG64(sw))
    W = np.empty((cfg.n, cfg.m), dtype=np.float32)
    rows = max(1, (1 << 24) // cfg.m)
    for r0 in range(0, cfg.n, rows):
        r1 = min(cfg.n, r0 + rows)
        W[r0:r1] = _draw(rng, cfg.w_dist, (r1 - r0, cfg.m)) * np.float32(cfg.w_std)
    ch = salient_weight_channels(cfg)
    if ch.size:
        W[:, ch] *= np.float32(cfg.w_salient_gain)
    if cfg.w_dtype == "f16":
        return np.clip(W, -65504.0, 65504.0).astype(np.float16)
    return W


def channel_scales(cfg: LayerConfig) -> np.ndarray:
    """Per-input-channel multiplier applied to X (float32, length m)."""
    _, sx, _ = cfg.seeds()
    rng = np.random.Generator(np.random.PCG64([sx, 0xC0FFEE]))
    if cfg.x_dist == "lognormal_scale":
        s = rng.lognormal(0.0, 1.0, size=cfg.m).astype(np.float32)
    else:
        s = np.ones(cfg.m, dtype=np.float32)
    ch = outlier_activation_channels(cfg)
    if ch.size:
        s[ch] *= np.float32(cfg.x_outlier_gain)
    return s


def mixing_factor(cfg: LayerConfig, rank: int = 32) -> np.ndarray:
    """R (m x rank) of the parity-only correlated variant X <- (I + 0.5 R R^T / sqrt(rank)) X."""
    _, sx, _ = cfg.seeds()
    rng = np.random.Generator(np.random.PCG64([sx, 0xABCD]))
    return rng.standard_normal((cfg.m, rank), dtype=np.float32)


def activation_chunk(cfg: LayerConfig, chunk: int, correlated: bool = False) -> np.ndarray:
    """Tokens [chunk*CHUNK_TOKENS, ...) of X as a float16 array of shape (m, tokens_in_chunk).

    Every chunk has its own generator, so chunks can be produced in any order.
    """
    _, sx, _ = cfg.seeds()
    t0 = chunk * CHUNK_TOKENS
    t1 = min(cfg.t, t0 + CHUNK_TOKENS)
    if t1 <= t0:
        raise IndexError("chunk beyond the end of X")
    rng = np.random.Generator(np.random.PCG64([sx, chunk]))
    x = _draw(rng, cfg.x_dist, (cfg.m, t1 - t0))
    x *= channel_scales(cfg)[:, None]
    if correlated:
        R = mixing_factor(cfg)
        x = x + (0.5 / np.sqrt(R.shape[1])) * (R @ (R.T @ x))
    return np.clip(x, -65504.0, 65504.0).astype(np.float16)


def n_chunks(cfg: LayerConfig) -> int:
    return (cfg.t + CHUNK_TOKENS - 1) // CHUNK_TOKENS


def activation_chunks(cfg: LayerConfig, correlated: bool = False) -> Iterator[np.ndarray]:
    for c in range(n_chunks(cfg)):
        yield activation_chunk(cfg, c, correlated)


def make_activations(cfg: LayerConfig, correlated: bool = False) -> np.ndarray:
    """All of X as one (m, t) float16 array (use the chunk iterator for the big configs)."""
    return np.concatenate(list(activation_chunks(cfg, correlated)), axis=1)
