"""Seeded synthetic layers shaped like Llama-family projections.

This module only draws random numbers; it holds none of the quantization
method's arithmetic.  Both the float64 CPU oracle (through the tests) and the
HIP path (tests, smoke, bench) are fed from here, so that the two sides see the
very same fp32 bytes.

Every array is a deterministic function of (config seed, stream id, chunk
index): weights come in chunks of ROW_CHUNK rows and activations in chunks of
TOKEN_CHUNK tokens, each chunk from its own child seed, so that any subset of
rows or tokens can be produced without producing the rest.

The layers stand in for the C4-calibrated Llama/Mistral layers the paper
quantizes (Section 4, "Baselines"): Gaussian bulk weights with a small
fraction of heavy-tailed entries, and activations with a few high-magnitude
input channels, which give the inverse-Hessian diagonal the few-outliers
shape the paper shows in Figure 1 (left).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Iterator, Optional, Sequence

import numpy as np

ROW_CHUNK = 256
TOKEN_CHUNK = 8192

_STREAM_W_BULK = 11
_STREAM_W_OUT = 12
_STREAM_CHAN = 21
_STREAM_X = 31


@dataclass(frozen=True)
class LayerConfig:
    name: str
    seed: int
    r: int                 # d_row, output channels (rows of W)
    c: int                 # d_col, input channels (columns of W)
    n_tokens: int
    mode: str              # "nu" (non-uniform) or "aff" (affine)
    bits: int
    group_size: int        # 0 = whole row
    block: int = 128
    damp: float = 0.01
    p: float = 4.0
    T: int = 2048
    w_sigma: float = 0.02
    w_outlier_frac: float = 0.0
    w_outlier_kind: str = "none"   # "normal" | "student_t3" | "none"
    w_outlier_scale: float = 0.0
    x_kind: str = "normal"         # "normal" | "silu_product"
    x_outlier_channels: int = 0
    x_outlier_scale: float = 1.0

    def scaled(self, **kw) -> "LayerConfig":
        """Same recipe at other sizes (fewer rows / tokens), same seed."""
        return replace(self, **kw)


CONFIGS = {
    "c1": LayerConfig("c1", 1001, 512, 512, 2048, "nu", 4, 0,
                      w_outlier_frac=0.01, w_outlier_kind="normal", w_outlier_scale=0.2,
                      x_outlier_channels=8, x_outlier_scale=20.0),
    "c2": LayerConfig("c2", 1002, 4096, 4096, 262144, "nu", 4, 0,
                      w_outlier_frac=0.005, w_outlier_kind="student_t3", w_outlier_scale=0.1,
                      x_outlier_channels=32, x_outlier_scale=50.0),
    "c3": LayerConfig("c3", 1003, 4096, 11008, 262144, "nu", 3, 0,
                      x_kind="silu_product"),
    "c4": LayerConfig("c4", 1004, 28672, 8192, 131072, "aff", 4, 128,
                      w_outlier_frac=0.005, w_outlier_kind="student_t3", w_outlier_scale=0.1,
                      x_outlier_channels=64, x_outlier_scale=30.0),
    "c5": LayerConfig("c5", 1005, 53248, 16384, 65536, "aff", 2, 64,
                      w_outlier_frac=0.005, w_outlier_kind="student_t3", w_outlier_scale=0.1,
                      x_outlier_channels=128, x_outlier_scale=40.0),
}
# The second run the fifth configuration asks for: 3-bit non-uniform, same layer.
CONFIGS["c5nu"] = CONFIGS["c5"].scaled(name="c5nu", mode="nu", bits=3, group_size=0)


def _rng(cfg: LayerConfig, stream: int, index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg.seed, stream, index])))


def weight_rows(cfg: LayerConfig, chunk: int) -> np.ndarray:
    """Rows [chunk*ROW_CHUNK, min(r, (chunk+1)*ROW_CHUNK)) of W, fp32, C-contiguous."""
    r0 = chunk * ROW_CHUNK
    n = min(cfg.r, r0 + ROW_CHUNK) - r0
    if n <= 0:
        raise IndexError("row chunk out of range")
    w = _rng(cfg, _STREAM_W_BULK, chunk).standard_normal((n, cfg.c), dtype=np.float32)
    w *= np.float32(cfg.w_sigma)
    if cfg.w_outlier_kind != "none" and cfg.w_outlier_frac > 0.0:
        g = _rng(cfg, _STREAM_W_OUT, chunk)
        mask = g.random((n, cfg.c), dtype=np.float32) < np.float32(cfg.w_outlier_frac)
        k = int(mask.sum())
        if cfg.w_outlier_kind == "normal":
            vals = g.standard_normal(k)
        elif cfg.w_outlier_kind == "student_t3":
            vals = g.standard_t(3.0, k)
        else:
            raise ValueError(cfg.w_outlier_kind)
        w[mask] = (vals * cfg.w_outlier_scale).astype(np.float32)
    return w


def weights(cfg: LayerConfig, rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """W [r x c] fp32, or only the listed rows (in the order given)."""
    n_chunks = (cfg.r + ROW_CHUNK - 1) // ROW_CHUNK
    if rows is None:
        return np.concatenate([weight_rows(cfg, k) for k in range(n_chunks)], axis=0)
    rows = np.asarray(rows, dtype=np.int64)
    out = np.empty((rows.size, cfg.c), dtype=np.float32)
    for k in np.unique(rows // ROW_CHUNK):
        blk = weight_rows(cfg, int(k))
        sel = np.nonzero(rows // ROW_CHUNK == k)[0]
        out[sel] = blk[rows[sel] - k * ROW_CHUNK]
    return out


def outlier_channels(cfg: LayerConfig) -> np.ndarray:
    if cfg.x_outlier_channels <= 0:
        return np.zeros(0, dtype=np.int64)
    ch = _rng(cfg, _STREAM_CHAN).choice(cfg.c, size=cfg.x_outlier_channels, replace=False)
    return np.sort(ch).astype(np.int64)


def n_token_chunks(cfg: LayerConfig) -> int:
    return (cfg.n_tokens + TOKEN_CHUNK - 1) // TOKEN_CHUNK


def activation_chunk(cfg: LayerConfig, chunk: int, out: Optional[np.ndarray] = None) -> np.ndarray:
    """Tokens [chunk*TOKEN_CHUNK, ...) of X as an [n x c] fp32 array (tokens are rows)."""
    t0 = chunk * TOKEN_CHUNK
    n = min(cfg.n_tokens, t0 + TOKEN_CHUNK) - t0
    if n <= 0:
        raise IndexError("token chunk out of range")
    g = _rng(cfg, _STREAM_X, chunk)
    if out is None:
        out = np.empty((n, cfg.c), dtype=np.float32)
    x = out[:n]
    g.standard_normal(out=x, dtype=np.float32)
    if cfg.x_kind == "silu_product":
        # gate-times-up shape of an MLP down-projection input: silu(a) * b
        b = g.standard_normal((n, cfg.c), dtype=np.float32)
        sig = 1.0 / (1.0 + np.exp(-x))
        x *= sig
        x *= b
    elif cfg.x_kind != "normal":
        raise ValueError(cfg.x_kind)
    ch = outlier_channels(cfg)
    if ch.size:
        x[:, ch] *= np.float32(cfg.x_outlier_scale)
    return x


def activation_chunks(cfg: LayerConfig) -> Iterator[np.ndarray]:
    for k in range(n_token_chunks(cfg)):
        yield activation_chunk(cfg, k)


def activations(cfg: LayerConfig) -> np.ndarray:
    """All of X [n_tokens x c]; only for configurations that fit host memory."""
    return np.concatenate(list(activation_chunks(cfg)), axis=0)


def sample_rows(cfg: LayerConfig, count: int, salt: int = 0) -> np.ndarray:
    """A seeded, sorted subset of row indices (for row-sampled comparisons)."""
    count = min(count, cfg.r)
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg.seed, 91, salt])))
    return np.sort(g.choice(cfg.r, size=count, replace=False)).astype(np.int64)
