"""Seeded synthetic inputs for the GQSA group-sparse GEMV path.

This module only draws random numbers and shapes them: dense fp32 weight
matrices, fp16 activation vectors and per-row kept-group counts.  It contains
none of the method's arithmetic (no saliency, no quantiser, no packing, no
product), so both the CPU oracle's tests and the HIP library's tests may feed
from it without sharing any computation.

The shapes are the public linear-layer dimensions of the LLaMA-7B and
LLaMA-3-8B decoder layers, which is what the paper's end-to-end tables
(Tab. 4, Tab. 13, Tab. 16) and its kernel benchmark (Sec. 4.4, the
(1,4096)x(4096,4096) GEMV) run on; the trained weights themselves are replaced
by Gaussian matrices with a few amplified columns standing in for the outlier
channels the paper discusses (App. "advantages of group quantization").
"""
from __future__ import annotations

import numpy as np

G_DEFAULT = 16

# name -> (N, K): output rows x reduction length of y = W x
LLAMA7B_LAYER = (
    ("q_proj", 4096, 4096),
    ("k_proj", 4096, 4096),
    ("v_proj", 4096, 4096),
    ("o_proj", 4096, 4096),
    ("gate_proj", 11008, 4096),
    ("up_proj", 11008, 4096),
    ("down_proj", 4096, 11008),
)

LLAMA3_8B_SHAPES = (
    ("qo_proj", 4096, 4096),
    ("kv_proj", 1024, 4096),
    ("gate_up_proj", 14336, 4096),
    ("down_proj", 4096, 14336),
)

IMBALANCED_SHAPES = (("imb_8k", 8192, 8192), ("imb_28k", 28672, 8192))

SMALL_BATCH_SHAPES = (("sb_4k", 4096, 4096), ("sb_14k", 14336, 4096))

SPARSITY_SWEEP = (0.0, 0.3, 0.5, 0.7)
BATCH_SWEEP = (1, 2, 4, 8, 16)


def config_seed(config: int, shape_index: int) -> int:
    """Seed convention: config c, shape index i -> 1000*c + 10*i (config 1 uses 0)."""
    if config == 1:
        return 0
    return 1000 * config + 10 * shape_index


def dense_weight(n: int, k: int, seed: int, outliers: bool = True,
                 sigma: float = 0.02, outlier_frac: float = 0.01,
                 outlier_gain: float = 20.0) -> np.ndarray:
    """Row-major fp32 [n, k] ~ N(0, sigma); optionally 1% of the columns scaled x20.

    The outlier columns are drawn after W from the same generator, so the pair
    (W, columns) is a function of the seed alone.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    w = rng.standard_normal((n, k), dtype=np.float32)
    w *= np.float32(sigma)
    if outliers:
        ncol = int(round(outlier_frac * k))
        if ncol > 0:
            cols = rng.choice(k, size=ncol, replace=False)
            w[:, cols] *= np.float32(outlier_gain)
    return w


def activations(batch: int, k: int, seed: int) -> np.ndarray:
    """fp16 [batch, k] ~ N(0, 1), drawn in fp32 and rounded once to fp16."""
    rng = np.random.Generator(np.random.PCG64(seed + 1))
    return rng.standard_normal((batch, k), dtype=np.float32).astype(np.float16)


def tiny_config():
    """Config 1: 256x256, no outliers, seed 0, batch 1."""
    w = dense_weight(256, 256, seed=0, outliers=False)
    x = activations(1, 256, seed=0)
    return w, x


def imbalanced_keep_counts(n: int, groups_per_row: int, seed: int,
                           frac_empty: float = 0.02,
                           frac_full: float = 0.02) -> np.ndarray:
    """Per-row kept-group counts for the imbalanced stress config.

    Kept fraction f ~ Beta(0.5, 0.5) per row, keep = rint(f * groups_per_row);
    then a random 2% of the rows are forced empty and a disjoint 2% forced full.
    """
    rng = np.random.Generator(np.random.PCG64(seed + 2))
    f = rng.beta(0.5, 0.5, size=n)
    keep = np.rint(f * groups_per_row).astype(np.int32)
    perm = rng.permutation(n)
    n_empty = int(round(frac_empty * n))
    n_full = int(round(frac_full * n))
    keep[perm[:n_empty]] = 0
    keep[perm[n_empty:n_empty + n_full]] = groups_per_row
    return keep


def unit_vector(k: int, index: int, batch: int = 1) -> np.ndarray:
    """fp16 [batch, k] with a single 1 at `index` in every batch row."""
    x = np.zeros((batch, k), dtype=np.float16)
    x[:, index] = np.float16(1.0)
    return x


def ones_vector(k: int, batch: int = 1) -> np.ndarray:
    return np.ones((batch, k), dtype=np.float16)


def dense_weight_chunked(n: int, k: int, seed: int, outliers: bool = True,
                         sigma: float = 0.02, outlier_frac: float = 0.01,
                         outlier_gain: float = 20.0, workers: int = 8) -> np.ndarray:
    """Same distribution as dense_weight, drawn in 16 independent row chunks so that several
    host threads can fill a large pool quickly.  The result depends on the seed only (the
    chunking is fixed), not on the number of workers.  Used for benchmark pools."""
    from concurrent.futures import ThreadPoolExecutor

    n_chunks = 16
    w = np.empty((n, k), dtype=np.float32)
    bounds = np.linspace(0, n, n_chunks + 1).astype(np.int64)

    def fill(j):
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, j])))
        part = w[bounds[j]:bounds[j + 1]]
        rng.standard_normal(part.shape, dtype=np.float32, out=part)
        part *= np.float32(sigma)

    with ThreadPoolExecutor(max_workers=max(1, workers)) as ex:
        list(ex.map(fill, range(n_chunks)))
    if outliers:
        ncol = int(round(outlier_frac * k))
        if ncol > 0:
            rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 9999])))
            cols = rng.choice(k, size=ncol, replace=False)
            w[:, cols] *= np.float32(outlier_gain)
    return w
