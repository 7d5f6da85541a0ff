"""Seeded synthetic inputs for the Hogbatch GPU batch-step workloads.

This module only *draws data*: feature matrices, labels, CSR batches and initial
weights, shaped like the paper's datasets (Table 2 of the paper: covtype 581,012x54,
w8a 64,700x300, real-sim 72,309x20,958) and like the five benchmark configurations.
It holds none of the method's arithmetic (no forward pass, no loss, no gradient, no
update) and is the only code shared by the CPU oracle's tests and the HIP path's tests.

Everything is numpy `default_rng` (PCG64) on the host, so both sides see identical bytes.
Seed streams: base + 1000*config + {0: data, 1: labels/teacher, 2: init}.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20200408

ACT_SIGMOID = 0
ACT_RELU = 1
LOSS_SOFTMAX_CE = 0
LOSS_LOGISTIC = 1
DTYPE_F32 = 0
DTYPE_BF16_F32MASTER = 1


@dataclass(frozen=True)
class Config:
    """One benchmark configuration (network + workload recipe)."""
    index: int
    name: str
    dims: tuple
    activation: int
    loss: int
    dtype: int
    n_examples: int
    batch: int
    lr: float
    sparse: bool = False
    extra: dict = field(default_factory=dict)


CONFIGS = {
    1: Config(1, "tiny-54-32-7", (54, 32, 7), ACT_SIGMOID, LOSS_SOFTMAX_CE, DTYPE_F32,
              4096, 64, 0.1),
    2: Config(2, "covtype-54-512x4-7", (54, 512, 512, 512, 512, 7), ACT_SIGMOID,
              LOSS_SOFTMAX_CE, DTYPE_F32, 581_012, 4096, 0.1 * 4096 / 256),
    3: Config(3, "w8a-300-1024x3-2", (300, 1024, 1024, 1024, 2), ACT_RELU, LOSS_LOGISTIC,
              DTYPE_F32, 350_000, 4096, 0.05),
    4: Config(4, "realsim-20958-512x3-2-csr", (20958, 512, 512, 512, 2), ACT_RELU,
              LOSS_LOGISTIC, DTYPE_F32, 72_000, 8192, 0.05, sparse=True),
    5: Config(5, "wide-2048-4096x3-1000-bf16", (2048, 4096, 4096, 4096, 1000), ACT_RELU,
              LOSS_SOFTMAX_CE, DTYPE_BF16_F32MASTER, 1_000_000, 16384, 0.05),
    # The networks of the paper's own experiments (Section 7.1, Table 2), on synthetic data of
    # their shapes: covtype with 6 hidden layers of 512 sigmoid units and 2 labels at the GPU
    # batch size the paper names (8192, Section 7.2), and the delicious-shaped net with 8 hidden
    # layers and a 983-way output.
    6: Config(6, "paper-covtype-54-512x6-2", (54,) + (512,) * 6 + (2,), ACT_SIGMOID,
              LOSS_SOFTMAX_CE, DTYPE_F32, 581_012, 8192, 0.1 * 8192 / 256),
    7: Config(7, "paper-delicious-500-512x8-983", (500,) + (512,) * 8 + (983,), ACT_SIGMOID,
              LOSS_SOFTMAX_CE, DTYPE_F32, 16_105, 2048, 0.1 * 2048 / 256),
}


def seed_for(config: int, stream: int) -> int:
    return BASE_SEED + 1000 * int(config) + int(stream)


def rng_for(config: int, stream: int) -> np.random.Generator:
    return np.random.default_rng(seed_for(config, stream))


# --------------------------------------------------------------------------- weights
def num_params(dims) -> int:
    return int(sum(dims[l] * dims[l - 1] + dims[l] for l in range(1, len(dims))))


def param_offsets(dims):
    """[(w_off, b_off)] per layer in the flat layout [W_1, b_1, W_2, b_2, ...]."""
    out, off = [], 0
    for l in range(1, len(dims)):
        w_off = off
        off += dims[l] * dims[l - 1]
        b_off = off
        off += dims[l]
        out.append((w_off, b_off))
    return out


def xavier_uniform_params(dims, rng: np.random.Generator, bias_scale: float = 0.0) -> np.ndarray:
    """Flat fp32 parameter vector: W_l ~ U(-a, a), a = sqrt(6/(d_{l-1}+d_l)).

    Biases are 0 by default; `bias_scale` > 0 draws them from U(-bias_scale, bias_scale)
    so that tests exercise the bias path with non-trivial values.
    """
    flat = np.zeros(num_params(dims), dtype=np.float32)
    for l, (w_off, b_off) in enumerate(param_offsets(dims), start=1):
        fan_in, fan_out = dims[l - 1], dims[l]
        a = np.sqrt(6.0 / (fan_in + fan_out))
        flat[w_off:w_off + fan_in * fan_out] = rng.uniform(-a, a, fan_in * fan_out).astype(np.float32)
        if bias_scale > 0.0:
            flat[b_off:b_off + fan_out] = rng.uniform(-bias_scale, bias_scale, fan_out).astype(np.float32)
    return flat


# --------------------------------------------------------------------------- dense data
def gaussian_features(n: int, d: int, rng: np.random.Generator) -> np.ndarray:
    return rng.standard_normal((n, d), dtype=np.float32)


def uniform_labels(n: int, k: int, rng: np.random.Generator) -> np.ndarray:
    return rng.integers(0, k, size=n, dtype=np.int32)


def covtype_like_features(n: int, rng: np.random.Generator) -> np.ndarray:
    """54 columns: 10 continuous U[0,1] + 44 binary indicators with p = 0.1."""
    x = np.empty((n, 54), dtype=np.float32)
    x[:, :10] = rng.random((n, 10), dtype=np.float32)
    x[:, 10:] = (rng.random((n, 44), dtype=np.float32) < 0.1).astype(np.float32)
    return x


def teacher_labels(x: np.ndarray, k: int, rng: np.random.Generator, hidden: int = 64) -> np.ndarray:
    """Labels = argmax of a fixed random tanh teacher net d-hidden-k (a data recipe,
    not the trained model)."""
    d = x.shape[1]
    w1 = rng.standard_normal((d, hidden))
    w2 = rng.standard_normal((hidden, k))
    out = np.empty(x.shape[0], dtype=np.int32)
    for s in range(0, x.shape[0], 65536):
        h = np.tanh(x[s:s + 65536].astype(np.float64) @ w1)
        out[s:s + 65536] = np.argmax(h @ w2, axis=1).astype(np.int32)
    return out


def normalised_gaussian_features(n: int, d: int, rng: np.random.Generator) -> np.ndarray:
    x = rng.standard_normal((n, d), dtype=np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True).astype(np.float32)
    return x


def noisy_linear_pm1_labels(x: np.ndarray, rng: np.random.Generator, flip: float = 0.1) -> np.ndarray:
    w = rng.standard_normal(x.shape[1])
    y = np.where(x.astype(np.float64) @ w >= 0.0, 1, -1).astype(np.int32)
    flips = rng.random(x.shape[0]) < flip
    y[flips] = -y[flips]
    return y


# --------------------------------------------------------------------------- CSR data
def zipf_csr(n_rows: int, n_cols: int, rng: np.random.Generator, mean_nnz: float = 50.0,
             max_nnz: int = 256):
    """real-sim-shaped CSR rows.

    nnz per row ~ Poisson(mean_nnz) clipped to [1, max_nnz]; column = pi(r) with rank r
    drawn from a truncated Zipf p(r) ~ 1/r on [1, n_cols] and pi a fixed random
    permutation (hot columns are scattered); duplicates within a row are merged; columns
    ascending per row; values LogNormal(0, 0.5), each row L2-normalised.
    Returns (row_ptr int32[n_rows+1], col_idx int32[nnz], vals float32[nnz]).
    """
    perm = rng.permutation(n_cols).astype(np.int64)
    ranks = np.arange(1, n_cols + 1, dtype=np.float64)
    cdf = np.cumsum(1.0 / ranks)
    cdf /= cdf[-1]
    draws = np.clip(rng.poisson(mean_nnz, size=n_rows), 1, max_nnz).astype(np.int64)
    row_ptr = np.zeros(n_rows + 1, dtype=np.int64)
    cols_out, vals_out = [], []
    for i in range(n_rows):
        u = rng.random(int(draws[i]))
        r = np.searchsorted(cdf, u, side="left")
        r = np.minimum(r, n_cols - 1)
        c = np.unique(perm[r])
        v = rng.lognormal(0.0, 0.5, size=c.size)
        v /= np.sqrt(np.sum(v * v))
        cols_out.append(c.astype(np.int32))
        vals_out.append(v.astype(np.float32))
        row_ptr[i + 1] = row_ptr[i] + c.size
    assert row_ptr[-1] < 2**31
    return (row_ptr.astype(np.int32), np.concatenate(cols_out), np.concatenate(vals_out))


def scramble_csr_rows(row_ptr, col_idx, vals, rng: np.random.Generator, dup_prob: float = 0.2):
    """The same batch with the entries of every row in random order and, with probability
    dup_prob per entry, an entry split into two entries of the same column whose fp32 values
    add up to (about) the original: a CSR batch as a caller may hand it over that has neither
    sorted nor merged its rows.  Returns (row_ptr, col_idx, vals) of the new batch."""
    cols_out, vals_out = [], []
    new_ptr = np.zeros(row_ptr.size, dtype=np.int64)
    for i in range(row_ptr.size - 1):
        s, e = int(row_ptr[i]), int(row_ptr[i + 1])
        c, v = col_idx[s:e].astype(np.int32), vals[s:e].astype(np.float32)
        split = rng.random(c.size) < dup_prob
        part = v[split] * rng.uniform(0.2, 0.8, int(split.sum())).astype(np.float32)
        rest = v.copy()
        rest[split] -= part
        c = np.concatenate([c, c[split]])
        v = np.concatenate([rest, part])
        order = rng.permutation(c.size)
        cols_out.append(c[order])
        vals_out.append(v[order])
        new_ptr[i + 1] = new_ptr[i] + c.size
    if not cols_out:
        return row_ptr.copy(), col_idx.copy(), vals.copy()
    return new_ptr.astype(np.int32), np.concatenate(cols_out).astype(np.int32), np.concatenate(vals_out).astype(np.float32)


def csr_pm1_labels(row_ptr, col_idx, vals, n_cols: int, rng: np.random.Generator) -> np.ndarray:
    w = rng.standard_normal(n_cols)
    contrib = vals.astype(np.float64) * w[col_idx]
    s = np.add.reduceat(contrib, row_ptr[:-1].astype(np.int64))
    return np.where(s >= 0.0, 1, -1).astype(np.int32)


def csr_to_dense(row_ptr, col_idx, vals, n_cols: int) -> np.ndarray:
    n = row_ptr.size - 1
    x = np.zeros((n, n_cols), dtype=np.float32)
    for i in range(n):
        s, e = int(row_ptr[i]), int(row_ptr[i + 1])
        x[i, col_idx[s:e]] = vals[s:e]
    return x


def csr_slice(row_ptr, col_idx, vals, start: int, stop: int):
    """Rows [start, stop) as a CSR batch with row_ptr rebased to 0."""
    s, e = int(row_ptr[start]), int(row_ptr[stop])
    return ((row_ptr[start:stop + 1] - row_ptr[start]).astype(np.int32),
            np.ascontiguousarray(col_idx[s:e]), np.ascontiguousarray(vals[s:e]))


# --------------------------------------------------------------------------- per-config
def make_dense_dataset(config: int, n: int | None = None):
    """(X float32 [n x d0], y int32 [n]) for dense configs 1, 2, 3, 5, 6, 7 (n rows; the
    config's full size when n is None)."""
    cfg = CONFIGS[config]
    n = cfg.n_examples if n is None else int(n)
    d0, k = cfg.dims[0], cfg.dims[-1]
    data_rng, label_rng = rng_for(config, 0), rng_for(config, 1)
    if config in (1, 5, 7):
        return gaussian_features(n, d0, data_rng), uniform_labels(n, k, label_rng)
    if config in (2, 6):
        x = covtype_like_features(n, data_rng)
        return x, teacher_labels(x, k, label_rng)
    if config == 3:
        x = normalised_gaussian_features(n, d0, data_rng)
        return x, noisy_linear_pm1_labels(x, label_rng)
    raise ValueError(f"config {config} is not a dense config")


def make_csr_dataset(config: int = 4, n: int | None = None):
    """(row_ptr, col_idx, vals, y) for the sparse-input config."""
    cfg = CONFIGS[config]
    if not cfg.sparse:
        raise ValueError(f"config {config} is not sparse")
    n = cfg.n_examples if n is None else int(n)
    row_ptr, col_idx, vals = zipf_csr(n, cfg.dims[0], rng_for(config, 0))
    y = csr_pm1_labels(row_ptr, col_idx, vals, cfg.dims[0], rng_for(config, 1))
    return row_ptr, col_idx, vals, y


def make_params(config: int, bias_scale: float = 0.0) -> np.ndarray:
    return xavier_uniform_params(CONFIGS[config].dims, rng_for(config, 2), bias_scale)


def adaptive_batch_ladder(min_b: int, max_b: int, alpha: float = 2.0):
    """Batch sizes Adaptive Hogbatch can hand the GPU worker: max_b / alpha^k clipped to
    [min_b, max_b] (Algorithm 2 of the paper; alpha defaults to 2)."""
    out, b = [], float(max_b)
    while True:
        bi = max(int(round(b)), int(min_b))
        if not out or out[-1] != bi:
            out.append(bi)
        if bi <= min_b:
            break
        b /= alpha
    return out
