"""Seeded synthetic inputs for Independent Subnet Training (IST).

This module only *draws data*: network shapes, initial weights, neuron
permutations, mini-batches and labels.  It contains none of the method's
arithmetic (no partition, no forward/backward, no update) so that both the CPU
oracle and the HIP path can be fed from it without sharing any logic.

The workloads stand in for the datasets the paper trains on (Section 3.1:
Google Speech Commands features, CIFAR10/ImageNet images, Amazon-670k sparse
features), none of which is available here; only their shapes and coarse value
distributions are reproduced.

All floating-point arrays are returned as float32 whose values are exactly
representable in the storage dtype of the configuration ("f32" or "bf16").
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import numpy as np

SEED_BASE = 19100212000


@dataclass(frozen=True)
class ISTConfig:
    """One workload: a fully connected net N_0 -> ... -> N_t split into S subnets."""
    name: str
    idx: int                      # 1-based index into the benchmark list
    dims: Tuple[int, ...]         # N_0 .. N_t
    S: int                        # number of subnets ("sites" n in the paper)
    B: int                        # mini-batch size
    k: int                        # local SGD steps per round (J in the paper)
    rounds: int
    dtype: str                    # "f32" | "bf16" storage
    input: str = "dense"          # "dense" | "csr"
    x_dist: str = "normal"        # "normal" | "uniform"
    lr: float = 0.01
    nnz_per_row: int = 75         # CSR only
    label_dist: str = "teacher"   # "teacher" | "zipf"
    init_gain: float = 1.0        # multiplies the Xavier bound of the initial weights

    @property
    def t(self) -> int:
        return len(self.dims) - 1

    def width(self, l: int) -> int:
        """Neurons of layer l held by one subnet (input/output layers are shared)."""
        if l == 0 or l == self.t:
            return self.dims[l]
        return self.dims[l] // self.S


CONFIGS = {
    "cfg1": ISTConfig("cfg1-tiny", 1, (64, 128, 128, 10), S=2, B=32, k=10, rounds=1,
                      dtype="f32", lr=0.05),
    "cfg2": ISTConfig("cfg2-speech-like", 2, (1024, 4096, 4096, 35), S=4, B=128, k=10,
                      rounds=20, dtype="f32"),
    "cfg3": ISTConfig("cfg3-image-like", 3, (3072, 8192, 8192, 10), S=8, B=128, k=20,
                      rounds=10, dtype="bf16", x_dist="uniform"),
    "cfg4": ISTConfig("cfg4-wide-stress", 4, (4096, 65536, 65536, 65536, 100), S=8, B=512,
                      k=10, rounds=1, dtype="bf16"),
    "cfg5": ISTConfig("cfg5-extreme-classification", 5, (135909, 1024, 670091), S=8, B=256,
                      k=5, rounds=1, dtype="bf16", input="csr", label_dist="zipf"),
    # beyond the five benchmark configurations: the paper's larger speech model (Section 3.1: three
    # hidden layers of 8192 neurons, 4096-dimensional features, 35 keywords); S, B, k are ours
    "speech8192": ISTConfig("speech-3x8192", 6, (4096, 8192, 8192, 8192, 35), S=8, B=128, k=10,
                            rounds=4, dtype="f32"),
}


def scaled(cfg: ISTConfig, **kw) -> ISTConfig:
    """A copy of a configuration with some fields replaced (reduced test shapes)."""
    return replace(cfg, **kw)


# --------------------------------------------------------------------------
# storage-dtype helpers (I/O plumbing, not method arithmetic)
# --------------------------------------------------------------------------
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rnd) >> 16).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def quantize(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float values to the storage dtype, returned as float32."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        return from_bf16_bits(to_bf16_bits(x)).reshape(x.shape)
    return x


def _rng(cfg: ISTConfig, rnd: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([SEED_BASE + 100 * cfg.idx + rnd, stream]))


# --------------------------------------------------------------------------
# the pieces
# --------------------------------------------------------------------------
def make_weights(cfg: ISTConfig, with_bias: bool = True, bias_scale: float = 0.0):
    """Xavier-uniform W_l [N_l][N_{l-1}], l = 1..t; biases zero (or small random
    values when bias_scale > 0, used by tests that must see biases move)."""
    g = _rng(cfg, 0, 1)
    Ws, bs = [], []
    for l in range(1, cfg.t + 1):
        fan_out, fan_in = cfg.dims[l], cfg.dims[l - 1]
        a = cfg.init_gain * np.sqrt(6.0 / (fan_in + fan_out))
        W = g.uniform(-a, a, size=(fan_out, fan_in)).astype(np.float32)
        Ws.append(quantize(W, cfg.dtype))
        if with_bias:
            b = (bias_scale * g.standard_normal(fan_out)).astype(np.float32)
            bs.append(quantize(b, cfg.dtype))
        else:
            bs.append(None)
    return Ws, bs


def make_perms(cfg: ISTConfig, rnd: int = 0) -> List[np.ndarray]:
    """One independent uniform random permutation of 0..N_l-1 per hidden layer."""
    g = _rng(cfg, rnd, 2)
    return [g.permutation(cfg.dims[l]).astype(np.int32) for l in range(1, cfg.t)]


def _teacher_labels(cfg: ISTConfig, X2d: np.ndarray) -> np.ndarray:
    g = _rng(cfg, 0, 3)
    hid = 128 if cfg.dims[0] <= 256 else 256
    T1 = g.standard_normal((cfg.dims[0], hid)).astype(np.float32) / np.sqrt(cfg.dims[0])
    T2 = g.standard_normal((hid, cfg.dims[-1])).astype(np.float32) / np.sqrt(hid)
    Xc = X2d - X2d.mean(axis=0, keepdims=True)
    return np.argmax(np.maximum(Xc @ T1, 0.0) @ T2, axis=1).astype(np.int32)


def make_dense_batches(cfg: ISTConfig, rnd: int = 0):
    """X [S][k][B][N_0] float32 (representable in cfg.dtype), y [S][k][B] int32."""
    g = _rng(cfg, rnd, 4)
    shape = (cfg.S, cfg.k, cfg.B, cfg.dims[0])
    if cfg.x_dist == "uniform":
        X = g.random(shape, dtype=np.float32)
    else:
        X = g.standard_normal(shape, dtype=np.float32)
    X = quantize(X, cfg.dtype)
    if cfg.label_dist == "zipf":
        y = _zipf_labels(cfg, g, cfg.S * cfg.k * cfg.B)
    else:
        y = _teacher_labels(cfg, X.reshape(-1, cfg.dims[0]))
    return X, y.reshape(cfg.S, cfg.k, cfg.B)


def _zipf_probs(n: int, alpha: float) -> np.ndarray:
    p = 1.0 / np.power(np.arange(1, n + 1, dtype=np.float64), alpha)
    return p / p.sum()


def _zipf_labels(cfg: ISTConfig, g: np.random.Generator, n: int) -> np.ndarray:
    C = cfg.dims[-1]
    ids = g.permutation(C)
    cdf = np.cumsum(_zipf_probs(C, 1.1))
    r = np.searchsorted(cdf, g.random(n), side="left").clip(0, C - 1)
    return ids[r].astype(np.int32)


def make_csr_batches(cfg: ISTConfig, rnd: int = 0):
    """Sparse batches: rowptr [S*k*B+1], colidx, vals (float32, representable in
    cfg.dtype), y [S][k][B].  Row r of the CSR is sample (s, j, b) with
    r = (s*k + j)*B + b.  Per row: nnz ~ Poisson(nnz_per_row) clamped to
    [1, N_0]; distinct column ids drawn from a Zipf(1.0) popularity over a
    shuffled id space, ascending; values lognormal(0,1), row L2-normalised."""
    g = _rng(cfg, rnd, 5)
    N0 = cfg.dims[0]
    rows = cfg.S * cfg.k * cfg.B
    ids = g.permutation(N0)
    cdf = np.cumsum(_zipf_probs(N0, 1.0))
    counts = np.clip(g.poisson(cfg.nnz_per_row, rows), 1, N0).astype(np.int64)
    rowptr = np.zeros(rows + 1, dtype=np.int64)
    cols_l, vals_l = [], []
    for r in range(rows):
        want = int(counts[r])
        got = np.empty(0, dtype=np.int64)
        while got.size < want:
            draw = np.searchsorted(cdf, g.random(2 * want), side="left").clip(0, N0 - 1)
            got = np.unique(np.concatenate([got, ids[draw]]))
            if got.size > want:
                got = np.sort(g.choice(got, want, replace=False))
        v = np.exp(g.standard_normal(want))
        v = v / np.sqrt(np.sum(v * v))
        cols_l.append(got)
        vals_l.append(v)
        rowptr[r + 1] = rowptr[r] + want
    colidx = np.concatenate(cols_l).astype(np.int32)
    vals = quantize(np.concatenate(vals_l).astype(np.float32), cfg.dtype)
    if cfg.label_dist == "zipf":
        y = _zipf_labels(cfg, g, rows)
    else:
        y = g.integers(0, cfg.dims[-1], rows).astype(np.int32)
    return rowptr.astype(np.int32), colidx, vals, y.reshape(cfg.S, cfg.k, cfg.B)


def csr_to_dense(rowptr, colidx, vals, n_cols: int) -> np.ndarray:
    """Expand a CSR matrix to dense float32 (test helper, small shapes only)."""
    rows = len(rowptr) - 1
    out = np.zeros((rows, n_cols), dtype=np.float32)
    for r in range(rows):
        sl = slice(rowptr[r], rowptr[r + 1])
        out[r, colidx[sl]] = vals[sl]
    return out
