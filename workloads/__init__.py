"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *prepares inputs*: a pruned, weight-shared layer matrix W
(fp32, exact zeros where pruned, a small set of shared values elsewhere) and a
dense batch X.  It contains none of the HAC / sHAC arithmetic (no Huffman
code, no bitstream, no dot product); both the CPU oracle's tests and the HIP
path consume the arrays it returns, so choices made here cannot affect parity.

The paper's timing experiment (Sect. V, "State-of-the-art comparison of HAC and
sHAC") uses trained VGG19 fully-connected matrices, pruned at p in 60..99 %
and quantized by clustering-based weight sharing with k = 32 / 256; those
weights are not available, so Gaussian matrices with the same pruning level
and number of shared values stand in for them.

Recipe (all of it deterministic given the seed):
  * W0 ~ N(0, sigma) fp32, `numpy.random.default_rng(1000*cfg + 0)`.
  * Magnitude pruning (Sect. III-B): q = round(p*n*m); the threshold is the
    q-th smallest |w|; an entry survives iff |w| is strictly greater.
  * Weight sharing over the survivors, one of
      - "uniform": k equal bins over [min, max] of the survivors, each
        survivor replaced by its bin's midpoint (fp64 -> fp32); empty bins
        simply never occur in W.
      - "kmeans": 1-D k-means (Sect. III-C1, CWS) on the survivors: quantile
        initialisation, Lloyd iterations in fp64 until assignment boundaries
        stop moving or 50 iterations, centroids rounded to fp32, identical
        centroids merged.
    A shared value never equals 0.0, so 0 stays the "pruned" symbol only.
  * X = max(N(0,1), 0) fp32, B x n row-major, `default_rng(1000*cfg + 1)`.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    cfg: int            # 1-based id, used for the seeds
    name: str
    n: int              # rows of W (= input features)
    m: int              # columns of W (= output features)
    sigma: float        # std-dev of the Gaussian W0
    prune: float        # fraction of entries set to zero
    k: int              # number of shared values asked for
    quant: str          # "uniform" | "kmeans"
    batches: Tuple[int, ...]   # batch sizes B the config names


CONFIGS: Dict[int, LayerConfig] = {
    1: LayerConfig(1, "tiny-500x300", 500, 300, 0.05, 0.70, 16, "uniform", (8,)),
    2: LayerConfig(2, "vgg16-fc3-4096x1000", 4096, 1000, 0.02, 0.90, 32, "kmeans", (64,)),
    3: LayerConfig(3, "hidden-fc-4096x4096", 4096, 4096, 0.01, 0.96, 256, "kmeans", (128,)),
    4: LayerConfig(4, "vgg16-fc1-25088x4096", 25088, 4096, 0.005, 0.98, 32, "uniform", (1, 32, 256)),
    5: LayerConfig(5, "conv3x3-512-im2col-4608x512", 4608, 512, 0.02, 0.60, 256, "kmeans", (12544,)),
}


def prune_magnitude(w0: np.ndarray, frac: float) -> np.ndarray:
    """Boolean mask of survivors: |w| strictly above the `frac` empirical
    percentile of |w| (ties at the threshold are pruned)."""
    total = w0.size
    q = int(round(frac * total))
    if q <= 0:
        return np.ones(w0.shape, dtype=bool)
    if q >= total:
        return np.zeros(w0.shape, dtype=bool)
    a = np.abs(w0).ravel()
    thr = np.partition(a, q - 1)[q - 1]
    return np.abs(w0) > thr


def share_uniform(vals: np.ndarray, k: int) -> np.ndarray:
    """Replace each value by the midpoint of its bin, k equal bins on [min,max]."""
    if vals.size == 0:
        return vals.astype(np.float32)
    lo = float(vals.min())
    hi = float(vals.max())
    if hi == lo:
        return np.full(vals.shape, np.float32(lo), dtype=np.float32)
    delta = (hi - lo) / k
    b = np.floor((vals.astype(np.float64) - lo) / delta).astype(np.int64)
    np.clip(b, 0, k - 1, out=b)
    mids = (lo + (np.arange(k, dtype=np.float64) + 0.5) * delta).astype(np.float32)
    return mids[b]


def share_kmeans(vals: np.ndarray, k: int, iters: int = 50) -> np.ndarray:
    """1-D k-means: replace each value by its (fp32) centroid."""
    if vals.size == 0:
        return vals.astype(np.float32)
    v = np.sort(vals.astype(np.float64))
    k = min(k, np.unique(v).size)
    cent = np.quantile(v, (np.arange(k) + 0.5) / k)
    csum = np.concatenate(([0.0], np.cumsum(v)))
    prev = None
    for _ in range(iters):
        bounds = 0.5 * (cent[:-1] + cent[1:])
        cut = np.searchsorted(v, bounds, side="right")     # v <= bound -> lower cluster
        edges = np.concatenate(([0], cut, [v.size]))
        cnt = np.diff(edges)
        tot = csum[edges[1:]] - csum[edges[:-1]]
        new = np.where(cnt > 0, tot / np.maximum(cnt, 1), cent)
        if prev is not None and np.array_equal(cut, prev):
            cent = new
            break
        prev = cut
        cent = new
    cent32 = np.unique(cent.astype(np.float32))
    bounds = 0.5 * (cent32[:-1].astype(np.float64) + cent32[1:].astype(np.float64))
    idx = np.searchsorted(bounds, vals.astype(np.float64), side="left")
    return cent32[idx]


def make_layer(n: int, m: int, sigma: float, prune: float, k: int, quant: str,
               seed: int) -> np.ndarray:
    """Pruned + weight-shared n x m fp32 matrix (C-contiguous, row-major)."""
    rng = np.random.default_rng(seed)
    w0 = (rng.standard_normal((n, m), dtype=np.float32) * np.float32(sigma)).astype(np.float32)
    keep = prune_magnitude(w0, prune)
    w = np.zeros((n, m), dtype=np.float32)
    surv = w0[keep]
    if quant == "uniform":
        shared = share_uniform(surv, k)
    elif quant == "kmeans":
        shared = share_kmeans(surv, k)
    else:
        raise ValueError(f"unknown quantizer {quant!r}")
    if shared.size and np.any(shared == 0.0):
        raise ValueError("a shared value rounded to 0.0; pick another k or seed")
    w[keep] = shared
    return w


def make_network(shapes, sigmas, prunes, k: int, quant: str, seed: int):
    """Layers pruned one by one (magnitude, fraction prunes[l]) and then weight-shared
    together: the survivors of all layers are quantized as one set with k representatives,
    the paper's "unified" quantization (Sect. V-H).  shapes[l] = (n_l, m_l), m_l = n_{l+1}."""
    rng = np.random.default_rng(seed)
    raw, keeps = [], []
    for (n, m), sigma, prune in zip(shapes, sigmas, prunes):
        w0 = (rng.standard_normal((n, m), dtype=np.float32) * np.float32(sigma)).astype(np.float32)
        raw.append(w0)
        keeps.append(prune_magnitude(w0, prune))
    pooled = np.concatenate([w0[keep] for w0, keep in zip(raw, keeps)])
    shared = share_uniform(pooled, k) if quant == "uniform" else share_kmeans(pooled, k)
    if shared.size and np.any(shared == 0.0):
        raise ValueError("a shared value rounded to 0.0; pick another k or seed")
    out, at = [], 0
    for w0, keep in zip(raw, keeps):
        w = np.zeros(w0.shape, dtype=np.float32)
        cnt = int(keep.sum())
        w[keep] = shared[at:at + cnt]
        at += cnt
        out.append(w)
    return out


def make_biases(shapes, seed: int):
    """One fp32 bias vector per layer, N(0, 0.1)."""
    rng = np.random.default_rng(seed)
    return [(rng.standard_normal(m, dtype=np.float32) * np.float32(0.1)).astype(np.float32) for _, m in shapes]


# Fully connected blocks for the chain of layers.  "vgg19-fc" has the shapes of the matrices the
# paper times (Sect. V-G: 512x4096, 4096x4096, 4096x10); "vgg16-fc" starts from the graded layer.
NETWORKS = {
    "tiny-fc": dict(shapes=((500, 300), (300, 120), (120, 10)), sigmas=(0.05, 0.06, 0.1),
                    prunes=(0.7, 0.7, 0.5), k=16, quant="uniform", seed=5001),
    "vgg19-fc": dict(shapes=((512, 4096), (4096, 4096), (4096, 10)), sigmas=(0.03, 0.01, 0.02),
                     prunes=(0.9, 0.96, 0.8), k=32, quant="uniform", seed=5002),
    "vgg16-fc": dict(shapes=((25088, 4096), (4096, 4096), (4096, 1000)), sigmas=(0.005, 0.01, 0.02),
                     prunes=(0.98, 0.96, 0.9), k=32, quant="uniform", seed=5003),
}


def network(name: str):
    """(layers, biases) of a named fully connected block."""
    c = NETWORKS[name]
    return (make_network(c["shapes"], c["sigmas"], c["prunes"], c["k"], c["quant"], c["seed"]),
            make_biases(c["shapes"], c["seed"] + 1))


def make_batch(B: int, n: int, seed: int) -> np.ndarray:
    """ReLU(N(0,1)) fp32 batch, B x n row-major."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, n), dtype=np.float32)
    np.maximum(x, 0.0, out=x)
    return x


def layer(cfg: int) -> np.ndarray:
    c = CONFIGS[cfg]
    return make_layer(c.n, c.m, c.sigma, c.prune, c.k, c.quant, 1000 * c.cfg + 0)


def batch(cfg: int, B: int | None = None) -> np.ndarray:
    c = CONFIGS[cfg]
    if B is None:
        B = c.batches[0]
    return make_batch(B, c.n, 1000 * c.cfg + 1)


def scaled(cfg: int, n: int, m: int, seed_offset: int = 7) -> np.ndarray:
    """Same recipe as config `cfg` but at another shape (parity-test sizes)."""
    c = CONFIGS[cfg]
    return make_layer(n, m, c.sigma, c.prune, c.k, c.quant, 1000 * c.cfg + seed_offset)


# ---- small structured matrices for edge cases (no randomness in the layout) ----

def edge_cases() -> Dict[str, np.ndarray]:
    """Degenerate matrices the formats must survive; values are shared ones."""
    rng = np.random.default_rng(424242)
    out: Dict[str, np.ndarray] = {}
    out["all_zero"] = np.zeros((7, 5), dtype=np.float32)
    out["one_value_dense"] = np.full((6, 4), 0.25, dtype=np.float32)
    d = rng.choice(np.array([-0.5, 0.125, 0.75, 1.5], dtype=np.float32), size=(9, 6))
    out["dense_no_zero"] = d.astype(np.float32)
    sc = np.zeros((11, 1), dtype=np.float32)
    sc[[0, 4, 10], 0] = [0.5, -0.5, 0.25]
    out["single_column"] = sc
    sr = np.zeros((1, 13), dtype=np.float32)
    sr[0, [1, 2, 12]] = [1.0, 2.0, 1.0]
    out["single_row"] = sr
    ec = np.zeros((8, 7), dtype=np.float32)          # empty first, middle and last columns
    ec[[1, 5], 1] = [0.5, 1.0]
    ec[[0, 7], 2] = [1.0, 1.0]
    ec[3, 4] = -2.0
    ec[[2, 3, 4], 5] = [0.5, 0.5, -2.0]
    out["empty_columns"] = ec
    one = np.zeros((5, 5), dtype=np.float32)
    one[[0, 2, 4], [1, 1, 3]] = 3.0                   # a single shared value (sHAC alphabet of 1)
    out["one_shared_value"] = one
    out["single_entry"] = np.array([[2.5]], dtype=np.float32)
    out["single_zero_entry"] = np.array([[0.0]], dtype=np.float32)
    return out


def stress_cases() -> Dict[str, np.ndarray]:
    """Larger structured matrices that push the format's limits (all deterministic)."""
    rng = np.random.default_rng(777)
    out: Dict[str, np.ndarray] = {}
    # every entry distinct: alphabet of n*m > 1024 symbols (the paper's Fact 1 setting)
    out["no_repeats_40x30"] = rng.permutation(np.arange(1, 1201, dtype=np.float32)).reshape(40, 30)
    # Fibonacci-like counts: a path-shaped Huffman tree, codewords up to 23 bits
    counts = [1, 1]
    while len(counts) < 24:
        counts.append(counts[-1] + counts[-2])
    vals = np.arange(1, len(counts) + 1, dtype=np.float32) * np.float32(0.25)
    col = np.concatenate([np.full(c, v, dtype=np.float32) for c, v in zip(counts, vals)])
    pad = (-col.size) % 8
    col = np.concatenate([col, np.zeros(pad, dtype=np.float32)])
    out["long_codes"] = rng.permutation(col).reshape(-1, 8)
    # tall and fairly dense: 17 row bits + > 2^15 stream bits per column (64-bit HAC chunk
    # entries) and > 2^16 bits of non-zero codes per column (32-bit sHAC chunk entries)
    tall = np.zeros((70000, 2), dtype=np.float32)
    mask = rng.random(tall.shape) < 0.5
    tall[mask] = rng.choice(np.array([-1.5, -0.5, 0.25, 0.75, 1.0, 2.0, 3.5, 4.0, 6.0], dtype=np.float32),
                            size=int(mask.sum()))
    out["tall_dense_70000x2"] = tall
    # dense clusters of rows far apart: small row gaps with a few enormous ones
    cl = np.zeros((300000, 3), dtype=np.float32)
    for j, starts in enumerate(((5, 120000, 299000), (0, 250000), (150000,))):
        for s0 in starts:
            rows = s0 + np.flatnonzero(rng.random(900) < 0.7)
            cl[rows, j] = rng.choice(np.array([-2.0, -1.0, 0.5, 1.5], dtype=np.float32), size=rows.size)
    out["clustered_rows_300000x3"] = cl
    # very wide and short: tens of thousands of columns of a few non-zeros each, many of them empty
    wide = np.zeros((24, 20000), dtype=np.float32)
    mask = rng.random(wide.shape) < 0.08
    wide[mask] = rng.choice(np.array([-3.0, -0.75, 0.125, 0.5, 2.5], dtype=np.float32), size=int(mask.sum()))
    out["wide_24x20000"] = wide
    return out


def random_cases(count: int, seed: int = 2024):
    """`count` small random matrices of varied shape, density, alphabet size and value skew
    (a seeded sweep for randomized parity tests): yields (name, W)."""
    rng = np.random.default_rng(seed)
    for i in range(count):
        n = int(rng.integers(1, 400))
        m = int(rng.integers(1, 90))
        dens = float(rng.choice([0.0, 0.01, 0.05, 0.3, 0.7, 1.0]))
        k = int(rng.choice([1, 2, 3, 17, 64, 300]))
        vals = np.unique(rng.standard_normal(k).astype(np.float32))
        vals = vals[vals != 0]
        if vals.size == 0:
            vals = np.array([1.0], dtype=np.float32)
        p = rng.random(vals.size) ** float(rng.choice([0.5, 1.0, 4.0]))       # flat to very skewed
        p /= p.sum()
        W = np.zeros((n, m), dtype=np.float32)
        mask = rng.random((n, m)) < dens
        W[mask] = rng.choice(vals, size=int(mask.sum()), p=p)
        yield f"rand{i}-{n}x{m}-d{dens}-k{k}", W


def paper_example_matrix() -> np.ndarray:
    """The 5x5 matrix of the paper's CSC example (Sect. IV-A, Example 1)."""
    return np.array([[1, 0, 4, 0, 0],
                     [0, 10, 0, 0, 0],
                     [2, 3, 0, 0, 5],
                     [0, 0, 0, 0, 0],
                     [0, 0, 0, 0, 6]], dtype=np.float32)
