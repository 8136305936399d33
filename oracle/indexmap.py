"""Index map (IM) representation of a weight-shared matrix (paper Sect. III-C1).

TEST INFRASTRUCTURE -- see oracle/__init__.py.

After weight sharing the k representatives are kept in a vector (c in the
paper) and every entry of W is replaced by a pointer into it: the index map
(Pi in the paper), stored with bbar bits per entry (8 when k <= 256).  The
occupancy ratio is (bbar*n*m + k*b) / (b*n*m) = bbar/b + k/(n*m).  The paper uses
this form for convolutional layers, which it quantizes without pruning
(Sect. V, the hybrid of index map for the convolutional part and HAC / sHAC for
the fully-connected part).

Readings: pointers are 0-based; the representatives are the distinct fp32
values that occur in W, the value 0.0 first when it occurs, then ascending --
the same numbering as the HAC alphabet, so Pi[i, j] is the HAC symbol of W[i, j].
bbar is 8 for k <= 256 and 16 for k <= 65536 ("even larger when k > 256").

The product is the plain definition: Y[b, j] = sum_i X[b, i] * c[Pi[i, j]].
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import huffman


@dataclass
class IndexMap:
    n: int
    m: int
    c: np.ndarray          # fp32 representatives
    pi: np.ndarray         # n x m pointers (uint8 or uint16)
    bbar: int              # bits per pointer


def im_encode(W: np.ndarray) -> IndexMap:
    W = huffman.normalise_values(W)
    n, m = W.shape
    vals = np.unique(W.ravel())                      # ascending
    if (vals == 0).any():
        vals = np.concatenate(([np.float32(0.0)], vals[vals != 0]))
    k = vals.size
    if k > 65536:
        raise ValueError("more than 65536 representatives")
    bbar = 8 if k <= 256 else 16
    pi = np.empty((n, m), dtype=np.uint8 if bbar == 8 else np.uint16)
    for idx, v in enumerate(vals):                   # one representative at a time, written out plainly
        pi[W == v] = idx
    return IndexMap(n=n, m=m, c=vals.astype(np.float32), pi=pi, bbar=bbar)


def im_decode(im: IndexMap) -> np.ndarray:
    return im.c[im.pi.astype(np.int64)]


def im_bits(im: IndexMap, b: int = 32) -> int:
    """bbar*n*m + k*b, the numerator of the paper's occupancy ratio."""
    return im.bbar * im.n * im.m + im.c.size * b


def dot_im(im: IndexMap, X: np.ndarray) -> np.ndarray:
    """Y = X . W with W looked up entry by entry (two memory accesses per weight)."""
    X = np.asarray(X, dtype=np.float64)
    Y = np.zeros((X.shape[0], im.m), dtype=np.float64)
    c = im.c.astype(np.float64)
    for j in range(im.m):
        Y[:, j] = X @ c[im.pi[:, j].astype(np.int64)]
    return Y
