"""Dot procedures on the compressed formats (what the paper's Algorithms 1, 2 and 3 return).

TEST INFRASTRUCTURE -- see oracle/__init__.py.

The result of all three is the plain product with the decoded matrix
(each algorithm's "Output" line): dense_dot below is that definition in fp64
and the parity reference.  dot_hac / dot_shac reach the same numbers straight
from the compressed form, without materialising W: a bit-serial walk of the
code tree hands out one symbol per codeword, and the columns of W are summed
as their symbols arrive (HAC: n symbols per column; sHAC: cb[j+1] - cb[j]
symbols, rows from ri).  Accumulation is fp64 throughout, in stream order.
"""
from __future__ import annotations

from typing import Iterator

import numpy as np

from . import huffman
from .formats import HAC, SHAC, WORD_BITS


def dense_dot(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Y = X.W by definition, fp64 accumulation of the fp32 operands."""
    return np.asarray(X, dtype=np.float64) @ np.asarray(W, dtype=np.float64)


def abs_dot(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """|X|.|W| in fp64: the scale against which a rounding error in Y is judged."""
    return np.abs(np.asarray(X, dtype=np.float64)) @ np.abs(np.asarray(W, dtype=np.float64))


def codewords(words: np.ndarray, code: huffman.HuffmanCode) -> Iterator[int]:
    """The symbols of a stream, one per codeword, for as long as the caller asks.

    The words are one long run of bits (first stream bit = most significant bit
    of word 0; a codeword may straddle two words).  Every bit moves one edge
    down the code tree -- 0 left, 1 right -- and a leaf ends the codeword.  The
    zero padding behind the last codeword is only reached by a caller that asks
    for more symbols than were stored.
    """
    k = code.k
    node = code.root
    for w in words:
        w = int(w)
        for t in range(WORD_BITS - 1, -1, -1):
            node = code.right[node - k] if (w >> t) & 1 else code.left[node - k]
            if node < k:
                yield node
                node = code.root


def dot_hac(h: HAC, x: np.ndarray) -> np.ndarray:
    """x^T W from the HAC stream (Sect. IV-B): the stream is W column after column, every
    entry a codeword, so column j is the next n symbols; each is multiplied with its row's x
    as it is decoded."""
    value = h.values.astype(np.float64)
    x = np.asarray(x, dtype=np.float64)
    stream = codewords(h.words, h.code)
    out = np.zeros(h.m, dtype=np.float64)
    for j in range(h.m):
        total = 0.0
        for i in range(h.n):
            total += x[i] * value[next(stream)]
        out[j] = total
    return out


def dot_shac(s: SHAC, x: np.ndarray) -> np.ndarray:
    """x^T W from the sHAC triple (Sect. IV-C): the stream holds the non-zeros only, in CSC
    order; column j owns positions cb[j] .. cb[j+1] - 1 (none for an empty column) and
    position p sits in row ri[p]."""
    value = s.values.astype(np.float64)
    x = np.asarray(x, dtype=np.float64)
    stream = codewords(s.words, s.code)
    out = np.zeros(s.m, dtype=np.float64)          # empty columns keep the value 0
    for j in range(s.m):
        total = 0.0
        for p in range(int(s.cb[j]), int(s.cb[j + 1])):
            total += x[s.ri[p]] * value[next(stream)]
        out[j] = total
    return out


def pardot(struct, X: np.ndarray, q: int = 1) -> np.ndarray:
    """Algorithm 3 (ParDot): the rows of X are dealt to q workers in runs of
    ceil(rows / q) consecutive rows; every row goes through the single-vector procedure on
    the whole compressed W.  (The runs are independent; here they simply follow each other.)"""
    X = np.asarray(X)
    rows = X.shape[0]
    dot = dot_hac if isinstance(struct, HAC) else dot_shac
    out = np.zeros((rows, struct.m), dtype=np.float64)
    if rows == 0:
        return out
    k = -(-rows // q)
    idx = [(t * k, min((t + 1) * k, rows)) for t in range(q) if t * k < rows]
    for start, end in idx:
        for i in range(start, end):
            out[i, :] = dot(struct, X[i, :])
    return out
