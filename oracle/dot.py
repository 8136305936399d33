"""Dot procedures on the compressed formats (paper Algorithms 1, 2 and 3).

TEST INFRASTRUCTURE -- see oracle/__init__.py.

The result of all three is the plain product with the decoded matrix
(each algorithm's "Output" line): dense_dot below is that definition in fp64.
Algorithms 1-3 are also taken step by step, with the paper's variable names,
as a second route to the same numbers.  Accumulation is fp64 throughout.
"""
from __future__ import annotations

from typing import Dict, Optional, Tuple

import numpy as np

from .formats import HAC, SHAC, WORD_BITS


def dense_dot(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Y = X.W by definition, fp64 accumulation of the fp32 operands."""
    return np.asarray(X, dtype=np.float64) @ np.asarray(W, dtype=np.float64)


def abs_dot(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """|X|.|W| in fp64: the scale against which a rounding error in Y is judged."""
    return np.abs(np.asarray(X, dtype=np.float64)) @ np.abs(np.asarray(W, dtype=np.float64))


def get_binary_seq(word: int) -> str:
    """Binary representation S of one memory word, first stream bit first."""
    return format(int(word), "b").zfill(WORD_BITS)


def ncw(S: str, rem: str, oset: int, Hinv: Dict[str, int]) -> Tuple[int, str, Optional[int]]:
    """Next code word (Sect. IV-B, "Dot product").

    Extends the unprocessed bits `rem` with bits of S from offset `oset`, one
    at a time, searching the decoding dictionary after every bit.  Returns
    (oset, rem, z): z is the decoded symbol and rem is empty again, or z is
    None (the paper's "null") when S is exhausted first -- the codeword
    continues in the next memory word and rem holds the bits read so far.
    """
    cur = rem
    while oset < len(S):
        cur += S[oset]
        oset += 1
        if cur in Hinv:
            return oset, "", Hinv[cur]
    return oset, cur, None


def dot_hac(h: HAC, x: np.ndarray) -> np.ndarray:
    """Algorithm 1 (Dot_HAC): x^T W from the HAC stream, one codeword at a time."""
    n, m = h.n, h.m
    Hinv = h.code.decoding_dictionary()
    Hval = h.values.astype(np.float64)
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros(m, dtype=np.float64)
    row, col = 0, 0
    acc = 0.0
    rem, oset = "", 0
    left = n * m                       # symbols still to decode: the padding is never read as data
    for i in range(h.N):
        if left == 0:
            break
        S = get_binary_seq(h.words[i])
        oset = 0
        while left > 0:
            oset, rem, z = ncw(S, rem, oset, Hinv)
            if z is None:
                break
            left -= 1
            acc += x[row] * Hval[z]
            row += 1
            if row == n:
                row = 0
                out[col] = acc
                col += 1
                acc = 0.0
    return out


def dot_shac(s: SHAC, x: np.ndarray) -> np.ndarray:
    """Algorithm 2 (Dot_sHAC): x^T W from the sHAC triple (C_HAC(nz), ri, cb)."""
    m = s.m
    Hinv = s.code.decoding_dictionary()
    Hval = s.values.astype(np.float64)
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros(m, dtype=np.float64)          # empty columns keep the value 0
    cb, ri = s.cb, s.ri
    pos, col = 0, 0
    acc = 0.0
    rem, oset = "", 0
    q = s.q
    for i in range(s.N1):
        if pos == q:
            break
        S = get_binary_seq(s.words[i])
        oset = 0
        while pos < q:
            oset, rem, z = ncw(S, rem, oset, Hinv)
            if z is None:
                break
            while cb[col + 1] == pos:            # skip empty columns
                col += 1
            acc += x[ri[pos]] * Hval[z]
            pos += 1
            if cb[col + 1] == pos:               # last non-zero of this column
                out[col] = acc
                acc = 0.0
                col += 1
    return out


def pardot(struct, X: np.ndarray, q: int = 1) -> np.ndarray:
    """Algorithm 3 (ParDot): the rows of X are split into q chunks of
    k = ceil(rows / q); every row goes through Dot on the whole compressed W.
    (The chunks are independent; here they simply run one after the other.)"""
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
