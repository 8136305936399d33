"""sHAC with an entropy-coded address map: Rice-coded row gaps.

TEST INFRASTRUCTURE -- see oracle/__init__.py.

This is an extension, not one of the paper's formats.  The paper keeps the row
index vector ri of sHAC uncompressed (Sect. IV-C) and only remarks, in the
footnote to Sect. IV-A, that ceil(log2 n) bits per index would do.  Here ri is
replaced by the gaps between consecutive non-zeros of a column, each written
with a Golomb-Rice code (Golomb 1966; Rice 1979: quotient in unary, remainder in
k plain bits), and the gap codeword is placed in the stream directly in front of
the Huffman codeword of the value it belongs to.  nz, its Huffman code and cb
are exactly those of sHAC.

Definition used by both this oracle and the library (the library's header
restates it; neither side imports the other):

  * CSC order (columns left to right, rows ascending).  For the non-zero at CSC
    position p in column j:  d_p = ri[p] - prev - 1, where prev = ri[p-1] if
    p-1 lies in the same column, else -1.  d_p >= 0.
  * Rice_k(d), q = d >> k:
        q < 31 : q bits '0', one bit '1', then the k low bits of d, MSB first
        q >= 31: 31 bits '0', one bit '1', then d as 32 bits, MSB first
    (a '1' always appears within 32 bits, so a decoder finds the quotient with
    one count-leading-zeros; the second form is an escape for huge gaps).
  * stream = concat over p of  Rice_k(d_p) || H(nz_p),  cut into 32-bit words,
    MSB first, last word zero padded -- the same word convention as HAC/sHAC.
  * k is the value in 0..15 that minimises the total number of gap bits; ties go
    to the smaller k.

Pins (tests/test_oracle_gapcode.py): hand-written codewords, the closed-form
length q + 1 + k, Kraft sums, the paper's 5x5 example worked by hand (32 bits in
all), the expected length k + 1/(1 - (1-s)^(2^k)) for geometric gaps, exhaustive
search for k, losslessness, and the product against the dense one.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import numpy as np

from . import formats, huffman

WORD_BITS = 32
Q_ESCAPE = 31          # quotients from here on use the escape form
K_MAX = 15


# --------------------------------------------------------------------------
# the gap code
# --------------------------------------------------------------------------

def rice_length(d: int, k: int) -> int:
    q = d >> k
    return q + 1 + k if q < Q_ESCAPE else Q_ESCAPE + 1 + 32


def rice_bits(d: int, k: int) -> str:
    """Codeword of d as a string of '0'/'1'."""
    if d < 0 or d >= 1 << 32:
        raise ValueError("gap out of range")
    q = d >> k
    if q < Q_ESCAPE:
        rem = format(d & ((1 << k) - 1), "b").zfill(k) if k else ""
        return "0" * q + "1" + rem
    return "0" * Q_ESCAPE + "1" + format(d, "b").zfill(32)


def rice_lengths(d: np.ndarray, k: int) -> np.ndarray:
    d = np.asarray(d, dtype=np.int64)
    q = d >> k
    return np.where(q < Q_ESCAPE, q + 1 + k, Q_ESCAPE + 1 + 32).astype(np.int64)


def best_k(d: np.ndarray) -> int:
    """k in 0..K_MAX with the fewest total gap bits (smallest such k)."""
    if np.asarray(d).size == 0:
        return 0
    totals = [int(rice_lengths(d, k).sum()) for k in range(K_MAX + 1)]
    return int(np.argmin(totals))            # argmin returns the first minimum


def column_gaps(ri: np.ndarray, cb: np.ndarray) -> np.ndarray:
    """d_p for every CSC position."""
    ri = np.asarray(ri, dtype=np.int64)
    d = np.empty(ri.size, dtype=np.int64)
    for j in range(cb.size - 1):
        lo, hi = int(cb[j]), int(cb[j + 1])
        prev = -1
        for p in range(lo, hi):
            d[p] = ri[p] - prev - 1
            prev = ri[p]
    return d


def column_gaps_fast(ri: np.ndarray, cb: np.ndarray) -> np.ndarray:
    """Same as column_gaps with array operations (for the large configurations)."""
    ri = np.asarray(ri, dtype=np.int64)
    if ri.size == 0:
        return np.zeros(0, dtype=np.int64)
    prev = np.empty_like(ri)
    prev[1:] = ri[:-1]
    prev[0] = -1
    starts = np.asarray(cb[:-1], dtype=np.int64)
    starts = starts[starts < ri.size]
    prev[starts] = -1                        # first non-zero of every non-empty column
    return ri - prev - 1


# --------------------------------------------------------------------------
# packing
# --------------------------------------------------------------------------

def pack_fields(values: np.ndarray, lens: np.ndarray) -> Tuple[np.ndarray, int]:
    """Concatenate bit fields (value, length <= 64), MSB first, into 32-bit words."""
    values = np.asarray(values, dtype=np.uint64)
    lens = np.asarray(lens, dtype=np.int64)
    if values.size == 0:
        return np.zeros(0, dtype=np.uint32), 0
    start = np.cumsum(lens) - lens
    nbits = int(start[-1] + lens[-1])
    nwords = -(-nbits // WORD_BITS)
    bits = np.zeros(nwords * WORD_BITS, dtype=np.uint8)
    for t in range(int(lens.max())):
        sel = lens > t
        shift = (lens[sel] - 1 - t).astype(np.uint64)
        bits[start[sel] + t] = ((values[sel] >> shift) & np.uint64(1)).astype(np.uint8)
    by = np.packbits(bits)
    w = by.reshape(-1, 4).astype(np.uint32)
    out = (w[:, 0] << 24) | (w[:, 1] << 16) | (w[:, 2] << 8) | w[:, 3]
    return out.astype(np.uint32), nbits


def pack_bitstring(bits: str) -> Tuple[np.ndarray, int]:
    nbits = len(bits)
    nwords = -(-nbits // WORD_BITS)
    bits = bits + "0" * (nwords * WORD_BITS - nbits)
    out = np.array([int(bits[i * WORD_BITS:(i + 1) * WORD_BITS], 2) for i in range(nwords)], dtype=np.uint32)
    return out, nbits


# --------------------------------------------------------------------------
# the format
# --------------------------------------------------------------------------

@dataclass
class SHACG:
    n: int
    m: int
    values: np.ndarray            # fp32 alphabet of the non-zero values, ascending
    freqs: np.ndarray
    code: huffman.HuffmanCode
    k: int                        # Rice parameter
    words: np.ndarray             # uint32[N]
    nbits: int
    gap_bits: int                 # part of nbits spent on the gap codewords
    cb: np.ndarray                # int64[m + 1]

    @property
    def N(self) -> int:
        return int(self.words.size)

    @property
    def q(self) -> int:
        return int(self.cb[-1])


def shacg_symbols(W: np.ndarray):
    """(values, sym, row, col, d): what a decoder must reproduce, in CSC order."""
    W = huffman.normalise_values(W)
    nz, ri, cb = formats.csc_arrays(W)
    values, _ = huffman.alphabet(nz)
    sym = formats.symbol_indices(nz, values)
    col = np.repeat(np.arange(W.shape[1], dtype=np.int64), np.diff(cb))
    return values, sym, ri, col, column_gaps_fast(ri, cb)


def shacg_encode(W: np.ndarray, k: int | None = None, reference_packer: bool = False) -> SHACG:
    W = huffman.normalise_values(W)
    n, m = W.shape
    nz, ri, cb = formats.csc_arrays(W)
    values, freqs = huffman.alphabet(nz)
    code = huffman.build(freqs.tolist())
    sym = formats.symbol_indices(nz, values)
    d = column_gaps(ri, cb) if reference_packer else column_gaps_fast(ri, cb)
    if k is None:
        k = best_k(d)
    glen = rice_lengths(d, k)
    if reference_packer:
        cws = code.codeword_strings()
        bits = "".join(rice_bits(int(d[p]), k) + cws[int(sym[p])] for p in range(sym.size))
        words, nbits = pack_bitstring(bits)
    else:
        q = d >> k
        esc = q >= Q_ESCAPE
        # gap field as one integer: the leading zeros come from the field being wider than its value
        rem = d & ((1 << k) - 1)
        gval = np.where(esc, (np.int64(1) << 32) | d, (np.int64(1) << k) | rem).astype(np.uint64)
        cw = np.array([c for c, _ in code.codes], dtype=np.uint64)
        ln = np.array([l for _, l in code.codes], dtype=np.int64)
        vals = np.empty(2 * sym.size, dtype=np.uint64)
        lens = np.empty(2 * sym.size, dtype=np.int64)
        vals[0::2], lens[0::2] = gval, glen
        if sym.size:
            vals[1::2], lens[1::2] = cw[sym], ln[sym]
        words, nbits = pack_fields(vals, lens)
    return SHACG(n=n, m=m, values=values, freqs=freqs, code=code, k=int(k), words=words, nbits=nbits,
                 gap_bits=int(glen.sum()), cb=cb)


class _BitReader:
    def __init__(self, words: np.ndarray):
        self.words = words
        self.pos = 0

    def bit(self) -> int:
        w = int(self.words[self.pos >> 5])
        b = (w >> (31 - (self.pos & 31))) & 1
        self.pos += 1
        return b

    def bits(self, count: int) -> int:
        v = 0
        for _ in range(count):
            v = (v << 1) | self.bit()
        return v


def _read_gap(r: _BitReader, k: int) -> int:
    q = 0
    while r.bit() == 0:
        q += 1
    if q < Q_ESCAPE:
        return (q << k) | r.bits(k)
    return r.bits(32)


def _read_symbol(r: _BitReader, code: huffman.HuffmanCode) -> int:
    node = code.root                        # a one-symbol alphabet has a root with two equal children
    while node >= code.k:
        node = code.right[node - code.k] if r.bit() else code.left[node - code.k]
    return node


def shacg_decode_csc(s: SHACG):
    """(sym, row, col) by reading the stream bit by bit."""
    q = s.q
    sym = np.empty(q, dtype=np.int64)
    row = np.empty(q, dtype=np.int64)
    col = np.empty(q, dtype=np.int64)
    r = _BitReader(s.words)
    for j in range(s.m):
        prev = -1
        for p in range(int(s.cb[j]), int(s.cb[j + 1])):
            prev = prev + 1 + _read_gap(r, s.k)
            row[p] = prev
            col[p] = j
            sym[p] = _read_symbol(r, s.code)
    if r.pos != s.nbits:
        raise ValueError("decoder did not end on the last stream bit")
    return sym, row, col


def shacg_decode(s: SHACG) -> np.ndarray:
    sym, row, col = shacg_decode_csc(s)
    W = np.zeros((s.n, s.m), dtype=np.float32)
    W[row, col] = s.values[sym]
    return W


def dot_shacg(s: SHACG, x: np.ndarray) -> np.ndarray:
    """x . W for one input vector, decoding the stream as it goes (the analogue of Algorithm 2)."""
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros(s.m, dtype=np.float64)
    r = _BitReader(s.words)
    for j in range(s.m):
        acc = 0.0
        prev = -1
        for _ in range(int(s.cb[j]), int(s.cb[j + 1])):
            prev = prev + 1 + _read_gap(r, s.k)
            acc += x[prev] * float(s.values[_read_symbol(r, s.code)])
        out[j] = acc
    return out


def shacg_paper_bits(s: SHACG, b: int = 32) -> int:
    """Size in the accounting of Corollary 2: stream words, the two dictionaries (6kb as in the
    paper's bound) and cb; there is no ri vector any more."""
    return b * s.N + 6 * len(s.values) * b + b * (s.m + 1)
