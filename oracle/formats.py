"""CSC, HAC and sHAC storage formats (paper Sect. IV-A, IV-B, IV-C).

TEST INFRASTRUCTURE -- see oracle/__init__.py.

HAC (Sect. IV-B): the entries of W, zeros included, are listed in column
order (Example 2), each is replaced by its Huffman codeword, the codewords are
concatenated into the bit stream HAC(W), and the stream is cut into
N = ceil(|HAC(W)| / b) words of b = 32 bits, the last one padded with zeros.

sHAC (Sect. IV-C): W is put in CSC form (nz, ri, cb as in Sect. IV-A); the
Huffman code is built over the non-zero values only and nz is stored as the
stream HAC(nz) in N1 = ceil(|HAC(nz)| / b) words; ri and cb are kept as they
are.  Indices are 0-based here (the paper's Example 1 prints them 1-based).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

from . import huffman

WORD_BITS = 32          # b: one memory word (the paper's FP32 setting)


# --------------------------------------------------------------------------
# plain CSC (Sect. IV-A)
# --------------------------------------------------------------------------

def column_order(W: np.ndarray) -> np.ndarray:
    """Entries of W in the column-order sequence of Example 2."""
    n, m = W.shape
    out = np.empty(n * m, dtype=W.dtype)
    for j in range(m):
        out[j * n:(j + 1) * n] = W[:, j]
    return out


def csc_arrays(W: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """nz (non-zero values by columns), ri (their rows), cb (column begins, m+1)."""
    n, m = W.shape
    nz: List[np.ndarray] = []
    ri: List[np.ndarray] = []
    cb = np.zeros(m + 1, dtype=np.int64)
    for j in range(m):
        rows = np.flatnonzero(W[:, j] != 0)
        nz.append(W[rows, j])
        ri.append(rows)
        cb[j + 1] = cb[j] + rows.size
    nzv = np.concatenate(nz) if nz else np.zeros(0, dtype=W.dtype)
    riv = np.concatenate(ri).astype(np.int64) if ri else np.zeros(0, dtype=np.int64)
    return nzv.astype(np.float32), riv, cb


# --------------------------------------------------------------------------
# symbol sequences and bit packing
# --------------------------------------------------------------------------

def symbol_indices(seq: np.ndarray, values: np.ndarray) -> np.ndarray:
    """Index in `values` of every element of `seq` (all must be present)."""
    if values.size == 0:
        return np.zeros(0, dtype=np.int64)
    sorter = np.argsort(values, kind="stable")
    pos = np.searchsorted(values, seq, sorter=sorter)
    idx = sorter[pos]
    if not np.array_equal(values[idx], seq):
        raise ValueError("sequence holds a value outside the alphabet")
    return idx.astype(np.int64)


def pack_stream_reference(symbols, code: huffman.HuffmanCode) -> Tuple[np.ndarray, int]:
    """Concatenate codewords and cut into 32-bit words -- written out literally.

    Builds the bit string character by character; only for small inputs.
    """
    words_of = code.codeword_strings()
    bits = "".join(words_of[int(s)] for s in symbols)
    nbits = len(bits)
    nwords = -(-nbits // WORD_BITS)
    bits = bits + "0" * (nwords * WORD_BITS - nbits)           # zero padding of the last word
    out = np.array([int(bits[i * WORD_BITS:(i + 1) * WORD_BITS], 2) for i in range(nwords)],
                   dtype=np.uint32)
    return out, nbits


def pack_stream(symbols: np.ndarray, code: huffman.HuffmanCode) -> Tuple[np.ndarray, int]:
    """Same result as pack_stream_reference, with array operations.

    Every symbol's codeword is written bit by bit at its start offset (the
    running sum of the lengths of the codewords before it).
    """
    symbols = np.asarray(symbols, dtype=np.int64)
    if symbols.size == 0:
        return np.zeros(0, dtype=np.uint32), 0
    cw = np.array([c for c, _ in code.codes], dtype=np.uint64)
    ln = np.array([l for _, l in code.codes], dtype=np.int64)
    lens = ln[symbols]
    cws = cw[symbols]
    start = np.cumsum(lens) - lens
    nbits = int(start[-1] + lens[-1])
    nwords = -(-nbits // WORD_BITS)
    bits = np.zeros(nwords * WORD_BITS, dtype=np.uint8)
    for t in range(int(lens.max())):                    # t-th bit of each codeword, from its MSB
        sel = lens > t
        shift = (lens[sel] - 1 - t).astype(np.uint64)
        bits[start[sel] + t] = ((cws[sel] >> shift) & np.uint64(1)).astype(np.uint8)
    by = np.packbits(bits)                               # first bit -> MSB of byte 0
    words = by.reshape(-1, 4).astype(np.uint32)
    out = (words[:, 0] << 24) | (words[:, 1] << 16) | (words[:, 2] << 8) | words[:, 3]
    return out.astype(np.uint32), nbits


def unpack_stream(words: np.ndarray, count: int, code: huffman.HuffmanCode) -> np.ndarray:
    """Decode `count` symbols by walking the code tree one bit at a time."""
    out = np.empty(count, dtype=np.int64)
    if count == 0:
        return out
    k = code.k
    node = code.root
    got = 0
    for w in words:
        w = int(w)
        for t in range(WORD_BITS - 1, -1, -1):
            bit = (w >> t) & 1
            node = code.right[node - k] if bit else code.left[node - k]
            if node < k:
                out[got] = node
                got += 1
                node = code.root
                if got == count:
                    return out
    raise ValueError("stream ended before all symbols were decoded")


# --------------------------------------------------------------------------
# HAC (Sect. IV-B)
# --------------------------------------------------------------------------

@dataclass
class HAC:
    n: int
    m: int
    values: np.ndarray            # fp32 alphabet, symbol order (H^-1 maps symbol -> value)
    freqs: np.ndarray
    code: huffman.HuffmanCode
    words: np.ndarray             # C_HAC(W): uint32[N]
    nbits: int                    # |HAC(W)|

    @property
    def N(self) -> int:
        return int(self.words.size)


def hac_encode(W: np.ndarray, reference_packer: bool = False) -> HAC:
    W = huffman.normalise_values(W)
    n, m = W.shape
    seq = column_order(W)
    values, freqs = huffman.alphabet(seq)
    code = huffman.build(freqs.tolist())
    sym = symbol_indices(seq, values)
    packer = pack_stream_reference if reference_packer else pack_stream
    words, nbits = packer(sym, code)
    return HAC(n, m, values, freqs, code, words, nbits)


def hac_symbols(W: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """(alphabet, symbol index of every entry in column order) -- the ground truth
    a decoder of any HAC stream of W must reproduce."""
    W = huffman.normalise_values(W)
    seq = column_order(W)
    values, _ = huffman.alphabet(seq)
    return values, symbol_indices(seq, values)


def hac_decode(h: HAC) -> np.ndarray:
    sym = unpack_stream(h.words, h.n * h.m, h.code)
    seq = h.values[sym] if h.values.size else np.zeros(0, dtype=np.float32)
    W = np.empty((h.n, h.m), dtype=np.float32)
    for j in range(h.m):
        W[:, j] = seq[j * h.n:(j + 1) * h.n]
    return W


# --------------------------------------------------------------------------
# sHAC (Sect. IV-C)
# --------------------------------------------------------------------------

@dataclass
class SHAC:
    n: int
    m: int
    values: np.ndarray            # fp32 alphabet of the non-zero values
    freqs: np.ndarray
    code: huffman.HuffmanCode
    words: np.ndarray             # C_HAC(nz): uint32[N1]
    nbits: int                    # |HAC(nz)|
    ri: np.ndarray                # row index of every non-zero (0-based)
    cb: np.ndarray                # column begins, m+1 entries (0-based), cb[m] = q

    @property
    def N1(self) -> int:
        return int(self.words.size)

    @property
    def q(self) -> int:
        return int(self.cb[-1])


def shac_encode(W: np.ndarray, reference_packer: bool = False) -> SHAC:
    W = huffman.normalise_values(W)
    n, m = W.shape
    nz, ri, cb = csc_arrays(W)
    values, freqs = huffman.alphabet(nz)
    code = huffman.build(freqs.tolist())
    sym = symbol_indices(nz, values)
    packer = pack_stream_reference if reference_packer else pack_stream
    words, nbits = packer(sym, code)
    return SHAC(n, m, values, freqs, code, words, nbits, ri, cb)


def shac_symbols(W: np.ndarray):
    """(alphabet, symbol index, row, column) of every non-zero in CSC order."""
    W = huffman.normalise_values(W)
    nz, ri, cb = csc_arrays(W)
    values, _ = huffman.alphabet(nz)
    col = np.repeat(np.arange(W.shape[1], dtype=np.int64), np.diff(cb))
    return values, symbol_indices(nz, values), ri, col


def shac_decode(s: SHAC) -> np.ndarray:
    sym = unpack_stream(s.words, s.q, s.code)
    W = np.zeros((s.n, s.m), dtype=np.float32)
    for j in range(s.m):
        for p in range(int(s.cb[j]), int(s.cb[j + 1])):
            W[int(s.ri[p]), j] = s.values[sym[p]]
    return W


# --------------------------------------------------------------------------
# stored size, as the paper accounts for it
# --------------------------------------------------------------------------

def hac_paper_bits(h: HAC, b: int = WORD_BITS) -> int:
    """Stream words plus both dictionaries at 3b bits per entry each (Fact 1's proof)."""
    return h.N * b + 6 * len(h.values) * b


def shac_paper_bits(s: SHAC, b: int = WORD_BITS) -> int:
    """Stream words, dictionaries at 6b per entry, ri and cb at b bits per element."""
    return s.N1 * b + 6 * len(s.values) * b + b * (s.q + s.m + 1)
