"""Huffman code over the distinct values of a matrix (paper Sect. IV-B).

TEST INFRASTRUCTURE -- see oracle/__init__.py.

The paper replaces each entry's address-map string a(z) by its Huffman
codeword H_W(z) [Huffman 1952] and quotes H <= average length <= H + 1.  The
construction here is the textbook one: repeatedly merge the two least frequent
nodes.  Codes are read off the tree (left edge = 0, right edge = 1); this is
deliberately *not* a canonical re-assignment, so the oracle's bitstream is an
independent one.
"""
from __future__ import annotations

import heapq
import math
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np


def normalise_values(W: np.ndarray) -> np.ndarray:
    """fp32 copy with -0.0 turned into +0.0; NaN / Inf are an error."""
    W = np.asarray(W, dtype=np.float32)
    if not np.all(np.isfinite(W)):
        raise ValueError("W contains NaN or Inf")
    return W + np.float32(0.0)          # -0.0 + 0.0 == +0.0, everything else unchanged


def alphabet(values: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Distinct fp32 values and their counts.

    Order: 0.0 first if it occurs, then the remaining values ascending.
    """
    vals, counts = np.unique(np.asarray(values, dtype=np.float32).ravel(), return_counts=True)
    z = np.flatnonzero(vals == 0.0)
    if z.size:
        i = int(z[0])
        order = np.concatenate(([i], np.arange(0, i), np.arange(i + 1, vals.size))).astype(np.int64)
        vals, counts = vals[order], counts[order]
    return vals.astype(np.float32), counts.astype(np.int64)


@dataclass
class HuffmanCode:
    """A prefix code for symbols 0..k-1.

    left/right: children of internal node (k + i); a child < k is a leaf.
    root: index of the root node.  codes[s] = (bits as int, length).
    """
    k: int
    left: List[int]
    right: List[int]
    root: int
    codes: List[Tuple[int, int]]

    @property
    def lengths(self) -> List[int]:
        return [l for _, l in self.codes]

    def codeword_strings(self) -> List[str]:
        return [format(c, "b").zfill(l) for c, l in self.codes]

    def decoding_dictionary(self) -> Dict[str, int]:
        """H^-1 as a map from codeword bit-string to symbol."""
        return {s: i for i, s in enumerate(self.codeword_strings())}


def build(freqs: Sequence[int]) -> HuffmanCode:
    """Huffman's algorithm.  freqs[i] > 0 is the count of symbol i."""
    k = len(freqs)
    if k == 0:
        return HuffmanCode(0, [], [], -1, [])
    if any(f <= 0 for f in freqs):
        raise ValueError("every symbol of the alphabet must occur")
    if k == 1:
        # degenerate source: one symbol, codeword "0" (the bit "1" is never written)
        return HuffmanCode(1, [0], [0], 1, [(0, 1)])
    heap = [(int(f), i) for i, f in enumerate(freqs)]      # (weight, node id); ties -> lower id
    heapq.heapify(heap)
    left: List[int] = []
    right: List[int] = []
    nxt = k
    while len(heap) > 1:
        wa, a = heapq.heappop(heap)
        wb, b = heapq.heappop(heap)
        left.append(a)
        right.append(b)
        heapq.heappush(heap, (wa + wb, nxt))
        nxt += 1
    root = heap[0][1]
    codes: List[Tuple[int, int]] = [(0, 0)] * k
    stack = [(root, 0, 0)]
    while stack:
        node, bits, depth = stack.pop()
        if node < k:
            codes[node] = (bits, depth)
        else:
            stack.append((left[node - k], bits << 1, depth + 1))
            stack.append((right[node - k], (bits << 1) | 1, depth + 1))
    return HuffmanCode(k, left, right, root, codes)


def cost(freqs: Sequence[int], lengths: Sequence[int]) -> int:
    """Total number of bits sum f_i * l_i."""
    return int(sum(int(f) * int(l) for f, l in zip(freqs, lengths)))


def entropy_bits(freqs: Sequence[int]) -> float:
    """Source entropy in bits per symbol (binary log, as everywhere in the paper)."""
    tot = float(sum(freqs))
    return -sum((f / tot) * math.log2(f / tot) for f in freqs if f > 0)


def kraft_numerator(lengths: Sequence[int]) -> Tuple[int, int]:
    """(sum 2^(Lmax - l_i), 2^Lmax): equal for a complete prefix code."""
    L = max(lengths)
    return sum(1 << (L - l) for l in lengths), 1 << L


def is_prefix_free(code: HuffmanCode) -> bool:
    words = code.codeword_strings()
    for i, a in enumerate(words):
        for j, b in enumerate(words):
            if i != j and b.startswith(a):
                return False
    return True
