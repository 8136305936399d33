"""Space bounds and occupancy formulas of the paper (Sect. III-C1, IV-A, IV-B, IV-C).

TEST INFRASTRUCTURE -- see oracle/__init__.py.

All logarithms are binary (Sect. III-A).  b is the word size in bits, s the
ratio of non-zero entries, k the number of distinct values.
"""
from __future__ import annotations

import math


def fact1_bits(n: int, m: int, b: int = 32) -> float:
    """Fact 1: dense W without repeated entries."""
    nm = n * m
    return nm * (1 + math.log2(nm)) + 6 * nm * b


def corollary1_bits(n: int, m: int, k: int, b: int = 32) -> float:
    """Corollary 1: |HAC(W)| <= nm(1 + log k) + 6kb for k distinct values."""
    return n * m * (1 + math.log2(k)) + 6 * k * b


def psi_hac_bound(n: int, m: int, k: int, b: int = 32) -> float:
    """Eq. (2): occupancy bound for HAC."""
    return (1 + math.log2(k)) / b + 6 * k / (n * m)


def fact2_bits(n: int, m: int, q: int, b: int = 32) -> float:
    """Fact 2 with q = s*n*m non-null elements, all distinct."""
    if q == 0:
        return b * (m + 1)
    return q * (1 + math.log2(q)) + b * (7 * q + m + 1)


def corollary2_bits(n: int, m: int, q: int, k: int, b: int = 32) -> float:
    """Corollary 2: |sHAC(W)| <= snm(1 + log k) + b(6k + snm + m + 1)."""
    return q * (1 + math.log2(k)) + b * (6 * k + q + m + 1)


def psi_shac_bound(n: int, m: int, s: float, k: int, b: int = 32) -> float:
    """Eq. (3): occupancy bound for sHAC."""
    return s * (1 + math.log2(k)) / b + (6 * k + m + 1) / (n * m) + s


def crossover_sparsity(n: int, m: int, k: int, b: int = 32) -> float:
    """Non-zero ratio below which Eq. (3) is smaller than Eq. (2) (end of Sect. IV-C)."""
    a = (1 + math.log2(k)) / b
    return (a - (m + 1) / (n * m)) / (1 + a)


def psi_csc(n: int, m: int, q: int) -> float:
    """Sect. IV-A: (2q + m + 1) / (nm)."""
    return (2 * q + m + 1) / (n * m)


def csc_break_even_s(n: int, m: int) -> float:
    """Sect. IV-A: psi_CSC < 1 iff s < 1/2 - (m+1)/(2nm)."""
    return 0.5 - (m + 1) / (2 * n * m)


def psi_index_map(n: int, m: int, k: int, bbar: int, b: int = 32) -> float:
    """Sect. III-C1: index map of bbar-bit pointers plus k representatives."""
    return bbar / b + k / (n * m)
