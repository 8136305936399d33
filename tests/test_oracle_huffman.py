"""Pins for oracle.huffman: the code must be an optimal complete prefix code.

What fixes it (none of these re-types the construction):
  * brute force over every Kraft-feasible length vector on tiny alphabets,
  * Kraft equality in exact integer arithmetic and pairwise prefix-freeness,
  * H <= average length <= H + 1 (paper Sect. IV-B),
  * 2^j equiprobable symbols -> every codeword has j bits (the index map case),
  * the length multisets forced by the paper's 5x5 example.
"""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import huffman


def brute_force_min_cost(freqs):
    k = len(freqs)
    best = None
    for lens in itertools.product(range(1, k), repeat=k):
        if sum(Fraction(1, 2 ** l) for l in lens) <= 1:
            c = sum(f * l for f, l in zip(freqs, lens))
            if best is None or c < best:
                best = c
    return best


FREQ_SETS = [
    [1, 1],
    [5, 1],
    [1, 1, 1],
    [1, 2, 3],
    [10, 1, 1],
    [1, 1, 1, 1],
    [1, 1, 2, 3],
    [7, 7, 7, 1],
    [1, 1, 2, 3, 5],          # Fibonacci-like skew: a path-shaped tree
    [4, 4, 4, 4, 4],
    [18, 1, 1, 1, 1],
    [1, 1, 2, 3, 5, 8],
    [3, 3, 3, 3, 3, 3],
    [100, 50, 20, 10, 5, 1],
    [2, 2, 3, 3, 4, 4],
]


@pytest.mark.parametrize("freqs", FREQ_SETS)
def test_cost_is_optimal_by_brute_force(freqs):
    code = huffman.build(freqs)
    assert huffman.cost(freqs, code.lengths) == brute_force_min_cost(freqs)


def test_cost_is_optimal_on_random_tiny_alphabets():
    rng = np.random.default_rng(5)
    for _ in range(40):
        k = int(rng.integers(2, 7))
        freqs = [int(v) for v in rng.integers(1, 30, size=k)]
        code = huffman.build(freqs)
        assert huffman.cost(freqs, code.lengths) == brute_force_min_cost(freqs), freqs


@pytest.mark.parametrize("k", [2, 3, 5, 8, 13, 33, 100, 257])
def test_kraft_equality_and_prefix_free(k):
    rng = np.random.default_rng(k)
    freqs = [int(v) for v in rng.integers(1, 1000, size=k)]
    code = huffman.build(freqs)
    num, den = huffman.kraft_numerator(code.lengths)
    assert num == den
    assert huffman.is_prefix_free(code)
    # codewords have the stated lengths and are distinct
    words = code.codeword_strings()
    assert len(set(words)) == k
    assert all(len(w) == l for w, l in zip(words, code.lengths))


def test_entropy_sandwich():
    rng = np.random.default_rng(11)
    for k in (2, 3, 9, 40, 257):
        for skew in (1.0, 3.0):
            freqs = [int(v) + 1 for v in (rng.random(k) ** skew * 10000)]
            code = huffman.build(freqs)
            H = huffman.entropy_bits(freqs)
            avg = huffman.cost(freqs, code.lengths) / sum(freqs)
            assert H - 1e-12 <= avg <= H + 1 + 1e-12


@pytest.mark.parametrize("j", [1, 2, 3, 5, 8])
def test_equiprobable_power_of_two_alphabet_is_fixed_length(j):
    code = huffman.build([7] * (2 ** j))
    assert set(code.lengths) == {j}


def test_single_symbol_alphabet_gets_one_bit():
    code = huffman.build([12])
    assert code.codes == [(0, 1)]
    assert code.decoding_dictionary() == {"0": 0}


def test_empty_alphabet():
    assert huffman.build([]).k == 0


def test_zero_frequency_is_rejected():
    with pytest.raises(ValueError):
        huffman.build([3, 0, 1])


def test_example_lengths(golden):
    d = golden("example_derived.txt")
    hac = huffman.build([18, 1, 1, 1, 1, 1, 1, 1])
    assert sorted(hac.lengths) == [int(v) for v in d["hac_sorted_lengths"]]
    assert hac.lengths[0] == 1                       # the zero symbol gets the 1-bit codeword
    shac = huffman.build([1] * 7)
    assert sorted(shac.lengths) == [int(v) for v in d["shac_sorted_lengths"]]


def test_alphabet_order_and_counts():
    vals, cnt = huffman.alphabet(np.array([0.5, 0.0, -1.0, 0.0, 0.5, 0.0, 2.0], dtype=np.float32))
    assert vals.tolist() == [0.0, -1.0, 0.5, 2.0]
    assert cnt.tolist() == [3, 1, 2, 1]
    vals, cnt = huffman.alphabet(np.array([3.0, -2.0, 3.0], dtype=np.float32))
    assert vals.tolist() == [-2.0, 3.0] and cnt.tolist() == [1, 2]


def test_negative_zero_and_non_finite():
    W = huffman.normalise_values(np.array([[-0.0, 1.0]], dtype=np.float32))
    assert not np.signbit(W[0, 0])
    for bad in (np.nan, np.inf, -np.inf):
        with pytest.raises(ValueError):
            huffman.normalise_values(np.array([[bad]], dtype=np.float32))


def test_entropy_closed_form():
    assert math.isclose(huffman.entropy_bits([1, 1, 1, 1]), 2.0)
    assert math.isclose(huffman.entropy_bits([18] + [1] * 7), 1.6415, abs_tol=5e-4)
