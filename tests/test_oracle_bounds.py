"""The paper's space bounds hold for what the oracle encoders produce, and the
closed forms in oracle.bounds behave as the text says.

Fact 1 / Corollary 1 / Eq. (2) (Sect. IV-B), Fact 2 / Corollary 2 / Eq. (3)
and the crossover (Sect. IV-C), psi_CSC (Sect. IV-A), index map (Sect. III-C1).
"""
import math

import numpy as np
import pytest

import workloads
from oracle import bounds, formats, huffman

B = 32


def layers():
    yield "cfg1", workloads.layer(1)
    yield "cfg2-small", workloads.scaled(2, 512, 125)
    yield "cfg3-small", workloads.scaled(3, 512, 512)
    yield "cfg4-small", workloads.scaled(4, 1568, 256)
    yield "cfg5-small", workloads.scaled(5, 576, 64)
    for name, W in workloads.edge_cases().items():
        yield name, W


@pytest.mark.parametrize("name,W", list(layers()), ids=[n for n, _ in layers()])
def test_corollaries_hold(name, W):
    n, m = W.shape
    h = formats.hac_encode(W)
    k = len(h.values)
    # pure stream part and the paper's full accounting (dictionaries at 6b per codeword)
    assert h.nbits <= n * m * (1 + math.log2(k))
    assert h.nbits + 6 * k * B <= bounds.corollary1_bits(n, m, k, B)
    assert formats.hac_paper_bits(h, B) <= bounds.corollary1_bits(n, m, k, B) + (B - 1)
    s = formats.shac_encode(W)
    q, ks = s.q, len(s.values)
    if q:
        assert s.nbits <= q * (1 + math.log2(ks))
        assert s.nbits + B * (6 * ks + q + m + 1) <= bounds.corollary2_bits(n, m, q, ks, B)
        assert formats.shac_paper_bits(s, B) <= bounds.corollary2_bits(n, m, q, ks, B) + (B - 1)
    # occupancy form of the same statements
    assert (h.nbits + 6 * k * B) / (B * n * m) <= bounds.psi_hac_bound(n, m, k, B) + 1e-15
    if q:
        occ = (s.nbits + B * (6 * ks + q + m + 1)) / (B * n * m)
        assert occ <= bounds.psi_shac_bound(n, m, q / (n * m), ks, B) + 1e-15


def test_fact1_and_fact2_on_matrices_without_repeats():
    rng = np.random.default_rng(3)
    W = rng.permutation(np.arange(1, 1 + 24 * 10, dtype=np.float32)).reshape(24, 10)
    h = formats.hac_encode(W)
    assert len(h.values) == W.size
    assert h.nbits + 6 * W.size * B <= bounds.fact1_bits(24, 10, B)
    Ws = W.copy()
    Ws[rng.random(W.shape) < 0.7] = 0.0
    s = formats.shac_encode(Ws)
    assert len(s.values) == s.q
    assert s.nbits + 6 * s.q * B + B * (s.q + 10 + 1) <= bounds.fact2_bits(24, 10, s.q, B)
    # Fact 1's bound exceeds the uncompressed size, as the paper remarks
    assert bounds.fact1_bits(24, 10, B) > B * W.size


def test_bounds_are_consistent_with_each_other():
    n, m, k = 4096, 1000, 32
    # Eq. (2) is Corollary 1 divided by b*n*m
    assert math.isclose(bounds.corollary1_bits(n, m, k, B) / (B * n * m),
                        bounds.psi_hac_bound(n, m, k, B))
    s = 0.1
    q = int(s * n * m)
    assert math.isclose(bounds.corollary2_bits(n, m, q, k, B) / (B * n * m),
                        bounds.psi_shac_bound(n, m, q / (n * m), k, B))
    # Corollary 1 with k = nm is Fact 1; Corollary 2 with k = snm is Fact 2
    assert math.isclose(bounds.corollary1_bits(7, 9, 63, B), bounds.fact1_bits(7, 9, B))
    assert math.isclose(bounds.corollary2_bits(7, 9, 20, 20, B), bounds.fact2_bits(7, 9, 20, B))


@pytest.mark.parametrize("n,m,k", [(4096, 1000, 32), (4096, 4096, 256), (25088, 4096, 32), (500, 300, 16)])
def test_crossover_separates_the_two_bounds(n, m, k):
    s_star = bounds.crossover_sparsity(n, m, k, B)
    assert 0 < s_star < 1
    for s in (0.5 * s_star, 0.99 * s_star):
        assert bounds.psi_shac_bound(n, m, s, k, B) < bounds.psi_hac_bound(n, m, k, B)
    for s in (1.01 * s_star, min(1.0, 2 * s_star)):
        assert bounds.psi_shac_bound(n, m, s, k, B) > bounds.psi_hac_bound(n, m, k, B)
    assert math.isclose(bounds.psi_shac_bound(n, m, s_star, k, B),
                        bounds.psi_hac_bound(n, m, k, B), rel_tol=1e-12)


def test_csc_and_index_map_closed_forms(golden):
    # Example 1: q = 7, m = 5, n = 5 -> (14 + 6) / 25
    assert bounds.psi_csc(5, 5, 7) == 20 / 25
    n, m = 100, 40
    s_be = bounds.csc_break_even_s(n, m)
    q = int(s_be * n * m)
    assert bounds.psi_csc(n, m, q) <= 1 < bounds.psi_csc(n, m, q + 1)
    # "when k <= 256, b-bar = 8 and b = 32 the occupancy is about 1/4"
    assert abs(bounds.psi_index_map(4096, 4096, 256, 8, 32) - 0.25) < 1e-4


def test_measured_stream_is_well_below_the_bound_on_sparse_layers():
    # the paper reports actual sizes 2x-6x (HAC) under Corollary 1; same trend here
    W = workloads.scaled(4, 1568, 256)
    h = formats.hac_encode(W)
    k = len(h.values)
    assert 2.0 < bounds.corollary1_bits(W.shape[0], W.shape[1], k, B) / (h.nbits + 6 * k * B)
    H = huffman.entropy_bits(h.freqs)
    assert H * W.size <= h.nbits <= (H + 1) * W.size
