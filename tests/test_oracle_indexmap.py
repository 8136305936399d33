"""Pins for the oracle's index map (Sect. III-C1)."""
import numpy as np
import pytest

import workloads
from oracle import bounds, formats, indexmap
from oracle import dot as odot


def test_paper_example_matrix_by_hand():
    # Example 1's matrix holds the values 0 1 2 3 4 5 6 10 -> pointers 0..7 in that order
    W = workloads.paper_example_matrix()
    im = indexmap.im_encode(W)
    assert im.c.tolist() == [0, 1, 2, 3, 4, 5, 6, 10] and im.bbar == 8
    expect = np.array([[1, 0, 4, 0, 0],
                       [0, 7, 0, 0, 0],
                       [2, 3, 0, 0, 5],
                       [0, 0, 0, 0, 0],
                       [0, 0, 0, 0, 6]])
    assert np.array_equal(im.pi, expect)
    assert np.array_equal(indexmap.im_decode(im), W)
    assert np.allclose(indexmap.dot_im(im, np.ones((1, 5))), [[3, 13, 4, 0, 11]])
    # occupancy: (8*25 + 8*32) / (32*25)
    assert indexmap.im_bits(im) == 8 * 25 + 8 * 32
    assert indexmap.im_bits(im) / (32 * 25) == pytest.approx(bounds.psi_index_map(5, 5, 8, 8))


def cases():
    for name, W in workloads.edge_cases().items():
        yield name, W
    yield "cfg1", workloads.layer(1)
    yield "cfg5-300x70", workloads.scaled(5, 300, 70)
    yield "no_repeats", workloads.stress_cases()["no_repeats_40x30"]


@pytest.mark.parametrize("name,W", list(cases()), ids=[c[0] for c in cases()])
def test_round_trip_symbols_and_product(name, W):
    im = indexmap.im_encode(W)
    n, m = W.shape
    assert np.array_equal(indexmap.im_decode(im).view(np.uint32), (W + np.float32(0)).view(np.uint32))
    values, sym = formats.hac_symbols(W)                       # same numbering as the HAC alphabet
    assert np.array_equal(im.c, values)
    assert np.array_equal(im.pi.astype(np.int64), sym.reshape(m, n).T)
    assert im.bbar == (8 if len(values) <= 256 else 16)
    assert indexmap.im_bits(im) / (32.0 * n * m) == pytest.approx(bounds.psi_index_map(n, m, len(values), im.bbar))
    X = workloads.make_batch(5, n, 3) - np.float32(0.3)
    assert np.allclose(indexmap.dot_im(im, X), odot.dense_dot(X, W), rtol=1e-12, atol=1e-12)


def test_quarter_occupancy_for_eight_bit_pointers():
    # quantized without pruning, as the paper does for convolutional layers: exactly k = 256 pointers
    W = workloads.make_layer(512, 256, 0.02, 0.0, 256, "kmeans", 12)
    im = indexmap.im_encode(W)
    assert im.bbar == 8 and im.c.size <= 256
    psi = indexmap.im_bits(im) / (32.0 * W.size)
    assert 0.25 < psi < 0.26                                   # "about 1/4" for k <= 256 and FP32 weights
