"""The synthetic layers have the structure the configurations name: sparsity,
number of shared values, exact zeros, determinism."""
import numpy as np
import pytest

import workloads


@pytest.mark.parametrize("cfg", [1, 2])
def test_layer_structure(cfg):
    c = workloads.CONFIGS[cfg]
    W = workloads.layer(cfg)
    assert W.shape == (c.n, c.m) and W.dtype == np.float32 and W.flags.c_contiguous
    nnz = np.count_nonzero(W)
    assert abs(nnz / W.size - (1 - c.prune)) < 1e-3
    shared = np.unique(W[W != 0])
    assert 2 <= shared.size <= c.k
    assert not np.any(np.signbit(W[W == 0]))
    assert np.array_equal(W, workloads.layer(cfg))          # same seed, same matrix


def test_batch_structure():
    X = workloads.batch(1)
    assert X.shape == (8, 500) and X.dtype == np.float32
    assert X.min() == 0.0 and 0.4 < np.mean(X == 0) < 0.6    # ReLU of a centred Gaussian
    assert np.array_equal(X, workloads.batch(1))


def test_pruning_keeps_strictly_larger_magnitudes():
    w = np.array([[0.1, -0.2, 0.2, 0.3, -0.4, 0.05]], dtype=np.float32)
    keep = workloads.prune_magnitude(w, 0.5)                 # 3 smallest |w| go: 0.05, 0.1, one 0.2
    assert keep.tolist() == [[False, False, False, True, True, False]]  # the tie at 0.2 is pruned too


def test_quantizers():
    v = np.linspace(-1, 1, 101).astype(np.float32)
    u = workloads.share_uniform(v, 4)
    assert np.unique(u).tolist() == [-0.75, -0.25, 0.25, 0.75]
    km = workloads.share_kmeans(np.array([0.0, 0.1, 0.2, 5.0, 5.1, 5.2], dtype=np.float32), 2)
    assert np.allclose(np.unique(km), [0.1, 5.1])
