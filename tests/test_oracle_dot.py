"""Pins for oracle.dot (Algorithms 1-3) and its C twin.

  * the dense fp64 product (numpy), which is what all three algorithms output,
  * scipy's CSC product (the paper's own reference for sparse dots),
  * the paper's 5x5 example: 1^T W = (3, 13, 4, 0, 11), column 4 empty,
  * identity batches recover W exactly (one term per sum),
  * linearity in X,
  * a transposed operand, a dropped empty-column step or a decoded padding bit
    would each break one of the above.
"""
import numpy as np
import pytest
import scipy.sparse

import workloads
from oracle import cnative, dot, formats, huffman


def example_matrix(golden):
    return np.array(golden("example1_csc.txt")["W"], dtype=np.float32)


def test_example_ones_vector(golden):
    W = example_matrix(golden)
    expect = golden("example_derived.txt")["ones_dot"]
    x = np.ones(5, dtype=np.float32)
    assert dot.dot_hac(formats.hac_encode(W), x).tolist() == expect
    assert dot.dot_shac(formats.shac_encode(W), x).tolist() == expect
    assert cnative.pardot(cnative.hac_encode(W), x)[0].tolist() == expect
    assert cnative.pardot(cnative.shac_encode(W), x)[0].tolist() == expect


def test_non_square_shapes_are_not_transposed():
    W = workloads.scaled(1, 37, 11)
    x = workloads.make_batch(1, 37, 3)[0]
    ref = dot.dense_dot(x[None, :], W)[0]
    assert ref.shape == (11,)
    np.testing.assert_allclose(dot.dot_hac(formats.hac_encode(W), x), ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dot.dot_shac(formats.shac_encode(W), x), ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("name", sorted(workloads.edge_cases().keys()))
def test_edge_cases_against_dense(name):
    W = workloads.edge_cases()[name]
    n, m = W.shape
    X = workloads.make_batch(3, n, 99) + np.float32(0.25)
    ref = dot.dense_dot(X, W)
    for enc in (formats.hac_encode, formats.shac_encode):
        got = dot.pardot(enc(W), X, q=2)
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    for enc in (cnative.hac_encode, cnative.shac_encode):
        got = cnative.pardot(enc(W), X, q=2)
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_identity_batch_recovers_w_exactly():
    W = workloads.scaled(2, 23, 17)
    eye = np.eye(23, dtype=np.float32)
    for enc in (formats.hac_encode, formats.shac_encode):
        got = dot.pardot(enc(W), eye, q=3)
        assert np.array_equal(got, W.astype(np.float64))
    assert np.array_equal(cnative.pardot(cnative.hac_encode(W), eye, q=4), W.astype(np.float64))
    assert np.array_equal(cnative.pardot(cnative.shac_encode(W), eye, q=4), W.astype(np.float64))


def test_linearity():
    W = workloads.scaled(3, 150, 40)
    X1 = workloads.make_batch(2, 150, 1).astype(np.float64)
    X2 = workloads.make_batch(2, 150, 2).astype(np.float64)
    a = 0.375
    h = formats.hac_encode(W)
    f = lambda X: np.stack([dot.dot_hac(h, x) for x in X])
    np.testing.assert_allclose(f(a * X1 + X2), a * f(X1) + f(X2), rtol=1e-12, atol=1e-12)


def test_config1_c_oracle_against_dense_and_scipy():
    W = workloads.layer(1)
    X = workloads.batch(1)
    ref = dot.dense_dot(X, W)
    tol = 1e-12 * dot.abs_dot(X, W).max()
    yh = cnative.pardot(cnative.hac_encode(W), X, q=4)
    ys = cnative.pardot(cnative.shac_encode(W), X, q=4)
    assert np.abs(yh - ref).max() <= tol
    assert np.abs(ys - ref).max() <= tol
    sp = (scipy.sparse.csc_matrix(W.astype(np.float64)).T @ X.astype(np.float64).T).T
    assert np.abs(ys - sp).max() <= tol


def test_python_and_c_algorithms_agree_on_a_slice_of_config1():
    W = workloads.layer(1)[:, :12]
    X = workloads.batch(1)[:2]
    for penc, cenc in ((formats.hac_encode, cnative.hac_encode),
                       (formats.shac_encode, cnative.shac_encode)):
        yp = dot.pardot(penc(W), X, q=2)
        yc = cnative.pardot(cenc(W), X, q=2)
        np.testing.assert_allclose(yp, yc, rtol=0, atol=1e-13)


def test_pardot_chunking_covers_every_row_once():
    W = workloads.scaled(1, 30, 9)
    X = workloads.make_batch(7, 30, 5)
    ref = dot.dense_dot(X, W)
    h = cnative.hac_encode(W)
    for q in (1, 2, 3, 7, 8, 16):
        np.testing.assert_allclose(cnative.pardot(h, X, q=q), ref, rtol=0, atol=1e-12)
    hp = formats.hac_encode(W)
    for q in (1, 3, 10):
        np.testing.assert_allclose(dot.pardot(hp, X, q=q), ref, rtol=0, atol=1e-12)


def test_codeword_straddling_two_words_is_decoded_once():
    # 30 one-bit codewords, then "110" across the word boundary, then "10"
    code = huffman.HuffmanCode(4, [2, 1, 0], [3, 4, 5], 6, [(0, 1), (2, 2), (6, 3), (7, 3)])
    assert code.decoding_dictionary() == {"0": 0, "10": 1, "110": 2, "111": 3}
    words = np.array([0b11, 0b010 << 29], dtype=np.uint32)
    stream = dot.codewords(words, code)
    assert [next(stream) for _ in range(32)] == [0] * 30 + [2, 1]


# ---- decode once, threads over columns (the per-column offsets of the paper's conclusions) ----

def test_column_offsets_are_the_cumulated_code_lengths():
    W = workloads.scaled(1, 70, 23)
    n, m = W.shape
    h = cnative.hac_encode(W)
    lens = np.array([l for _, l in h.code.codes], dtype=np.int64)
    values, sym = formats.hac_symbols(W)
    per_col = lens[sym].reshape(m, n).sum(axis=1)
    assert cnative.column_offsets(h).tolist() == np.concatenate(([0], np.cumsum(per_col))).tolist()
    s = cnative.shac_encode(W)
    slens = np.array([l for _, l in s.code.codes], dtype=np.int64)
    svalues, ssym, srow, scol = formats.shac_symbols(W)
    per_col = np.bincount(scol, weights=slens[ssym], minlength=m).astype(np.int64)
    assert cnative.column_offsets(s).tolist() == np.concatenate(([0], np.cumsum(per_col))).tolist()
    assert cnative.column_offsets(h)[-1] == h.nbits and cnative.column_offsets(s)[-1] == s.nbits


@pytest.mark.parametrize("name", sorted(workloads.edge_cases()) + ["cfg1-slice", "cfg5-slice"])
def test_column_parallel_dot_is_the_dense_product(name):
    if name == "cfg1-slice":
        W = workloads.scaled(1, 120, 37)
    elif name == "cfg5-slice":
        W = workloads.scaled(5, 90, 21)
    else:
        W = workloads.edge_cases()[name]
    X = workloads.make_batch(5, W.shape[0], 31)
    X[2] = -X[2]                                              # signs on both sides
    ref = dot.dense_dot(X, W)
    for enc in (cnative.hac_encode, cnative.shac_encode):
        st = enc(W)
        one = cnative.coldot(st, X, q=1)
        np.testing.assert_allclose(one, ref, rtol=0, atol=1e-12 * max(1.0, float(np.abs(ref).max())))
        for q in (2, 3, 64):                                  # the split over threads changes nothing, bit for bit
            assert np.array_equal(cnative.coldot(st, X, q=q), one)
        # and it is Algorithm 3's result (same products, same order within a column)
        np.testing.assert_allclose(one, cnative.pardot(st, X, q=2), rtol=0, atol=1e-12 * max(1.0, float(np.abs(ref).max())))


def test_column_parallel_dot_identity_and_shape():
    W = workloads.edge_cases()["empty_columns"]
    eye = np.eye(W.shape[0], dtype=np.float32)
    for enc in (cnative.hac_encode, cnative.shac_encode):
        assert np.array_equal(cnative.coldot(enc(W), eye, q=3), W.astype(np.float64))
    W = workloads.scaled(2, 33, 7)                             # n != m: a transposed operand cannot pass
    X = workloads.make_batch(4, 33, 2)
    assert cnative.coldot(cnative.hac_encode(W), X, q=2).shape == (4, 7)
