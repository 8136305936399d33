"""Pins for oracle.formats: CSC, HAC and sHAC encoders / decoders.

  * the paper's Example 1 (CSC arrays) and Example 2 (column-order sequence),
  * the stream lengths those examples force (derived by hand, see the fixture),
  * scipy's CSC arrays (an independent library routine),
  * bit-exact round trips on the edge cases and on configuration 1,
  * the array packer against the literally written-out packer,
  * the first bit of the stream is the top bit of word 0, padding bits are 0.
"""
import numpy as np
import pytest
import scipy.sparse

import workloads
from oracle import cnative, formats, huffman


def example_matrix(golden):
    return np.array(golden("example1_csc.txt")["W"], dtype=np.float32)


def test_example1_csc_arrays(golden):
    g = golden("example1_csc.txt")
    W = example_matrix(golden)
    nz, ri, cb = formats.csc_arrays(W)
    assert nz.tolist() == g["nz"]
    assert (ri + 1).tolist() == g["ri"]              # the paper counts from 1
    assert (cb + 1).tolist() == g["cb"]
    assert cb[-1] - cb[0] == len(nz)                 # cb_{m+1} = cb_1 + |nz|


def test_example2_column_order(golden):
    W = example_matrix(golden)
    seq = formats.column_order(W)
    assert seq.tolist() == golden("example2_address_map.txt")["sequence"]
    assert np.count_nonzero(seq == 0) == 18


def test_example_stream_lengths(golden):
    d = golden("example_derived.txt")
    W = example_matrix(golden)
    h = formats.hac_encode(W)
    assert h.nbits == int(d["hac_total_bits"][0])
    assert h.N == int(d["hac_words"][0])
    assert len(h.values) == 8 and h.values[0] == 0.0       # seven values plus the zero
    s = formats.shac_encode(W)
    assert s.nbits == int(d["shac_total_bits"][0])
    assert s.N1 == int(d["shac_words"][0])
    assert len(s.values) == 7
    assert np.array_equal(formats.hac_decode(h), W)
    assert np.array_equal(formats.shac_decode(s), W)


def test_bit_order_and_padding():
    # two symbols, zero more frequent: codes are 1 bit each; stream = one bit per entry
    W = np.array([[0.0], [2.0], [0.0], [0.0], [2.0]], dtype=np.float32)
    h = formats.hac_encode(W)
    bit_of = {v: h.code.codes[i][0] for i, v in enumerate(h.values.tolist())}
    expect = "".join(str(bit_of[v]) for v in W[:, 0].tolist())
    assert h.nbits == 5 and h.N == 1
    assert format(int(h.words[0]), "032b") == expect + "0" * 27


@pytest.mark.parametrize("name", sorted(workloads.edge_cases().keys()))
def test_round_trip_edge_cases(name):
    W = workloads.edge_cases()[name]
    h = formats.hac_encode(W)
    assert np.array_equal(formats.hac_decode(h).view(np.uint32), W.view(np.uint32))
    s = formats.shac_encode(W)
    assert np.array_equal(formats.shac_decode(s).view(np.uint32), W.view(np.uint32))
    assert s.q == np.count_nonzero(W)
    if s.q == 0:
        assert s.N1 == 0 and s.nbits == 0


def test_all_zero_matrix_is_one_bit_per_entry():
    W = workloads.edge_cases()["all_zero"]
    h = formats.hac_encode(W)
    assert h.nbits == W.size and h.values.tolist() == [0.0]


@pytest.mark.parametrize("nbits_mod", [0, 1])
def test_stream_length_multiple_of_word_and_one_more(nbits_mod):
    # all-zero column vectors: exactly one bit per entry
    W = np.zeros((64 + nbits_mod, 1), dtype=np.float32)
    h = formats.hac_encode(W)
    assert h.nbits == 64 + nbits_mod
    assert h.N == 2 + nbits_mod
    assert np.array_equal(formats.hac_decode(h), W)


def test_packers_agree_and_config1_round_trip():
    W = workloads.layer(1)
    h = formats.hac_encode(W)
    h_ref = formats.hac_encode(W[:, :20], reference_packer=True)
    h_arr = formats.hac_encode(W[:, :20])
    assert h_ref.nbits == h_arr.nbits and np.array_equal(h_ref.words, h_arr.words)
    s_ref = formats.shac_encode(W[:, :20], reference_packer=True)
    s_arr = formats.shac_encode(W[:, :20])
    assert s_ref.nbits == s_arr.nbits and np.array_equal(s_ref.words, s_arr.words)
    assert np.array_equal(formats.hac_decode(h).view(np.uint32), W.view(np.uint32))
    s = formats.shac_encode(W)
    assert np.array_equal(formats.shac_decode(s).view(np.uint32), W.view(np.uint32))
    # total bits = sum f_i l_i
    assert h.nbits == huffman.cost(h.freqs, h.code.lengths)
    assert s.nbits == huffman.cost(s.freqs, s.code.lengths)


def test_csc_matches_scipy():
    W = workloads.scaled(2, 257, 93)
    nz, ri, cb = formats.csc_arrays(W)
    ref = scipy.sparse.csc_matrix(W)
    ref.sort_indices()
    assert np.array_equal(nz, ref.data)
    assert np.array_equal(ri, ref.indices)
    assert np.array_equal(cb, ref.indptr)


def test_symbol_ground_truth_matches_decoded_stream():
    W = workloads.scaled(3, 300, 41)
    values, sym = formats.hac_symbols(W)
    h = formats.hac_encode(W)
    assert np.array_equal(values, h.values)
    assert np.array_equal(formats.unpack_stream(h.words, W.size, h.code), sym)
    values, sym, row, col = formats.shac_symbols(W)
    assert np.array_equal(W[row, col], values[sym])
    s = formats.shac_encode(W)
    assert np.array_equal(formats.unpack_stream(s.words, s.q, s.code), sym)


def test_c_oracle_matches_python_oracle():
    for W in (workloads.scaled(1, 211, 57), workloads.scaled(3, 190, 77),
              workloads.edge_cases()["empty_columns"], workloads.edge_cases()["dense_no_zero"]):
        hp, hc = formats.hac_encode(W), cnative.hac_encode(W)
        assert hp.nbits == hc.nbits and np.array_equal(hp.words, hc.words)
        sp, sc = formats.shac_encode(W), cnative.shac_encode(W)
        assert sp.nbits == sc.nbits and np.array_equal(sp.words, sc.words)
        assert np.array_equal(sp.ri, sc.ri) and np.array_equal(sp.cb, sc.cb)
        assert np.array_equal(cnative.unpack(hc.words, W.size, hc.code),
                              formats.unpack_stream(hp.words, W.size, hp.code))


def test_stream_ending_early_is_an_error():
    W = workloads.scaled(1, 64, 8)
    h = formats.hac_encode(W)
    with pytest.raises(ValueError):
        formats.unpack_stream(h.words[:-1], W.size, h.code)
