"""Pins for the oracle of the unified dictionary (Sect. V-H) and of the chain of layers."""
import numpy as np
import pytest

import workloads
from oracle import dot as odot
from oracle import formats, huffman, unified

from test_oracle_huffman import brute_force_min_cost


def small_layers(seed=3, shapes=((40, 30), (30, 20), (20, 12)), k=6, prune=0.7):
    """Layers quantized together: all draw from one set of k representatives."""
    rng = np.random.default_rng(seed)
    reps = np.sort(rng.normal(0, 0.1, k)).astype(np.float32)
    Ws = []
    for n, m in shapes:
        W = reps[rng.integers(0, k, size=(n, m))]
        W[rng.random((n, m)) < prune] = 0.0
        Ws.append(W.astype(np.float32))
    return Ws


def test_two_layer_example_worked_by_hand(golden):
    g = golden("unified_dictionary.txt")
    W0 = np.array([g["layer0_row0"], g["layer0_row1"]], dtype=np.float32)
    W1 = np.array([g["layer1_row0"], g["layer1_row1"]], dtype=np.float32)
    u = unified.unified_encode(["hac", "shac"], [W0, W1], reference_packer=True)
    assert u.values.tolist() == g["pooled_values"]
    assert u.freqs.tolist() == g["pooled_counts"]
    assert u.code.lengths == [int(v) for v in g["code_lengths"]]
    assert [s.nbits for s in u.layers] == [int(v) for v in g["layer_bits"]]
    assert [s.words.size for s in u.layers] == [int(v) for v in g["layer_words"]]
    assert unified.unified_paper_bits(u) == int(g["unified_bits"][0])
    assert unified.separate_paper_bits(["hac", "shac"], [W0, W1]) == int(g["separate_bits"][0])
    acts = unified.chain(np.array([g["chain_x"]]), [W0, W1],
                         [np.array(g["chain_bias0"]), None], [True, False])
    assert acts[0].tolist() == [g["chain_after0"]]
    assert acts[1].tolist() == [g["chain_after1"]]


@pytest.mark.parametrize("kinds", [("hac", "hac", "hac"), ("shac", "shac", "shac"), ("hac", "shac", "hac")])
def test_pooled_counts_and_shared_code(kinds):
    Ws = small_layers()
    u = unified.unified_encode(kinds, Ws)
    # counted directly, value by value
    total = 0
    for v, f in zip(u.values, u.freqs):
        c = 0
        for kind, W in zip(kinds, Ws):
            c += int(np.sum(W == v)) if (kind == "hac" or v != 0) else 0
        assert c == int(f)
        total += c
    assert total == sum(W.size if kind == "hac" else int(np.count_nonzero(W)) for kind, W in zip(kinds, Ws))
    # one code: prefix-free, complete, and every layer carries it
    assert huffman.is_prefix_free(u.code)
    num, den = huffman.kraft_numerator(u.code.lengths)
    assert num == den
    for s in u.layers:
        assert s.code is u.code and s.values is u.values
    # the bits of all streams together are the cost of the code on the pooled source
    assert sum(s.nbits for s in u.layers) == huffman.cost(u.freqs, u.code.lengths)
    H = huffman.entropy_bits(u.freqs)
    avg = sum(s.nbits for s in u.layers) / float(u.freqs.sum())
    assert H - 1e-12 <= avg <= H + 1


def test_shared_code_is_optimal_for_the_pool_only():
    Ws = small_layers(seed=5, k=5)
    kinds = ["hac", "shac", "hac"]
    u = unified.unified_encode(kinds, Ws)
    assert huffman.cost(u.freqs, u.code.lengths) == brute_force_min_cost(u.freqs.tolist())
    # no layer gets shorter than with a code of its own
    for kind, W, s in zip(kinds, Ws, u.layers):
        own = formats.hac_encode(W) if kind == "hac" else formats.shac_encode(W)
        assert s.nbits >= own.nbits
    # equal histograms up to a factor: the shared code costs each layer exactly its own optimum
    W = Ws[0]
    u2 = unified.unified_encode(["hac", "hac"], [W, np.concatenate([W, W], axis=1)])
    own = formats.hac_encode(W)
    assert u2.layers[0].nbits == own.nbits and u2.layers[1].nbits == 2 * own.nbits


@pytest.mark.parametrize("reference_packer", [False, True])
def test_round_trip_and_algorithms_on_shared_code(reference_packer):
    Ws = small_layers(seed=11, shapes=((17, 9), (9, 14), (14, 5)))
    kinds = ["hac", "shac", "shac"]
    u = unified.unified_encode(kinds, Ws, reference_packer=reference_packer)
    rng = np.random.default_rng(2)
    for l, (kind, W) in enumerate(zip(kinds, Ws)):
        assert np.array_equal(unified.unified_decode(u, l), W)
        x = rng.normal(size=W.shape[0])
        y = odot.dot_hac(u.layers[l], x) if kind == "hac" else odot.dot_shac(u.layers[l], x)
        ref = x @ W.astype(np.float64)
        assert np.allclose(y, ref, rtol=0, atol=1e-12 * max(1.0, np.abs(ref).max()))
    # both packers write the same words
    u_other = unified.unified_encode(kinds, Ws, reference_packer=not reference_packer)
    for a, b in zip(u.layers, u_other.layers):
        assert np.array_equal(a.words, b.words) and a.nbits == b.nbits


def test_dictionary_counted_once():
    # layers over one value set (zero and every representative occur in each): (L - 1) * 6kb saved
    rng = np.random.default_rng(8)
    reps = np.array([-0.5, 0.25, 1.0], dtype=np.float32)
    Ws = []
    for n, m in ((12, 10), (10, 8), (8, 6), (6, 9)):
        W = reps[rng.integers(0, 3, size=(n, m))]
        W[rng.random((n, m)) < 0.5] = 0.0
        W[0, 0], W[1, 0], W[2, 0], W[3, 0] = 0.0, reps[0], reps[1], reps[2]
        Ws.append(W)
    kinds = ["hac"] * 4
    u = unified.unified_encode(kinds, Ws)
    k = 4
    separate_words = sum(formats.hac_encode(W).N for W in Ws)
    unified_words = sum(s.N for s in u.layers)
    assert unified.separate_paper_bits(kinds, Ws) == 32 * separate_words + 4 * 6 * k * 32
    assert unified.unified_paper_bits(u) == 32 * unified_words + 6 * k * 32
    # the words themselves can only grow (a layer's own code is optimal for it)
    assert unified_words >= separate_words - len(Ws)      # rounding to whole words per layer


def test_index_map_layers_share_the_value_list():
    from oracle import indexmap
    rng = np.random.default_rng(12)
    Ws = small_layers(seed=41, shapes=((30, 20), (20, 16), (16, 9)), k=6, prune=0.6)
    conv = rng.choice(np.array([-0.75, -0.1, 0.3, 0.9, Ws[0][Ws[0] != 0][0]], dtype=np.float32), size=(27, 30))  # unpruned, one value shared
    kinds = ["im", "hac", "shac", "hac"]
    layers = [conv] + Ws
    u = unified.unified_encode(kinds, layers)
    # the code and the streams are those of the network without the index-map layer
    u0 = unified.unified_encode(kinds[1:], Ws)
    assert np.array_equal(u.values, u0.values) and np.array_equal(u.freqs, u0.freqs)
    assert u.code.lengths == u0.code.lengths
    for a, b in zip(u.layers[1:], u0.layers):
        assert np.array_equal(a.words, b.words)
    # extras: exactly the values no stream holds, ascending, appended after the alphabet
    assert u.extras.tolist() == sorted(set(np.unique(conv).tolist()) - set(u.values.tolist()))
    assert len(u.extras) == 4 and u.value_list.size == u.values.size + 4
    im = u.layers[0]
    assert im.bbar == 8 and int(im.pi.max()) < u.value_list.size
    assert np.array_equal(unified.unified_decode(u, 0), conv)
    assert np.array_equal(u.value_list[im.pi.astype(np.int64)], conv)
    x = rng.normal(size=(3, 27))
    assert np.allclose(indexmap.dot_im(im, x), x @ conv.astype(np.float64), rtol=0, atol=1e-12)
    # size: the other layers as before, bbar*n*m for the map, b per extra value
    assert unified.unified_paper_bits(u) == unified.unified_paper_bits(u0) + 8 * conv.size + 32 * 4
    # an extra 0.0 goes first among the extras; more than 256 values need 16-bit pointers
    convz = conv.copy(); convz[0, 0] = 0.0
    uz = unified.unified_encode(["im", "shac"], [convz, Ws[1]])
    assert uz.extras[0] == 0.0 and np.all(np.diff(uz.extras[1:]) > 0)
    assert np.array_equal(unified.unified_decode(uz, 0), convz)
    many = (np.arange(1, 301, dtype=np.float32) / 7).reshape(20, 15)
    um = unified.unified_encode(["im", "hac"], [many, Ws[0]])
    assert um.layers[0].bbar == 16 and np.array_equal(unified.unified_decode(um, 0), many)
    # alone, an index-map layer is the plain index map of Sect. III-C1
    alone = unified.unified_encode(["im"], [convz])
    ref = indexmap.im_encode(convz)
    assert alone.values.size == 0 and np.array_equal(alone.value_list, ref.c) and np.array_equal(alone.layers[0].pi, ref.pi)
    assert unified.unified_paper_bits(alone) == indexmap.im_bits(ref)


def test_chain_against_nested_products_and_linear_collapse():
    rng = np.random.default_rng(4)
    Ws = small_layers(seed=21, shapes=((25, 18), (18, 11), (11, 7)))
    bs = [rng.normal(size=18), None, rng.normal(size=7)]
    X = np.maximum(rng.normal(size=(5, 25)), 0)
    acts = unified.chain(X, Ws, bs, [True, True, False])
    a0 = np.maximum(X @ Ws[0].astype(np.float64) + bs[0], 0)
    a1 = np.maximum(a0 @ Ws[1].astype(np.float64), 0)
    a2 = a1 @ Ws[2].astype(np.float64) + bs[2]
    for got, ref in zip(acts, (a0, a1, a2)):
        assert np.array_equal(got, ref)
    # without activations and biases the chain is one matrix
    lin = unified.chain(X, Ws, [None] * 3, [False] * 3)[-1]
    M = Ws[0].astype(np.float64) @ Ws[1].astype(np.float64) @ Ws[2].astype(np.float64)
    assert np.allclose(lin, X @ M, rtol=1e-12, atol=1e-14)
    # an identity layer changes nothing; a negative bias under max(., 0) clamps
    I = np.eye(7, dtype=np.float32)
    ext = unified.chain(X, Ws + [I], bs + [None], [True, True, False, False])
    assert np.array_equal(ext[-1], acts[-1])
    clamp = unified.chain(X, Ws + [I], bs + [np.full(7, -1e9)], [True, True, False, True])
    assert np.count_nonzero(clamp[-1]) == 0


def test_chain_bound_covers_fp32_evaluation():
    # a float32 evaluation of the chain stays inside the bound for rel = 1e-5 and escapes a bound 1000x smaller
    rng = np.random.default_rng(6)
    Ws = small_layers(seed=31, shapes=((300, 200), (200, 150), (150, 40)), prune=0.5)
    bs = [rng.normal(size=200).astype(np.float32), rng.normal(size=150).astype(np.float32), None]
    relu = [True, True, False]
    X = np.maximum(rng.normal(size=(7, 300)), 0).astype(np.float32)
    ref = unified.chain(X, Ws, bs, relu)
    bound = unified.chain_bound(X, Ws, bs, relu, rel=1e-5)
    A = X
    for l, (W, b, r) in enumerate(zip(Ws, bs, relu)):
        A = A @ W
        if b is not None:
            A = A + b[None, :]
        if r:
            A = np.maximum(A, np.float32(0))
        assert A.dtype == np.float32
        err = np.abs(A.astype(np.float64) - ref[l])
        assert np.all(err <= bound[l])
    tight = unified.chain_bound(X, Ws, bs, relu, rel=1e-11, eps=0.0)
    assert np.any(err > tight[-1])
    # no error in, none allowed out: rel = 0 and eps = 0 give a zero bound
    zero = unified.chain_bound(X, Ws, bs, relu, rel=0.0, eps=0.0)
    assert all(np.count_nonzero(e) == 0 for e in zero)
