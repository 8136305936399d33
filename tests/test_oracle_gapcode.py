"""Pins for the oracle of the gap-coded sHAC address map (an extension of Sect. IV-C)."""
import itertools

import numpy as np
import pytest

import workloads
from oracle import dot as odot
from oracle import formats, gapcode, huffman


def bits_of(vals):
    return "".join(str(int(v)) for v in vals)


def test_handwritten_codewords(golden):
    g = golden("rice_gap_code.txt")
    for key, val in g.items():
        if not key.startswith("k") or key.endswith("_length"):
            continue
        k, d = int(key[1:key.index("_")]), int(key[key.index("_d") + 2:])
        assert gapcode.rice_bits(d, k) == bits_of(val), key
        assert gapcode.rice_length(d, k) == len(val), key
    assert gapcode.rice_length(495, 4) == int(g["k4_d495_length"][0])
    assert gapcode.rice_length(496, 4) == int(g["k4_d496_length"][0])
    assert gapcode.rice_length(31, 0) == int(g["k0_d31_length"][0])
    assert gapcode.rice_length(30, 0) == int(g["k0_d30_length"][0])
    esc = gapcode.rice_bits(31, 0)
    assert esc == "0" * 31 + "1" + format(31, "032b")


@pytest.mark.parametrize("k", [0, 1, 2, 3, 5])
def test_lengths_closed_form_and_prefix_free(k):
    lim = 31 << k
    words = [gapcode.rice_bits(d, k) for d in range(min(lim + 40, 1200))]
    for d, w in enumerate(words):
        q = d >> k
        assert len(w) == (q + 1 + k if q < 31 else 64)
        assert len(w) == gapcode.rice_length(d, k)
        assert int(gapcode.rice_lengths(np.array([d]), k)[0]) == len(w)
    # no codeword is a prefix of another
    srt = sorted(words)
    for a, b in zip(srt, srt[1:]):
        assert not b.startswith(a)
    # Kraft: the plain forms fill 1 - 2^-31 of the code space, all escapes together 2^-32 * 2^32 * 2^-32
    kraft = sum(2.0 ** -(q + 1 + k) for q in range(31)) * (1 << k)
    assert abs(kraft - (1 - 2.0 ** -31)) < 1e-12


def test_paper_example_worked_by_hand(golden):
    g = golden("rice_gap_code.txt")
    W = workloads.paper_example_matrix()
    nz, ri, cb = formats.csc_arrays(W)
    d = gapcode.column_gaps(ri, cb)
    assert d.tolist() == [int(v) for v in g["example1_gaps"]]
    assert np.array_equal(d, gapcode.column_gaps_fast(ri, cb))
    assert gapcode.best_k(d) == int(g["example1_best_k"][0])
    s = gapcode.shacg_encode(W)
    assert s.k == 0 and s.gap_bits == int(g["example1_gap_bits"][0])
    assert s.nbits == int(g["example1_total_bits"][0]) and s.N == int(g["example1_words"][0])
    # the two packers agree, and the stream starts with gap "1" followed by the first value's codeword
    r = gapcode.shacg_encode(W, reference_packer=True)
    assert np.array_equal(r.words, s.words) and r.nbits == s.nbits
    first = s.code.codeword_strings()[int(formats.symbol_indices(nz, s.values)[0])]
    assert format(int(s.words[0]), "032b").startswith("1" + first)
    assert np.array_equal(gapcode.shacg_decode(s), W)
    assert np.allclose(gapcode.dot_shacg(s, np.ones(5)), [3, 13, 4, 0, 11])


def all_cases():
    for name, W in workloads.edge_cases().items():
        yield name, W
    yield "cfg1", workloads.layer(1)
    yield "cfg2-300x40", workloads.scaled(2, 300, 40)
    yield "cfg4-2500x12", workloads.scaled(4, 2500, 12)
    yield "cfg5-200x30", workloads.scaled(5, 200, 30)


@pytest.mark.parametrize("name,W", list(all_cases()), ids=[c[0] for c in all_cases()])
def test_lossless_and_consistent(name, W):
    s = gapcode.shacg_encode(W)
    values, sym, row, col, d = gapcode.shacg_symbols(W)
    dsym, drow, dcol = gapcode.shacg_decode_csc(s)
    assert np.array_equal(dsym, sym) and np.array_equal(drow, row) and np.array_equal(dcol, col)
    Wd = gapcode.shacg_decode(s)
    assert np.array_equal(Wd.view(np.uint32), huffman.normalise_values(W).view(np.uint32))
    # bits: gap part + value part, the value part being sHAC's stream length
    sh = formats.shac_encode(W)
    assert s.nbits == s.gap_bits + sh.nbits
    assert s.gap_bits == int(gapcode.rice_lengths(d, s.k).sum())
    assert s.N == -(-s.nbits // 32)
    if W.size <= 4000:
        r = gapcode.shacg_encode(W, reference_packer=True)
        assert np.array_equal(r.words, s.words) and r.k == s.k


def test_best_k_is_the_exhaustive_minimum():
    rng = np.random.default_rng(5)
    for mean in (0.3, 2.0, 17.0, 400.0, 9000.0):
        d = rng.geometric(1.0 / (1.0 + mean), size=3000) - 1
        totals = [sum(gapcode.rice_length(int(x), k) for x in d) for k in range(16)]
        assert gapcode.best_k(d) == int(np.argmin(totals))
        for k in (0, 3, 7):
            s_fast = int(gapcode.rice_lengths(d, k).sum())
            assert s_fast == totals[k]


def test_expected_length_for_geometric_gaps():
    """Gaps of a Bernoulli(s) column are geometric; a Rice code then costs k + 1/(1 - (1-s)^(2^k))
    bits on average (quotient geometric with success probability 1 - (1-s)^(2^k))."""
    rng = np.random.default_rng(11)
    n, m, s = 200000, 4, 0.02
    W = np.zeros((n, m), dtype=np.float32)
    W[rng.random((n, m)) < s] = 1.0
    enc = gapcode.shacg_encode(W)
    k = enc.k
    expect = {kk: kk + 1.0 / (1.0 - (1.0 - s) ** (2 ** kk)) for kk in range(16)}
    assert k == min(expect, key=expect.get)                       # the formula's own best k
    per_gap = enc.gap_bits / enc.q
    assert abs(per_gap - expect[k]) / expect[k] < 0.01
    # within 5 % of the entropy of the gap distribution, H(s)/s bits
    h = (-s * np.log2(s) - (1 - s) * np.log2(1 - s)) / s
    assert h <= per_gap <= 1.05 * h


def test_brute_force_decoding_of_tiny_streams():
    """Every way of cutting the bit string into (gap, value) codewords that is consistent with the
    code tables yields the same parse: try all splits for tiny matrices."""
    rng = np.random.default_rng(3)
    for _ in range(20):
        W = np.zeros((6, 3), dtype=np.float32)
        mask = rng.random(W.shape) < 0.4
        W[mask] = rng.choice(np.array([0.5, 1.0, 2.0], dtype=np.float32), size=int(mask.sum()))
        s = gapcode.shacg_encode(W, k=1, reference_packer=True)
        bits = "".join(format(int(w), "032b") for w in s.words)[:s.nbits]
        cws = s.code.codeword_strings()
        gapwords = {gapcode.rice_bits(d, 1): d for d in range(6)}

        def parses(pos, left):
            if left == 0:
                return [[]] if pos == len(bits) else []
            out = []
            for gw, d in gapwords.items():
                if bits.startswith(gw, pos):
                    for sy, cw in enumerate(cws):
                        if bits.startswith(cw, pos + len(gw)):
                            for rest in parses(pos + len(gw) + len(cw), left - 1):
                                out.append([(d, sy)] + rest)
            return out

        found = parses(0, s.q)
        assert len(found) == 1
        values, sym, row, col, d = gapcode.shacg_symbols(W)
        assert [p[0] for p in found[0]] == d.tolist() and [p[1] for p in found[0]] == sym.tolist()


def test_dot_matches_dense_and_size_is_below_corollary_2():
    from oracle import bounds
    for cfg, shape in ((1, None), (2, (400, 60)), (4, (3000, 20))):
        W = workloads.layer(cfg) if shape is None else workloads.scaled(cfg, *shape)
        n, m = W.shape
        s = gapcode.shacg_encode(W)
        x = workloads.make_batch(1, n, 9)[0] - np.float32(0.25)
        ref = odot.dense_dot(x[None, :], W)[0]
        got = gapcode.dot_shacg(s, x)
        assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)
        sh = formats.shac_encode(W)
        assert gapcode.shacg_paper_bits(s) < formats.shac_paper_bits(sh)
        k = len(s.values)
        assert gapcode.shacg_paper_bits(s) <= bounds.corollary2_bits(n, m, s.q, k)


def test_gap_code_beats_fixed_width_fields_on_the_five_configs_shapes():
    for cfg, shape in ((1, None), (2, (2048, 100)), (3, (2048, 100)), (4, (25088, 16)), (5, (4608, 16))):
        W = workloads.layer(cfg) if shape is None else workloads.scaled(cfg, *shape)
        n = W.shape[0]
        s = gapcode.shacg_encode(W)
        fixed = s.q * max(1, int(np.ceil(np.log2(n))))
        assert s.gap_bits < fixed
