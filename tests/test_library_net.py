"""Host side of the network blob (one dictionary for all layers, Sect. V-H) against the oracle."""
import ctypes as C

import numpy as np
import pytest

import paper_2108_12704_amd as hac
from oracle import formats, gapcode, huffman, unified

from test_library_host import codes_from_blob, header_fields, oracle_decode_bits
from test_oracle_unified import small_layers

KIND = {hac.HAC_FORMAT_HAC: "hac", hac.HAC_FORMAT_SHAC: "shac", hac.HAC_FORMAT_IM: "im"}


def test_net_structs_match_binding():
    assert header_fields("hac_net_t") == [f[0] for f in hac.Net._fields_]
    assert header_fields("hac_net_stats_t") == [f[0] for f in hac.NetStats._fields_]
    assert C.sizeof(hac.Net) == 256 and C.sizeof(hac.Desc) == 256


class _LayerView:
    """What codes_from_blob needs, for the shared tables of a network blob."""

    def __init__(self, nb, desc):
        self.desc, self._nb = desc, nb

    def section(self, off_field, dtype, count):
        return self._nb.section(self.desc, off_field, dtype, count)


@pytest.mark.parametrize("fmts,ri_coding", [
    ((1, 1, 1), 0), ((2, 2, 2), 0), ((1, 2, 1), 0), ((2, 1, 2), 1), ((2, 2, 2), 1)])
def test_net_blob_against_oracle(fmts, ri_coding):
    Ws = small_layers(seed=13, shapes=((60, 33), (33, 41), (41, 9)), k=9, prune=0.8)
    nb = hac.hac_net_encode(Ws, fmts, ri_coding=ri_coding)
    assert nb.validate(deep=True) == 0
    kinds = [KIND[f] for f in fmts]
    u = unified.unified_encode(kinds, Ws)
    net = nb.net
    assert net.n_layers == 3 and net.k_sym == len(u.values) and net.has_zero == int(u.values[0] == 0.0)
    cb = nb.section(nb.layers[0], "off_codebook", np.float32, int(net.k_sym))
    assert np.array_equal(cb, u.values)
    lens, words = codes_from_blob(_LayerView(nb, nb.layers[0]))
    # any optimal code has the oracle's cost on the pooled counts
    assert huffman.cost(u.freqs, lens) == huffman.cost(u.freqs, u.code.lengths)
    assert max(lens) == net.lmax
    total = 0
    for l, (d, kind, W) in enumerate(zip(nb.layers, kinds, Ws)):
        assert d.dict_shared == 1 and d.blob_bytes == nb.nbytes
        assert (d.n, d.m) == W.shape and d.nnz == np.count_nonzero(W)
        for f in ("off_codebook", "off_codelen", "off_canon", "off_symsort", "off_lut"):
            assert getattr(d, f) == getattr(net, f)
        # symbols of the layer's stream, decoded bit by bit with the shared code's dictionary
        stream = nb.section(d, "off_stream", np.uint32, int(d.n_words))
        if kind == "hac":
            sym_ref = formats.symbol_indices(formats.column_order(W), u.values)
            assert d.total_bits == int(np.sum(lens[sym_ref]))
            assert np.array_equal(oracle_decode_bits(stream, sym_ref.size, words), sym_ref)
            Wd, sym = nb.decode_host(l)
            assert np.array_equal(sym, sym_ref)
        else:
            nz, ri, cbeg = formats.csc_arrays(W)
            sym_ref = formats.symbol_indices(nz, u.values)
            Wd, sym, row, col = nb.decode_host(l)
            assert np.array_equal(sym, sym_ref) and np.array_equal(row, ri)
            assert np.array_equal(nb.section(d, "off_col_pos", np.uint32, W.shape[1] + 1), cbeg)
            if ri_coding:
                gaps = gapcode.column_gaps(ri, cbeg)
                assert d.rice_k == gapcode.best_k(gaps)
                assert d.gap_bits == int(gapcode.rice_lengths(gaps, int(d.rice_k)).sum())
                assert d.total_bits == int(np.sum(lens[sym_ref])) + d.gap_bits
            else:
                assert d.total_bits == int(np.sum(lens[sym_ref]))
                assert np.array_equal(oracle_decode_bits(stream, sym_ref.size, words), sym_ref)
        assert np.array_equal(Wd, W)
        total += int(d.total_bits) - int(d.gap_bits)
    assert total == huffman.cost(u.freqs, u.code.lengths)
    st = nb.stats()
    assert st.n_layers == 3 and st.entries == sum(W.size for W in Ws) and st.nnz == sum(np.count_nonzero(W) for W in Ws)
    assert st.symbols == int(u.freqs.sum())
    assert abs(st.entropy_bits - huffman.entropy_bits(u.freqs)) < 1e-12
    assert st.entropy_bits - 1e-12 <= st.avg_code_bits <= st.entropy_bits + 1
    if not ri_coding:
        assert st.paper_bits == unified.unified_paper_bits(u)
        assert st.stream_bits == sum(s.nbits for s in u.layers)


def hybrid_layers(seed=12, zero_in_map=False):
    """An unpruned 'convolutional' matrix over a few representatives (one of them shared with the
    pruned layers) in front of three pruned layers."""
    rng = np.random.default_rng(seed)
    Ws = small_layers(seed=41, shapes=((30, 20), (20, 16), (16, 9)), k=6, prune=0.6)
    reps = np.array([-0.75, -0.1, 0.3, 0.9, Ws[0][Ws[0] != 0][0]], dtype=np.float32)
    conv = rng.choice(reps, size=(27, 30))
    if zero_in_map:
        conv[rng.random(conv.shape) < 0.1] = 0.0
    return [conv] + Ws


@pytest.mark.parametrize("fmts,zero_in_map", [((3, 1, 2, 1), False), ((3, 2, 2, 2), True), ((3, 1, 1, 2), True),
                                               ((3, 3, 2, 2), False)])
def test_index_map_layers_in_a_network_blob(fmts, zero_in_map):
    layers = hybrid_layers(zero_in_map=zero_in_map)
    nb = hac.hac_net_encode(layers, fmts)
    assert nb.validate(deep=True) == 0
    u = unified.unified_encode([KIND[f] for f in fmts], layers)
    net = nb.net
    assert net.k_sym == len(u.values) and net.k_values == u.value_list.size
    assert np.array_equal(nb.section(nb.layers[0], "off_codebook", np.float32, int(net.k_values)), u.value_list)
    for l, (f, W, d) in enumerate(zip(fmts, layers, nb.layers)):
        if f != hac.HAC_FORMAT_IM:
            assert np.array_equal(nb.decode_host(l)[0], W)
            assert d.total_bits == u.layers[l].nbits
            continue
        im = u.layers[l]
        assert d.dict_shared == 1 and d.k_sym == net.k_values and d.ent_bits == im.bbar
        assert d.total_bits == im.bbar * W.size and d.nnz == np.count_nonzero(W)
        Wd, ptr = nb.decode_host(l)
        assert np.array_equal(Wd, W)
        assert np.array_equal(ptr.reshape(W.shape[1], W.shape[0]).T, im.pi)
        # padding columns of the map hold 0
        pitch = int(d.idx_pitch)
        raw = nb.section(d, "off_stream", np.uint8 if d.ent_bits == 8 else np.uint16, W.shape[0] * pitch).reshape(W.shape[0], pitch)
        assert np.array_equal(raw[:, :W.shape[1]], im.pi) and not raw[:, W.shape[1]:].any()
    st = nb.stats()
    assert st.paper_bits == unified.unified_paper_bits(u)
    assert st.entries == sum(W.size for W in layers) and st.symbols == int(u.freqs.sum())
    if u.freqs.size:
        assert abs(st.entropy_bits - huffman.entropy_bits(u.freqs)) < 1e-12


def test_network_of_index_maps_only_and_wide_pointers():
    from oracle import indexmap
    conv = hybrid_layers(zero_in_map=True)[0]
    nb = hac.hac_net_encode([conv, conv.T.copy()], (3, 3))
    assert nb.validate(deep=True) == 0 and nb.net.k_sym == 0
    ref = indexmap.im_encode(conv)
    assert np.array_equal(nb.section(nb.layers[0], "off_codebook", np.float32, int(nb.net.k_values)), ref.c)
    assert np.array_equal(nb.decode_host(0)[1].reshape(conv.shape[1], conv.shape[0]).T, ref.pi)
    many = (np.arange(1, 301, dtype=np.float32) / 7).reshape(20, 15)
    W = small_layers(seed=3, shapes=((15, 8),))[0]
    nb = hac.hac_net_encode([many, W], (3, 1))
    assert nb.validate(deep=True) == 0 and nb.layers[0].ent_bits == 16
    assert np.array_equal(nb.decode_host(0)[0], many) and np.array_equal(nb.decode_host(1)[0], W)
    u = unified.unified_encode(["im", "hac"], [many, W])
    assert nb.stats().paper_bits == unified.unified_paper_bits(u)


def test_damaged_value_list_and_index_map_are_rejected():
    lib = hac.load_library()
    layers = hybrid_layers(zero_in_map=True)
    nb = hac.hac_net_encode(layers, (3, 2, 2, 2))
    good = nb.data
    assert nb.net.k_values > nb.net.k_sym and nb.net.has_zero == 0

    def check(mutate, deep=1):
        b = good.copy()
        mutate(b)
        return lib.hac_net_validate(b.ctypes.data, b.size, deep)

    cb_off, k, kv = int(nb.net.off_codebook), int(nb.net.k_sym), int(nb.net.k_values)

    def poke_value(i, v):
        def f(b): b[cb_off + 4 * i:cb_off + 4 * i + 4].view(np.float32)[0] = v
        return f

    cb = good[cb_off:cb_off + 4 * kv].view(np.float32)
    assert cb[k] == 0.0                                              # the extra 0.0 comes first
    assert check(poke_value(k + 1, np.nan), 0) == -3
    assert check(poke_value(k + 2, cb[k + 1]), 0) == -3              # not ascending
    assert check(poke_value(kv - 1, cb[0]), 0) == -3                 # repeats a shared symbol's value
    assert check(poke_value(kv - 1, 0.0), 0) == -3                   # 0.0 anywhere but first
    d0 = nb.layers[0]
    off = int(d0.off_stream)

    def poke_map(at, v):
        def f(b): b[off + at] = v
        return f

    assert check(poke_map(0, kv)) == -3                              # pointer past the list
    assert check(poke_map(int(d0.m), 1)) == -3                       # padding column not 0
    first_nz = int(np.flatnonzero(layers[0][0] != 0)[0])
    assert check(poke_map(first_nz, k)) == -3                        # a non-zero turned into 0.0: nnz no longer matches
    net_off = {f[0]: getattr(hac.Net, f[0]).offset for f in hac.Net._fields_}

    def set_u32(o, v):
        def f(b): b[o:o + 4].view(np.uint32)[0] = v
        return f

    assert check(set_u32(net_off["k_values"], kv + 1)) == -3
    assert check(set_u32(net_off["k_values"], k - 1 if k else 0xffffffff)) == -3
    assert check(set_u32(net_off["reserved32"], 1)) == -3


def test_single_layer_net_has_the_layers_own_stream():
    W = small_layers(seed=2)[0]
    for fmt, enc in ((hac.HAC_FORMAT_HAC, hac.hac_encode), (hac.HAC_FORMAT_SHAC, hac.shac_encode)):
        nb = hac.hac_net_encode([W], [fmt])
        b = enc(W)
        d, e = nb.layers[0], b.desc
        for f in ("n", "m", "nnz", "total_bits", "n_words", "k_sym", "lmax", "chunk", "n_chunks", "ent_bits", "ri_bits",
                  "has_zero", "zero_len", "max_col_bits", "max_col_nnz"):
            assert getattr(d, f) == getattr(e, f), f
        for f, dt, cnt in (("off_stream", np.uint32, int(e.n_words)), ("off_col_bit", np.uint32, W.shape[1] + 1),
                           ("off_codebook", np.float32, int(e.k_sym)), ("off_lut", np.uint32, 1 << int(e.lut_bits))):
            assert np.array_equal(nb.section(d, f, dt, cnt), b.section(f, dt, cnt)), f


def test_unused_symbols_and_empty_layers():
    # layer 1 uses two of the values only and has an empty column; layer 2 is all zero
    W0 = small_layers(seed=4, shapes=((20, 12),), k=7, prune=0.3)[0]
    vals = np.unique(W0[W0 != 0])
    W1 = np.zeros((12, 6), dtype=np.float32)
    W1[0, 0], W1[5, 0], W1[7, 2], W1[11, 5] = vals[0], vals[-1], vals[0], vals[-1]
    W2 = np.zeros((6, 4), dtype=np.float32)
    for fmts in ((1, 1, 1), (1, 2, 2), (2, 2, 2), (2, 1, 2)):
        nb = hac.hac_net_encode([W0, W1, W2], fmts)
        assert nb.validate(deep=True) == 0, fmts
        for l, W in enumerate((W0, W1, W2)):
            assert np.array_equal(nb.decode_host(l)[0], W)
        u = unified.unified_encode([KIND[f] for f in fmts], [W0, W1, W2])
        assert nb.stats().paper_bits == unified.unified_paper_bits(u)
    # every layer empty and sHAC: no symbol at all
    nb = hac.hac_net_encode([W2, W2.T.copy()], (2, 2))
    assert nb.validate(deep=True) == 0 and nb.net.k_sym == 0
    assert np.count_nonzero(nb.decode_host(1)[0]) == 0


def test_argument_and_format_errors():
    lib = hac.load_library()
    W = small_layers(seed=1)[0]
    with pytest.raises(hac.HacError):
        hac.hac_net_encode([W], [4])
    with pytest.raises(hac.HacError):
        hac.hac_net_encode([W], [hac.HAC_FORMAT_SHAC], ri_bits=2)           # too narrow for 40 rows
    bad = W.copy(); bad[0, 0] = np.inf
    with pytest.raises(hac.HacError):
        hac.hac_net_encode([W, bad], [1, 1])
    nb = hac.hac_net_encode([W, W.T.copy()], [1, 2])
    single = hac.hac_encode(W)
    # a network blob is not a layer blob and the other way round
    assert lib.hac_validate(nb.data.ctypes.data, nb.data.size, 1) == -3
    assert lib.hac_net_validate(single.data.ctypes.data, single.data.size, 1) == -3
    d = hac.Desc()
    assert lib.hac_net_layer(nb.data.ctypes.data, nb.data.size, 2, C.byref(d)) == -1
    assert lib.hac_net_validate(nb.data.ctypes.data, 100, 1) == -3
    assert lib.hac_net_validate(nb.data.ctypes.data, nb.data.size - 256, 1) == -3


def test_damaged_network_blobs_are_rejected():
    lib = hac.load_library()
    Ws = small_layers(seed=9)
    nb = hac.hac_net_encode(Ws, [1, 2, 2], ri_coding=0)
    good = nb.data
    assert lib.hac_net_validate(good.ctypes.data, good.size, 1) == 0

    def check(mutate):
        b = good.copy()
        mutate(b)
        return lib.hac_net_validate(b.ctypes.data, b.size, 1)

    def set_u32(off, v):
        def f(b): b[off:off + 4].view(np.uint32)[0] = v
        return f

    def set_u64(off, v):
        def f(b): b[off:off + 8].view(np.uint64)[0] = v
        return f

    net_off = {f[0]: getattr(hac.Net, f[0]).offset for f in hac.Net._fields_}
    desc_off = {f[0]: getattr(hac.Desc, f[0]).offset for f in hac.Desc._fields_}
    assert check(set_u32(net_off["n_layers"], 4)) == -3                      # a header that is not there
    assert check(set_u32(net_off["n_layers"], 0)) == -3
    assert check(set_u64(net_off["off_lut"], int(nb.net.off_lut) + 256)) == -3
    assert check(set_u32(net_off["k_sym"], int(nb.net.k_sym) + 1)) == -3
    assert check(set_u64(net_off["blob_bytes"], good.size + 256)) == -3
    base1 = int(nb.net.off_layers) + 256
    assert check(set_u32(base1 + desc_off["dict_shared"], 0)) == -3
    assert check(set_u64(base1 + desc_off["off_codebook"], int(nb.layers[1].off_stream))) == -3
    assert check(set_u64(base1 + desc_off["off_stream"], 0)) == -3           # into the headers
    assert check(set_u64(base1 + desc_off["off_stream"], good.size)) == -3
    assert check(set_u64(base1 + desc_off["total_bits"], int(nb.layers[1].total_bits) + 1)) == -3
    assert check(set_u64(base1 + desc_off["nnz"], int(nb.layers[1].nnz) + 1)) == -3
    # a flipped stream bit: another symbol or a broken walk -- the deep check or the decoder must notice a change
    b = good.copy()
    off = int(nb.layers[2].off_stream)
    b[off] ^= 0x80
    rc = lib.hac_net_validate(b.ctypes.data, b.size, 1)
    if rc == 0:
        W = np.empty(Ws[2].shape, dtype=np.float32)
        assert lib.hac_net_decode_host(b.ctypes.data, b.size, 2, W.ctypes.data_as(C.POINTER(C.c_float)), None, None, None) == 0
        assert not np.array_equal(W, Ws[2])
    # the codebook must stay ascending
    b = good.copy()
    cb = b[int(nb.net.off_codebook):int(nb.net.off_codebook) + 4 * int(nb.net.k_sym)].view(np.float32)
    cb[1], cb[2] = cb[2], cb[1]
    assert lib.hac_net_validate(b.ctypes.data, b.size, 0) == -3


def _layer_structs(descs, acts=None):
    arr = (hac.Layer * len(descs))()
    for i, d in enumerate(descs):
        arr[i].desc = C.pointer(d)
        arr[i].d_blob = 256                      # never dereferenced by the calls below
        arr[i].activation = 0 if acts is None else acts[i]
    return arr


def test_chain_workspace_and_argument_checks_on_the_host():
    """What hac_forward decides before it touches the GPU: shapes, workspace, argument errors."""
    lib = hac.load_library()
    Ws = small_layers(seed=6, shapes=((300, 200), (200, 120), (120, 10)))
    nb = hac.hac_net_encode(Ws, (1, 2, 1))
    descs = nb.layers
    arr = _layer_structs(descs)
    # B = 1: a row is its own feature-major copy, so only the two activation buffers remain
    need1 = lib.hac_forward_workspace_bytes(arr, 3, 1)
    assert need1 == 2 * 256 * ((4 * 1 * 200 + 255) // 256)
    # B = 40 -> padded to 64 batch columns; the input of layer 0 is re-laid out, the others arrive feature-major
    need = lib.hac_forward_workspace_bytes(arr, 3, 40)
    act = 256 * ((4 * 64 * 200 + 255) // 256)
    assert need == 2 * act + hac.hac_workspace_bytes(descs[0], 40)
    # one layer: exactly the dot's workspace
    assert lib.hac_forward_workspace_bytes(arr, 1, 40) == hac.hac_workspace_bytes(descs[0], 40)
    assert lib.hac_forward_workspace_bytes(arr, 3, 0) == 0
    # argument errors (all found before any device work)
    assert lib.hac_forward_workspace_bytes(None, 3, 8) == 0
    assert lib.hac_forward_workspace_bytes(arr, 0, 8) == 0 and lib.hac_forward_workspace_bytes(arr, 257, 8) == 0
    assert lib.hac_forward(arr, 3, 256, 0, 300, 256, 10, None, 0, None) == 0                    # B = 0: nothing to do
    assert lib.hac_forward(None, 3, 256, 8, 300, 256, 10, None, 0, None) == -1
    assert lib.hac_forward(arr, 3, None, 8, 300, 256, 10, 256, need, None) == -1                # no X
    assert lib.hac_forward(arr, 3, 256, 8, 299, 256, 10, 256, need, None) == -1                 # ldx < n
    assert lib.hac_forward(arr, 3, 256, 8, 300, 256, 9, 256, need, None) == -1                  # ldy < m
    assert lib.hac_forward(arr, 3, 256, 8, 300, 256, 10, None, 0, None) == -6                   # no workspace
    assert lib.hac_forward(arr, 3, 256, -1, 300, 256, 10, 256, need, None) == -1
    swapped = _layer_structs([descs[1], descs[0], descs[2]])
    assert lib.hac_forward_workspace_bytes(swapped, 3, 8) == 0                                   # shapes do not chain
    assert lib.hac_forward(swapped, 3, 256, 8, 200, 256, 10, 256, need, None) == -1
    bad = _layer_structs(descs, acts=[0, 7, 0])
    assert lib.hac_forward(bad, 3, 256, 8, 300, 256, 10, 256, need, None) == -1
    arr[2].reserved = 1
    assert lib.hac_forward(arr, 3, 256, 8, 300, 256, 10, 256, need, None) == -1
    arr[2].reserved = 0
    arr[1].d_blob = None
    assert lib.hac_forward(arr, 3, 256, 8, 300, 256, 10, 256, need, None) == -1
