"""Host side of libhac (no GPU): the C ABI loads and exports what include/hac.h
declares; the encoders produce streams the oracle agrees with (same symbols,
same number of bits, decodable by the oracle's bit-by-bit decoder); validation
rejects damaged blobs instead of reading out of bounds."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

import paper_2108_12704_amd as hac
import workloads
from oracle import bounds, formats, huffman

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hac.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:s?hac|im)_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = hac.load_library()
    names = declared_functions()
    assert set(names) == set(hac.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def header_fields(struct_name):
    text = open(os.path.join(ROOT, "include", "hac.h")).read()
    body = text[:text.index("} " + struct_name + ";")]
    body = body[body.rindex("typedef struct {") + len("typedef struct {"):]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    return re.findall(r"\b([a-z_][a-z_0-9]*)(?:\[\d+\])?\s*[;,]", body)


def test_header_struct_matches_binding():
    assert header_fields("hac_desc_t") == [f[0] for f in hac.Desc._fields_]
    assert header_fields("hac_opts_t") == [f[0] for f in hac.Opts._fields_]
    assert header_fields("hac_launch_t") == [f[0] for f in hac.Launch._fields_]
    assert header_fields("hac_stats_t") == [f[0] for f in hac.Stats._fields_]


def codes_from_blob(blob):
    d = blob.desc
    k = int(d.k_sym)
    lens = blob.section("off_codelen", np.uint8, k).astype(int)
    symsort = blob.section("off_symsort", np.uint32, k)
    canon = blob.section("off_canon", np.uint32, 99)
    words = {}
    for l in range(1, 33):
        for r in range(int(canon[33 + l])):
            s = int(symsort[int(canon[66 + l]) + r])
            assert lens[s] == l
            words[format(int(canon[l]) + r, "b").zfill(l)] = s
    return lens, words


def chunk_entries(blob):
    """[(relative bit offset, first row)] per chunk, unpacked from the blob."""
    d = blob.desc
    nch = int(d.n_chunks)
    if d.format == hac.HAC_FORMAT_HAC or d.ri_coding == hac.RI_RICE:
        if d.ent_bits == 32:
            e = blob.section("off_chunk_ent", np.uint32, nch)
            rb = int(d.row_bits)
            return [(int(v) >> rb, int(v) & ((1 << rb) - 1)) for v in e]
        e = blob.section("off_chunk_ent", np.uint32, 2 * nch).reshape(-1, 2)
        return [(int(r[1]), int(r[0])) for r in e]
    dt = np.uint16 if d.ent_bits == 16 else np.uint32
    return [(int(v), 0) for v in blob.section("off_chunk_ent", dt, nch)]


def oracle_decode_bits(stream_words, count, words):
    """Bit-by-bit decode with a codeword dictionary (the oracle's NCW idea)."""
    out = np.empty(count, dtype=np.int64)
    cur, got = "", 0
    for w in stream_words:
        for ch in format(int(w), "032b"):
            cur += ch
            if cur in words:
                out[got] = words[cur]
                got += 1
                cur = ""
                if got == count:
                    return out
    assert got == count
    return out


def small_layers():
    yield "cfg1", workloads.layer(1)
    yield "cfg3-small", workloads.scaled(3, 700, 50)
    yield "cfg5-small", workloads.scaled(5, 300, 40)
    for name, W in workloads.edge_cases().items():
        yield name, W


LAYERS = list(small_layers())
IDS = [n for n, _ in LAYERS]


@pytest.mark.parametrize("name,W", LAYERS, ids=IDS)
def test_hac_blob_against_oracle(name, W):
    n, m = W.shape
    blob = hac.hac_encode(W, chunk_nnz=3)
    assert blob.validate(deep=True) == 0
    d = blob.desc
    values, sym = formats.hac_symbols(W)
    oh = formats.hac_encode(W)
    assert int(d.total_bits) == oh.nbits                       # same optimal cost sum f_i l_i
    assert int(d.n_words) == oh.N
    assert int(d.k_sym) == len(values) and int(d.nnz) == np.count_nonzero(W)
    assert np.array_equal(blob.section("off_codebook", np.float32, len(values)), values)
    Wd, symd = blob.decode_host()
    assert np.array_equal(Wd.view(np.uint32), W.view(np.uint32))
    assert np.array_equal(symd, sym)
    lens, words = codes_from_blob(blob)
    assert huffman.cost(oh.freqs, lens) == oh.nbits
    stream = blob.section("off_stream", np.uint32, int(d.n_words))
    assert np.array_equal(oracle_decode_bits(stream, n * m, words), sym)
    # padding bits of the last word are zero
    pad = int(d.n_words) * 32 - int(d.total_bits)
    if pad:
        assert int(stream[-1]) & ((1 << pad) - 1) == 0
    # index: per column its first bit / first non-zero / first chunk; per chunk of C non-zeros the
    # bit right after the previous non-zero's codeword (column start for the first) and the row there
    C = int(d.chunk)
    cum = np.concatenate(([0], np.cumsum(lens[sym])))
    isnz = values[sym] != 0
    nzcum = np.concatenate(([0], np.cumsum(isnz)))
    col_start = np.arange(m + 1) * n
    col_bit = blob.section("off_col_bit", np.uint32, m + 1)
    col_pos = blob.section("off_col_pos", np.uint32, m + 1)
    col_chunk = blob.section("off_col_chunk", np.uint32, m + 1)
    assert np.array_equal(col_bit, cum[col_start])
    assert np.array_equal(col_pos, nzcum[col_start])
    counts = np.diff(nzcum[col_start])
    assert np.array_equal(np.diff(col_chunk), -(-counts // C))
    assert int(d.max_col_nnz) == counts.max() and int(d.max_col_bits) == np.diff(cum[col_start]).max()
    ents = chunk_entries(blob)
    g = 0
    for j in range(m):
        nzidx = np.flatnonzero(isnz[j * n:(j + 1) * n])
        for k in range(0, len(nzidx), C):
            start = 0 if k == 0 else nzidx[k - 1] + 1            # first symbol decoded by this chunk
            assert ents[g] == (cum[j * n + start] - cum[j * n], start), (j, k)
            g += 1
    assert g == int(d.n_chunks)


@pytest.mark.parametrize("name,W", LAYERS, ids=IDS)
def test_shac_blob_against_oracle(name, W):
    n, m = W.shape
    blob = hac.shac_encode(W, chunk_nnz=8)
    assert blob.validate(deep=True) == 0
    d = blob.desc
    values, sym, row, col = formats.shac_symbols(W)
    os_ = formats.shac_encode(W)
    assert int(d.total_bits) == os_.nbits and int(d.n_words) == os_.N1
    assert int(d.nnz) == os_.q and int(d.k_sym) == len(values)
    Wd, symd, rowd, cold = blob.decode_host()
    assert np.array_equal(Wd.view(np.uint32), W.view(np.uint32))
    assert np.array_equal(symd, sym) and np.array_equal(rowd, row) and np.array_equal(cold, col)
    assert np.array_equal(blob.section("off_col_pos", np.uint32, m + 1), os_.cb)       # the paper's cb
    lens_s = blob.section("off_codelen", np.uint8, len(values)).astype(int)
    cum = np.concatenate(([0], np.cumsum(lens_s[sym]))) if os_.q else np.zeros(1, dtype=int)
    col_bit = blob.section("off_col_bit", np.uint32, m + 1)
    assert np.array_equal(col_bit, cum[os_.cb])
    ents = chunk_entries(blob)
    g = 0
    for j in range(m):
        for p in range(int(os_.cb[j]), int(os_.cb[j + 1]), int(d.chunk)):
            assert ents[g] == (cum[p] - cum[os_.cb[j]], 0)
            g += 1
    assert g == int(d.n_chunks)
    assert int(d.ri_bits) == max(1, math.ceil(math.log2(n))) if n > 1 else int(d.ri_bits) == 1
    if os_.q:
        lens, words = codes_from_blob(blob)
        stream = blob.section("off_stream", np.uint32, int(d.n_words))
        assert np.array_equal(oracle_decode_bits(stream, os_.q, words), sym)


@pytest.mark.parametrize("name,W", LAYERS, ids=IDS)
def test_rice_coded_shac_blob_against_oracle(name, W):
    """sHAC with Rice-coded row gaps (extension): same bits, same k, same decoded CSC as the oracle;
    the stream parses gap by gap with the oracle's codeword strings; index entries point at gap starts."""
    from oracle import gapcode
    n, m = W.shape
    blob = hac.shac_encode(W, chunk_nnz=7, ri_coding=hac.RI_RICE)
    assert blob.validate(deep=True) == 0
    d = blob.desc
    og = gapcode.shacg_encode(W)
    values, sym, row, col, gaps = gapcode.shacg_symbols(W)
    assert int(d.ri_coding) == hac.RI_RICE and int(d.ri_bits) == 0 and int(d.off_ri) == 0
    assert int(d.total_bits) == og.nbits and int(d.gap_bits) == og.gap_bits and int(d.n_words) == og.N
    assert int(d.rice_k) == og.k and int(d.nnz) == og.q and int(d.k_sym) == len(values)
    Wd, symd, rowd, cold = blob.decode_host()
    assert np.array_equal(Wd.view(np.uint32), W.view(np.uint32))
    assert np.array_equal(symd, sym) and np.array_equal(rowd, row) and np.array_equal(cold, col)
    assert np.array_equal(blob.section("off_col_pos", np.uint32, m + 1), og.cb)
    lens_s = blob.section("off_codelen", np.uint8, len(values)).astype(int)
    per = gapcode.rice_lengths(gaps, og.k) + (lens_s[sym] if og.q else 0)
    cum = np.concatenate(([0], np.cumsum(per))).astype(np.int64)
    assert np.array_equal(blob.section("off_col_bit", np.uint32, m + 1), cum[og.cb])
    ents = chunk_entries(blob)
    g = 0
    for j in range(m):
        for p in range(int(og.cb[j]), int(og.cb[j + 1]), int(d.chunk)):
            base_row = 0 if p == og.cb[j] else int(row[p - 1]) + 1
            assert ents[g] == (cum[p] - cum[og.cb[j]], base_row)
            g += 1
    assert g == int(d.n_chunks)
    if og.q:
        # parse the library's stream with the oracle's gap codewords and the blob's own value codewords
        lens, words = codes_from_blob(blob)
        stream = blob.section("off_stream", np.uint32, int(d.n_words))
        bits = "".join(format(int(w), "032b") for w in stream)
        pos = 0
        for p in range(og.q):
            gw = gapcode.rice_bits(int(gaps[p]), og.k)
            assert bits.startswith(gw, pos), p
            pos += len(gw)
            cur = ""
            while cur not in words:
                cur += bits[pos]; pos += 1
            assert words[cur] == sym[p]
        assert pos == og.nbits and set(bits[pos:]) <= {"0"}
    st = blob.stats()
    assert st.ri_bytes == 0 and st.paper_bits == gapcode.shacg_paper_bits(og)
    assert st.paper_bits <= st.bound_bits
    assert blob.nbytes <= hac.shac_encode(W, chunk_nnz=7).nbytes


def test_rice_coding_argument_checks_and_damage():
    import ctypes as C
    W = workloads.scaled(4, 900, 30)
    with pytest.raises(hac.HacError):
        hac.shac_encode(W, ri_coding=2)
    with pytest.raises(hac.HacError):
        hac.shac_encode(W, ri_coding=hac.RI_RICE, ri_bits=32)
    lib = hac.load_library()
    out, size = C.c_void_p(), C.c_size_t()
    opts = hac.Opts(0, 0, 0, hac.RI_RICE)
    Wc = np.ascontiguousarray(W)
    rc = lib.hac_encode(Wc.ctypes.data_as(C.POINTER(C.c_float)), 900, 30, 30, C.byref(opts), C.byref(out), C.byref(size))
    assert rc == -1 and not out.value
    blob = hac.shac_encode(W, ri_coding=hac.RI_RICE)
    assert blob.validate(deep=True) == 0
    off = int(blob.desc.off_stream)

    def damaged(at, value=None, flip=0, deep=1):
        b = blob.data.copy()
        b[at] = value if value is not None else b[at] ^ flip
        return lib.hac_validate(b.ctypes.data, b.size, deep)

    for byte in (0, 5, 40):
        assert damaged(off + byte, flip=0x10) in (0, -3)    # decodes to some other matrix or fails, never crashes
    assert damaged(off, flip=0x80) == -3                    # first gap codeword now disagrees with the index / counts
    assert damaged(hac.Desc.rice_k.offset, value=16, deep=0) == -3
    assert damaged(hac.Desc.gap_bits.offset, flip=1) == -3
    assert damaged(hac.Desc.ri_coding.offset, value=0) == -3


def test_rice_escape_form_for_huge_gaps():
    from oracle import gapcode
    W = workloads.stress_cases()["clustered_rows_300000x3"]
    og = gapcode.shacg_encode(W)
    values, sym, row, col, gaps = gapcode.shacg_symbols(W)
    assert int((gaps >> og.k).max()) >= 31                   # the escape form occurs
    blob = hac.shac_encode(W, ri_coding=hac.RI_RICE)
    assert blob.validate(deep=True) == 0
    assert int(blob.desc.total_bits) == og.nbits and int(blob.desc.rice_k) == og.k
    _, symd, rowd, cold = blob.decode_host(want_w=False)
    assert np.array_equal(symd, sym) and np.array_equal(rowd, row) and np.array_equal(cold, col)


def im_cases():
    for name, W in LAYERS:
        yield name, W
    yield "no_repeats", workloads.stress_cases()["no_repeats_40x30"]
    yield "unpruned", workloads.make_layer(130, 77, 0.02, 0.0, 64, "kmeans", 3)


@pytest.mark.parametrize("name,W", list(im_cases()), ids=[c[0] for c in im_cases()])
def test_index_map_blob_against_oracle(name, W):
    from oracle import indexmap
    n, m = W.shape
    blob = hac.im_encode(W)
    assert blob.validate(deep=True) == 0
    d = blob.desc
    im = indexmap.im_encode(W)
    assert int(d.format) == hac.HAC_FORMAT_IM and int(d.ent_bits) == im.bbar and int(d.k_sym) == im.c.size
    assert int(d.total_bits) == im.bbar * n * m and int(d.nnz) == np.count_nonzero(W)
    assert int(d.idx_pitch) == -(-m // 16) * 16
    assert np.array_equal(blob.section("off_codebook", np.float32, im.c.size), im.c)
    dt = np.uint8 if im.bbar == 8 else np.uint16
    pi = blob.section("off_stream", dt, n * int(d.idx_pitch)).reshape(n, int(d.idx_pitch))
    assert np.array_equal(pi[:, :m], im.pi) and not pi[:, m:].any()
    Wd, sym = blob.decode_host()
    assert np.array_equal(Wd.view(np.uint32), (W + np.float32(0)).view(np.uint32))
    assert np.array_equal(sym.reshape(m, n).T, im.pi.astype(np.int32))
    st = blob.stats()
    assert st.paper_bits == indexmap.im_bits(im)
    assert st.paper_bits / (32.0 * n * m) == pytest.approx(bounds.psi_index_map(n, m, im.c.size, im.bbar))
    assert st.avg_code_bits == im.bbar and 0.0 <= st.entropy_bits <= im.bbar


def test_index_map_argument_checks_and_damage():
    import ctypes as C
    lib = hac.load_library()
    W = workloads.scaled(5, 60, 20)
    Wc = np.ascontiguousarray(W)
    out, size = C.c_void_p(), C.c_size_t()
    opts = hac.Opts(0, 0, 0, 0)
    f32p = C.POINTER(C.c_float)
    assert lib.im_encode(Wc.ctypes.data_as(f32p), 60, 20, 20, C.byref(opts), C.byref(out), C.byref(size)) == -1
    assert lib.im_encode(Wc.ctypes.data_as(f32p), 60, 20, 10, None, C.byref(out), C.byref(size)) == -1
    bad = Wc.copy(); bad[3, 3] = np.inf
    assert lib.im_encode(bad.ctypes.data_as(f32p), 60, 20, 20, None, C.byref(out), C.byref(size)) == -1
    many = np.arange(1, 70001, dtype=np.float32).reshape(700, 100)          # more than 65536 representatives
    assert lib.im_encode(many.ctypes.data_as(f32p), 700, 100, 100, None, C.byref(out), C.byref(size)) == -4
    blob = hac.im_encode(W)
    d = blob.desc

    def damaged(at, value, deep=1):
        b = blob.data.copy()
        b[at] = value
        return lib.hac_validate(b.ctypes.data, b.size, deep)

    assert damaged(int(d.off_stream) + 5, 255) == -3                        # pointer past the representatives
    assert damaged(int(d.off_stream) + 25, 1) == -3                         # padding column not zero
    assert damaged(hac.Desc.ent_bits.offset, 12, deep=0) == -3
    assert damaged(hac.Desc.idx_pitch.offset, 16, deep=0) == -3
    assert damaged(int(d.off_codebook) + 3, 0x7f, deep=0) == -3             # representatives no longer ascending
    assert lib.hac_validate(blob.data.ctypes.data, blob.data.size - 256, 1) == -3


def test_route_choice_on_the_full_size_layers():
    """hac_dot_route is host-side logic: the 40 % dense conv-shaped layer at its batch of 12544 goes
    to the matrix cores, the 98 % sparse layer never does, and forcing works either way."""
    b5 = hac.shac_encode(workloads.layer(5))
    assert hac.hac_dot_route(b5.desc, 12544) == 1
    assert hac.hac_dot_route(b5.desc, 8) == 0
    assert hac.hac_workspace_bytes(b5.desc, 12544) == (4608 * 512 * 2 + 255) // 256 * 256      # 257 pointers: 16 bits
    b4 = hac.shac_encode(workloads.scaled(4, 25088, 256))
    for B in (1, 32, 256, 4096):
        assert hac.hac_dot_route(b4.desc, B) == 0
    assert hac.hac_dot_route(b4.desc, 256, hac.Launch(variant=0x800)) == 1
    assert hac.hac_dot_route(b5.desc, 12544, hac.Launch(variant=0x400)) == 0
    im = hac.im_encode(workloads.scaled(5, 300, 40))
    with pytest.raises(hac.HacError):
        hac.hac_dot_route(im.desc, 8)


def test_randomized_blobs_against_oracle():
    """A seeded sweep over shapes, densities, alphabet sizes and skews: every format's blob validates,
    holds as many bits as the oracle's encoding, and decodes to the oracle's symbols."""
    from oracle import gapcode, indexmap
    for name, W in workloads.random_cases(60):
        n, m = W.shape
        opts = dict(chunk_nnz=int(np.random.default_rng(len(name)).choice([0, 1, 5, 64])))
        hb = hac.hac_encode(W, **opts)
        sb = hac.shac_encode(W, **opts)
        gb = hac.shac_encode(W, ri_coding=hac.RI_RICE, **opts)
        ib = hac.im_encode(W)
        for b in (hb, sb, gb, ib):
            assert b.validate(deep=True) == 0, name
        values, sym = formats.hac_symbols(W)
        assert int(hb.desc.total_bits) == formats.hac_encode(W).nbits, name
        Wd, symd = hb.decode_host()
        assert np.array_equal(Wd.view(np.uint32), W.view(np.uint32)) and np.array_equal(symd, sym), name
        svalues, ssym, srow, scol = formats.shac_symbols(W)
        assert int(sb.desc.total_bits) == formats.shac_encode(W).nbits, name
        for b in (sb, gb):
            Wd, symd, rowd, cold = b.decode_host()
            assert np.array_equal(Wd.view(np.uint32), W.view(np.uint32)), name
            assert np.array_equal(symd, ssym) and np.array_equal(rowd, srow) and np.array_equal(cold, scol), name
        og = gapcode.shacg_encode(W)
        assert (int(gb.desc.total_bits), int(gb.desc.rice_k)) == (og.nbits, og.k), name
        Wd, symd = ib.decode_host()
        assert np.array_equal(Wd.view(np.uint32), W.view(np.uint32)), name
        assert np.array_equal(symd.reshape(m, n).T, indexmap.im_encode(W).pi.astype(np.int32)), name


def test_choose_format_follows_the_bound_crossover():
    """The library's rule against the oracle's closed form and against the two bounds themselves."""
    for n, m, k in ((500, 300, 16), (4096, 1000, 32), (4096, 4096, 256), (25088, 4096, 32), (64, 64, 2)):
        s_star = bounds.crossover_sparsity(n, m, k)
        for s in (0.0, 0.5 * s_star, 0.99 * s_star, 1.01 * s_star, min(1.0, 3 * s_star), 1.0):
            nnz = int(s * n * m)
            got = hac.hac_choose_format(n, m, nnz, k)
            smaller = bounds.psi_shac_bound(n, m, nnz / (n * m), k) < bounds.psi_hac_bound(n, m, k)
            assert got == (hac.HAC_FORMAT_SHAC if smaller else hac.HAC_FORMAT_HAC), (n, m, k, s)
    with pytest.raises(hac.HacError):
        hac.hac_choose_format(0, 5, 0, 2)
    with pytest.raises(hac.HacError):
        hac.hac_choose_format(5, 5, 26, 2)


def test_ri_bits_32_and_small_tables_still_round_trip():
    W = workloads.scaled(3, 260, 33)
    for kw in (dict(ri_bits=32), dict(lut_bits=2), dict(chunk_nnz=1), dict(chunk_nnz=65536)):
        blob = hac.shac_encode(W, **kw)
        assert blob.validate(deep=True) == 0
        assert np.array_equal(blob.decode_host()[0], W)
    for kw in (dict(lut_bits=1), dict(lut_bits=12), dict(chunk_nnz=1), dict(chunk_nnz=65536)):
        blob = hac.hac_encode(W, **kw)
        assert blob.validate(deep=True) == 0
        assert np.array_equal(blob.decode_host()[0], W)


def test_long_codewords_use_the_second_level():
    # Fibonacci-like counts force a path-shaped tree: lengths up to k - 1
    counts = [1, 1, 2, 3, 5, 8, 13, 21, 34, 55, 89, 144, 233, 377, 610]
    vals = np.arange(1, len(counts) + 1, dtype=np.float32)
    col = np.concatenate([np.full(c, v, dtype=np.float32) for c, v in zip(counts, vals)])
    rng = np.random.default_rng(0)
    W = rng.permutation(col).reshape(-1, 1)
    W = np.concatenate([W, np.zeros_like(W)], axis=1)
    blob = hac.shac_encode(W, lut_bits=4)
    assert int(blob.desc.lmax) == len(counts) - 1
    assert blob.validate(deep=True) == 0
    assert np.array_equal(blob.decode_host()[0], W)


@pytest.mark.parametrize("name", sorted(workloads.stress_cases().keys()))
def test_stress_cases_round_trip(name):
    W = workloads.stress_cases()[name]
    hb = hac.hac_encode(W)
    sb = hac.shac_encode(W)
    assert hb.validate(deep=True) == 0 and sb.validate(deep=True) == 0
    assert np.array_equal(hb.decode_host()[0].view(np.uint32), W.view(np.uint32))
    assert np.array_equal(sb.decode_host()[0].view(np.uint32), W.view(np.uint32))
    oh, os_ = formats.hac_symbols(W), formats.shac_symbols(W)
    assert np.array_equal(hb.decode_host(want_w=False)[1], oh[1])
    assert np.array_equal(sb.decode_host(want_w=False)[1], os_[1])
    if name == "no_repeats_40x30":
        assert int(hb.desc.k_sym) == 1200                       # above the 1024 symbols kept in LDS
    if name == "long_codes":
        assert int(sb.desc.lmax) >= 20 and int(sb.desc.lmax) > int(sb.desc.lut_bits)
    if name == "tall_dense_70000x2":
        assert int(hb.desc.ent_bits) == 64 and int(sb.desc.ent_bits) == 32


def test_stats_and_corollary_bounds():
    W = workloads.layer(1)
    n, m = W.shape
    hb = hac.hac_encode(W)
    st = hb.stats()
    k = int(hb.desc.k_sym)
    assert st.stream_bits == hb.desc.total_bits
    assert st.paper_bits <= bounds.corollary1_bits(n, m, k) + 31
    assert math.isclose(st.bound_bits, bounds.corollary1_bits(n, m, k))
    assert st.entropy_bits <= st.avg_code_bits <= st.entropy_bits + 1
    assert st.blob_bytes == hb.nbytes and math.isclose(st.psi, hb.nbytes / (4 * n * m))
    sb = hac.shac_encode(W, ri_bits=32)
    ss = sb.stats()
    q, ks = int(sb.desc.nnz), int(sb.desc.k_sym)
    assert ss.paper_bits <= bounds.corollary2_bits(n, m, q, ks) + 31
    assert math.isclose(ss.bound_bits, bounds.corollary2_bits(n, m, q, ks))
    # with ceil(log2 n)-bit row indices the stored blob, chunk index included, is below the bound too
    sb2 = hac.shac_encode(W)
    assert 8 * sb2.nbytes <= bounds.corollary2_bits(n, m, q, ks)
    assert 8 * hb.nbytes <= bounds.corollary1_bits(n, m, k)


def test_invalid_arguments():
    lib = hac.load_library()
    W = np.ones((3, 3), dtype=np.float32)
    out, size = C.c_void_p(), C.c_size_t()
    f32p = C.POINTER(C.c_float)
    assert lib.hac_encode(None, 3, 3, 3, None, C.byref(out), C.byref(size)) == -1
    assert lib.hac_encode(W.ctypes.data_as(f32p), 0, 3, 3, None, C.byref(out), C.byref(size)) == -1
    assert lib.shac_encode(W.ctypes.data_as(f32p), 3, 3, 2, None, C.byref(out), C.byref(size)) == -1
    for bad in (np.nan, np.inf):
        Wb = W.copy()
        Wb[1, 1] = bad
        with pytest.raises(hac.HacError) as e:
            hac.hac_encode(Wb)
        assert e.value.status == -1
    with pytest.raises(hac.HacError):
        hac.shac_encode(np.ones((300, 2), dtype=np.float32), ri_bits=8)     # 300 rows need 9 bits
    assert lib.hac_strerror(-3).decode() == "blob fails validation"
    assert lib.hac_strerror(12345) is not None
    lib.hac_free(None)


def test_encoders_run_concurrently_from_threads():
    # no global mutable state: eight threads encoding different layers (the foreign calls release
    # the interpreter lock) must produce the bytes of the same encodes done one after the other
    import threading
    work = []
    for t in range(8):
        W = workloads.make_layer(300 + 17 * t, 40 + t, 0.02, 0.8, 8 + t, "uniform", 900 + t)
        enc = (hac.hac_encode, hac.shac_encode, hac.im_encode)[t % 3]
        work.append((enc, W, enc(W).data.tobytes()))
    wrong = []

    def worker(enc, W, expect):
        for _ in range(5):
            if enc(W).data.tobytes() != expect:
                wrong.append(enc.__name__)

    threads = [threading.Thread(target=worker, args=w) for w in work]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not wrong, wrong


def test_planning_calls_survive_implausible_headers():
    # hac_workspace_bytes / hac_dot_route / hac_forward_workspace_bytes size launches from header
    # fields; a header with zero or absurd fields must give "no answer", not a division by zero
    import random
    rnd = random.Random(5)
    W = workloads.make_layer(60, 20, 0.02, 0.7, 8, "uniform", 3)
    good = {"hac": hac.hac_encode(W).desc, "shac": hac.shac_encode(W).desc, "im": hac.im_encode(W).desc}
    lib = hac.load_library()
    for name, d0 in good.items():
        assert hac.hac_workspace_bytes(d0, 40) >= 0
        for field, _ in hac.Desc._fields_:
            for value in (0, 1, 0xffffffff, 0x7fffffff, rnd.getrandbits(31)):
                d = hac.Desc.from_buffer_copy(bytes(d0))
                try:
                    setattr(d, field, value)
                except (TypeError, ValueError):           # array fields
                    continue
                for B in (1, 8, 40, 300):
                    lib.hac_workspace_bytes(C.byref(d), B)
                    lib.hac_dot_route(C.byref(d), B, None)
                    layer = hac.Layer()
                    layer.desc = C.pointer(d)
                    layer.d_blob = 256                    # never dereferenced by the size query
                    lib.hac_forward_workspace_bytes(C.byref(layer), 1, B)
        for field in ("n", "m", "chunk", "magic", "version"):
            d = hac.Desc.from_buffer_copy(bytes(d0))
            setattr(d, field, 0)
            if field == "chunk" and name == "im":
                continue
            assert lib.hac_workspace_bytes(C.byref(d), 40) == 0, (name, field)
            if name != "im":
                assert lib.hac_dot_route(C.byref(d), 40, None) < 0, (name, field)
            # the device calls turn such a header down before anything is launched (fake, aligned
            # pointers: they are never dereferenced on the host)
            f = {"hac": lib.hac_dot, "shac": lib.shac_dot, "im": lib.im_dot}[name]
            assert f(C.byref(d), 4096, 8192, 40, 100, 12288, 100, 16384, 1 << 20, None, None) == -1, (name, field)


def test_negative_zero_is_stored_as_zero():
    W = np.array([[-0.0, 1.0], [0.0, -0.0]], dtype=np.float32)
    for enc in (hac.hac_encode, hac.shac_encode):
        Wd = enc(W).decode_host()[0]
        assert np.array_equal(Wd.view(np.uint32), np.array([[0.0, 1.0], [0.0, 0.0]], dtype=np.float32).view(np.uint32))


def test_strided_input():
    big = workloads.scaled(1, 40, 30)
    W = big[:, 5:17]
    assert np.array_equal(hac.hac_encode(W).decode_host()[0], W)
    assert np.array_equal(hac.shac_encode(W).decode_host()[0], W)


@pytest.mark.parametrize("enc", [hac.hac_encode, hac.shac_encode])
def test_damaged_blobs_are_rejected(enc):
    lib = hac.load_library()
    W = workloads.scaled(1, 120, 17)
    blob = enc(W)
    good = blob.data
    assert lib.hac_validate(good.ctypes.data, good.size, 1) == 0
    # truncated
    assert lib.hac_validate(good.ctypes.data, 100, 1) == -3
    assert lib.hac_validate(good.ctypes.data, good.size - 256, 1) == -3
    assert lib.hac_validate(None, 1000, 1) == -1
    d = blob.desc

    def damaged(mutate):
        b = good.copy()
        mutate(b)
        return lib.hac_validate(b.ctypes.data, b.size, 1)

    def poke32(off, value):
        def f(b):
            b[off:off + 4] = np.frombuffer(np.uint32(value).tobytes(), dtype=np.uint8)
        return f

    assert damaged(poke32(0, 0xdeadbeef)) == -3                              # magic
    assert damaged(poke32(int(d.off_col_bit) + 4, 0x7fffffff)) == -3         # column start past the end
    assert damaged(poke32(int(d.off_chunk_ent), 0x00010001)) == -3           # first chunk not at its column's start
    assert damaged(poke32(int(d.off_codelen), 0x01010101)) == -3             # lengths no longer a complete code
    assert damaged(poke32(int(d.off_lut), 0xffffffff)) == -3                 # first-level table
    off_field = hac.Desc.off_stream.offset
    assert damaged(poke32(off_field, int(d.blob_bytes))) == -3               # section outside the blob
    if d.format == hac.HAC_FORMAT_SHAC:
        assert damaged(poke32(int(d.off_col_pos) + 4, int(d.nnz) + 5)) == -3 # cb not monotone
        assert damaged(poke32(int(d.off_ri), 0xffffffff)) == -3              # row index >= n
    else:
        assert damaged(poke32(int(d.off_col_pos) + 8, 0)) == -3
    # flipping stream bits either still decodes to *a* matrix (deep check passes or fails) but never crashes
    b = good.copy()
    b[int(d.off_stream):int(d.off_stream) + 8] ^= 0xff
    assert lib.hac_validate(b.ctypes.data, b.size, 1) in (0, -3)


def test_random_damage_never_crashes_validation_or_decode():
    """Random bit and byte damage anywhere in a blob (half of it in the header and tables): the deep
    check either rejects the blob or accepts it, and what it accepts the sequential decoder walks
    without leaving the matrix (an out-of-range row, column or symbol would write outside the buffers
    this test hands it and bring the process down)."""
    lib = hac.load_library()
    rng = np.random.default_rng(20240611)
    W = workloads.scaled(1, 120, 17)
    blobs = [hac.hac_encode(W), hac.shac_encode(W), hac.shac_encode(W, ri_coding=hac.RI_RICE), hac.im_encode(W),
             hac.hac_encode(W, chunk_nnz=4), hac.shac_encode(W, ri_bits=32)]

    def damage(b):
        for _ in range(int(rng.integers(1, 4))):
            pos = int(rng.integers(0, min(4096, b.size))) if rng.random() < 0.5 else int(rng.integers(0, b.size))
            if rng.random() < 0.3:
                b[pos] = np.uint8(rng.integers(0, 256))
            else:
                b[pos] ^= np.uint8(1 << int(rng.integers(0, 8)))

    accepted = 0
    for blob in blobs:
        for _ in range(1500):
            b = blob.data.copy()
            damage(b)
            rc = lib.hac_validate(b.ctypes.data, b.size, 1)
            assert rc in (0, -3)
            if rc == 0:
                accepted += 1
                got = hac.Blob(b)
                if (int(got.desc.n), int(got.desc.m)) != W.shape:
                    # only the row count of an address-map blob can change and stay consistent: the same
                    # non-zeros in a taller matrix (every other format codes all n * m entries)
                    assert got.desc.format == hac.HAC_FORMAT_SHAC and int(got.desc.m) == W.shape[1]
                    continue
                assert got.decode_host()[0].shape == W.shape
    net = hac.hac_net_encode([W, workloads.scaled(2, 17, 9)], [hac.HAC_FORMAT_HAC, hac.HAC_FORMAT_SHAC])
    for _ in range(1500):
        b = net.data.copy()
        damage(b)
        rc = lib.hac_net_validate(b.ctypes.data, b.size, 1)
        assert rc in (0, -3)
        if rc == 0:
            accepted += 1
            got = hac.NetBlob(b)
            for l in range(len(got.layers)):
                got.decode_host(l)
    assert accepted > 100                                              # damage in padding and in stream bits that still decode


# ---- the optional row index (hac_opts_t.chunk_rows) -----------------------------------------

def row_index_entries(blob):
    """(rel_bit, rel_pos) arrays of shape (m, nq + 1) from a blob's row index."""
    d = blob.desc
    n, m, cr = int(d.n), int(d.m), int(d.chunk_rows)
    nq = -(-n // cr)
    if int(d.rent_bits) == 32:
        raw = blob.section("off_row_ent", np.uint32, m * (nq + 1)).reshape(m, nq + 1)
        pb = int(d.rpos_bits)
        return (raw >> pb).astype(np.int64), (raw & ((1 << pb) - 1)).astype(np.int64)
    raw = blob.section("off_row_ent", np.uint32, 2 * m * (nq + 1)).reshape(m, nq + 1, 2)
    return raw[:, :, 1].astype(np.int64), raw[:, :, 0].astype(np.int64)


def fullest_tile(W, cr):
    n, m = W.shape
    worst = 0
    for j0 in range(0, m, 16):
        for r0 in range(0, n, 4 * cr):
            worst = max(worst, int(np.count_nonzero(W[r0:r0 + 4 * cr, j0:j0 + 16])))
    return min(worst, 65535)


@pytest.mark.parametrize("name,W", LAYERS, ids=IDS)
@pytest.mark.parametrize("cr", [4, 12, "auto", "n"])
def test_row_index_against_oracle(name, W, cr):
    """Entry q of column j: the bits the oracle's symbols of rows < q*chunk_rows occupy under the blob's
    code lengths, and how many of them are non-zero; the header's fullest tile by direct count."""
    n, m = W.shape
    want = hac.CHUNK_ROWS_AUTO if cr == "auto" else n if cr == "n" else cr
    if isinstance(cr, int) and cr > n:
        pytest.skip("chunk_rows above n is refused")
    values, sym = formats.hac_symbols(W)
    svalues, ssym, srow, scol = formats.shac_symbols(W)
    for fmt in ("hac", "shac"):
        blob = hac.hac_encode(W, chunk_rows=want) if fmt == "hac" else hac.shac_encode(W, chunk_rows=want)
        assert blob.validate(deep=True) == 0
        d = blob.desc
        crr = int(d.chunk_rows)
        assert 1 <= crr <= n and (crr == n or crr % 4 == 0)
        if isinstance(cr, int):
            assert crr == cr
        nq = -(-n // crr)
        rel_bit, rel_pos = row_index_entries(blob)
        lens, _ = codes_from_blob(blob)
        colbit = blob.section("off_col_bit", np.uint32, m + 1).astype(np.int64)
        for j in range(m):
            rows_nz = np.flatnonzero(W[:, j])
            if fmt == "hac":
                cum = np.concatenate(([0], np.cumsum(lens[sym[j * n:(j + 1) * n]])))
            else:
                cum_nz = np.concatenate(([0], np.cumsum(lens[ssym[scol == j]])))
            for q in range(nq + 1):
                r = min(q * crr, n)
                above = int(np.searchsorted(rows_nz, r))
                assert rel_pos[j, q] == above, (fmt, j, q)
                assert rel_bit[j, q] == (cum[r] if fmt == "hac" else cum_nz[above]), (fmt, j, q)
            assert rel_bit[j, nq] == colbit[j + 1] - colbit[j]
        assert int(d.max_tile_nnz) == fullest_tile(W, crr)
        assert blob.stats().row_index_bytes == m * (nq + 1) * int(d.rent_bits) // 8
        # the blob without the option is the same blob minus that section
        plain = hac.hac_encode(W) if fmt == "hac" else hac.shac_encode(W)
        assert int(plain.desc.chunk_rows) == 0 and plain.stats().row_index_bytes == 0
        assert np.array_equal(plain.decode_host()[1], blob.decode_host()[1])


def test_row_index_options_and_damage():
    W = workloads.scaled(2, 96, 40)
    for bad in (3, 6, 97, 1000):                              # not a multiple of 4, or above n
        with pytest.raises(hac.HacError) as err:
            hac.hac_encode(W, chunk_rows=bad)
        assert err.value.status == -1
    with pytest.raises(hac.HacError) as err:                   # Rice-coded gaps carry no row index
        hac.shac_encode(W, ri_coding=hac.RI_RICE, chunk_rows=8)
    assert err.value.status == -1
    for enc in (hac.hac_encode, hac.shac_encode):
        blob = enc(W, chunk_rows=8)
        off = int(blob.desc.off_row_ent)
        for at in (off + 4, off + 4 * 13, off + 4 * (13 * 9)):
            data = blob.data.copy()
            data[at] ^= 0x10
            rc = hac.load_library().hac_validate(data.ctypes.data, data.size, 1)
            assert rc == -3, at
        # the header's fullest tile is checked by the deep validation
        data = blob.data.copy()
        view = hac.Desc.from_buffer(data)
        view.max_tile_nnz += 1
        assert hac.load_library().hac_validate(data.ctypes.data, data.size, 0) == 0
        assert hac.load_library().hac_validate(data.ctypes.data, data.size, 1) == -3


def test_network_blob_layers_carry_the_row_index():
    Ws, _ = workloads.network("tiny-fc")
    nb = hac.hac_net_encode(Ws, (hac.HAC_FORMAT_HAC, hac.HAC_FORMAT_SHAC, hac.HAC_FORMAT_HAC), chunk_rows=hac.CHUNK_ROWS_AUTO)
    assert nb.validate(deep=True) == 0
    for l, d in enumerate(nb.layers):
        assert int(d.chunk_rows) > 0 and int(d.off_row_ent) > 0
        assert int(d.max_tile_nnz) == fullest_tile(Ws[l], int(d.chunk_rows))


# ---- chunk sizes per column (hac_opts_t.chunk_nnz = HAC_CHUNK_PER_COLUMN) ----

def uneven_columns():
    """columns of very different lengths: empty, short (chunks of 4), and long ones whose chunk size
    is ceil(non-zeros / 64)"""
    rng = np.random.default_rng(77)
    n, m = 1500, 11
    dens = [0.0, 0.01, 0.05, 0.17, 0.171, 0.3, 0.5, 0.8, 1.0, 0.0, 0.43]
    W = np.zeros((n, m), dtype=np.float32)
    vals = np.array([-1.5, -0.25, 0.5, 0.75, 2.0], dtype=np.float32)
    for j, p in enumerate(dens):
        mask = rng.random(n) < p
        W[mask, j] = vals[rng.integers(0, len(vals), int(mask.sum()))]
    return W


def chunk_size_of(desc, cnt):
    c = int(desc.chunk)
    base = c & 0x7fffffff
    return max(base, -(-int(cnt) // 64)) if c & hac.CHUNK_FLAG_PER_COLUMN else base


def test_per_column_chunk_sizes_against_oracle():
    W = uneven_columns()
    n, m = W.shape
    counts = np.count_nonzero(W, axis=0)
    assert counts.max() > 64 * 4 and len({max(4, -(-int(c) // 64)) for c in counts}) >= 5
    # HAC
    blob = hac.hac_encode(W, chunk_nnz=hac.CHUNK_PER_COLUMN)
    assert blob.validate(deep=True) == 0
    d = blob.desc
    assert int(d.chunk) == hac.CHUNK_FLAG_PER_COLUMN | 4
    values, sym = formats.hac_symbols(W)
    lens, words = codes_from_blob(blob)
    cum = np.concatenate(([0], np.cumsum(lens[sym])))
    isnz = values[sym] != 0
    col_chunk = blob.section("off_col_chunk", np.uint32, m + 1)
    ents = chunk_entries(blob)
    g = 0
    for j in range(m):
        C = chunk_size_of(d, counts[j])
        assert C == max(4, -(-int(counts[j]) // 64))
        assert int(col_chunk[j]) == g and -(-int(counts[j]) // C) <= 64
        nzidx = np.flatnonzero(isnz[j * n:(j + 1) * n])
        for k in range(0, len(nzidx), C):
            start = 0 if k == 0 else nzidx[k - 1] + 1
            assert ents[g] == (cum[j * n + start] - cum[j * n], start), (j, k)
            g += 1
    assert g == int(d.n_chunks) == int(col_chunk[m])
    Wd, symd = blob.decode_host()
    assert np.array_equal(Wd.view(np.uint32), W.view(np.uint32)) and np.array_equal(symd, sym)
    # sHAC with ri fields, and with Rice-coded gaps
    os_ = formats.shac_encode(W)
    for kw in ({}, {"ri_coding": hac.RI_RICE}):
        blob = hac.shac_encode(W, chunk_nnz=hac.CHUNK_PER_COLUMN, **kw)
        assert blob.validate(deep=True) == 0
        d = blob.desc
        col_chunk = blob.section("off_col_chunk", np.uint32, m + 1)
        expect = np.concatenate(([0], np.cumsum([-(-int(c) // chunk_size_of(d, c)) for c in counts])))
        assert np.array_equal(col_chunk, expect) and int(d.n_chunks) == expect[-1]
        Wd, symd, rowd, cold = blob.decode_host()
        assert np.array_equal(Wd.view(np.uint32), W.view(np.uint32))
        if not kw:
            values_s, sym_s, row, col = formats.shac_symbols(W)
            lens_s = blob.section("off_codelen", np.uint8, len(values_s)).astype(int)
            cum_s = np.concatenate(([0], np.cumsum(lens_s[sym_s])))
            ents = chunk_entries(blob)
            g = 0
            for j in range(m):
                for p in range(int(os_.cb[j]), int(os_.cb[j + 1]), chunk_size_of(d, counts[j])):
                    assert ents[g] == (cum_s[p] - cum_s[os_.cb[j]], 0)
                    g += 1
            assert g == int(d.n_chunks)
    # a damaged chunk count is caught, and the option is refused where it makes no sense
    bad = hac.hac_encode(W, chunk_nnz=hac.CHUNK_PER_COLUMN)
    raw = bytearray(bad.data.tobytes())
    off = int(bad.desc.off_col_chunk) + 4 * 5
    raw[off] ^= 1
    assert hac.Blob(np.frombuffer(bytes(raw), dtype=np.uint8).copy()).validate(deep=False) != 0
    with pytest.raises(hac.HacError):
        hac.hac_encode(W, chunk_nnz=70000)
