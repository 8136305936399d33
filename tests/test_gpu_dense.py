"""GPU parity of the matrix-core paths: im_dot (index map, Sect. III-C1) and the dense
route of hac_dot / shac_dot (decode to an index map, then fp32 MFMA tiles).

Same bar as the vector path: |Y - Yref|_ij <= 1e-5 (|X| . |W|)_ij and
max |Y - Yref| <= 1e-5 max |Yref|, Yref the dense fp64 product of the oracle.
"""
import numpy as np
import pytest

import workloads
from oracle import dot as odot
from oracle import indexmap

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5
SPARSE, DENSE = 0x400, 0x800


@pytest.fixture(scope="module")
def hac():
    import paper_2108_12704_amd as lib
    lib.load_library()
    assert torch.cuda.is_available(), "GPU tests need a device"
    return lib


def dev():
    return torch.device("cuda:0")


def check_y(Y, X, W, what=""):
    ref = odot.dense_dot(X, W)
    scale = odot.abs_dot(X, W)
    got = Y.detach().cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape, what
    err = np.abs(got - ref)
    bad = err > TOL * scale + 1e-37
    assert not bad.any(), f"{what}: {int(bad.sum())} entries off, worst {float((err / (scale + 1e-300)).max()):.3e}"
    if ref.size and np.abs(ref).max() > 0:
        assert err.max() <= TOL * np.abs(ref).max(), what


def dense_layers():
    yield "cfg5-640x33", workloads.scaled(5, 640, 33)
    yield "cfg5-300x129", workloads.scaled(5, 300, 129)
    yield "cfg5-97x200", workloads.scaled(5, 97, 200)
    yield "cfg5-2100x40", workloads.scaled(5, 2100, 40)                                # K loop split into 8
    yield "unpruned-257x256", workloads.make_layer(257, 256, 0.02, 0.0, 64, "kmeans", 5)
    yield "cfg1", workloads.layer(1)
    yield "no_repeats_40x30", workloads.stress_cases()["no_repeats_40x30"]             # 16-bit pointers
    rng = np.random.default_rng(8)
    yield "distinct-100x60", rng.permutation(np.arange(1, 6001, dtype=np.float32)).reshape(100, 60) / np.float32(64)
    for name, W in workloads.edge_cases().items():
        yield name, W


LAYERS = list(dense_layers())
IDS = [c[0] for c in LAYERS]
BATCHES = [1, 2, 5, 8, 9, 64, 127, 128, 129, 300]


@pytest.mark.parametrize("name,W", LAYERS, ids=IDS)
def test_im_dot_parity(hac, name, W):
    n, m = W.shape
    blob = hac.im_encode(W)
    im = indexmap.im_encode(W)
    assert int(blob.desc.ent_bits) == im.bbar and int(blob.desc.k_sym) == im.c.size
    db = blob.to_device(dev())
    for B in BATCHES:
        print(f"[case] im_dot {name} {W.shape} B={B}", flush=True)
        X = workloads.make_batch(B, n, 31 + B) - np.float32(0.125)
        Y = hac.im_dot(db, torch.from_numpy(X).to(dev()))
        torch.cuda.synchronize()
        check_y(Y, X, W, f"im {name} B={B}")


def test_im_dot_small_batch_on_a_tall_map_with_a_long_value_list(hac):
    """At most 32 rows of X against a tall index map: the blocks of the small-batch kernel then hold
    close to a thousand rows of X, the partial sums of their row groups and the representatives in
    LDS, more than a kernel gets without asking for it."""
    W = workloads.make_layer(25088, 64, 0.02, 0.0, 256, "kmeans", 77)
    blob = hac.im_encode(W)
    assert int(blob.desc.k_sym) >= 200
    db = blob.to_device(dev())
    for B in (32, 9):
        print(f"[case] im_dot tall map B={B}", flush=True)
        X = workloads.make_batch(B, W.shape[0], 12 + B)
        Y = hac.im_dot(db, torch.from_numpy(X).to(dev()))
        torch.cuda.synchronize()
        check_y(Y, X, W, f"tall map B={B}")
    # the same shape as the dense route of a pruned layer forced at a small batch
    Wp = workloads.make_layer(25088, 64, 0.02, 0.6, 256, "kmeans", 78)
    dbp = hac.hac_encode(Wp).to_device(dev())
    X = workloads.make_batch(32, Wp.shape[0], 5)
    print("[case] dense route forced at B=32 on a tall layer", flush=True)
    Y = hac.hac_dot(dbp, torch.from_numpy(X).to(dev()), launch=hac.Launch(variant=DENSE))
    torch.cuda.synchronize()
    check_y(Y, X, Wp, "dense route tall")


def test_im_dot_strided_and_unaligned(hac):
    W = workloads.scaled(5, 301, 70)
    db = hac.im_encode(W).to_device(dev())
    for rows in (40, 6):                                          # the matrix-core kernel, and the one for small batches
        Xbig = torch.from_numpy(workloads.make_batch(rows, 310, 2)).to(dev())
        Ybig = torch.full((rows, 90), 3.0, device=dev())
        for shift in (0, 1, 4):
            X = Xbig[:, shift:shift + 301]                       # ldx = 310, pointer offset by `shift` floats
            Y = Ybig[:, 7:77]
            hac.im_dot(db, X, Y=Y)
            torch.cuda.synchronize()
            check_y(Y, X.cpu().numpy(), W, f"rows {rows} shift {shift}")
            assert torch.all(Ybig[:, :7] == 3.0) and torch.all(Ybig[:, 77:] == 3.0)


@pytest.mark.parametrize("name,W", LAYERS, ids=IDS)
def test_dense_route_matches_the_oracle(hac, name, W):
    n, m = W.shape
    blobs = [("hac", hac.hac_dot, hac.hac_encode(W)), ("shac", hac.shac_dot, hac.shac_encode(W)),
             ("shac/rice", hac.shac_dot, hac.shac_encode(W, ri_coding=1)),
             ("hac c=3", hac.hac_dot, hac.hac_encode(W, chunk_nnz=3))]
    for what, f, blob in blobs:
        db = blob.to_device(dev())
        for B in (1, 3, 8, 9, 33, 128, 200):
            print(f"[case] dense route {what} {name} {W.shape} B={B}", flush=True)
            X = workloads.make_batch(B, n, 3 + B) - np.float32(0.2)
            Y = f(db, torch.from_numpy(X).to(dev()), launch=hac.Launch(variant=DENSE))
            torch.cuda.synchronize()
            check_y(Y, X, W, f"{what} dense {name} B={B}")


def test_dense_route_decode_without_its_lds_copies(hac):
    # the decode kernel keeps a block's stream words, ri fields and the column index in LDS when
    # they fit; these layers do not fit: 256 chunks of a very sparse, tall HAC layer span more
    # stream words than the staging area, 256 chunks of 100 non-zeros carry more ri bits than
    # theirs, and a layer with more than 8191 columns has too long an index
    tall = workloads.make_layer(30000, 24, 0.02, 0.999, 8, "uniform", 71)
    fat = workloads.make_layer(2000, 300, 0.02, 0.5, 16, "uniform", 72)
    wide = workloads.make_layer(24, 9000, 0.02, 0.7, 8, "uniform", 73)
    cases = [("tall", tall, hac.hac_encode(tall), hac.hac_dot), ("tall/rice", tall, hac.shac_encode(tall, ri_coding=1), hac.shac_dot),
             ("fat ri", fat, hac.shac_encode(fat, chunk_nnz=100), hac.shac_dot),
             ("wide", wide, hac.hac_encode(wide), hac.hac_dot), ("wide", wide, hac.shac_encode(wide), hac.shac_dot)]
    for what, W, blob, f in cases:
        db = blob.to_device(dev())
        for B in (1, 33):
            print(f"[case] dense route, decode from the blob: {what} {W.shape} B={B}", flush=True)
            X = workloads.make_batch(B, W.shape[0], 9 + B) - np.float32(0.2)
            Y = f(db, torch.from_numpy(X).to(dev()), launch=hac.Launch(variant=DENSE))
            torch.cuda.synchronize()
            check_y(Y, X, W, f"{what} B={B}")


def test_route_selection_and_workspace(hac):
    W = workloads.scaled(5, 2100, 70)                        # 40 % non-zero
    n, m = W.shape
    pitch = 80
    for enc, f in ((hac.hac_encode, hac.hac_dot), (hac.shac_encode, hac.shac_dot)):
        b = enc(W)
        bits = 8 if int(b.desc.k_sym) + (0 if enc is hac.hac_encode else 1) <= 256 else 16
        idx_bytes = (n * pitch * bits // 8 + 255) // 256 * 256
        db = b.to_device(dev())
        for B in (40, 256, 700):
            X = workloads.make_batch(B, n, 1)
            Xd = torch.from_numpy(X).to(dev())
            route = hac.hac_dot_route(b.desc, B)
            need = hac.hac_workspace_bytes(b.desc, B)
            if route == 0:
                assert need == 4 * n * (-(-B // 256) * 256 if B > 256 else 1 << (B - 1).bit_length())
            else:
                assert need >= idx_bytes                                       # index map (+ partial tiles)
            dense = hac.Launch(variant=DENSE)
            assert hac.hac_dot_route(b.desc, B, dense) == 1 and hac.hac_dot_route(b.desc, B, hac.Launch(variant=SPARSE)) == 0
            assert hac.hac_workspace_bytes(b.desc, B, dense) >= idx_bytes
            Y0 = f(db, Xd)
            Yd = f(db, Xd, launch=dense)
            Ys = f(db, Xd, launch=hac.Launch(variant=SPARSE))
            torch.cuda.synchronize()
            for Y, what in ((Y0, "default"), (Yd, "dense"), (Ys, "sparse")):
                check_y(Y, X, W, f"{f.__name__} {what} B={B}")
            assert torch.equal(Y0, Yd if route == 1 else Ys)                   # the default is one of the two, bit for bit
            assert torch.equal(Yd, f(db, Xd, launch=dense))                    # split-K parts are added in a fixed order
        Xd = torch.from_numpy(workloads.make_batch(256, n, 1)).to(dev())
        small = torch.empty(256, dtype=torch.uint8, device=dev())
        with pytest.raises(hac.HacError) as e:
            f(db, Xd, workspace=small, launch=hac.Launch(variant=DENSE))
        assert e.value.status == -6
        with pytest.raises(hac.HacError) as e:
            f(db, Xd, launch=hac.Launch(variant=SPARSE | DENSE))
        assert e.value.status == -1


def test_im_dot_argument_checks(hac):
    import ctypes as C
    lib = hac.load_library()
    W = workloads.scaled(5, 100, 20)
    ib = hac.im_encode(W).to_device(dev())
    hb = hac.hac_encode(W).to_device(dev())
    X = torch.zeros((4, 100), device=dev())
    with pytest.raises(hac.HacError) as e:
        hac.im_dot(hb, X)                                    # a HAC blob
    assert e.value.status == -1
    with pytest.raises(hac.HacError) as e:
        hac.hac_dot(ib, X)                                   # an index map given to hac_dot
    assert e.value.status == -1
    Y = torch.empty((4, 20), device=dev())
    assert lib.im_dot(C.byref(ib.desc), ib.tensor.data_ptr(), X.data_ptr(), 4, 50, Y.data_ptr(), 20, None, 0, None, None) == -1
    assert lib.im_dot(C.byref(ib.desc), ib.tensor.data_ptr(), None, 0, 100, None, 20, None, 0, None, None) == 0
    tall = hac.im_encode(workloads.scaled(5, 2100, 20))      # few tiles, long K: partial tiles need a workspace
    assert hac.hac_workspace_bytes(tall.desc, 4) > 0
    td = tall.to_device(dev())
    X = torch.zeros((4, 2100), device=dev())
    assert lib.im_dot(C.byref(td.desc), td.tensor.data_ptr(), X.data_ptr(), 4, 2100, Y.data_ptr(), 20, None, 0, None, None) == -6
    torch.cuda.synchronize()
