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
    yield "unpruned-257x256", workloads.make_layer(257, 256, 0.02, 0.0, 64, "kmeans", 5)
    yield "cfg1", workloads.layer(1)
    yield "no_repeats_40x30", workloads.stress_cases()["no_repeats_40x30"]             # 16-bit pointers
    rng = np.random.default_rng(8)
    yield "distinct-100x60", rng.permutation(np.arange(1, 6001, dtype=np.float32)).reshape(100, 60) / np.float32(64)
    for name, W in workloads.edge_cases().items():
        yield name, W


LAYERS = list(dense_layers())
IDS = [c[0] for c in LAYERS]
BATCHES = [1, 5, 64, 127, 128, 129, 300]


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


def test_im_dot_strided_and_unaligned(hac):
    W = workloads.scaled(5, 301, 70)
    db = hac.im_encode(W).to_device(dev())
    Xbig = torch.from_numpy(workloads.make_batch(40, 310, 2)).to(dev())
    Ybig = torch.full((40, 90), 3.0, device=dev())
    for shift in (0, 1, 4):
        X = Xbig[:, shift:shift + 301]                       # ldx = 310, pointer offset by `shift` floats
        Y = Ybig[:, 7:77]
        hac.im_dot(db, X, Y=Y)
        torch.cuda.synchronize()
        check_y(Y, X.cpu().numpy(), W, f"shift {shift}")
        assert torch.all(Ybig[:, :7] == 3.0) and torch.all(Ybig[:, 77:] == 3.0)


@pytest.mark.parametrize("name,W", LAYERS, ids=IDS)
def test_dense_route_matches_the_oracle(hac, name, W):
    n, m = W.shape
    blobs = [("hac", hac.hac_dot, hac.hac_encode(W)), ("shac", hac.shac_dot, hac.shac_encode(W)),
             ("shac/rice", hac.shac_dot, hac.shac_encode(W, ri_coding=1)),
             ("hac c=3", hac.hac_dot, hac.hac_encode(W, chunk_nnz=3))]
    for what, f, blob in blobs:
        db = blob.to_device(dev())
        for B in (1, 33, 128, 200):
            print(f"[case] dense route {what} {name} {W.shape} B={B}", flush=True)
            X = workloads.make_batch(B, n, 3 + B) - np.float32(0.2)
            Y = f(db, torch.from_numpy(X).to(dev()), launch=hac.Launch(variant=DENSE))
            torch.cuda.synchronize()
            check_y(Y, X, W, f"{what} dense {name} B={B}")


def test_route_selection_and_workspace(hac):
    import ctypes as C
    W = workloads.scaled(5, 640, 70)                         # 40 % non-zero
    Ws = workloads.scaled(4, 640, 70)                        # 2 % non-zero
    pitch = 80
    for enc in (hac.hac_encode, hac.shac_encode):
        b = enc(W)
        assert hac.hac_workspace_bytes(b.desc, 127) == 4 * 640 * 128          # sparse: feature-major X
        bits = 8 if int(b.desc.k_sym) + (0 if enc is hac.hac_encode else 1) <= 256 else 16
        assert hac.hac_workspace_bytes(b.desc, 128) == (640 * pitch * bits // 8 + 255) // 256 * 256   # dense: the index map
        assert hac.hac_workspace_bytes(enc(Ws).desc, 4096) == 4 * 640 * 4096  # sparse layers stay on the sparse route
        db = b.to_device(dev())
        X = workloads.make_batch(256, 640, 1)
        Xd = torch.from_numpy(X).to(dev())
        f = hac.hac_dot if enc is hac.hac_encode else hac.shac_dot
        Yd = f(db, Xd)                                                         # dense by default
        Ys = f(db, Xd, launch=hac.Launch(variant=SPARSE))
        torch.cuda.synchronize()
        check_y(Yd, X, W, "default")
        check_y(Ys, X, W, "forced sparse")
        small = torch.empty(256, dtype=torch.uint8, device=dev())
        with pytest.raises(hac.HacError) as e:
            f(db, Xd, workspace=small)
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
    torch.cuda.synchronize()
