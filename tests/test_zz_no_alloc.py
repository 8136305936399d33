"""hac_dot_noalloc: the dot call whose workspace is a fixed array inside the library.

Called through the C ABI twice in a row on one GPU, the second time with a smaller batch, and
compared with hac_dot / shac_dot on a caller-owned workspace (the same kernels, so bit for bit)
and with the oracle's fp64 product under the usual gate.
"""
import ctypes as C

import numpy as np
import pytest

import workloads
from oracle import dot as odot

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def hac():
    import paper_2108_12704_amd as lib
    lib.load_library()
    assert torch.cuda.is_available(), "GPU tests need a device"
    return lib


def gate(Y, X, W, what):
    ref = odot.dense_dot(X, W)
    scale = odot.abs_dot(X, W)
    err = np.abs(Y.cpu().numpy().astype(np.float64) - ref)
    assert not (err > TOL * scale + 1e-37).any(), what
    assert err.max() <= TOL * np.abs(ref).max(), what


@pytest.mark.parametrize("fmt", ["hac", "shac", "shac-rice"])
def test_two_calls_in_a_row_second_smaller(hac, fmt):
    dev = torch.device("cuda:0")
    W = workloads.scaled(2, 2100, 333)
    if fmt == "hac":
        blob, ref_dot = hac.hac_encode(W), hac.hac_dot
    else:
        blob, ref_dot = hac.shac_encode(W, ri_coding=1 if fmt == "shac-rice" else 0), hac.shac_dot
    db = blob.to_device(dev)
    for B in (64, 9):                                    # both need the workspace (9 rows x 2100 does not fit LDS)
        print(f"[case] hac_dot_noalloc {fmt} B={B}", flush=True)
        assert 0 < hac.hac_workspace_bytes(blob.desc, B) <= hac.NOALLOC_WORKSPACE_BYTES
        X = workloads.make_batch(B, W.shape[0], 77 + B)
        Xd = torch.from_numpy(X).to(dev)
        Y = torch.full((B, W.shape[1]), float("nan"), dtype=torch.float32, device=dev)
        hac.hac_dot_noalloc(db, Xd, Y)
        want = ref_dot(db, Xd)
        torch.cuda.synchronize()
        assert torch.equal(Y, want), (fmt, B)
        gate(Y, X, W, (fmt, B))


def test_dense_route_and_limit(hac):
    dev = torch.device("cuda:0")
    W = workloads.scaled(5, 640, 96)
    blob = hac.hac_encode(W)
    db = blob.to_device(dev)
    launch = hac.Launch(variant=0x800)                    # dense route: index map and partial sums in the array
    for B in (200, 40):
        print(f"[case] hac_dot_noalloc dense route B={B}", flush=True)
        X = workloads.make_batch(B, W.shape[0], 5 + B)
        Xd = torch.from_numpy(X).to(dev)
        Y = torch.full((B, W.shape[1]), float("nan"), dtype=torch.float32, device=dev)
        hac.hac_dot_noalloc(db, Xd, Y, launch=launch)
        want = hac.hac_dot(db, Xd, launch=launch)
        torch.cuda.synchronize()
        assert torch.equal(Y, want), B
        gate(Y, X, W, ("dense", B))
    # a product whose workspace exceeds the array is refused, and nothing is launched
    tall = hac.shac_encode(workloads.make_layer(25088, 16, 0.005, 0.98, 32, "uniform", 11))
    B = 256
    assert hac.hac_workspace_bytes(tall.desc, B) > hac.NOALLOC_WORKSPACE_BYTES
    X = torch.zeros((B, 25088), dtype=torch.float32, device=dev)
    Y = torch.full((B, 16), 7.0, dtype=torch.float32, device=dev)
    with pytest.raises(hac.HacError) as err:
        hac.hac_dot_noalloc(tall.to_device(dev), X, Y)
    assert err.value.status == -6
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())
    # an index-map blob is not a HAC / sHAC blob
    im = hac.im_encode(W)
    with pytest.raises(hac.HacError) as err:
        hac.hac_dot_noalloc(im.to_device(dev), torch.zeros((4, 640), dtype=torch.float32, device=dev),
                            torch.zeros((4, 96), dtype=torch.float32, device=dev))
    assert err.value.status == -1
