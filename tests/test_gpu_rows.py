"""GPU parity of the row-blocked batch kernel (blobs with a row index), through the C ABI.

Y against the oracle's dense fp64 product, element by element, with the usual gate; the kernel is
forced with the launch flag so that small batches and small matrices reach it too, at sizes that
span several sessions, several slabs of rows, ragged ends and several batch tiles.
"""
import numpy as np
import pytest

import workloads
from oracle import dot as odot

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5
ROWS, NO_ROWS = 0x2000, 0x4000


@pytest.fixture(scope="module")
def hac():
    import paper_2108_12704_amd as lib
    lib.load_library()
    assert torch.cuda.is_available(), "GPU tests need a device"
    return lib


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


def encoders(hac):
    return (("hac", hac.hac_encode, hac.hac_dot), ("shac", hac.shac_encode, hac.shac_dot),
            ("shac32", lambda W, **kw: hac.shac_encode(W, ri_bits=32, **kw), hac.shac_dot))


CASES = [
    # name, W, chunk_rows, batches, sessions per block
    ("cfg4-3000x300", lambda: workloads.scaled(4, 3000, 300), 40, (200, 256, 300), (0, 1, 3, 1000)),
    ("cfg4-1001x65-auto", lambda: workloads.scaled(4, 1001, 65), "auto", (129, 7), (0,)),
    ("cfg3-1100x70", lambda: workloads.scaled(3, 1100, 70), 100, (256,), (0, 2)),
    ("cfg2-700x529", lambda: workloads.scaled(2, 700, 529), 24, (130,), (0, 1)),
    ("cfg5-640x33", lambda: workloads.scaled(5, 640, 33), 8, (513,), (0, 5)),
    ("cfg1", lambda: workloads.layer(1), 20, (8, 260), (0,)),
    ("cfg4-400x40-one-entry", lambda: workloads.scaled(4, 400, 40), "n", (131,), (0,)),
]


@pytest.mark.parametrize("name,make,cr,batches,spbs", CASES, ids=[c[0] for c in CASES])
def test_rows_kernel_against_oracle(hac, name, make, cr, batches, spbs):
    dev = torch.device("cuda:0")
    W = make()
    n, m = W.shape
    chunk_rows = hac.CHUNK_ROWS_AUTO if cr == "auto" else n if cr == "n" else cr
    for fmt, enc, dot in encoders(hac):
        blob = enc(W, chunk_rows=chunk_rows)
        db = blob.to_device(dev)
        for B in batches:
            X = workloads.make_batch(B, n, 100 + B)
            Xd = torch.from_numpy(X).to(dev)
            for spb in spbs:
                print(f"[case] rows kernel {name} {fmt} chunk_rows={int(blob.desc.chunk_rows)} B={B} sessions/block={spb}", flush=True)
                launch = hac.Launch(variant=ROWS, sessions_per_block=spb)
                Y = dot(db, Xd, launch=launch)
                torch.cuda.synchronize()
                check_y(Y, X, W, f"{name} {fmt} B={B} spb={spb}")


def test_rows_kernel_edge_cases(hac):
    """Degenerate matrices (empty columns first and last, one row, one column, all zero, no zero, one
    shared value) and a strided X / Y."""
    dev = torch.device("cuda:0")
    for name, W in workloads.edge_cases().items():
        n, m = W.shape
        for cr in (hac.CHUNK_ROWS_AUTO, n, 4 if n > 4 else n):
            for fmt, enc, dot in encoders(hac)[:2]:
                blob = enc(W, chunk_rows=cr)
                db = blob.to_device(dev)
                for B in (1, 130):
                    print(f"[case] rows kernel edge {name} {W.shape} {fmt} chunk_rows={int(blob.desc.chunk_rows)} B={B}", flush=True)
                    X = workloads.make_batch(B, n, 7)
                    Y = dot(db, torch.from_numpy(X).to(dev), launch=hac.Launch(variant=ROWS))
                    torch.cuda.synchronize()
                    check_y(Y, X, W, f"{name} {fmt} B={B}")
    W = workloads.scaled(4, 777, 91)
    n, m = W.shape
    B = 150
    X = workloads.make_batch(B, n, 3)
    for fmt, enc, dot in encoders(hac)[:2]:
        db = enc(W, chunk_rows=16).to_device(dev)
        Xbig = torch.full((B, n + 5), float("nan"), dtype=torch.float32, device=dev)
        Xbig[:, :n] = torch.from_numpy(X).to(dev)
        Ybig = torch.full((B, m + 3), -7.0, dtype=torch.float32, device=dev)
        print(f"[case] rows kernel strided {fmt}", flush=True)
        dot(db, Xbig[:, :n], Y=Ybig[:, :m], launch=hac.Launch(variant=ROWS))     # rows of X not 16-byte aligned
        torch.cuda.synchronize()
        check_y(Ybig[:, :m], X, W, f"strided {fmt}")
        assert bool((Ybig[:, m:] == -7.0).all())


def test_rows_kernel_is_on_request_only_and_reproducible(hac):
    dev = torch.device("cuda:0")
    W = workloads.scaled(4, 2000, 520)
    n, m = W.shape
    blob = hac.hac_encode(W, chunk_rows=hac.CHUNK_ROWS_AUTO)
    db = blob.to_device(dev)
    X = workloads.make_batch(256, n, 5)
    Xd = torch.from_numpy(X).to(dev)
    print("[case] rows kernel on request", flush=True)
    rows = hac.Launch(variant=ROWS)
    assert hac.hac_workspace_bytes(blob.desc, 256, rows) != hac.hac_workspace_bytes(blob.desc, 256)
    Y0 = hac.hac_dot(db, Xd)                                     # the default: the column kernels
    Y1 = hac.hac_dot(db, Xd, launch=rows)
    Y2 = hac.hac_dot(db, Xd, launch=hac.Launch(variant=NO_ROWS))
    Y3 = hac.hac_dot(db, Xd, launch=rows)
    torch.cuda.synchronize()
    assert torch.equal(Y0, Y2)
    assert torch.equal(Y1, Y3)                                  # same kernel, same order of additions
    check_y(Y0, X, W, "default")
    check_y(Y1, X, W, "rows kernel")
    # a blob without a row index cannot be sent there
    plain = hac.hac_encode(W).to_device(dev)
    with pytest.raises(hac.HacError) as err:
        hac.hac_dot(plain, Xd, launch=rows)
    assert err.value.status == -1
