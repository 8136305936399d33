"""GPU parity for blobs whose columns have chunk sizes of their own (HAC_CHUNK_PER_COLUMN).

Columns of very different lengths (empty, a few non-zeros, up to every row), so that the chunk size
differs from column to column and wavefronts that own several columns mix them: Y against the
oracle's dense product and, with unit vectors, against the rows of W bit for bit, through the
small-batch, batch, short-X and dense-route kernels; the decode entry points against the oracle's
symbols; the device encoder against the host encoder byte for byte.
"""
import numpy as np
import pytest

import workloads
from oracle import dot as odot
from oracle import formats

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def hac():
    import paper_2108_12704_amd as lib
    lib.load_library()
    assert torch.cuda.is_available(), "GPU tests need a device"
    return lib


def uneven(n, m, seed):
    rng = np.random.default_rng(seed)
    dens = rng.choice([0.0, 0.004, 0.02, 0.1, 0.2, 0.45, 0.9, 1.0], size=m)
    vals = np.array([-2.0, -0.5, -0.125, 0.25, 0.75, 1.5, 3.0], dtype=np.float32)
    W = np.zeros((n, m), dtype=np.float32)
    for j, p in enumerate(dens):
        mask = rng.random(n) < p
        W[mask, j] = vals[rng.integers(0, len(vals), int(mask.sum()))]
    return W


def check_y(Y, X, W, what):
    ref = odot.dense_dot(X, W)
    scale = odot.abs_dot(X, W)
    err = np.abs(Y.detach().cpu().numpy().astype(np.float64) - ref)
    bad = err > TOL * scale + 1e-37
    assert not bad.any(), f"{what}: {int(bad.sum())} entries off"


CASES = [("1200x70", 1200, 70, 1), ("2600x33", 2600, 33, 2), ("700x150", 700, 150, 3)]


@pytest.mark.parametrize("name,n,m,seed", CASES, ids=[c[0] for c in CASES])
def test_dot_with_per_column_chunks(hac, name, n, m, seed):
    dev = torch.device("cuda:0")
    W = uneven(n, m, seed)
    encs = (("hac", lambda: hac.hac_encode(W, chunk_nnz=hac.CHUNK_PER_COLUMN), hac.hac_dot),
            ("shac", lambda: hac.shac_encode(W, chunk_nnz=hac.CHUNK_PER_COLUMN), hac.shac_dot),
            ("shac-rice", lambda: hac.shac_encode(W, chunk_nnz=hac.CHUNK_PER_COLUMN, ri_coding=hac.RI_RICE), hac.shac_dot))
    rng = np.random.default_rng(seed)
    for fmt, enc, dot in encs:
        blob = enc()
        assert int(blob.desc.chunk) & hac.CHUNK_FLAG_PER_COLUMN
        db = blob.to_device(dev)
        for B in (1, 3, 8, 32, 70, 256):
            X = workloads.make_batch(B, n, 10 * seed + B) - np.float32(0.25)
            Xd = torch.from_numpy(X).to(dev)
            for launch in (hac.Launch(variant=0x400), hac.Launch(variant=0x400, cols_per_wave=3), hac.Launch(variant=0x800)):
                print(f"[case] per-column chunks {name} {fmt} B={B} variant={launch.variant:#x} cpw={launch.cols_per_wave}", flush=True)
                Y = dot(db, Xd, launch=launch)
                torch.cuda.synchronize()
                check_y(Y, X, W, f"{name} {fmt} B={B}")
        # unit vectors: the rows of W back, bit for bit
        rows = np.sort(rng.choice(n, size=96, replace=False))
        X = np.zeros((96, n), dtype=np.float32)
        X[np.arange(96), rows] = 1.0
        for B in (1, 4, 96):
            print(f"[case] per-column chunks one-hot {name} {fmt} B={B}", flush=True)
            Y = dot(db, torch.from_numpy(X[:B]).to(dev), launch=hac.Launch(variant=0x400))
            torch.cuda.synchronize()
            assert np.array_equal(Y.cpu().numpy(), W[rows[:B], :]), (name, fmt, B)


def test_decode_and_device_encoder_with_per_column_chunks(hac):
    dev = torch.device("cuda:0")
    W = uneven(1800, 60, 5)
    values, sym = formats.hac_symbols(W)
    blob = hac.hac_encode(W, chunk_nnz=hac.CHUNK_PER_COLUMN)
    print("[case] per-column chunks hac_decode_dev", flush=True)
    Wd, symd = hac.hac_decode_dev(blob.to_device(dev))
    torch.cuda.synchronize()
    assert np.array_equal(Wd.cpu().numpy(), W)
    assert np.array_equal(symd.cpu().numpy(), sym)
    sblob = hac.shac_encode(W, chunk_nnz=hac.CHUNK_PER_COLUMN)
    print("[case] per-column chunks shac_decode_dev", flush=True)
    nz, ssym, row, col = hac.shac_decode_dev(sblob.to_device(dev))
    torch.cuda.synchronize()
    values_s, sym_s, row_s, col_s = formats.shac_symbols(W)
    assert np.array_equal(ssym.cpu().numpy(), sym_s) and np.array_equal(row.cpu().numpy(), row_s)
    assert np.array_equal(col.cpu().numpy(), col_s) and np.array_equal(nz.cpu().numpy(), values_s[sym_s])
    for fmt, host in ((hac.HAC_FORMAT_HAC, blob), (hac.HAC_FORMAT_SHAC, sblob)):
        print(f"[case] per-column chunks hac_encode_dev format {fmt}", flush=True)
        dblob = hac.hac_encode_dev(torch.from_numpy(W).to(dev), fmt=fmt, chunk_nnz=hac.CHUNK_PER_COLUMN)
        torch.cuda.synchronize()
        assert np.array_equal(dblob.tensor.cpu().numpy(), host.data), fmt
