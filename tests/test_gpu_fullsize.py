"""GPU parity at the configurations' full sizes, in the launch configuration the
benchmark times (default encoder options, default launch).

Decode: every decoded value / symbol / index against the oracle's ground truth
(bit-exact).  Y: a sample of output columns (all batch rows, or a sample of them
for the largest batch) against the dense fp64 product computed one column at a
time, to the tolerance of test_gpu_parity.
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
    assert torch.cuda.is_available()
    return lib


_layers = {}


def layer(cfg):
    if cfg not in _layers:
        _layers.clear()                       # keep one big matrix at a time
        _layers[cfg] = workloads.layer(cfg)
    return _layers[cfg]


def check_sampled(Y, X, W, cols, rows, what):
    Ys = Y[rows][:, cols].cpu().numpy().astype(np.float64)
    Xs = X[rows]
    Ws = W[:, cols]
    ref = odot.dense_dot(Xs, Ws)
    scale = odot.abs_dot(Xs, Ws)
    err = np.abs(Ys - ref)
    bad = err > TOL * scale + 1e-37
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} sampled outputs off"
    assert err.max() <= TOL * np.abs(ref).max(), what


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_dot(hac, cfg):
    c = workloads.CONFIGS[cfg]
    W = layer(cfg)
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(cfg)
    cols = np.sort(rng.choice(c.m, size=min(c.m, 96), replace=False))
    cols = np.unique(np.concatenate((cols, [0, c.m - 1])))
    hb = hac.hac_encode(W)
    sb = hac.shac_encode(W)
    gb = hac.shac_encode(W, ri_coding=hac.RI_RICE)          # Rice-coded row gaps (extension)
    assert hb.validate(deep=False) == 0 and sb.validate(deep=False) == 0 and gb.validate(deep=False) == 0
    dh, ds, dg = hb.to_device(dev), sb.to_device(dev), gb.to_device(dev)
    # beside the benchmark's batches, on the large layer: a ragged small batch (two lanes per row
    # group) and one that ends in a tile with two of its eight passes
    for B in list(c.batches) + ([5, 300] if cfg == 4 else []):
        print(f"[case] full cfg{cfg} B={B}", flush=True)
        X = workloads.make_batch(B, c.n, 1000 * cfg + 1)
        rows = np.arange(B) if B <= 256 else np.unique(np.concatenate((rng.choice(B, 254, replace=False), [0, B - 1])))
        Xd = torch.from_numpy(X).to(dev)
        Yh = hac.hac_dot(dh, Xd)
        Ys = hac.shac_dot(ds, Xd)
        Yg = hac.shac_dot(dg, Xd)
        torch.cuda.synchronize()
        check_sampled(Yh, X, W, cols, rows, f"hac cfg{cfg} B={B}")
        check_sampled(Ys, X, W, cols, rows, f"shac cfg{cfg} B={B}")
        check_sampled(Yg, X, W, cols, rows, f"shac/rice cfg{cfg} B={B}")
        assert torch.isfinite(Yg).all()
        assert (Yh - Yg).abs().max().item() <= 4 * TOL * max(Yh.abs().max().item(), 1e-30)
        del Yg
        # properties that hold at any size: Y is finite everywhere, and the two formats, which
        # hold the same matrix, agree to rounding on every output (not only the sampled ones)
        assert torch.isfinite(Yh).all() and torch.isfinite(Ys).all()
        assert (Yh - Ys).abs().max().item() <= 4 * TOL * max(Yh.abs().max().item(), 1e-30)
        del Xd, Yh, Ys


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_decode(hac, cfg):
    c = workloads.CONFIGS[cfg]
    W = layer(cfg)
    dev = torch.device("cuda:0")
    print(f"[case] full decode cfg{cfg}", flush=True)
    values, sym = formats.hac_symbols(W)
    hb = hac.hac_encode(W)
    Wd, symd = hac.hac_decode_dev(hb.to_device(dev))
    torch.cuda.synchronize()
    assert torch.equal(Wd.view(torch.int32), torch.from_numpy(W.view(np.int32)).to(dev))
    assert torch.equal(symd, torch.from_numpy(sym.astype(np.int32)).to(dev))
    assert np.array_equal(hb.section("off_codebook", np.float32, len(values)), values)
    del Wd, symd
    values, sym, row, col = formats.shac_symbols(W)
    sb = hac.shac_encode(W)
    nz, symd, rowd, cold = hac.shac_decode_dev(sb.to_device(dev))
    torch.cuda.synchronize()
    assert np.array_equal(symd.cpu().numpy().astype(np.int64), sym)
    assert np.array_equal(rowd.cpu().numpy().astype(np.int64), row)
    assert np.array_equal(cold.cpu().numpy().astype(np.int64), col)
    assert np.array_equal(nz.cpu().numpy().view(np.uint32), values[sym].view(np.uint32))
    del nz, symd, rowd, cold
    gb = hac.shac_encode(W, ri_coding=hac.RI_RICE)
    nz, symd, rowd, cold = hac.shac_decode_dev(gb.to_device(dev))
    torch.cuda.synchronize()
    assert np.array_equal(symd.cpu().numpy().astype(np.int64), sym)
    assert np.array_equal(rowd.cpu().numpy().astype(np.int64), row)
    assert np.array_equal(cold.cpu().numpy().astype(np.int64), col)
    assert np.array_equal(nz.cpu().numpy().view(np.uint32), values[sym].view(np.uint32))
