"""GPU parity: layers of a network blob (one shared dictionary, Sect. V-H) and the chain of
layers hac_forward.

Per-layer products keep the bar of the single-layer tests.  The chain is compared with the
oracle's fp64 chain inside the forward error bound that follows from that bar
(oracle.unified.chain_bound with rel = 1e-5), and bit for bit with the same layers multiplied
one call at a time.
"""
import ctypes as C

import numpy as np
import pytest

import workloads
from oracle import dot as odot
from oracle import formats, unified

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5
HAC, SHAC = 1, 2
KIND = {HAC: "hac", SHAC: "shac"}


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
    err = np.abs(got - ref)
    bad = err > TOL * scale + 1e-37
    assert not bad.any(), f"{what}: {int(bad.sum())} entries off"
    if ref.size and np.abs(ref).max() > 0:
        assert err.max() <= TOL * np.abs(ref).max(), what


def check_chain(Y, X, Ws, bs, relu, what=""):
    ref = unified.chain(X, Ws, bs, relu)[-1]
    bound = unified.chain_bound(X, Ws, bs, relu, rel=TOL)[-1]
    got = Y.detach().cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape, what
    err = np.abs(got - ref)
    bad = err > bound + 1e-37
    assert not bad.any(), f"{what}: {int(bad.sum())} entries outside the bound, worst ratio {float((err / (bound + 1e-300)).max()):.3e}"


@pytest.mark.parametrize("fmts,ri_coding", [((HAC, HAC, HAC), 0), ((SHAC, SHAC, SHAC), 0), ((HAC, SHAC, HAC), 0),
                                            ((SHAC, HAC, SHAC), 1)])
@pytest.mark.parametrize("B", [1, 3, 40])
def test_layers_of_a_network_blob(hac, fmts, ri_coding, B):
    Ws, _ = workloads.network("tiny-fc")
    nb = hac.hac_net_encode(Ws, fmts, ri_coding=ri_coding)
    assert nb.validate(deep=True) == 0
    dls = nb.to_device(dev())
    assert all(dl.tensor.data_ptr() == dls[0].tensor.data_ptr() for dl in dls)          # one device copy
    u_values, _ = unified.pooled_alphabet([KIND[f] for f in fmts], Ws)
    for l, (fmt, W, dl) in enumerate(zip(fmts, Ws, dls)):
        X = workloads.make_batch(B, W.shape[0], 90 + l)
        dot = hac.hac_dot if fmt == HAC else hac.shac_dot
        Y = dot(dl, torch.from_numpy(X).to(dev()))
        torch.cuda.synchronize()
        check_y(Y, X, W, f"layer {l} fmt {fmt} B {B}")
        # the device decoder reproduces the symbols of the shared alphabet, bit-exact
        if fmt == HAC:
            Wd, sym = hac.hac_decode_dev(dl)
            torch.cuda.synchronize()
            ref = formats.symbol_indices(formats.column_order(W), u_values)
            assert np.array_equal(sym.cpu().numpy().astype(np.int64), ref)
            assert np.array_equal(Wd.cpu().numpy(), W)
        else:
            nz, sym, row, col = hac.shac_decode_dev(dl)
            torch.cuda.synchronize()
            nz_ref, ri, cb = formats.csc_arrays(W)
            assert np.array_equal(sym.cpu().numpy().astype(np.int64), formats.symbol_indices(nz_ref, u_values))
            assert np.array_equal(row.cpu().numpy().astype(np.int64), ri)
            assert np.array_equal(nz.cpu().numpy(), nz_ref)


def _layers(hac, dls, bs, relu):
    return [(dl, None if b is None else torch.from_numpy(b).to(dev()), bool(r)) for dl, b, r in zip(dls, bs, relu)]


def _one_call_at_a_time(hac, fmts, dls, bs, relu, X):
    A = torch.from_numpy(X).to(dev())
    for fmt, dl, b, r in zip(fmts, dls, bs, relu):
        dot = {HAC: hac.hac_dot, SHAC: hac.shac_dot, 3: hac.im_dot}[fmt]
        A = dot(dl, A)
        if b is not None:
            A = A + torch.from_numpy(b).to(dev())[None, :]
        if r:
            A = torch.clamp_min(A, 0.0)
    return A


@pytest.mark.parametrize("B", [1, 2, 4, 5, 32, 70, 300, 513])
@pytest.mark.parametrize("fmts", [(HAC, HAC, HAC), (SHAC, SHAC, SHAC), (HAC, SHAC, HAC)])
def test_chain_on_a_network_blob(hac, fmts, B):
    Ws, bs = workloads.network("tiny-fc")
    bs = [bs[0], None, bs[2]]
    relu = [True, True, False]
    nb = hac.hac_net_encode(Ws, fmts)
    dls = nb.to_device(dev())
    X = workloads.make_batch(B, Ws[0].shape[0], 17)
    Y = hac.hac_forward(_layers(hac, dls, bs, relu), torch.from_numpy(X).to(dev()))
    torch.cuda.synchronize()
    check_chain(Y, X, Ws, bs, relu, f"fmts {fmts} B {B}")
    Yseq = _one_call_at_a_time(hac, fmts, dls, bs, relu, X)
    torch.cuda.synchronize()
    assert torch.equal(Y, Yseq), "the chain differs from its layers multiplied one call at a time"


def test_chain_of_separate_blobs_with_an_index_map_in_the_middle(hac):
    # sparse -> index map (row-major, matrix cores) -> sparse: both kinds of hand-over
    Ws, bs = workloads.network("tiny-fc")
    relu = [True, False, True]
    blobs = [hac.hac_encode(Ws[0]), hac.im_encode(Ws[1]), hac.shac_encode(Ws[2], ri_coding=hac.RI_RICE)]
    dls = [b.to_device(dev()) for b in blobs]
    for B in (1, 7, 64, 260):
        X = workloads.make_batch(B, Ws[0].shape[0], 23)
        Y = hac.hac_forward(_layers(hac, dls, bs, relu), torch.from_numpy(X).to(dev()))
        torch.cuda.synchronize()
        check_chain(Y, X, Ws, bs, relu, f"B {B}")
        Yseq = _one_call_at_a_time(hac, (HAC, 3, SHAC), dls, bs, relu, X)
        torch.cuda.synchronize()
        assert torch.equal(Y, Yseq)


def test_hybrid_network_blob_index_map_then_compressed_layers(hac):
    # Sect. V-K: an unpruned layer as index map and pruned layers as HAC / sHAC, one value list
    rng = np.random.default_rng(3)
    Ws, bs = workloads.network("tiny-fc")
    reps = np.concatenate([np.unique(Ws[0][Ws[0] != 0])[:3], np.array([-0.31, 0.07, 0.5], dtype=np.float32)])
    conv = rng.choice(reps, size=(260, 500)).astype(np.float32)                 # 260 -> 500 in front of tiny-fc
    layers = [conv] + Ws
    fmts = (3, HAC, SHAC, HAC)
    nb = hac.hac_net_encode(layers, fmts)
    assert nb.validate(deep=True) == 0 and nb.net.k_values > nb.net.k_sym
    dls = nb.to_device(dev())
    bs = [None] + bs
    relu = [True, True, True, False]
    for B in (1, 9, 64, 300):
        X = workloads.make_batch(B, 260, 51)
        Y0 = hac.im_dot(dls[0], torch.from_numpy(X).to(dev()))
        torch.cuda.synchronize()
        check_y(Y0, X, conv, f"index-map layer of the network blob, B {B}")
        Y = hac.hac_forward(_layers(hac, dls, bs, relu), torch.from_numpy(X).to(dev()))
        torch.cuda.synchronize()
        check_chain(Y, X, layers, bs, relu, f"hybrid chain B {B}")
        assert torch.equal(Y, _one_call_at_a_time(hac, fmts, dls, bs, relu, X))


def test_randomized_chains(hac):
    # seeded sweep: 1-5 layers of random widths (1 included), densities (0 and 1 included), formats
    # (HAC, sHAC with fields or Rice-coded gaps, index map), biases, activations and batch sizes,
    # as one network blob or as separate blobs
    rng = np.random.default_rng(20240607)
    for case in range(40):
        L = int(rng.integers(1, 6))
        widths = [int(rng.choice([1, 2, 7, 33, 64, 129, 300])) for _ in range(L + 1)]
        k = int(rng.choice([1, 3, 17, 200]))
        reps = np.unique((rng.normal(0, 0.2, k) + 0.01).astype(np.float32))
        reps = reps[reps != 0]
        Ws = []
        for l in range(L):
            dens = float(rng.choice([0.0, 0.02, 0.3, 1.0]))
            W = reps[rng.integers(0, reps.size, size=(widths[l], widths[l + 1]))].astype(np.float32)
            W[rng.random(W.shape) >= dens] = 0.0
            Ws.append(np.ascontiguousarray(W))
        fmts = [int(rng.choice([HAC, SHAC, 3])) for _ in range(L)]
        rice = int(rng.integers(0, 2))
        bs = [None if rng.random() < 0.4 else rng.normal(0, 0.1, widths[l + 1]).astype(np.float32) for l in range(L)]
        relu = [bool(rng.integers(0, 2)) for _ in range(L)]
        B = int(rng.choice([1, 2, 3, 4, 6, 31, 32, 33, 100, 257, 600]))
        print(f"[case] chain {case}: widths {widths} fmts {fmts} rice {rice} B {B}", flush=True)
        if rng.random() < 0.5:
            dls = hac.hac_net_encode(Ws, fmts, ri_coding=rice).to_device(dev())
        else:
            enc = {HAC: lambda W: hac.hac_encode(W), SHAC: lambda W: hac.shac_encode(W, ri_coding=rice), 3: hac.im_encode}
            dls = [enc[f](W).to_device(dev()) for f, W in zip(fmts, Ws)]
        X = workloads.make_batch(B, widths[0], 1000 + case)
        Y = hac.hac_forward(_layers(hac, dls, bs, relu), torch.from_numpy(X).to(dev()))
        torch.cuda.synchronize()
        check_chain(Y, X, Ws, bs, relu, f"case {case}")
        assert torch.equal(Y, _one_call_at_a_time(hac, fmts, dls, bs, relu, X)), f"case {case}"


def test_single_layer_chain_equals_dot_with_epilogue(hac):
    W = workloads.layer(1)
    b = workloads.make_biases(((W.shape[0], W.shape[1]),), 3)[0]
    dl = hac.shac_encode(W).to_device(dev())
    for B in (1, 8, 33):
        X = workloads.make_batch(B, W.shape[0], 4)
        Y = hac.hac_forward([(dl, torch.from_numpy(b).to(dev()), True)], torch.from_numpy(X).to(dev()))
        torch.cuda.synchronize()
        check_chain(Y, X, [W], [b], [True])
        # no bias, no activation: exactly shac_dot
        Y0 = hac.hac_forward([(dl, None, False)], torch.from_numpy(X).to(dev()))
        assert torch.equal(Y0, hac.shac_dot(dl, torch.from_numpy(X).to(dev())))


def test_chain_padded_rows_and_strides(hac):
    # X and Y with leading dimensions larger than their widths; the padding of Y stays untouched
    Ws, bs = workloads.network("tiny-fc")
    relu = [True, True, True]
    dls = hac.hac_net_encode(Ws, (HAC, HAC, SHAC)).to_device(dev())
    B = 37
    X = workloads.make_batch(B, Ws[0].shape[0], 5)
    Xp = torch.zeros((B, Ws[0].shape[0] + 12), device=dev())
    Xp[:, :Ws[0].shape[0]] = torch.from_numpy(X).to(dev())
    Yp = torch.full((B, Ws[2].shape[1] + 6), -7.0, device=dev())
    hac.hac_forward(_layers(hac, dls, bs, relu), Xp[:, :Ws[0].shape[0]], Y=Yp[:, :Ws[2].shape[1]])
    torch.cuda.synchronize()
    check_chain(Yp[:, :Ws[2].shape[1]], X, Ws, bs, relu)
    assert torch.all(Yp[:, Ws[2].shape[1]:] == -7.0)


def test_chain_argument_checks(hac):
    lib = hac.load_library()
    Ws, bs = workloads.network("tiny-fc")
    dls = hac.hac_net_encode(Ws, (HAC, HAC, HAC)).to_device(dev())
    X = torch.from_numpy(workloads.make_batch(8, Ws[0].shape[0], 1)).to(dev())
    # layers that do not chain
    with pytest.raises(hac.HacError) as e:
        hac.hac_forward([(dls[0], None, False), (dls[2], None, False)], X)
    assert e.value.status == -1
    # workspace too small / missing
    layers = [(dl, None, True) for dl in dls]
    arr = hac._layer_array(layers)
    need = lib.hac_forward_workspace_bytes(arr, 3, 8)
    assert need > 0
    Y = torch.empty((8, Ws[2].shape[1]), device=dev())
    ws = torch.empty(need, dtype=torch.uint8, device=dev())
    args = (arr, 3, X.data_ptr(), 8, X.stride(0), Y.data_ptr(), Y.stride(0))
    assert lib.hac_forward(*args, ws.data_ptr(), need - 1, None) == -6
    assert lib.hac_forward(*args, None, 0, None) == -6
    assert lib.hac_forward(*args, ws.data_ptr() + 4, need, None) == -1            # misaligned
    assert lib.hac_forward(arr, 0, X.data_ptr(), 8, X.stride(0), Y.data_ptr(), Y.stride(0), ws.data_ptr(), need, None) == -1
    assert lib.hac_forward(arr, 3, X.data_ptr(), 8, 10, Y.data_ptr(), Y.stride(0), ws.data_ptr(), need, None) == -1
    arr[1].activation = 9
    assert lib.hac_forward(*args, ws.data_ptr(), need, None) == -1
    arr[1].activation = 1
    assert lib.hac_forward(arr, 3, X.data_ptr(), 0, X.stride(0), Y.data_ptr(), Y.stride(0), None, 0, None) == 0   # B = 0
    assert lib.hac_forward(*args, ws.data_ptr(), need, None) == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("B", [1, 3, 6, 32, 256])
def test_chain_full_size_vgg19_block(hac, B):
    # the fully connected block whose matrices the paper times (512x4096, 4096x4096, 4096x10)
    Ws, bs = workloads.network("vgg19-fc")
    relu = [True, True, False]
    fmts = [hac.hac_choose_format(W.shape[0], W.shape[1], int(np.count_nonzero(W)), 32) for W in Ws]
    nb = hac.hac_net_encode(Ws, fmts)
    dls = nb.to_device(dev())
    X = workloads.make_batch(B, 512, 77)
    Y = hac.hac_forward(_layers(hac, dls, bs, relu), torch.from_numpy(X).to(dev()))
    torch.cuda.synchronize()
    check_chain(Y, X, Ws, bs, relu, f"B {B}")
    assert torch.equal(Y, _one_call_at_a_time(hac, fmts, dls, bs, relu, X))
