"""GPU parity: the HIP path against the CPU oracle, through the C ABI.

Decoded symbols, values and indices must match the oracle bit for bit.
Y must satisfy, with fp32 accumulation,
    |Y - Yref|_ij <= 1e-5 * (|X| . |W|)_ij      (componentwise), and
    max |Y - Yref| <= 1e-5 * max |Yref|,
where Yref is the dense fp64 product with the matrix that was encoded.
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


def layer_cases():
    yield "cfg1", workloads.layer(1)
    yield "cfg2-700x129", workloads.scaled(2, 700, 129)
    yield "cfg3-1100x70", workloads.scaled(3, 1100, 70)
    yield "cfg4-3000x65", workloads.scaled(4, 3000, 65)
    yield "cfg5-640x33", workloads.scaled(5, 640, 33)
    for name, W in workloads.edge_cases().items():
        yield name, W


CASES = list(layer_cases())
CASE_IDS = [c[0] for c in CASES]


@pytest.mark.parametrize("name,W", CASES, ids=CASE_IDS)
def test_hac_decode_bit_exact(hac, name, W):
    print(f"[case] hac_decode {name} {W.shape}", flush=True)
    values, sym = formats.hac_symbols(W)
    for kw in (dict(), dict(chunk_nnz=1), dict(chunk_nnz=37), dict(lut_bits=3)):
        blob = hac.hac_encode(W, **kw)
        Wd, symd = hac.hac_decode_dev(blob.to_device(dev()))
        torch.cuda.synchronize()
        assert np.array_equal(Wd.cpu().numpy().view(np.uint32), W.view(np.uint32)), kw
        assert np.array_equal(symd.cpu().numpy().astype(np.int64), sym), kw


@pytest.mark.parametrize("name,W", CASES, ids=CASE_IDS)
def test_shac_decode_bit_exact(hac, name, W):
    print(f"[case] shac_decode {name} {W.shape}", flush=True)
    values, sym, row, col = formats.shac_symbols(W)
    for kw in (dict(), dict(chunk_nnz=5), dict(ri_bits=32), dict(lut_bits=2),
               dict(ri_coding=1), dict(ri_coding=1, chunk_nnz=3), dict(ri_coding=1, lut_bits=2, chunk_nnz=1000)):
        blob = hac.shac_encode(W, **kw)
        nz, symd, rowd, cold = hac.shac_decode_dev(blob.to_device(dev()))
        torch.cuda.synchronize()
        assert np.array_equal(symd.cpu().numpy().astype(np.int64), sym), kw
        assert np.array_equal(rowd.cpu().numpy().astype(np.int64), row), kw
        assert np.array_equal(cold.cpu().numpy().astype(np.int64), col), kw
        assert np.array_equal(nz.cpu().numpy().view(np.uint32), values[sym].view(np.uint32)), kw


BATCHES = [1, 2, 3, 8, 31, 32, 64, 65, 128, 200, 256, 300]


@pytest.mark.parametrize("name,W", CASES, ids=CASE_IDS)
def test_dot_parity_small(hac, name, W):
    n, m = W.shape
    hb = hac.hac_encode(W).to_device(dev())
    sb = hac.shac_encode(W).to_device(dev())
    gb = hac.shac_encode(W, ri_coding=1).to_device(dev())               # Rice-coded row gaps
    for B in BATCHES:
        print(f"[case] dot {name} {W.shape} B={B}", flush=True)
        X = workloads.make_batch(B, n, 77 + B) - np.float32(0.125)      # a few negative inputs too
        Xd = torch.from_numpy(X).to(dev())
        Yh = hac.hac_dot(hb, Xd)
        Ys = hac.shac_dot(sb, Xd)
        Yg = hac.shac_dot(gb, Xd)
        torch.cuda.synchronize()
        check_y(Yh, X, W, f"hac {name} B={B}")
        check_y(Ys, X, W, f"shac {name} B={B}")
        check_y(Yg, X, W, f"shac/rice {name} B={B}")


@pytest.mark.parametrize("name", sorted(workloads.stress_cases().keys()))
def test_stress_cases(hac, name):
    """Alphabets above 1024 symbols, codewords beyond the first-level table, 64-bit chunk entries,
    columns with far more than 64 chunks."""
    W = workloads.stress_cases()[name]
    n, m = W.shape
    print(f"[case] stress {name} {W.shape}", flush=True)
    values, sym = formats.hac_symbols(W)
    hb, sb = hac.hac_encode(W), hac.shac_encode(W)
    Wd, symd = hac.hac_decode_dev(hb.to_device(dev()))
    nz, ssym, srow, scol = hac.shac_decode_dev(sb.to_device(dev()))
    torch.cuda.synchronize()
    assert np.array_equal(Wd.cpu().numpy().view(np.uint32), W.view(np.uint32))
    assert np.array_equal(symd.cpu().numpy().astype(np.int64), sym)
    svalues, s_sym, s_row, s_col = formats.shac_symbols(W)
    assert np.array_equal(ssym.cpu().numpy().astype(np.int64), s_sym)
    assert np.array_equal(srow.cpu().numpy().astype(np.int64), s_row)
    assert np.array_equal(scol.cpu().numpy().astype(np.int64), s_col)
    assert np.array_equal(nz.cpu().numpy().view(np.uint32), svalues[s_sym].view(np.uint32))
    gb = hac.shac_encode(W, ri_coding=1)
    nz, ssym, srow, scol = hac.shac_decode_dev(gb.to_device(dev()))
    torch.cuda.synchronize()
    assert np.array_equal(ssym.cpu().numpy().astype(np.int64), s_sym)
    assert np.array_equal(srow.cpu().numpy().astype(np.int64), s_row)
    assert np.array_equal(scol.cpu().numpy().astype(np.int64), s_col)
    dh, ds, dg = hb.to_device(dev()), sb.to_device(dev()), gb.to_device(dev())
    for B in (1, 5, 32, 70):
        X = workloads.make_batch(B, n, 11 + B) - np.float32(0.25)
        Xd = torch.from_numpy(X).to(dev())
        Yh = hac.hac_dot(dh, Xd)
        Ys = hac.shac_dot(ds, Xd)
        Yg = hac.shac_dot(dg, Xd)
        torch.cuda.synchronize()
        check_y(Yh, X, W, f"hac {name} B={B}")
        check_y(Ys, X, W, f"shac {name} B={B}")
        check_y(Yg, X, W, f"shac/rice {name} B={B}")


def test_randomized_parity(hac):
    """Seeded sweep: random shapes, densities, alphabets and skews x all formats x a few batch sizes."""
    rng = np.random.default_rng(99)
    for name, W in workloads.random_cases(40, seed=77):
        n, m = W.shape
        chunk = int(rng.choice([0, 0, 1, 7, 200, hac.CHUNK_PER_COLUMN]))
        blobs = [(hac.hac_dot, hac.hac_encode(W, chunk_nnz=chunk)), (hac.shac_dot, hac.shac_encode(W, chunk_nnz=chunk)),
                 (hac.shac_dot, hac.shac_encode(W, chunk_nnz=chunk, ri_coding=1)), (hac.im_dot, hac.im_encode(W))]
        for B in (1, int(rng.integers(2, 5)), int(rng.integers(5, 140))):
            print(f"[case] random {name} chunk={chunk} B={B}", flush=True)
            X = workloads.make_batch(B, n, B + n) - np.float32(0.3)
            Xd = torch.from_numpy(X).to(dev())
            variant = int(rng.choice([0, 0x400, 0x800]))
            for f, blob in blobs:
                db = blob.to_device(dev())
                Y = f(db, Xd) if f is hac.im_dot else f(db, Xd, launch=hac.Launch(variant=variant))
                torch.cuda.synchronize()
                check_y(Y, X, W, f"{f.__name__} {name} B={B} variant={variant:#x}")


def test_dot_other_encoder_options(hac):
    W = workloads.scaled(3, 1500, 90)
    n, m = W.shape
    X8 = workloads.make_batch(8, n, 3)
    blobs = [(hac.hac_dot, hac.hac_encode(W, chunk_nnz=1)),
             (hac.hac_dot, hac.hac_encode(W, chunk_nnz=100)),
             (hac.hac_dot, hac.hac_encode(W, chunk_nnz=4096, lut_bits=2)),
             (hac.shac_dot, hac.shac_encode(W, chunk_nnz=3)),
             (hac.shac_dot, hac.shac_encode(W, chunk_nnz=1000, ri_bits=32, lut_bits=4))]
    for f, blob in blobs:
        db = blob.to_device(dev())
        for X in (X8[:1], X8):
            print(f"[case] options {f.__name__} chunk={blob.desc.chunk} B={X.shape[0]}", flush=True)
            Y = f(db, torch.from_numpy(X).to(dev()))
            torch.cuda.synchronize()
            check_y(Y, X, W, f.__name__)


def test_short_x_kept_in_lds_matches_the_relayout_route(hac):
    """2 to 8 batch rows over a short X run with X copied into LDS by every block and no workspace;
    HAC_LAUNCH_NO_X_LDS (0x1000) sends them through the re-layout instead.  Same kernel arithmetic up to
    4 rows (bitwise equal), another summation order from 5 rows on."""
    no_lds = hac.Launch(variant=0x1000)
    for name, W in (("cfg1", workloads.layer(1)), ("cfg2-1000x77", workloads.scaled(2, 1000, 77)),
                    ("cfg5-640x33", workloads.scaled(5, 640, 33)), ("cfg3-4096x50", workloads.scaled(3, 4096, 50))):
        n = W.shape[0]
        for enc, dot, kw in ((hac.hac_encode, hac.hac_dot, {}), (hac.shac_encode, hac.shac_dot, {}),
                             (hac.shac_encode, hac.shac_dot, dict(ri_coding=hac.RI_RICE))):
            blob = enc(W, **kw)
            db = blob.to_device(dev())
            for B in (2, 3, 4, 5, 8):
                in_lds = hac.hac_workspace_bytes(blob.desc, B) == 0
                assert in_lds == (n * (2 if B <= 2 else 4 if B <= 4 else 8) <= 8192), (name, B)
                assert hac.hac_workspace_bytes(blob.desc, B, no_lds) > 0
                X = workloads.make_batch(B, n, 60 + B) - np.float32(0.2)
                Xd = torch.from_numpy(X).to(dev())
                print(f"[case] x in lds {name} {dot.__name__} {kw} B={B} in_lds={in_lds}", flush=True)
                Y = dot(db, Xd)
                Yold = dot(db, Xd, launch=no_lds)
                torch.cuda.synchronize()
                check_y(Y, X, W, f"{name} B={B}")
                check_y(Yold, X, W, f"{name} B={B} re-layout")
                if B <= 4:
                    assert torch.equal(Y, Yold), (name, B)
    # strided X and Y
    W = workloads.layer(1)
    db = hac.shac_encode(W).to_device(dev())
    X = workloads.make_batch(6, W.shape[0], 9)
    Xp = torch.zeros((6, W.shape[0] + 7), device=dev())
    Xp[:, :W.shape[0]] = torch.from_numpy(X).to(dev())
    Yp = torch.full((6, W.shape[1] + 3), -3.0, device=dev())
    hac.shac_dot(db, Xp[:, :W.shape[0]], Y=Yp[:, :W.shape[1]])
    torch.cuda.synchronize()
    check_y(Yp[:, :W.shape[1]], X, W, "strided")
    assert torch.all(Yp[:, W.shape[1]:] == -3.0)


def test_workspace_left_overs_do_not_reach_the_result(hac):
    """Panels of the re-laid-out X that hold only padding rows are neither written nor read: a
    workspace full of NaN must not show in Y (batches that are not a multiple of 32 or of 256)."""
    W = workloads.scaled(3, 900, 130)
    n = W.shape[0]
    for enc, dot in ((hac.hac_encode, hac.hac_dot), (hac.shac_encode, hac.shac_dot)):
        blob = enc(W)
        db = blob.to_device(dev())
        for B in (9, 33, 70, 129, 257, 300):
            X = workloads.make_batch(B, n, 80 + B)
            ws = torch.full((hac.hac_workspace_bytes(blob.desc, B) // 4,), float("nan"), device=dev())
            Y = dot(db, torch.from_numpy(X).to(dev()), workspace=ws.view(torch.uint8))
            torch.cuda.synchronize()
            assert not torch.isnan(Y).any(), (dot.__name__, B)
            check_y(Y, X, W, f"{dot.__name__} B={B}")


def test_launch_overrides_do_not_change_the_result(hac):
    W = workloads.scaled(5, 900, 77)          # ~360 non-zeros per column
    n, m = W.shape
    X = workloads.make_batch(40, n, 9)
    Xd = torch.from_numpy(X).to(dev())
    rice_encode = lambda W: hac.shac_encode(W, ri_coding=1)
    for enc, f in ((hac.hac_encode, hac.hac_dot), (hac.shac_encode, hac.shac_dot), (rice_encode, hac.shac_dot)):
        db = enc(W).to_device(dev())
        for cpw, wpb, cap, sbuf in ((1, 1, 64, 0), (3, 2, 64, 16), (7, 4, 128, 64), (32, 4, 2048, 4096), (5, 16, 256, 0),
                                    (2, 3, 1024, 0)):
            print(f"[case] launch {f.__name__} cpw={cpw} wpb={wpb} cap={cap} sbuf={sbuf}", flush=True)
            launch = hac.Launch(cols_per_wave=cpw, waves_per_block=wpb)
            launch.list_entries = cap          # list capacity: small values force several windows per column
            launch.staging_words = sbuf         # staging buffer: small values force the unstaged reader
            launch.pass_width = 64 if cpw == 7 else 0     # batch columns per pass
            Y = f(db, Xd, launch=launch)
            Y1 = f(db, Xd[:1], launch=launch)
            torch.cuda.synchronize()
            check_y(Y, X, W, f"{f.__name__} cpw={cpw}")
            check_y(Y1, X[:1], W, f"{f.__name__} B=1 cpw={cpw}")


def test_small_batches_through_both_kernels(hac):
    """B <= 4 has a kernel of its own; the list-based kernel must still serve it on request."""
    for name, W in (("cfg4-3000x65", workloads.scaled(4, 3000, 65)), ("cfg5-640x33", workloads.scaled(5, 640, 33)),
                    ("empty_columns", workloads.edge_cases()["empty_columns"])):
        n, m = W.shape
        for enc, f, kw in ((hac.hac_encode, hac.hac_dot, dict()), (hac.shac_encode, hac.shac_dot, dict()),
                           (hac.hac_encode, hac.hac_dot, dict(chunk_nnz=1)), (hac.shac_encode, hac.shac_dot, dict(chunk_nnz=2)),
                           (hac.shac_encode, hac.shac_dot, dict(ri_coding=1)),
                           (hac.shac_encode, hac.shac_dot, dict(ri_coding=1, chunk_nnz=2))):
            db = enc(W, **kw).to_device(dev())
            for B in (1, 2, 3, 4):
                X = workloads.make_batch(B, n, 5 + B) - np.float32(0.5)
                Xd = torch.from_numpy(X).to(dev())
                for variant, cpw in ((0, 0), (0x200, 0), (0, 5), (0x200, 3)):
                    print(f"[case] small {f.__name__} {name} B={B} variant={variant:#x} cpw={cpw} {kw}", flush=True)
                    Y = f(db, Xd, launch=hac.Launch(cols_per_wave=cpw, variant=variant))
                    torch.cuda.synchronize()
                    check_y(Y, X, W, f"{f.__name__} {name} B={B} variant={variant:#x}")


def test_identity_batch_recovers_w_bit_exact(hac):
    W = workloads.scaled(2, 96, 50)
    eye = torch.eye(96, dtype=torch.float32, device=dev())
    for enc, f in ((hac.hac_encode, hac.hac_dot), (hac.shac_encode, hac.shac_dot)):
        Y = f(enc(W).to_device(dev()), eye)
        torch.cuda.synchronize()
        assert np.array_equal(Y.cpu().numpy().view(np.uint32), W.view(np.uint32))


def test_results_are_bitwise_reproducible(hac):
    W = workloads.scaled(4, 2048, 128)
    X = torch.from_numpy(workloads.make_batch(32, 2048, 1)).to(dev())
    for enc, f in ((hac.hac_encode, hac.hac_dot), (hac.shac_encode, hac.shac_dot)):
        db = enc(W).to_device(dev())
        for Xb in (X, X[:1]):
            a = f(db, Xb).clone()
            b = f(db, Xb).clone()
            torch.cuda.synchronize()
            assert torch.equal(a, b)


def test_calls_from_several_threads_on_their_own_streams(hac):
    # the header promises that calls on distinct arguments may run concurrently: four host threads,
    # each with its own stream, blob, X, Y and workspace, must each reproduce the single-thread bits
    import threading
    jobs = []
    for t, (enc, f, B) in enumerate(((hac.hac_encode, hac.hac_dot, 1), (hac.shac_encode, hac.shac_dot, 3),
                                     (hac.hac_encode, hac.hac_dot, 40), (hac.shac_encode, hac.shac_dot, 300))):
        W = workloads.scaled(4, 1500 + 100 * t, 90 + t)
        blob = enc(W)
        db = blob.to_device(dev())
        X = torch.from_numpy(workloads.make_batch(B, W.shape[0], 50 + t)).to(dev())
        ws = torch.empty(max(hac.hac_workspace_bytes(blob.desc, B), 256), dtype=torch.uint8, device=dev())
        expect = f(db, X, workspace=ws).clone()
        torch.cuda.synchronize()
        check_y(expect, X.cpu().numpy(), W, f"{f.__name__} B={B}")
        jobs.append((f, db, X, ws, expect, torch.cuda.Stream()))
    failures = []

    def worker(f, db, X, ws, expect, stream):
        try:
            Y = torch.empty_like(expect)
            for _ in range(25):
                Y.fill_(float("nan"))
                stream.wait_stream(torch.cuda.current_stream())
                f(db, X, Y=Y, workspace=ws, stream=stream)
                stream.synchronize()
                if not torch.equal(Y, expect):
                    failures.append(f.__name__)
                    return
        except Exception as e:                            # a thread's exception would otherwise be lost
            failures.append(repr(e))

    threads = [threading.Thread(target=worker, args=j) for j in jobs]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not failures, failures


def test_batch_beyond_65536_rows_on_both_routes(hac):
    # more batch rows than a grid dimension has entries: 257 tiles of 256 batch columns on the sparse
    # route, 2049 row tiles on the matrix cores, the index map's small layout left far behind
    W = workloads.layer(1)
    B = 65537
    X = workloads.make_batch(B, W.shape[0], 77) - np.float32(0.25)
    Xd = torch.from_numpy(X).to(dev())
    for name, enc, f in (("hac", hac.hac_encode, hac.hac_dot), ("shac", hac.shac_encode, hac.shac_dot),
                         ("im", hac.im_encode, hac.im_dot)):
        db = enc(W).to_device(dev())
        for variant in ((0,) if name == "im" else (0x400, 0x800)):
            print(f"[case] {name} B={B} variant={variant:#x}", flush=True)
            Y = f(db, Xd) if name == "im" else f(db, Xd, launch=hac.Launch(variant=variant))
            torch.cuda.synchronize()
            check_y(Y, X, W, f"{name} B={B} variant={variant:#x}")


def test_strided_x_and_y(hac):
    W = workloads.scaled(1, 200, 40)
    Xbig = torch.from_numpy(workloads.make_batch(16, 260, 4)).to(dev())
    X = Xbig[:, 30:230]                                   # ldx = 260
    Ybig = torch.full((16, 64), 7.0, device=dev())
    Y = Ybig[:, 8:48]                                     # ldy = 64
    for enc, f in ((hac.hac_encode, hac.hac_dot), (hac.shac_encode, hac.shac_dot)):
        f(enc(W).to_device(dev()), X, Y=Y)
        torch.cuda.synchronize()
        check_y(Y, X.cpu().numpy(), W, f.__name__)
        assert torch.all(Ybig[:, :8] == 7.0) and torch.all(Ybig[:, 48:] == 7.0)


def test_error_paths(hac):
    import ctypes as C
    lib = hac.load_library()
    W = workloads.scaled(1, 100, 20)
    hb = hac.hac_encode(W).to_device(dev())
    sb = hac.shac_encode(W).to_device(dev())
    X = torch.zeros((4, 100), device=dev())
    with pytest.raises(hac.HacError) as e:
        hac.shac_dot(hb, X)                                # HAC blob given to the sHAC entry point
    assert e.value.status == -1
    with pytest.raises(hac.HacError) as e:
        hac.hac_dot(sb, X)
    assert e.value.status == -1
    small = torch.empty(256, dtype=torch.uint8, device=dev())
    with pytest.raises(hac.HacError) as e:
        hac.hac_dot(hb, torch.zeros((40, 100), device=dev()), workspace=small)     # 40 rows need a re-laid-out copy
    assert e.value.status == -6
    with pytest.raises(hac.HacError) as e:
        hac.hac_dot(hb, X, workspace=small, launch=hac.Launch(variant=0x1000))    # so do 4 rows when X may not go to LDS
    assert e.value.status == -6
    assert hac.hac_workspace_bytes(hb.desc, 4) == 0 and hac.hac_workspace_bytes(hb.desc, 4, hac.Launch(variant=0x1000)) > 0
    Y = torch.empty((4, 20), device=dev())
    args = (C.byref(hb.desc), hb.tensor.data_ptr(), X.data_ptr(), 4, 50, Y.data_ptr(), 20, None, 0, None, None)
    assert lib.hac_dot(*args) == -1                        # ldx < n
    # B = 0 is a no-op
    assert lib.hac_dot(C.byref(hb.desc), hb.tensor.data_ptr(), None, 0, 100, None, 20, None, 0, None, None) == 0
    torch.cuda.synchronize()
