"""The production kernels' decoders, checked value by value through the C ABI.

With unit vectors as the rows of X (row b of X is e_r(b)), row b of Y = X.W is row r(b) of W, and a
sum with one non-zero term is exact: every entry of Y must equal the entry of W it stands for, bit
for bit (-0.0 never occurs in W).  A wrong symbol, row, column boundary or zero run anywhere in a
kernel's own decode loop shows up as a wrong entry, which a tolerance on random X could hide when
two representatives lie close together.  Covered: the small-batch kernel (B <= 4), the short-X
kernel, the single- and multi-pass batch kernels, the list kernel on request, the row-blocked
kernel, Rice-coded gaps, the dense route (its decode-to-index-map kernel plus the matrix-core
contraction) and the index-map product.  Expected values come from W itself.
"""
import numpy as np
import pytest

import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

LIST, SPARSE, DENSE, ROWS = 0x200, 0x400, 0x800, 0x2000


@pytest.fixture(scope="module")
def hac():
    import paper_2108_12704_amd as lib
    lib.load_library()
    assert torch.cuda.is_available(), "GPU tests need a device"
    return lib


def unit_rows(rows, n):
    X = np.zeros((len(rows), n), dtype=np.float32)
    X[np.arange(len(rows)), rows] = 1.0
    return X


def check_rows(hac, dot, db, W, rows, launch, what):
    dev = torch.device("cuda:0")
    n, m = W.shape
    X = unit_rows(rows, n)
    print(f"[case] one-hot {what} B={len(rows)}", flush=True)
    Y = dot(db, torch.from_numpy(X).to(dev), **({"launch": launch} if launch is not None else {}))
    torch.cuda.synchronize()
    got = Y.cpu().numpy()
    want = W[rows, :]
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"{what}: {len(bad)} entries differ, first at batch row {bad[0][0]} (row {rows[bad[0][0]]} of W), column {bad[0][1]}: {got[tuple(bad[0])]!r} != {want[tuple(bad[0])]!r}"


def row_sets(n, rng):
    """all rows of W in batches that reach every kernel: 1, 3 (small), 8 (short X / single pass), 33 .. 256 (multi-pass)"""
    perm = rng.permutation(n)
    sets, at = [], 0
    for size in (1, 3, 8, 32, 96, 256):
        if at >= n:
            break
        sets.append(perm[at:at + size]); at += size
    while at < n:
        sets.append(perm[at:at + 256]); at += 256
    return [np.sort(s) for s in sets]


CASES = [
    ("cfg4-1500x130", lambda: workloads.scaled(4, 1500, 130)),
    ("cfg3-600x200", lambda: workloads.scaled(3, 600, 200)),
    ("cfg2-300x77", lambda: workloads.scaled(2, 300, 77)),
    ("cfg5-500x96", lambda: workloads.scaled(5, 500, 96)),
]


@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
def test_sparse_kernels_reproduce_w_row_by_row(hac, name, make):
    dev = torch.device("cuda:0")
    W = make()
    n, m = W.shape
    rng = np.random.default_rng(11)
    sets = row_sets(n, rng)
    encoders = (("hac", lambda: hac.hac_encode(W), hac.hac_dot),
                ("shac", lambda: hac.shac_encode(W), hac.shac_dot),
                ("shac-rice", lambda: hac.shac_encode(W, ri_coding=1), hac.shac_dot),
                ("hac-chunk3", lambda: hac.hac_encode(W, chunk_nnz=3), hac.hac_dot))
    for fmt, enc, dot in encoders:
        db = enc().to_device(dev)
        for rows in sets:
            check_rows(hac, dot, db, W, rows, hac.Launch(variant=SPARSE), f"{name} {fmt} sparse")
        # the list kernel where the small-batch kernel is the default, and two columns per wavefront
        check_rows(hac, dot, db, W, sets[1], hac.Launch(variant=SPARSE | LIST), f"{name} {fmt} list kernel")
        check_rows(hac, dot, db, W, sets[-1], hac.Launch(variant=SPARSE, cols_per_wave=2), f"{name} {fmt} 2 columns per wave")


def test_row_blocked_kernel_reproduces_w(hac):
    dev = torch.device("cuda:0")
    W = workloads.scaled(4, 1500, 130)
    n, m = W.shape
    sets = row_sets(n, np.random.default_rng(12))
    for fmt, enc, dot in (("hac", hac.hac_encode, hac.hac_dot), ("shac", hac.shac_encode, hac.shac_dot)):
        db = enc(W, chunk_rows=hac.CHUNK_ROWS_AUTO).to_device(dev)
        for rows in sets[3:]:
            check_rows(hac, dot, db, W, rows, hac.Launch(variant=ROWS), f"{fmt} row-blocked")


@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
def test_dense_route_and_index_map_reproduce_w(hac, name, make):
    dev = torch.device("cuda:0")
    W = make()
    n, m = W.shape
    sets = row_sets(n, np.random.default_rng(13))
    for fmt, enc, dot in (("hac", hac.hac_encode, hac.hac_dot), ("shac", hac.shac_encode, hac.shac_dot)):
        db = enc(W).to_device(dev)
        for rows in sets[2:]:
            check_rows(hac, dot, db, W, rows, hac.Launch(variant=DENSE), f"{name} {fmt} dense route")
    db = hac.im_encode(W).to_device(dev)
    for rows in sets:
        check_rows(hac, hac.im_dot, db, W, rows, None, f"{name} index map")
