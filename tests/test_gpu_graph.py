"""The library's calls inside a captured HIP graph: the benchmark times graph replays, so every
replay must give what the eager call gives.  Each graph is replayed several times with eager
work of the same library and synchronisations in between, on fresh inputs, and every replay is
compared bit for bit with the eager result (and once with the oracle)."""
import numpy as np
import pytest

import workloads
from oracle import dot as odot

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hac():
    import paper_2108_12704_amd as lib
    lib.load_library()
    assert torch.cuda.is_available(), "GPU tests need a device"
    return lib


def dev():
    return torch.device("cuda:0")


def replay_and_compare(hac, build_call, make_input, label):
    """build_call(X, Y) launches the work on the current stream; X, Y are static tensors."""
    X, Y = make_input(0)
    stream = torch.cuda.Stream(device=dev())
    with torch.cuda.stream(stream):
        build_call(X, Y)                                    # warm-up outside capture (sets kernel attributes)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            build_call(X, Y)
        for rep in range(1, 5):
            Xn, _ = make_input(rep)
            X.copy_(Xn)
            Y.fill_(float("nan"))
            graph.replay()
            stream.synchronize()
            got = Y.clone()
            # eager work of the library between replays: the same call on the same buffers
            Y.fill_(float("nan"))
            build_call(X, Y)
            stream.synchronize()
            assert torch.equal(got, Y), f"{label}: replay {rep} differs from the eager call"
    return X, Y


@pytest.mark.parametrize("B", [1, 3, 32, 300])
def test_dot_calls_replayed_from_a_graph(hac, B):
    W = workloads.scaled(4, 3000, 257)
    blobs = {"hac": (hac.hac_dot, hac.hac_encode(W)), "shac": (hac.shac_dot, hac.shac_encode(W)),
             "rice": (hac.shac_dot, hac.shac_encode(W, ri_coding=hac.RI_RICE)), "im": (hac.im_dot, hac.im_encode(W))}
    for name, (fn, blob) in blobs.items():
        db = blob.to_device(dev())
        ws = torch.empty(max(hac.hac_workspace_bytes(blob.desc, B), 256), dtype=torch.uint8, device=dev())

        def make_input(rep):
            X = torch.from_numpy(workloads.make_batch(B, W.shape[0], 40 + rep)).to(dev())
            return X, torch.empty((B, W.shape[1]), device=dev())

        def call(X, Y, fn=fn, db=db, ws=ws):
            fn(db, X, Y=Y, workspace=ws)

        X, Y = replay_and_compare(hac, call, make_input, f"{name} B={B}")
        ref = odot.dense_dot(X.cpu().numpy(), W)
        scale = odot.abs_dot(X.cpu().numpy(), W)
        assert np.all(np.abs(Y.cpu().numpy().astype(np.float64) - ref) <= 1e-5 * scale + 1e-37), name


def test_dense_route_and_chain_replayed_from_a_graph(hac):
    # the dense route (fill + decode to an index map + matrix-core tiles + split-K reduction) ...
    W = workloads.scaled(5, 640, 96)
    blob = hac.hac_encode(W)
    db = blob.to_device(dev())
    dense = hac.Launch(variant=0x800)
    B = 200
    ws = torch.empty(max(hac.hac_workspace_bytes(blob.desc, B, dense), 256), dtype=torch.uint8, device=dev())

    def make_input(rep):
        return (torch.from_numpy(workloads.make_batch(B, W.shape[0], 70 + rep)).to(dev()),
                torch.empty((B, W.shape[1]), device=dev()))

    replay_and_compare(hac, lambda X, Y: hac.hac_dot(db, X, Y=Y, workspace=ws, launch=dense), make_input, "dense route")

    # ... and a chain of layers on a network blob
    Ws, bs = workloads.network("tiny-fc")
    dls = hac.hac_net_encode(Ws, (1, 2, 1)).to_device(dev())
    layers = [(dl, torch.from_numpy(b).to(dev()), True) for dl, b in zip(dls, bs)]
    for Bc in (1, 40):
        wsc = torch.empty(max(hac.hac_forward_workspace_bytes(layers, Bc), 256), dtype=torch.uint8, device=dev())

        def make_chain_input(rep, Bc=Bc):
            return (torch.from_numpy(workloads.make_batch(Bc, Ws[0].shape[0], 90 + rep)).to(dev()),
                    torch.empty((Bc, Ws[-1].shape[1]), device=dev()))

        replay_and_compare(hac, lambda X, Y, wsc=wsc: hac.hac_forward(layers, X, Y=Y, workspace=wsc), make_chain_input,
                           f"chain B={Bc}")

