#!/usr/bin/env python3
"""Benchmark of the compressed dot product Y = X.W on one MI355X.

Workload: the VGG16-FC1-shaped layer (25088 x 4096, 98 % pruned, k = 32 shared
values by uniform binning), synthetic and seeded.  One *step* is one pass of
the whole hot path over that layer: hac_dot and shac_dot for each of the three
batch sizes the configuration names (B = 1, 32, 256) -- six products, each
decoding its compressed stream on the fly.

Metric: algorithmic HBM bytes moved per second,
    bytes(call) = stream + code tables + chunk index (+ ri + cb) + 4*B*n + 4*B*m,
each counted once, summed over the six calls of a step and divided by the step
time.  Inputs are resident in device memory before the timed region.  To keep
the 256 MB last-level cache from serving everything, the step rotates through
enough distinct copies of the blobs and of X / Y to exceed it.

Timing: HIP events on the launch stream around exactly K steps (each step is
replayed from a captured HIP graph so the host's launch rate is not what is
measured; --no-graph times eager launches instead).  The dominant kernel's own
average duration is measured the same way on a graph that holds only that
kernel, and is what `roofline.achieved` is computed from.

The CPU oracle (Algorithms 1-3 taken literally, oracle/c) is timed beside it on
a bounded sample as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0                 # MI355X HBM3E
MFMA_FP32_PEAK_TFLOPS = 157.3         # MI355X dense fp32 matrix peak
L2_GATHER_PEAK_TBPS = round(64 * 256 * 2.4e9 / 1e12, 1)      # 39.3: what the 256 L1s can take from the L2s
LLC_BYTES = 256 << 20                 # last-level (Infinity) cache to rotate past


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload id (4 = VGG16-FC1-shaped layer)")
    ap.add_argument("--batches", type=str, default="", help="comma list; default: the config's batch sizes")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of graph replays")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--hot", action="store_true", help="no rotation: same buffers every step (cache-resident)")
    ap.add_argument("--chunk-nnz", type=int, default=0)
    ap.add_argument("--only", type=str, default="", help="restrict the step to 'hac' or 'shac'")
    ap.add_argument("--extras", action="store_true",
                    help="also report cache-resident timings, the decode-only kernels' symbol rate and CPU context "
                         "rows (decode once + dense product, numpy dense, scipy CSC); adds about a minute")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a 256 MiB device-to-device copy 4 times before the timed region "
                         "(a kernel of known traffic for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def algorithmic_bytes(stats, desc, B):
    blob = stats.stream_bytes + stats.table_bytes + stats.index_bytes + stats.ri_bytes + stats.cb_bytes
    return int(blob + 4 * B * int(desc.n) + 4 * B * int(desc.m))


class Call:
    """One (format, B) product with its rotating device buffers."""

    def __init__(self, hac, fmt, blob, B, rot, Xhost, dev, torch, launch=None):
        self.fmt, self.B = fmt, B
        self.fn = hac.hac_dot if fmt == "hac" else hac.shac_dot
        self.stats = blob.stats()
        self.desc = blob.desc
        self.bytes = algorithmic_bytes(self.stats, blob.desc, B)
        self.blobs = [blob.to_device(dev) for _ in range(rot)]
        self.X = [torch.from_numpy(Xhost[:B]).to(dev).clone() for _ in range(rot)]
        self.Y = [torch.empty((B, int(blob.desc.m)), dtype=torch.float32, device=dev) for _ in range(rot)]
        need = hac.hac_workspace_bytes(blob.desc, B, launch)
        self.ws = [torch.empty(max(need, 256), dtype=torch.uint8, device=dev) for _ in range(rot)]
        self.rot = rot
        # the dot kernel can be timed alone (X already feature-major in the workspace) only where a
        # call re-lays X out first: not at B = 1, with a short X kept in LDS, or on the dense route
        self.relayout = B > 1 and need > 0 and hac.hac_dot_route(blob.desc, B) == 0

    def run(self, i, launch=None):
        j = i % self.rot
        self.fn(self.blobs[j], self.X[j], Y=self.Y[j], workspace=self.ws[j], launch=launch)

    def kernels(self, hac, launch=None):
        """Names of the kernels one call launches, as the library reports them after an eager call."""
        self.run(0, launch)
        return hac.hac_last_kernels()


def time_region(torch, body, iters, warmup, use_graph, rot):
    """Average milliseconds per body(i) call over exactly `iters` calls, HIP events on the current stream.

    With graphs, one captured graph holds `rot` consecutive calls (one per buffer set) and is
    replayed iters // rot times; the remaining iters % rot calls are launched eagerly.
    """
    stream = torch.cuda.current_stream()
    for i in range(warmup):
        body(i)
    torch.cuda.synchronize()
    graph = None
    if use_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for j in range(rot):
                body(j)
        graph.replay()
        torch.cuda.synchronize()
    t0 = torch.cuda.Event(enable_timing=True)
    t1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0.record(stream)
    done = 0
    if graph is not None:
        for _ in range(iters // rot):
            graph.replay()
        done = (iters // rot) * rot
    for i in range(done, iters):
        body(i)
    t1.record(stream)
    torch.cuda.synchronize()
    return t0.elapsed_time(t1) / iters


def time_spread(torch, body, replays, use_graph, rot):
    """(min, median) milliseconds per body(i) call over `replays` groups of `rot` calls, each group
    (one graph replay, or rot eager calls) between its own pair of events; everything is queued
    before the first wait, so the groups run back to back.  Beside time_region's mean, not instead."""
    stream = torch.cuda.current_stream()
    graph = None
    if use_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for j in range(rot):
                body(j)
        graph.replay()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(replays + 1)]
    marks[0].record(stream)
    for r in range(replays):
        if graph is not None:
            graph.replay()
        else:
            for j in range(rot):
                body(j)
        marks[r + 1].record(stream)
    torch.cuda.synchronize()
    per_call = sorted(marks[r].elapsed_time(marks[r + 1]) / rot for r in range(replays))
    return per_call[0], per_call[len(per_call) // 2]


def measured_traffic(cfg_id, fmt, B):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by the copy calibration) from the
    committed rocprofv3 counter summary, or None when that summary has no line for this kernel."""
    path = os.path.join(ROOT, "profiles", f"pmc_hbm_traffic_cfg{cfg_id}.md")
    key = f"| {fmt}_dot | {B} |"
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith(key):
                    cells = [c.strip() for c in line.strip().strip("|").split("|")]
                    return int(float(cells[-1]))
    except OSError:
        return None
    return None


def extras(torch, hac, calls, hb, sb, W, Xhost, dev, use_graph, iters):
    """Figures that are context for the headline number, not part of it."""
    out = {}
    reuse = hac.Launch()
    reuse.variant = 0x100
    hot = []
    for c in calls:                                    # same buffers every launch: everything cache-resident
        ms = time_region(torch, lambda i, c=c: c.fn(c.blobs[0], c.X[0], Y=c.Y[0], workspace=c.ws[0],
                                                    launch=reuse if c.relayout else None), iters, 5, use_graph, 8)
        hot.append({"format": c.fmt, "B": c.B, "kernel_ms": round(ms, 5),
                    "kernel_hbm_frac": round(c.bytes / ms / 1e6 / HBM_PEAK_GBS, 4)})
    out["hot"] = hot
    # sHAC with Rice-coded row gaps (an extension beyond the paper's two formats): same protocol as `detail`
    W_, dev_ = W, dev
    gb = hac.shac_encode(W_, ri_coding=hac.RI_RICE)
    rot = calls[0].rot
    rice = []
    for B in sorted({c.B for c in calls}):
        c = Call(hac, "shac", gb, B, rot, Xhost, dev_, torch)
        ms = time_region(torch, lambda i, c=c: c.run(i), iters, 5, use_graph, rot)
        ms_k = time_region(torch, lambda i, c=c: c.run(i, reuse), iters, 5, use_graph, rot) if c.relayout else ms
        rice.append({"B": B, "ms": round(ms, 5), "kernel_ms": round(ms_k, 5), "bytes": c.bytes,
                     "kernel_hbm_frac": round(c.bytes / ms_k / 1e6 / HBM_PEAK_GBS, 4)})
        del c
    out["shac_rice_gaps"] = {"blob_bytes": gb.nbytes, "rice_k": int(gb.desc.rice_k),
                             "gap_bits_per_nonzero": round(int(gb.desc.gap_bits) / max(int(gb.desc.nnz), 1), 3),
                             "calls": rice}
    # the row-blocked kernel (blobs with a row index; rows of X in LDS, column sums in registers): on
    # request only, because it is slower on this layer; timed here so that the record stays current
    rows_k = []
    rows_launch = hac.Launch(variant=0x2000)
    Bmax = max(c.B for c in calls)
    for fmt, enc in (("hac", hac.hac_encode), ("shac", hac.shac_encode)):
        rb_ = enc(W_, chunk_rows=hac.CHUNK_ROWS_AUTO)
        c = Call(hac, fmt, rb_, Bmax, rot, Xhost, dev_, torch, launch=rows_launch)
        ms = time_region(torch, lambda i, c=c: c.run(i, rows_launch), iters, 5, use_graph, rot)
        rows_k.append({"format": fmt, "B": Bmax, "ms": round(ms, 5), "chunk_rows": int(rb_.desc.chunk_rows),
                       "row_index_bytes": int(rb_.stats().row_index_bytes), "kernels": c.kernels(hac, rows_launch)})
        del c
    out["row_blocked_kernel"] = rows_k
    # decode-only kernels (test entry points): symbols and stream bits per second
    dec = []
    for fmt, blob in (("hac", hb), ("shac", sb)):
        db = blob.to_device(dev)
        n, m, nnz = int(blob.desc.n), int(blob.desc.m), int(blob.desc.nnz)
        if fmt == "hac":
            body = lambda i, db=db: hac.hac_decode_dev(db)
            symbols = n * m
        else:
            body = lambda i, db=db: hac.shac_decode_dev(db)
            symbols = nnz
        ms = time_region(torch, body, 20, 3, False, 1)
        dec.append({"format": fmt, "ms": round(ms, 4), "symbols_per_s": round(symbols / ms * 1e3, 1),
                    "nonzeros_per_s": round(nnz / ms * 1e3, 1),
                    "stream_bits_per_s": round(int(blob.desc.total_bits) / ms * 1e3, 1)})
    out["decode_only"] = dec
    # the GPU-side encoder (the step before the path): W already on the device -> blob on the device,
    # against the host encoder on the same matrix; one library call per encode, buffers allocated before
    import ctypes as C
    lib = hac.load_library()
    Wd_enc = torch.from_numpy(W).to(dev)
    n_, m_ = W.shape
    ws_enc = torch.empty(lib.hac_encode_dev_workspace_bytes(n_, m_), dtype=torch.uint8, device=dev)
    enc = {}
    for name, fmt, host_enc, host_blob in (("hac", hac.HAC_FORMAT_HAC, hac.hac_encode, hb), ("shac", hac.HAC_FORMAT_SHAC, hac.shac_encode, sb)):
        t = time.perf_counter()
        host_enc(W)
        host_ms = 1e3 * (time.perf_counter() - t)
        out_blob = torch.empty(host_blob.nbytes, dtype=torch.uint8, device=dev)
        d_ = hac.Desc()

        def encode_once():
            rc = lib.hac_encode_dev(fmt, Wd_enc.data_ptr(), n_, m_, m_, None, out_blob.data_ptr(), out_blob.numel(),
                                    C.byref(d_), ws_enc.data_ptr(), ws_enc.numel(), None)
            if rc:
                raise RuntimeError(f"hac_encode_dev: {rc}")

        encode_once()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(5):
            encode_once()                               # the call synchronises by itself
        dev_ms = 1e3 * (time.perf_counter() - t) / 5
        enc[name] = {"device_ms": round(dev_ms, 3), "host_ms": round(host_ms, 1),
                     "identical_to_host_blob": bool(np.array_equal(out_blob.cpu().numpy(), host_blob.data))}
    out["gpu_encoder"] = enc
    del Wd_enc, ws_enc, out_blob
    # a fully connected block as one chain (hac_forward) on a network blob with one shared dictionary,
    # against the same layers multiplied one call at a time with bias and ReLU as separate passes
    import workloads
    Ws, bs = workloads.network("vgg16-fc")
    fmts = [hac.hac_choose_format(w.shape[0], w.shape[1], int(np.count_nonzero(w)), 32) for w in Ws]
    nb = hac.hac_net_encode(Ws, fmts)
    own = [(hac.hac_encode if f == hac.HAC_FORMAT_HAC else hac.shac_encode)(w) for f, w in zip(fmts, Ws)]
    dls = nb.to_device(dev)
    dbias = [torch.from_numpy(b).to(dev) for b in bs]
    relu = [True, True, False]
    layers = list(zip(dls, dbias, relu))
    chain = []
    for B in sorted({c.B for c in calls}):
        X = torch.from_numpy(workloads.make_batch(B, Ws[0].shape[0], 31)).to(dev)
        Y = torch.empty((B, Ws[-1].shape[1]), dtype=torch.float32, device=dev)
        ws = torch.empty(max(hac.hac_forward_workspace_bytes(layers, B), 256), dtype=torch.uint8, device=dev)
        ms_chain = time_region(torch, lambda i: hac.hac_forward(layers, X, Y=Y, workspace=ws), iters, 5, use_graph, 4)
        wss = [torch.empty(max(hac.hac_workspace_bytes(dl.desc, B), 256), dtype=torch.uint8, device=dev) for dl in dls]
        Ys = [torch.empty((B, w.shape[1]), dtype=torch.float32, device=dev) for w in Ws]

        def separate(i):
            A = X
            for l, (dl, f) in enumerate(zip(dls, fmts)):
                (hac.hac_dot if f == hac.HAC_FORMAT_HAC else hac.shac_dot)(dl, A, Y=Ys[l], workspace=wss[l])
                Ys[l].add_(dbias[l])
                if relu[l]:
                    Ys[l].clamp_min_(0.0)
                A = Ys[l]

        ms_sep = time_region(torch, separate, iters, 5, use_graph, 4)
        chain.append({"B": B, "chain_ms": round(ms_chain, 5), "one_call_per_layer_ms": round(ms_sep, 5)})
    out["chain_vgg16_fc"] = {"layers": [list(w.shape) for w in Ws], "formats": fmts,
                             "network_blob_bytes": nb.nbytes, "separate_blob_bytes": sum(b.nbytes for b in own),
                             "calls": chain}
    # the paper's own timing set-up (Sect. V-G): 8 input vectors against the three fully connected
    # matrices of VGG19 (synthetic layers of those shapes, k = 32), every format of this library
    # beside the vendor's dense GEMM on the decoded matrix; psi = stored bytes / dense bytes
    shapes = []
    for (n_, m_) in ((512, 4096), (4096, 4096), (4096, 10)):
        for prune in (0.9, 0.99):
            Wp = workloads.make_layer(n_, m_, 0.02, prune, 32, "uniform", 4242)
            Xp = torch.from_numpy(workloads.make_batch(8, n_, 3)).to(dev)
            Yp = torch.empty((8, m_), dtype=torch.float32, device=dev)
            row = {"shape": [n_, m_], "pruned": prune}
            for name, enc, dot in (("hac", hac.hac_encode, hac.hac_dot), ("shac", hac.shac_encode, hac.shac_dot),
                                   ("im", hac.im_encode, hac.im_dot)):
                b_ = enc(Wp)
                db_ = b_.to_device(dev)
                ws_ = torch.empty(max(hac.hac_workspace_bytes(b_.desc, 8), 256), dtype=torch.uint8, device=dev)
                row[name + "_us"] = round(1e3 * time_region(torch, lambda i: dot(db_, Xp, Y=Yp, workspace=ws_), iters, 5, use_graph, 8), 2)
                row[name + "_psi"] = round(b_.nbytes / (4.0 * n_ * m_), 4)
            Wpd = torch.from_numpy(Wp).to(dev)
            row["dense_fp32_matmul_us"] = round(1e3 * time_region(torch, lambda i: torch.matmul(Xp, Wpd, out=Yp), iters, 5, use_graph, 8), 2)
            shapes.append(row)
    out["paper_shapes_8_vectors"] = shapes
    # GPU context: the same product with W decompressed to dense fp32 (torch.matmul, the vendor's
    # GEMM) and as an uncompressed CSR matrix (torch.sparse, the vendor's SpMM); neither is the
    # paper's method, both need W in HBM at 4 bytes (dense) or 8 bytes (CSR) per stored entry
    Wd = torch.from_numpy(W).to(dev)
    gpu_ctx = {"dense_bytes": int(W.size * 4), "csr_bytes": int(np.count_nonzero(W)) * 8 + 4 * (W.shape[0] + 1), "calls": []}
    import warnings
    try:
        with warnings.catch_warnings():
            warnings.simplefilter("ignore")                           # torch announces that sparse CSR is in beta
            Wt_csr = Wd.t().contiguous().to_sparse_csr()              # Y^T = W^T . X^T
    except Exception:                                                 # sparse CSR unavailable in this build
        Wt_csr = None
    for B in sorted({c.B for c in calls}):
        X = torch.from_numpy(Xhost[:B]).to(dev)
        Yd = torch.empty((B, W.shape[1]), dtype=torch.float32, device=dev)
        ms_dense = time_region(torch, lambda i: torch.matmul(X, Wd, out=Yd), 20, 3, False, 1)
        row = {"B": B, "dense_fp32_matmul_ms": round(ms_dense, 4)}
        if Wt_csr is not None:
            try:
                Xt = X.t().contiguous()
                row["csr_spmm_ms"] = round(time_region(torch, lambda i: torch.sparse.mm(Wt_csr, Xt), 20, 3, False, 1), 4)
            except Exception:
                row["csr_spmm_ms"] = None
        gpu_ctx["calls"].append(row)
    out["gpu_context"] = gpu_ctx
    del Wd, Wt_csr
    # CPU context on this host
    from oracle import cnative
    import scipy.sparse as sp
    B = min(32, Xhost.shape[0])
    X = np.ascontiguousarray(Xhost[:B])
    oh = cnative.hac_encode(W)
    n, m = W.shape
    t = time.perf_counter()
    sym = cnative.unpack(oh.words, n * m, oh.code)
    Wdec = np.ascontiguousarray(oh.values[sym].reshape(m, n).T)
    t_unpack = time.perf_counter() - t
    t = time.perf_counter()
    X @ Wdec
    t_mm = time.perf_counter() - t
    t = time.perf_counter()
    X @ W
    t_dense = time.perf_counter() - t
    Wc = sp.csc_matrix(W)
    t = time.perf_counter()
    (Wc.T @ X.T).T
    t_csc = time.perf_counter() - t
    out["cpu_context"] = {
        "B": B, "decode_once_then_dense_ms": round(1e3 * (t_unpack + t_mm), 2),
        "decode_once_ms": round(1e3 * t_unpack, 2), "numpy_dense_fp32_ms": round(1e3 * t_dense, 2),
        "scipy_csc_ms": round(1e3 * t_csc, 2),
        "note": "decode once = the oracle's tree-walk decoder over the whole HAC stream on one core, then numpy X@W",
    }
    return out


def cpu_baseline(W, Xs, cores):
    """The oracle's literal Algorithm 3 (q = cores threads) on 4 * cores rows of X, both formats
    (about a quarter of a core-second per row and format on the large layer)."""
    from oracle import cnative
    oh = cnative.hac_encode(W)
    osh = cnative.shac_encode(W)
    n, m = W.shape
    rows = min(4 * cores, Xs.shape[0])
    X = np.ascontiguousarray(Xs[:rows])
    t = time.perf_counter()
    cnative.pardot(oh, X, q=cores)
    th = time.perf_counter() - t
    t = time.perf_counter()
    cnative.pardot(osh, X, q=cores)
    ts = time.perf_counter() - t
    k_h, k_s = len(oh.values), len(osh.values)
    # bytes on the oracle's own structures: stream words + codebook/tree + (ri, cb as stored) + X + Y
    bh = 4 * oh.N + 12 * k_h + 4 * rows * n + 8 * rows * m
    bs = 4 * osh.N1 + 12 * k_s + 8 * osh.q + 8 * (m + 1) + 4 * rows * n + 8 * rows * m
    return {
        "value": round((bh + bs) / (th + ts) / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
        "sample": f"Algorithm 3 with q={cores} threads over {rows} rows of X, literal Algorithm 1 (HAC, "
                  f"{th:.2f} s) and Algorithm 2 (sHAC, {ts:.2f} s) on the full layer; W is re-decoded per row",
        "hac_ms_per_row_per_core": round(1e3 * th * min(cores, rows) / rows, 2),
        "shac_ms_per_row_per_core": round(1e3 * ts * min(cores, rows) / rows, 2),
        "dense_equiv_gflops": round(2.0 * 2 * rows * n * m / (th + ts) / 1e9, 3),
    }


def cpu_baseline_b(W, Xhost, batches, cores):
    """The variant the paper's conclusions propose, in the oracle's plain C: per-column bit offsets
    (found once, not timed: they belong to the stored form like the library's index), every codeword
    decoded once per product and applied to all rows of X, threads over ranges of columns.  The whole
    step (every batch size, both formats), fp64 accumulation."""
    from oracle import cnative
    n, m = W.shape
    total_bytes, total_s, rows = 0, 0.0, []
    for name, enc in (("hac", cnative.hac_encode), ("shac", cnative.shac_encode)):
        st = enc(W)
        t = time.perf_counter()
        colbit = cnative.column_offsets(st)
        t_off = time.perf_counter() - t
        k = len(st.values)
        for B in batches:
            X = np.ascontiguousarray(Xhost[:B])
            t = time.perf_counter()
            cnative.coldot(st, X, q=cores, colbit=colbit)
            dt = time.perf_counter() - t
            by = 4 * len(st.words) + 12 * k + 8 * (m + 1) + 4 * B * n + 8 * B * m
            if name == "shac":
                by += 8 * st.q + 8 * (m + 1)
            total_bytes += by
            total_s += dt
            rows.append({"format": name, "B": B, "ms": round(1e3 * dt, 2)})
        rows.append({"format": name, "column_offsets_ms_one_core_not_timed": round(1e3 * t_off, 1)})
    return {
        "value": round(total_bytes / total_s / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
        "sample": "the whole step: decode once per product, all rows of X per non-zero, threads over column ranges "
                  "from per-column bit offsets",
        "step_ms": round(1e3 * total_s, 1), "products": rows,
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); no multi-GPU path exists", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2108_12704_amd as hac
    import workloads

    hac.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = workloads.CONFIGS[args.config]
    batches = [int(b) for b in args.batches.split(",")] if args.batches else list(cfg.batches)
    t_start = time.perf_counter()
    W = workloads.layer(args.config)
    Xhost = workloads.make_batch(max(batches), cfg.n, 1000 * cfg.cfg + 1)
    hb = hac.hac_encode(W, chunk_nnz=args.chunk_nnz)
    sb = hac.shac_encode(W, chunk_nnz=args.chunk_nnz)
    t_prep = time.perf_counter() - t_start

    fmts = [f for f in ("hac", "shac") if not args.only or f == args.only]
    per_set = sum((hb.nbytes if f == "hac" else sb.nbytes) for f in fmts) * len(batches) + \
        sum(4 * B * (cfg.n + cfg.m) * len(fmts) for B in batches)
    rot = 1 if args.hot else max(2, -(-int(1.25 * LLC_BYTES) // per_set))
    calls = [Call(hac, f, hb if f == "hac" else sb, B, rot, Xhost, dev, torch) for B in batches for f in fmts]
    use_graph = not args.no_graph
    # graphs cannot be captured on the default stream: all launches and events go to this one
    work_stream = torch.cuda.Stream(device=dev)
    torch.cuda.synchronize()
    torch.cuda.set_stream(work_stream)

    if args.calibration_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def step(i):
        for c in calls:
            c.run(i)

    ms_step = time_region(torch, step, args.steps, args.warmup, use_graph, rot)
    step_min, step_med = time_spread(torch, step, 30, use_graph, rot)      # after the timed region, not part of it
    step_bytes = sum(c.bytes for c in calls)
    value = step_bytes / (ms_step * 1e-3) / 1e9
    dense_flop = sum(2.0 * c.B * cfg.n * cfg.m for c in calls)
    true_flop = sum(2.0 * c.B * int(c.desc.nnz) for c in calls)

    # every call on its own, same protocol (graph of that call only)
    detail = []
    for c in calls:
        ms = time_region(torch, lambda i, c=c: c.run(i), max(args.steps, 50), 5, use_graph, rot)
        reuse = hac.Launch()
        reuse.variant = 0x100                       # feature-major X already in the workspace: dot kernel alone
        ms_k = ms if not c.relayout else time_region(torch, lambda i, c=c: c.run(i, reuse), max(args.steps, 50), 5,
                                               use_graph, rot)
        ms_min, ms_med = time_spread(torch, lambda i, c=c: c.run(i), 30, use_graph, rot)
        detail.append({
            "format": c.fmt, "B": c.B, "ms": round(ms, 5), "min_ms": round(ms_min, 5), "median_ms": round(ms_med, 5),
            "kernel_ms": round(ms_k, 5),
            "bytes": c.bytes, "GBps": round(c.bytes / ms / 1e6, 1),
            "hbm_frac": round(c.bytes / ms / 1e6 / HBM_PEAK_GBS, 4),
            "kernel_hbm_frac": round(c.bytes / ms_k / 1e6 / HBM_PEAK_GBS, 4),
            "dense_equiv_gflops": round(2.0 * c.B * cfg.n * cfg.m / ms / 1e6, 1),
            "true_gflops": round(2.0 * c.B * int(c.desc.nnz) / ms / 1e6, 1),
        })
    for c, d in zip(calls, detail):
        d["kernels"] = c.kernels(hac)
    torch.cuda.synchronize()
    dom = max(detail, key=lambda d: d["kernel_ms"])
    dom_desc = hb.desc if dom["format"] == "hac" else sb.desc
    dense = hac.hac_dot_route(dom_desc, dom["B"]) == 1
    traffic = measured_traffic(cfg.cfg, dom["format"], dom["B"])
    traffic_source = (f"profiles/pmc_hbm_traffic_cfg{cfg.cfg}.md (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, each scaled by a "
                      "copy of known size; a committed summary, not collected in this run)") if traffic is not None else None
    # the dot kernel proper is the last launch of the call (a re-layout or decode pass may come first)
    kname = [k for k in dom["kernels"] if "reduce" not in k][-1] if dom["kernels"] else "?"
    if dense:
        # the dense route's dominant kernel is a contraction on the matrix cores: beside the flops of the
        # dense product it runs, the flops the method itself needs (2 B nnz) are reported: the method is
        # not credited with multiplications by zero
        flops = 2.0 * dom["B"] * cfg.n * cfg.m
        true_flops = 2.0 * dom["B"] * int(dom_desc.nnz)
        roofline = {
            "bound": "mfma", "kernel": f"{kname} ({dom['format']}_dot dense route, B={dom['B']})",
            "achieved": round(true_flops / dom["kernel_ms"] / 1e9, 2), "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(true_flops / dom["kernel_ms"] / 1e9 / MFMA_FP32_PEAK_TFLOPS, 4),
            "traffic": traffic, "traffic_source": traffic_source, "launch_ms": dom["kernel_ms"],
            "algorithmic_flops": true_flops, "executed_flops": flops,
            "executed_frac": round(flops / dom["kernel_ms"] / 1e9 / MFMA_FP32_PEAK_TFLOPS, 4),
        }
    else:
        xlds = 2 <= dom["B"] <= 8 and hac.hac_workspace_bytes(dom_desc, dom["B"]) == 0
        roofline = {
            "bound": "hbm", "kernel": f"{kname} ({dom['format']}_dot, B={dom['B']})",
            "achieved": round(dom["bytes"] / dom["kernel_ms"] / 1e6, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(dom["bytes"] / dom["kernel_ms"] / 1e6 / HBM_PEAK_GBS, 4),
            "traffic": traffic, "traffic_source": traffic_source,
            "launch_ms": dom["kernel_ms"], "algorithmic_bytes": dom["bytes"],
        }
        # What binds this kernel in practice is not HBM but the vector memory path from the L2s: every
        # non-zero fetches 4 bytes of X per (padded) batch column.  Peak: 64 bytes per clock and CU from
        # L1, 256 CUs at 2.4 GHz.
        Bpad = (dom["B"] + 31) // 32 * 32 if dom["B"] > 4 else dom["B"]
        gather = 4.0 * int(dom_desc.nnz) * Bpad
        if not xlds:                              # (a short X kept in LDS is not gathered from the L2s)
            roofline["l2_gather"] = {"bytes": int(gather), "achieved_TBps": round(gather / dom["kernel_ms"] / 1e9, 2),
                                     "peak_TBps": L2_GATHER_PEAK_TBPS,
                                     "frac": round(gather / dom["kernel_ms"] / 1e9 / L2_GATHER_PEAK_TBPS, 4)}

    out = {
        "metric": "compressed X.W throughput: algorithmic HBM GB/s", "value": round(value, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 5),
        "step_ms_min": round(step_min, 5), "step_ms_median": round(step_med, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": f"cfg{cfg.cfg} {cfg.name}: W {cfg.n}x{cfg.m} N(0,{cfg.sigma}) pruned {cfg.prune:.0%}, "
                        f"k={cfg.k} {cfg.quant}; X ReLU(N(0,1)) fp32; step = " +
                        " + ".join(f"{f}_dot(B={B})" for B in batches for f in fmts),
            "batches": batches, "formats": fmts, "rotation_sets": rot, "graph_replay": use_graph,
            "hac_chunk_nnz": int(hb.desc.chunk), "shac_chunk_nnz": int(sb.desc.chunk),
            "shac_ri_bits": int(sb.desc.ri_bits),
            "hac_blob_bytes": hb.nbytes, "shac_blob_bytes": sb.nbytes, "nnz": int(hb.desc.nnz),
        },
        "hbm_frac": round(value / HBM_PEAK_GBS, 4),
        "dense_equiv_gflops": round(dense_flop / ms_step / 1e6, 1),
        "true_gflops": round(true_flop / ms_step / 1e6, 1),
        "roofline": roofline,
        "detail": detail,
        "prep_seconds": round(t_prep, 2),
    }
    if args.extras:
        out["extras"] = extras(torch, hac, calls, hb, sb, W, Xhost, dev, use_graph, max(args.steps, 50))
    if not args.no_cpu_baseline:
        cores = min(len(os.sched_getaffinity(0)), 16)
        out["cpu_baseline"] = cpu_baseline(W, Xhost, cores)
        out["cpu_baseline_b"] = cpu_baseline_b(W, Xhost, batches, cores)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
