"""Thin Python binding of libhac (see include/hac.h for the contract).

Argument marshalling only: encoders run in the C++ host library, every step
of Y = X.W runs in the HIP kernels.  PyTorch supplies device memory and the
stream.  There is no CPU fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhac.so")
_lib: Optional[C.CDLL] = None

HAC_FORMAT_HAC = 1
HAC_FORMAT_SHAC = 2
HAC_FORMAT_IM = 3

EXPORTS = (
    "hac_encode", "shac_encode", "hac_free", "hac_validate", "hac_describe", "hac_stats",
    "hac_decode_host", "hac_workspace_bytes", "hac_workspace_bytes_for", "hac_dot_route", "hac_dot", "shac_dot", "hac_decode_dev",
    "shac_decode_dev", "hac_strerror", "hac_last_hip_error", "im_encode", "im_dot",
    "hac_encode_dev", "hac_encode_dev_workspace_bytes", "hac_choose_format",
    "hac_net_encode", "hac_net_describe", "hac_net_layer", "hac_net_validate", "hac_net_stats",
    "hac_net_decode_host", "hac_forward", "hac_forward_workspace_bytes", "hac_dot_noalloc", "hac_last_kernels",
)


class HacError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().hac_strerror(status).decode()
        extra = ""
        if status == -5:
            extra = f" (hipError {load_library().hac_last_hip_error()})"
        super().__init__(f"{where}: {msg}{extra} [{status}]")


class Opts(C.Structure):
    _fields_ = [("chunk_nnz", C.c_uint32), ("ri_bits", C.c_uint32),
                ("lut_bits", C.c_uint32), ("ri_coding", C.c_uint32), ("chunk_rows", C.c_uint32)]


class Desc(C.Structure):
    _fields_ = [("magic", C.c_uint32), ("version", C.c_uint32), ("format", C.c_uint32),
                ("header_bytes", C.c_uint32),
                ("n", C.c_uint64), ("m", C.c_uint64), ("nnz", C.c_uint64),
                ("total_bits", C.c_uint64), ("n_words", C.c_uint64),
                ("k_sym", C.c_uint32), ("lmax", C.c_uint32), ("lut_bits", C.c_uint32),
                ("has_zero", C.c_uint32), ("zero_len", C.c_uint32), ("chunk", C.c_uint32),
                ("ri_bits", C.c_uint32), ("ent_bits", C.c_uint32),
                ("n_chunks", C.c_uint64),
                ("off_codebook", C.c_uint64), ("off_codelen", C.c_uint64), ("off_canon", C.c_uint64),
                ("off_symsort", C.c_uint64), ("off_lut", C.c_uint64), ("off_stream", C.c_uint64),
                ("off_col_chunk", C.c_uint64), ("off_col_pos", C.c_uint64), ("off_col_bit", C.c_uint64),
                ("off_chunk_ent", C.c_uint64), ("off_ri", C.c_uint64),
                ("blob_bytes", C.c_uint64), ("max_col_bits", C.c_uint64), ("max_col_nnz", C.c_uint64),
                ("row_bits", C.c_uint32), ("ri_coding", C.c_uint32),
                ("rice_k", C.c_uint32), ("dict_shared", C.c_uint32),
                ("gap_bits", C.c_uint64), ("idx_pitch", C.c_uint64), ("off_row_ent", C.c_uint64),
                ("chunk_rows", C.c_uint32), ("rent_bits", C.c_uint8), ("rpos_bits", C.c_uint8),
                ("max_tile_nnz", C.c_uint16)]


class Stats(C.Structure):
    _fields_ = [("stream_bits", C.c_uint64), ("stream_bytes", C.c_uint64),
                ("table_bytes", C.c_uint64), ("index_bytes", C.c_uint64),
                ("ri_bytes", C.c_uint64), ("cb_bytes", C.c_uint64), ("blob_bytes", C.c_uint64),
                ("paper_bits", C.c_uint64), ("bound_bits", C.c_double),
                ("entropy_bits", C.c_double), ("avg_code_bits", C.c_double), ("psi", C.c_double),
                ("row_index_bytes", C.c_uint64)]


class Net(C.Structure):
    _fields_ = [("magic", C.c_uint32), ("version", C.c_uint32), ("header_bytes", C.c_uint32),
                ("n_layers", C.c_uint32), ("blob_bytes", C.c_uint64), ("off_layers", C.c_uint64),
                ("off_codebook", C.c_uint64), ("off_codelen", C.c_uint64), ("off_canon", C.c_uint64),
                ("off_symsort", C.c_uint64), ("off_lut", C.c_uint64),
                ("k_sym", C.c_uint32), ("lmax", C.c_uint32), ("lut_bits", C.c_uint32), ("has_zero", C.c_uint32),
                ("k_values", C.c_uint32), ("reserved32", C.c_uint32), ("reserved", C.c_uint64 * 20)]


class NetStats(C.Structure):
    _fields_ = [("n_layers", C.c_uint64), ("entries", C.c_uint64), ("nnz", C.c_uint64), ("symbols", C.c_uint64),
                ("stream_bits", C.c_uint64), ("table_bytes", C.c_uint64), ("blob_bytes", C.c_uint64),
                ("paper_bits", C.c_uint64), ("entropy_bits", C.c_double), ("avg_code_bits", C.c_double),
                ("psi", C.c_double)]


class Layer(C.Structure):
    _fields_ = [("desc", C.POINTER(Desc)), ("d_blob", C.c_void_p), ("d_bias", C.c_void_p),
                ("activation", C.c_uint32), ("reserved", C.c_uint32)]


ACT_NONE, ACT_RELU = 0, 1


class Launch(C.Structure):
    _fields_ = [("cols_per_wave", C.c_uint32), ("waves_per_block", C.c_uint32),
                ("variant", C.c_uint32), ("list_entries", C.c_uint32), ("staging_words", C.c_uint32),
                ("pass_width", C.c_uint32), ("free_running", C.c_uint32), ("tile_width", C.c_uint32),
                ("sessions_per_block", C.c_uint32)]


assert C.sizeof(Desc) == 256


def load_library() -> C.CDLL:
    """Load libhac.so from the package directory; raise if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python __graft_entry__.py` (build) first")
    lib = C.CDLL(_LIB_PATH)
    vp, f32p, i32p = C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_int32)
    enc_args = [f32p, C.c_int64, C.c_int64, C.c_int64, C.POINTER(Opts),
                C.POINTER(vp), C.POINTER(C.c_size_t)]
    lib.hac_encode.argtypes = enc_args
    lib.shac_encode.argtypes = enc_args
    lib.im_encode.argtypes = enc_args
    lib.hac_encode_dev_workspace_bytes.argtypes = [C.c_int64, C.c_int64]
    lib.hac_encode_dev_workspace_bytes.restype = C.c_size_t
    lib.hac_encode_dev.argtypes = [C.c_uint32, vp, C.c_int64, C.c_int64, C.c_int64, C.POINTER(Opts), vp, C.c_size_t,
                                   C.POINTER(Desc), vp, C.c_size_t, vp]
    lib.hac_choose_format.argtypes = [C.c_int64, C.c_int64, C.c_uint64, C.c_uint32]
    lib.hac_net_encode.argtypes = [C.c_uint32, C.POINTER(C.c_uint32), C.POINTER(f32p), C.POINTER(C.c_int64),
                                   C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(Opts),
                                   C.POINTER(vp), C.POINTER(C.c_size_t)]
    lib.hac_net_describe.argtypes = [vp, C.c_size_t, C.POINTER(Net)]
    lib.hac_net_layer.argtypes = [vp, C.c_size_t, C.c_uint32, C.POINTER(Desc)]
    lib.hac_net_validate.argtypes = [vp, C.c_size_t, C.c_int]
    lib.hac_net_stats.argtypes = [vp, C.c_size_t, C.POINTER(NetStats)]
    lib.hac_net_decode_host.argtypes = [vp, C.c_size_t, C.c_uint32, f32p, i32p, i32p, i32p]
    lib.hac_forward_workspace_bytes.argtypes = [C.POINTER(Layer), C.c_uint32, C.c_int64]
    lib.hac_forward_workspace_bytes.restype = C.c_size_t
    lib.hac_forward.argtypes = [C.POINTER(Layer), C.c_uint32, vp, C.c_int64, C.c_int64, vp, C.c_int64,
                                vp, C.c_size_t, vp]
    lib.hac_free.argtypes = [vp]
    lib.hac_free.restype = None
    lib.hac_validate.argtypes = [vp, C.c_size_t, C.c_int]
    lib.hac_describe.argtypes = [vp, C.c_size_t, C.POINTER(Desc)]
    lib.hac_stats.argtypes = [vp, C.c_size_t, C.POINTER(Stats)]
    lib.hac_decode_host.argtypes = [vp, C.c_size_t, f32p, i32p, i32p, i32p]
    lib.hac_workspace_bytes.argtypes = [C.POINTER(Desc), C.c_int64]
    lib.hac_workspace_bytes.restype = C.c_size_t
    lib.hac_workspace_bytes_for.argtypes = [C.POINTER(Desc), C.c_int64, C.POINTER(Launch)]
    lib.hac_workspace_bytes_for.restype = C.c_size_t
    lib.hac_dot_route.argtypes = [C.POINTER(Desc), C.c_int64, C.POINTER(Launch)]
    dot_args = [C.POINTER(Desc), vp, vp, C.c_int64, C.c_int64, vp, C.c_int64,
                vp, C.c_size_t, C.POINTER(Launch), vp]
    lib.hac_dot.argtypes = dot_args
    lib.shac_dot.argtypes = dot_args
    lib.im_dot.argtypes = dot_args
    lib.hac_dot_noalloc.argtypes = [C.POINTER(Desc), vp, vp, C.c_int64, C.c_int64, vp, C.c_int64, C.POINTER(Launch), vp]
    lib.hac_decode_dev.argtypes = [C.POINTER(Desc), vp, vp, vp, vp]
    lib.shac_decode_dev.argtypes = [C.POINTER(Desc), vp, vp, vp, vp, vp, vp]
    lib.hac_strerror.argtypes = [C.c_int]
    lib.hac_strerror.restype = C.c_char_p
    lib.hac_last_hip_error.argtypes = []
    lib.hac_last_kernels.argtypes = []
    lib.hac_last_kernels.restype = C.c_char_p
    for name in EXPORTS:
        getattr(lib, name)
    _lib = lib
    return lib


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise HacError(rc, where)


class Blob:
    """A host blob (numpy uint8 copy of what the encoder returned) and its header."""

    def __init__(self, data: np.ndarray):
        self.data = np.ascontiguousarray(data, dtype=np.uint8)
        self.desc = Desc()
        _check(load_library().hac_describe(self.data.ctypes.data, self.data.size, C.byref(self.desc)),
               "hac_describe")

    @property
    def nbytes(self) -> int:
        return int(self.data.size)

    def validate(self, deep: bool = True) -> int:
        return load_library().hac_validate(self.data.ctypes.data, self.data.size, int(deep))

    def stats(self) -> Stats:
        st = Stats()
        _check(load_library().hac_stats(self.data.ctypes.data, self.data.size, C.byref(st)), "hac_stats")
        return st

    def section(self, off_field: str, dtype, count: int) -> np.ndarray:
        off = int(getattr(self.desc, off_field))
        return self.data[off:off + count * np.dtype(dtype).itemsize].view(dtype)

    def decode_host(self, want_w: bool = True):
        """The library's sequential CPU decoder: (W, sym[, row, col])."""
        d = self.desc
        n, m, q = int(d.n), int(d.m), int(d.nnz)
        W = np.empty((n, m), dtype=np.float32) if want_w else None
        f32p, i32p = C.POINTER(C.c_float), C.POINTER(C.c_int32)
        wp = W.ctypes.data_as(f32p) if want_w else None
        if d.format in (HAC_FORMAT_HAC, HAC_FORMAT_IM):
            sym = np.empty(n * m, dtype=np.int32)
            _check(load_library().hac_decode_host(self.data.ctypes.data, self.data.size, wp,
                                                  sym.ctypes.data_as(i32p), None, None), "hac_decode_host")
            return W, sym
        sym = np.empty(max(q, 1), dtype=np.int32)
        row = np.empty(max(q, 1), dtype=np.int32)
        col = np.empty(max(q, 1), dtype=np.int32)
        _check(load_library().hac_decode_host(self.data.ctypes.data, self.data.size, wp,
                                              sym.ctypes.data_as(i32p), row.ctypes.data_as(i32p),
                                              col.ctypes.data_as(i32p)), "hac_decode_host")
        return W, sym[:q], row[:q], col[:q]

    def to_device(self, device=None) -> "DeviceBlob":
        import torch
        t = torch.from_numpy(self.data).to(device if device is not None else "cuda")
        return DeviceBlob(self.desc, t)


class DeviceBlob:
    """The blob's bytes in device memory (a torch uint8 tensor) plus the host header."""

    def __init__(self, desc: Desc, tensor):
        if tensor.data_ptr() % 256:
            raise ValueError("device blob must be 256-byte aligned")
        self.desc = desc
        self.tensor = tensor

    @property
    def n(self) -> int:
        return int(self.desc.n)

    @property
    def m(self) -> int:
        return int(self.desc.m)


class NetBlob:
    """A host network blob: L layers written with one shared dictionary (Sect. V-H)."""

    def __init__(self, data: np.ndarray):
        self.data = np.ascontiguousarray(data, dtype=np.uint8)
        self.net = Net()
        lib = load_library()
        _check(lib.hac_net_describe(self.data.ctypes.data, self.data.size, C.byref(self.net)), "hac_net_describe")
        self.layers = []
        for l in range(int(self.net.n_layers)):
            d = Desc()
            _check(lib.hac_net_layer(self.data.ctypes.data, self.data.size, l, C.byref(d)), "hac_net_layer")
            self.layers.append(d)

    @property
    def nbytes(self) -> int:
        return int(self.data.size)

    def validate(self, deep: bool = True) -> int:
        return load_library().hac_net_validate(self.data.ctypes.data, self.data.size, int(deep))

    def stats(self) -> NetStats:
        st = NetStats()
        _check(load_library().hac_net_stats(self.data.ctypes.data, self.data.size, C.byref(st)), "hac_net_stats")
        return st

    def section(self, desc, off_field: str, dtype, count: int) -> np.ndarray:
        off = int(getattr(desc, off_field))
        return self.data[off:off + count * np.dtype(dtype).itemsize].view(dtype)

    def decode_host(self, layer: int, want_w: bool = True):
        """The library's sequential CPU decoder on one layer: (W, sym[, row, col])."""
        d = self.layers[layer]
        n, m, q = int(d.n), int(d.m), int(d.nnz)
        W = np.empty((n, m), dtype=np.float32) if want_w else None
        f32p, i32p = C.POINTER(C.c_float), C.POINTER(C.c_int32)
        wp = W.ctypes.data_as(f32p) if want_w else None
        lib = load_library()
        if d.format in (HAC_FORMAT_HAC, HAC_FORMAT_IM):
            sym = np.empty(n * m, dtype=np.int32)
            _check(lib.hac_net_decode_host(self.data.ctypes.data, self.data.size, layer, wp,
                                           sym.ctypes.data_as(i32p), None, None), "hac_net_decode_host")
            return W, sym
        sym = np.empty(max(q, 1), dtype=np.int32)
        row = np.empty(max(q, 1), dtype=np.int32)
        col = np.empty(max(q, 1), dtype=np.int32)
        _check(lib.hac_net_decode_host(self.data.ctypes.data, self.data.size, layer, wp, sym.ctypes.data_as(i32p),
                                       row.ctypes.data_as(i32p), col.ctypes.data_as(i32p)), "hac_net_decode_host")
        return W, sym[:q], row[:q], col[:q]

    def to_device(self, device=None):
        """One device copy of the whole blob; returns a DeviceBlob per layer, all sharing it."""
        import torch
        t = torch.from_numpy(self.data).to(device if device is not None else "cuda")
        return [DeviceBlob(d, t) for d in self.layers]


RI_FIELDS, RI_RICE = 0, 1


CHUNK_ROWS_AUTO = 0xFFFFFFFF
CHUNK_PER_COLUMN = 0xFFFFFFFF        # Opts.chunk_nnz: every column its own chunk size
CHUNK_FLAG_PER_COLUMN = 0x80000000   # in Desc.chunk


def hac_net_encode(Ws, formats, chunk_nnz: int = 0, ri_bits: int = 0, lut_bits: int = 0,
                   ri_coding: int = RI_FIELDS, chunk_rows: int = 0) -> NetBlob:
    """Layers Ws[l] (n_l x m_l float32, host), formats[l] in (HAC_FORMAT_HAC, HAC_FORMAT_SHAC, HAC_FORMAT_IM)
    -> network blob."""
    lib = load_library()
    L = len(Ws)
    if L != len(formats):
        raise ValueError("one format per layer")
    keep = []
    for W in Ws:
        W = np.asarray(W)
        if W.dtype != np.float32 or W.ndim != 2:
            raise TypeError("every W must be a 2-D float32 array")
        keep.append(np.ascontiguousarray(W))
    f32p = C.POINTER(C.c_float)
    ptrs = (f32p * L)(*[W.ctypes.data_as(f32p) for W in keep])
    fm = (C.c_uint32 * L)(*[int(f) for f in formats])
    ns = (C.c_int64 * L)(*[W.shape[0] for W in keep])
    ms = (C.c_int64 * L)(*[W.shape[1] for W in keep])
    opts = Opts(chunk_nnz, ri_bits, lut_bits, ri_coding, chunk_rows)
    out, size = C.c_void_p(), C.c_size_t()
    _check(lib.hac_net_encode(L, fm, ptrs, ns, ms, ms, C.byref(opts), C.byref(out), C.byref(size)), "hac_net_encode")
    try:
        data = np.ctypeslib.as_array(C.cast(out, C.POINTER(C.c_uint8)), shape=(size.value,)).copy()
    finally:
        lib.hac_free(out)
    return NetBlob(data)


def _encode(fn_name: str, W: np.ndarray, chunk_nnz=0, ri_bits=0, lut_bits=0, ri_coding=0, chunk_rows=0) -> Blob:
    lib = load_library()
    W = np.asarray(W)
    if W.dtype != np.float32 or W.ndim != 2:
        raise TypeError("W must be a 2-D float32 array")
    if W.strides[1] != 4 or W.strides[0] % 4 or W.strides[0] < 4 * W.shape[1]:
        W = np.ascontiguousarray(W)
    ldw = W.strides[0] // 4
    opts = Opts(chunk_nnz, ri_bits, lut_bits, ri_coding, chunk_rows)
    out = C.c_void_p()
    size = C.c_size_t()
    rc = getattr(lib, fn_name)(W.ctypes.data_as(C.POINTER(C.c_float)), W.shape[0], W.shape[1], ldw,
                               C.byref(opts), C.byref(out), C.byref(size))
    _check(rc, fn_name)
    try:
        data = np.ctypeslib.as_array(C.cast(out, C.POINTER(C.c_uint8)), shape=(size.value,)).copy()
    finally:
        lib.hac_free(out)
    return Blob(data)


def hac_encode(W: np.ndarray, chunk_nnz: int = 0, lut_bits: int = 0, chunk_rows: int = 0) -> Blob:
    """W (n x m float32, host) -> HAC blob."""
    return _encode("hac_encode", W, chunk_nnz=chunk_nnz, lut_bits=lut_bits, chunk_rows=chunk_rows)


def shac_encode(W: np.ndarray, chunk_nnz: int = 0, ri_bits: int = 0, lut_bits: int = 0,
                ri_coding: int = RI_FIELDS, chunk_rows: int = 0) -> Blob:
    """W (n x m float32, host) -> sHAC blob."""
    return _encode("shac_encode", W, chunk_nnz=chunk_nnz, ri_bits=ri_bits, lut_bits=lut_bits, ri_coding=ri_coding,
                   chunk_rows=chunk_rows)


def im_encode(W: np.ndarray) -> Blob:
    """W (n x m float32, host) -> index-map blob (Sect. III-C1)."""
    W = np.asarray(W)
    if W.dtype != np.float32 or W.ndim != 2:
        raise TypeError("W must be a 2-D float32 array")
    W = np.ascontiguousarray(W)
    lib = load_library()
    out, size = C.c_void_p(), C.c_size_t()
    rc = lib.im_encode(W.ctypes.data_as(C.POINTER(C.c_float)), W.shape[0], W.shape[1], W.shape[1], None,
                       C.byref(out), C.byref(size))
    _check(rc, "im_encode")
    try:
        data = np.ctypeslib.as_array(C.cast(out, C.POINTER(C.c_uint8)), shape=(size.value,)).copy()
    finally:
        lib.hac_free(out)
    return Blob(data)


def hac_workspace_bytes(desc: Desc, B: int, launch: Optional["Launch"] = None) -> int:
    """Workspace bytes of a dot call; with `launch`, for that launch's route."""
    if launch is None:
        return int(load_library().hac_workspace_bytes(C.byref(desc), B))
    return int(load_library().hac_workspace_bytes_for(C.byref(desc), B, C.byref(launch)))


def _stream_handle(stream) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _dot(fn_name: str, dblob: DeviceBlob, X, Y=None, workspace=None, launch: Optional[Launch] = None,
         stream=None):
    import torch
    lib = load_library()
    if X.dtype != torch.float32 or X.dim() != 2 or not X.is_cuda:
        raise TypeError("X must be a 2-D float32 CUDA tensor")
    if X.stride(1) != 1:
        X = X.contiguous()
    B, n = X.shape
    if n != dblob.n:
        raise ValueError("X has the wrong width")
    if Y is None:
        Y = torch.empty((B, dblob.m), dtype=torch.float32, device=X.device)
    elif Y.dtype != torch.float32 or Y.shape != (B, dblob.m) or Y.stride(1) != 1 or not Y.is_cuda:
        raise TypeError("Y must be a B x m float32 CUDA tensor with unit column stride")
    need = hac_workspace_bytes(dblob.desc, B, launch)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    ldx = X.stride(0) if B > 1 else max(n, 1)
    ldy = Y.stride(0) if B > 1 else max(dblob.m, 1)
    rc = getattr(lib, fn_name)(C.byref(dblob.desc), dblob.tensor.data_ptr(), X.data_ptr(), B, ldx,
                               Y.data_ptr(), ldy, ws_ptr, ws_bytes,
                               C.byref(launch) if launch is not None else None,
                               _stream_handle(stream))
    _check(rc, fn_name)
    return Y


def hac_dot(dblob: DeviceBlob, X, Y=None, workspace=None, launch=None, stream=None):
    """Y = X . W for a HAC blob on the device (asynchronous on the stream)."""
    return _dot("hac_dot", dblob, X, Y, workspace, launch, stream)


def shac_dot(dblob: DeviceBlob, X, Y=None, workspace=None, launch=None, stream=None):
    """Y = X . W for an sHAC blob on the device (asynchronous on the stream)."""
    return _dot("shac_dot", dblob, X, Y, workspace, launch, stream)


def hac_last_kernels() -> list:
    """Names of the kernels this thread's last dot call launched, in order."""
    text = load_library().hac_last_kernels().decode()
    return [t for t in text.split("; ") if t]


NOALLOC_WORKSPACE_BYTES = 16 << 20


def hac_dot_noalloc(dblob: DeviceBlob, X, Y, launch: Optional[Launch] = None, stream=None):
    """hac_dot / shac_dot (by the blob's format) with the workspace inside the library: the call
    allocates nothing, so X and Y must be given, contiguous along their rows."""
    import torch
    lib = load_library()
    if X.dtype != torch.float32 or X.dim() != 2 or not X.is_cuda or X.stride(1) != 1:
        raise TypeError("X must be a 2-D float32 CUDA tensor with unit column stride")
    B, n = X.shape
    if n != dblob.n:
        raise ValueError("X has the wrong width")
    if Y.dtype != torch.float32 or Y.shape != (B, dblob.m) or Y.stride(1) != 1 or not Y.is_cuda:
        raise TypeError("Y must be a B x m float32 CUDA tensor with unit column stride")
    ldx = X.stride(0) if B > 1 else max(n, 1)
    ldy = Y.stride(0) if B > 1 else max(dblob.m, 1)
    rc = lib.hac_dot_noalloc(C.byref(dblob.desc), dblob.tensor.data_ptr(), X.data_ptr(), B, ldx, Y.data_ptr(), ldy,
                             C.byref(launch) if launch is not None else None, _stream_handle(stream))
    _check(rc, "hac_dot_noalloc")
    return Y


def hac_encode_dev(W, fmt: int = HAC_FORMAT_HAC, chunk_nnz: int = 0, ri_bits: int = 0, lut_bits: int = 0,
                   ri_coding: int = 0, stream=None) -> DeviceBlob:
    """Encode a device matrix (2-D float32 CUDA tensor, unit column stride) on the device.

    Calls the library twice: once to learn the blob's size, once to fill it.  Synchronises the stream.
    """
    import torch
    if W.dtype != torch.float32 or W.dim() != 2 or not W.is_cuda or W.stride(1) != 1:
        raise TypeError("W must be a 2-D float32 CUDA tensor with unit column stride")
    lib = load_library()
    n, m = W.shape
    ldw = W.stride(0) if n > 1 else max(m, 1)
    ws = torch.empty(lib.hac_encode_dev_workspace_bytes(n, m), dtype=torch.uint8, device=W.device)
    opts = Opts(chunk_nnz, ri_bits, lut_bits, ri_coding)
    desc = Desc()
    sh = _stream_handle(stream)
    rc = lib.hac_encode_dev(fmt, W.data_ptr(), n, m, ldw, C.byref(opts), None, 0, C.byref(desc), ws.data_ptr(), ws.numel(), sh)
    if rc != -6:
        _check(rc, "hac_encode_dev")
    blob = torch.empty(int(desc.blob_bytes), dtype=torch.uint8, device=W.device)
    _check(lib.hac_encode_dev(fmt, W.data_ptr(), n, m, ldw, C.byref(opts), blob.data_ptr(), blob.numel(), C.byref(desc),
                              ws.data_ptr(), ws.numel(), sh), "hac_encode_dev")
    return DeviceBlob(desc, blob)


def hac_choose_format(n: int, m: int, nnz: int, k: int) -> int:
    """HAC_FORMAT_HAC or HAC_FORMAT_SHAC by the paper's bound-based rule (end of Sect. IV-C)."""
    rc = load_library().hac_choose_format(n, m, nnz, k)
    if rc < 0:
        _check(rc, "hac_choose_format")
    return rc


def hac_dot_route(desc: Desc, B: int, launch: Optional["Launch"] = None) -> int:
    """0 = sparse route (vector FMAs per non-zero), 1 = dense route (index map + matrix cores)."""
    rc = load_library().hac_dot_route(C.byref(desc), B, C.byref(launch) if launch is not None else None)
    if rc < 0:
        _check(rc, "hac_dot_route")
    return rc


def im_dot(dblob: DeviceBlob, X, Y=None, workspace=None, stream=None):
    """Y = X . W for an index-map blob on the device (asynchronous on the stream)."""
    return _dot("im_dot", dblob, X, Y, workspace, None, stream)


def _layer_array(layers):
    """layers: sequence of (DeviceBlob, bias tensor or None, relu flag)."""
    import torch
    arr = (Layer * len(layers))()
    for i, (dblob, bias, relu) in enumerate(layers):
        if bias is not None and (bias.dtype != torch.float32 or bias.numel() != dblob.m or not bias.is_contiguous()
                                 or not bias.is_cuda):
            raise TypeError("bias must be a contiguous float32 CUDA tensor of m elements")
        arr[i].desc = C.pointer(dblob.desc)
        arr[i].d_blob = dblob.tensor.data_ptr()
        arr[i].d_bias = bias.data_ptr() if bias is not None else None
        arr[i].activation = ACT_RELU if relu else ACT_NONE
    return arr


def hac_forward_workspace_bytes(layers, B: int) -> int:
    arr = _layer_array(layers)
    return int(load_library().hac_forward_workspace_bytes(arr, len(layers), B))


def hac_forward(layers, X, Y=None, workspace=None, stream=None):
    """Y = act_L(... act_0(X . W_0 + b_0) ... . W_L + b_L); layers: (DeviceBlob, bias or None, relu) per layer."""
    import torch
    lib = load_library()
    if X.dtype != torch.float32 or X.dim() != 2 or not X.is_cuda:
        raise TypeError("X must be a 2-D float32 CUDA tensor")
    if X.stride(1) != 1:
        X = X.contiguous()
    B = X.shape[0]
    m_out = layers[-1][0].m
    if Y is None:
        Y = torch.empty((B, m_out), dtype=torch.float32, device=X.device)
    elif Y.dtype != torch.float32 or Y.shape != (B, m_out) or Y.stride(1) != 1 or not Y.is_cuda:
        raise TypeError("Y must be a B x m float32 CUDA tensor with unit column stride")
    arr = _layer_array(layers)
    need = int(lib.hac_forward_workspace_bytes(arr, len(layers), B))
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    ldx = X.stride(0) if B > 1 else max(X.shape[1], 1)
    ldy = Y.stride(0) if B > 1 else max(m_out, 1)
    rc = lib.hac_forward(arr, len(layers), X.data_ptr(), B, ldx, Y.data_ptr(), ldy, ws_ptr, ws_bytes,
                         _stream_handle(stream))
    _check(rc, "hac_forward")
    return Y


def hac_decode_dev(dblob: DeviceBlob, stream=None):
    """TEST ONLY: (W n x m float32, sym int32[n*m] in column order) as the device decoder sees them."""
    import torch
    dev = dblob.tensor.device
    W = torch.empty((dblob.n, dblob.m), dtype=torch.float32, device=dev)
    sym = torch.empty(dblob.n * dblob.m, dtype=torch.int32, device=dev)
    _check(load_library().hac_decode_dev(C.byref(dblob.desc), dblob.tensor.data_ptr(), W.data_ptr(),
                                         sym.data_ptr(), _stream_handle(stream)), "hac_decode_dev")
    return W, sym


def shac_decode_dev(dblob: DeviceBlob, stream=None):
    """TEST ONLY: (nz float32, sym, row, col int32), each nnz long, CSC order."""
    import torch
    dev = dblob.tensor.device
    q = int(dblob.desc.nnz)
    nz = torch.empty(max(q, 1), dtype=torch.float32, device=dev)
    sym = torch.empty(max(q, 1), dtype=torch.int32, device=dev)
    row = torch.empty(max(q, 1), dtype=torch.int32, device=dev)
    col = torch.empty(max(q, 1), dtype=torch.int32, device=dev)
    _check(load_library().shac_decode_dev(C.byref(dblob.desc), dblob.tensor.data_ptr(), nz.data_ptr(),
                                          sym.data_ptr(), row.data_ptr(), col.data_ptr(),
                                          _stream_handle(stream)), "shac_decode_dev")
    return nz[:q], sym[:q], row[:q], col[:q]
