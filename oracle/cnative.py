"""ctypes wrapper around oracle/c/oracle.c (plain C twin of the Python oracle).

TEST INFRASTRUCTURE -- see oracle/__init__.py.  Used where Python loops are
too slow (full-size layers, the benchmark's cpu_baseline leg).  The Huffman
code always comes from oracle.huffman; the C side only packs, unpacks and
runs Algorithms 1-3, plus the variant the paper's conclusions propose
(per-column bit offsets, threads over columns: column_offsets, coldot).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

from . import formats, huffman
from .formats import HAC, SHAC

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "c", "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib: Optional[C.CDLL] = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-shared", "-fPIC", "-pthread", _SRC, "-o", _LIB])
    return _LIB


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _p(a: np.ndarray, t):
    return a.ctypes.data_as(C.POINTER(t))


def _tree(code: huffman.HuffmanCode):
    left = np.ascontiguousarray(code.left, dtype=np.int32)
    right = np.ascontiguousarray(code.right, dtype=np.int32)
    return left, right


def _code_arrays(code: huffman.HuffmanCode):
    cw = np.array([c for c, _ in code.codes], dtype=np.uint32)
    ln = np.array([l for _, l in code.codes], dtype=np.int32)
    if ln.size and ln.max() > 32:
        raise ValueError("codeword longer than 32 bits")
    return cw, ln


def hac_encode(W: np.ndarray) -> HAC:
    W = np.ascontiguousarray(huffman.normalise_values(W))
    n, m = W.shape
    values, freqs = huffman.alphabet(W)
    code = huffman.build(freqs.tolist())
    cw, ln = _code_arrays(code)
    nbits_expected = huffman.cost(freqs, ln)
    cap = -(-nbits_expected // 32)
    words = np.zeros(cap, dtype=np.uint32)
    nbits = C.c_int64(0)
    rc = lib().oracle_hac_encode(_p(W, C.c_float), C.c_int64(n), C.c_int64(m),
                                 _p(values, C.c_float), _p(cw, C.c_uint32), _p(ln, C.c_int32),
                                 C.c_int32(len(values)), _p(words, C.c_uint32), C.c_int64(cap),
                                 C.byref(nbits))
    if rc:
        raise RuntimeError(f"oracle_hac_encode failed: {rc}")
    return HAC(n, m, values, freqs, code, words, int(nbits.value))


def shac_encode(W: np.ndarray) -> SHAC:
    W = np.ascontiguousarray(huffman.normalise_values(W))
    n, m = W.shape
    nzv = W[W != 0]
    values, freqs = huffman.alphabet(nzv)
    code = huffman.build(freqs.tolist())
    cw, ln = _code_arrays(code)
    q = int(nzv.size)
    cap = -(-huffman.cost(freqs, ln) // 32) if q else 0
    words = np.zeros(max(cap, 1), dtype=np.uint32)
    ri = np.zeros(max(q, 1), dtype=np.int64)
    cb = np.zeros(m + 1, dtype=np.int64)
    nbits = C.c_int64(0)
    vals_arg = values if values.size else np.zeros(1, dtype=np.float32)
    cw_arg = cw if cw.size else np.zeros(1, dtype=np.uint32)
    ln_arg = ln if ln.size else np.zeros(1, dtype=np.int32)
    rc = lib().oracle_shac_encode(_p(W, C.c_float), C.c_int64(n), C.c_int64(m),
                                  _p(vals_arg, C.c_float), _p(cw_arg, C.c_uint32),
                                  _p(ln_arg, C.c_int32), C.c_int32(len(values)),
                                  _p(words, C.c_uint32), C.c_int64(cap), C.byref(nbits),
                                  _p(ri, C.c_int64), C.c_int64(q), _p(cb, C.c_int64))
    if rc:
        raise RuntimeError(f"oracle_shac_encode failed: {rc}")
    return SHAC(n, m, values, freqs, code, words[:cap], int(nbits.value), ri[:q], cb)


def unpack(words: np.ndarray, count: int, code: huffman.HuffmanCode) -> np.ndarray:
    left, right = _tree(code)
    out = np.zeros(max(count, 1), dtype=np.int32)
    w = np.ascontiguousarray(words, dtype=np.uint32)
    if w.size == 0:
        w = np.zeros(1, dtype=np.uint32)
    rc = lib().oracle_unpack(_p(w, C.c_uint32), C.c_int64(words.size), C.c_int64(count),
                             _p(left, C.c_int32), _p(right, C.c_int32),
                             C.c_int32(code.k), C.c_int32(code.root), _p(out, C.c_int32))
    if rc:
        raise RuntimeError("oracle_unpack: stream ended early")
    return out[:count].astype(np.int64)


def pardot(struct, X: np.ndarray, q: int = 1) -> np.ndarray:
    """Algorithm 3 in C with q threads; X is B x n fp32, result B x m fp64."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    if X.ndim == 1:
        X = X[None, :]
    rows, n = X.shape
    if n != struct.n:
        raise ValueError("X has the wrong width")
    out = np.zeros((rows, struct.m), dtype=np.float64)
    if rows == 0 or struct.m == 0:
        return out
    code = struct.code
    if code.k == 0:                               # nothing stored: W is all zero
        return out
    left, right = _tree(code)
    values = np.ascontiguousarray(struct.values, dtype=np.float32)
    words = np.ascontiguousarray(struct.words, dtype=np.uint32)
    if words.size == 0:
        words = np.zeros(1, dtype=np.uint32)
    common = (_p(left, C.c_int32), _p(right, C.c_int32), C.c_int32(code.k), C.c_int32(code.root),
              _p(values, C.c_float), _p(X, C.c_float), C.c_int64(rows), C.c_int64(n),
              C.c_int64(struct.n), C.c_int64(struct.m), C.c_int32(q), _p(out, C.c_double))
    if isinstance(struct, HAC):
        rc = lib().oracle_pardot_hac(_p(words, C.c_uint32), C.c_int64(struct.words.size), *common)
    else:
        ri = np.ascontiguousarray(struct.ri, dtype=np.int64)
        if ri.size == 0:
            ri = np.zeros(1, dtype=np.int64)
        cb = np.ascontiguousarray(struct.cb, dtype=np.int64)
        rc = lib().oracle_pardot_shac(_p(words, C.c_uint32), C.c_int64(struct.words.size),
                                      _p(ri, C.c_int64), _p(cb, C.c_int64), *common)
    if rc:
        raise RuntimeError(f"oracle pardot failed: {rc}")
    return out


def column_offsets(struct) -> np.ndarray:
    """Bit offset at which every column's codewords begin (m + 1 entries; the last is the stream's
    length): the per-column offsets the paper's conclusions propose, found by one sequential pass."""
    code = struct.code
    out = np.zeros(struct.m + 1, dtype=np.int64)
    if code.k == 0:
        return out
    left, right = _tree(code)
    words = np.ascontiguousarray(struct.words, dtype=np.uint32)
    if words.size == 0:
        words = np.zeros(1, dtype=np.uint32)
    tree = (_p(left, C.c_int32), _p(right, C.c_int32), C.c_int32(code.k), C.c_int32(code.root))
    if isinstance(struct, HAC):
        rc = lib().oracle_hac_column_offsets(_p(words, C.c_uint32), C.c_int64(struct.nbits), *tree,
                                             C.c_int64(struct.n), C.c_int64(struct.m), _p(out, C.c_int64))
    else:
        cb = np.ascontiguousarray(struct.cb, dtype=np.int64)
        rc = lib().oracle_shac_column_offsets(_p(words, C.c_uint32), C.c_int64(struct.nbits), _p(cb, C.c_int64), *tree,
                                              C.c_int64(struct.m), _p(out, C.c_int64))
    if rc:
        raise RuntimeError("column offsets: the stream does not hold the expected number of codewords")
    return out


def coldot(struct, X: np.ndarray, q: int = 1, colbit: Optional[np.ndarray] = None) -> np.ndarray:
    """Y = X.W with every codeword decoded once and applied to all rows of X, q threads over ranges
    of columns (each starts at its column's bit offset).  X is B x n fp32, the result B x m fp64."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    if X.ndim == 1:
        X = X[None, :]
    rows, n = X.shape
    if n != struct.n:
        raise ValueError("X has the wrong width")
    out = np.zeros((rows, struct.m), dtype=np.float64)
    code = struct.code
    if rows == 0 or struct.m == 0 or code.k == 0:
        return out
    if colbit is None:
        colbit = column_offsets(struct)
    colbit = np.ascontiguousarray(colbit, dtype=np.int64)
    left, right = _tree(code)
    values = np.ascontiguousarray(struct.values, dtype=np.float32)
    words = np.ascontiguousarray(struct.words, dtype=np.uint32)
    if words.size == 0:
        words = np.zeros(1, dtype=np.uint32)
    if isinstance(struct, HAC):
        ri_p, cb_p, keep = None, None, ()
    else:
        ri = np.ascontiguousarray(struct.ri, dtype=np.int64)
        if ri.size == 0:
            ri = np.zeros(1, dtype=np.int64)
        cb = np.ascontiguousarray(struct.cb, dtype=np.int64)
        ri_p, cb_p, keep = _p(ri, C.c_int64), _p(cb, C.c_int64), (ri, cb)
    rc = lib().oracle_coldot(_p(words, C.c_uint32), _p(colbit, C.c_int64), ri_p, cb_p,
                             _p(left, C.c_int32), _p(right, C.c_int32), C.c_int32(code.k), C.c_int32(code.root),
                             _p(values, C.c_float), _p(X, C.c_float), C.c_int64(rows), C.c_int64(n),
                             C.c_int64(struct.n), C.c_int64(struct.m), C.c_int32(q), _p(out, C.c_double))
    del keep
    if rc:
        raise RuntimeError(f"oracle coldot failed: {rc}")
    return out
