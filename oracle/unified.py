"""One dictionary for all the layers of a network, and a chain of layers.

TEST INFRASTRUCTURE -- see oracle/__init__.py.

Unified dictionary (paper Sect. V-H, "Evaluation of global and per-layer
quantization"; used for the whole network in Sect. V-K):
when the layers of a network are quantized together they draw their weights
from one set of representatives, and the paper then stores one dictionary for
the whole network in place of one per layer.  Written out for HAC / sHAC:

  * every layer contributes the symbols it writes into its own stream -- all
    n*m entries (zeros included) for a HAC layer, the q non-zeros for an sHAC
    layer -- to one pooled source;
  * the alphabet is the set of values of the pooled source, numbered as
    everywhere else (0.0 first when it occurs, then ascending), and one Huffman
    code is built from the pooled counts;
  * each layer's stream is HAC(W) / HAC(nz) of Sect. IV-B / IV-C written with
    that shared code; ri and cb of an sHAC layer are untouched;
  * the stored size counts the two dictionaries once (6kb bits, as in the proof
    of Fact 1) plus every layer's words (and ri, cb for sHAC).

The paper does not say what is pooled when HAC and sHAC layers are mixed; the
reading above makes the shared code optimal for the concatenation of all the
streams that are written with it.

Index-map layers (the hybrid of Sect. V-K: index map for the convolutional part,
HAC / sHAC for the fully connected part, "sharing the same representatives"):
an index-map layer (Sect. III-C1) writes no codewords, so it adds nothing to the
pooled source; its pointers index the network's one value list, which is the
shared alphabet followed by the values that occur in index-map layers only
(0.0 first if it is one of them, then ascending).  A pointer takes 8 bits when
the list has at most 256 entries, else 16.  Size: bbar*n*m per index-map layer,
and b bits per extra value (they are in no dictionary, only in the value vector,
as in the paper's index-map accounting).

Chain of layers (not in the paper, which gives the product of one layer only):
X_0 = X,  X_{l+1} = act_l(X_l . W_l + b_l)  with act_l the identity or
max(., 0), b_l an optional row vector; evaluated in fp64.  `chain_bound`
propagates the element-wise error a path may make when each of its products is
within rel * (|X|.|W|) of the exact one.

Pins (tests/test_oracle_unified.py): index-map layers reduce to oracle.indexmap
when alone, point below the list's length, decode to W, leave the code of the
other layers untouched, and cost bbar*n*m + b per extra value; a two-layer example worked by hand,
pooled counts against a direct count, optimality of the shared code for the
pooled source and sub-optimality per layer (never shorter than the layer's own
code, equal when the layers have proportional histograms), bit-exact round
trips, Algorithms 1 / 2 on a shared-code layer against the dense product, the
saving of (L - 1) * 6kb for layers over one value set, and the chain against
nested numpy products, a hand-computed 2-layer case and a linear (no
activation) chain that collapses to one matrix.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import formats, huffman
from .formats import HAC, SHAC, WORD_BITS
from .indexmap import IndexMap


@dataclass
class Unified:
    values: np.ndarray            # shared fp32 alphabet
    freqs: np.ndarray             # pooled counts
    code: huffman.HuffmanCode     # the one code
    kinds: List[str]              # "hac" / "shac" / "im" per layer
    layers: list                  # HAC / SHAC structures whose values/code are the shared ones; IndexMap
    extras: np.ndarray = None     # values that occur in index-map layers only

    @property
    def value_list(self) -> np.ndarray:
        if self.extras is None or self.extras.size == 0:
            return self.values
        return np.concatenate([self.values, self.extras]).astype(np.float32)


def layer_source(kind: str, W: np.ndarray) -> np.ndarray:
    """The value sequence a layer writes into its stream."""
    W = huffman.normalise_values(W)
    if kind == "hac":
        return formats.column_order(W)
    if kind == "shac":
        return formats.csc_arrays(W)[0]
    if kind == "im":
        return np.zeros(0, dtype=np.float32)         # pointers, no codewords
    raise ValueError("kind must be 'hac', 'shac' or 'im'")


def pooled_alphabet(kinds: Sequence[str], Ws: Sequence[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    pool = [layer_source(k, W) for k, W in zip(kinds, Ws)]
    allv = np.concatenate(pool) if pool else np.zeros(0, dtype=np.float32)
    return huffman.alphabet(allv)


def unified_encode(kinds: Sequence[str], Ws: Sequence[np.ndarray], reference_packer: bool = False) -> Unified:
    if len(kinds) != len(Ws):
        raise ValueError("one kind per layer")
    values, freqs = pooled_alphabet(kinds, Ws)
    code = huffman.build(freqs.tolist())
    packer = formats.pack_stream_reference if reference_packer else formats.pack_stream
    # values of index-map layers that no stream holds: appended to the list, 0.0 first, then ascending
    im_vals = [np.unique(huffman.normalise_values(W)) for kind, W in zip(kinds, Ws) if kind == "im"]
    extras = np.zeros(0, dtype=np.float32)
    if im_vals:
        cand = np.unique(np.concatenate(im_vals))
        cand = cand[~np.isin(cand, values)]
        extras = np.concatenate([cand[cand == 0], cand[cand != 0]]).astype(np.float32)
    value_list = np.concatenate([values, extras]).astype(np.float32)
    if value_list.size > 65536 and im_vals:
        raise ValueError("more than 65536 values for 16-bit pointers")
    bbar = 8 if value_list.size <= 256 else 16
    layers = []
    for kind, W in zip(kinds, Ws):
        W = huffman.normalise_values(W)
        n, m = W.shape
        if kind == "im":
            pi = np.empty((n, m), dtype=np.uint8 if bbar == 8 else np.uint16)
            for idx, v in enumerate(value_list):
                pi[W == v] = idx
            layers.append(IndexMap(n=n, m=m, c=value_list, pi=pi, bbar=bbar))
        elif kind == "hac":
            sym = formats.symbol_indices(formats.column_order(W), values)
            words, nbits = packer(sym, code)
            layers.append(HAC(n, m, values, freqs, code, words, nbits))
        else:
            nz, ri, cb = formats.csc_arrays(W)
            sym = formats.symbol_indices(nz, values)
            words, nbits = packer(sym, code)
            layers.append(SHAC(n, m, values, freqs, code, words, nbits, ri, cb))
    return Unified(values, freqs, code, list(kinds), layers, extras)


def unified_decode(u: Unified, layer: int) -> np.ndarray:
    s = u.layers[layer]
    if u.kinds[layer] == "im":
        return s.c[s.pi.astype(np.int64)]
    return formats.hac_decode(s) if u.kinds[layer] == "hac" else formats.shac_decode(s)


def unified_paper_bits(u: Unified, b: int = WORD_BITS) -> int:
    """Stored size with the dictionaries counted once."""
    total = 6 * len(u.values) * b + (0 if u.extras is None else len(u.extras)) * b
    for kind, s in zip(u.kinds, u.layers):
        if kind == "im":
            total += s.bbar * s.n * s.m
        elif kind == "hac":
            total += s.N * b
        else:
            total += s.N1 * b + b * (s.q + s.m + 1)
    return total


def separate_paper_bits(kinds: Sequence[str], Ws: Sequence[np.ndarray], b: int = WORD_BITS) -> int:
    """Stored size when every layer keeps a code and dictionaries of its own."""
    total = 0
    from . import indexmap
    for kind, W in zip(kinds, Ws):
        if kind == "im":
            total += indexmap.im_bits(indexmap.im_encode(W), b)
        elif kind == "hac":
            total += formats.hac_paper_bits(formats.hac_encode(W), b)
        else:
            total += formats.shac_paper_bits(formats.shac_encode(W), b)
    return total


# --------------------------------------------------------------------------
# chain of layers
# --------------------------------------------------------------------------

def chain(X: np.ndarray, Ws: Sequence[np.ndarray], biases: Sequence[Optional[np.ndarray]],
          relu: Sequence[bool]) -> List[np.ndarray]:
    """Activations after every layer, fp64.  Ws[l] is n_l x m_l with m_l = n_{l+1}."""
    A = np.asarray(X, dtype=np.float64)
    out = []
    for W, b, r in zip(Ws, biases, relu):
        A = A @ np.asarray(W, dtype=np.float64)
        if b is not None:
            A = A + np.asarray(b, dtype=np.float64)[None, :]
        if r:
            A = np.maximum(A, 0.0)
        out.append(A)
    return out


def chain_bound(X: np.ndarray, Ws: Sequence[np.ndarray], biases: Sequence[Optional[np.ndarray]],
                relu: Sequence[bool], rel: float, eps: float = 2.0 ** -24) -> List[np.ndarray]:
    """Element-wise bound on |computed - exact| after every layer.

    If the input of layer l is off by at most E (element-wise) and the layer's own
    product is within rel * (|X|.|W|) of the exact product of the input it was
    given, then its output is off by at most
        E.|W| + rel * ((|X| + E).|W|) + eps * (|X.W| + |b|)    (the bias add rounds once)
    and max(., 0) does not increase an error.
    """
    A = np.asarray(X, dtype=np.float64)
    E = np.zeros_like(A)
    out = []
    for W, b, r in zip(Ws, biases, relu):
        W64 = np.asarray(W, dtype=np.float64)
        absW = np.abs(W64)
        P = A @ W64
        Enew = E @ absW + rel * ((np.abs(A) + E) @ absW)
        if b is not None:
            b64 = np.asarray(b, dtype=np.float64)[None, :]
            Enew = Enew + eps * (np.abs(P) + np.abs(b64) + Enew)
            P = P + b64
        if r:
            P = np.maximum(P, 0.0)
        A, E = P, Enew
        out.append(E)
    return out
