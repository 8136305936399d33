"""CPU oracle for the HAC / sHAC compressed dot product.  TEST INFRASTRUCTURE.

A plain, slow, obviously-correct implementation of what the hot path
computes, written from the paper (arXiv 2108.12704, Sect. IV) and from
nothing else.  Only the tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product (the HIP library and its Python
binding) never does, and this package never imports the product.

Modules
  huffman   classic Huffman code over the values that occur in W (Sect. IV-B)
  formats   CSC (Sect. IV-A), HAC (Sect. IV-B) and sHAC (Sect. IV-C) encoders
            and bit-by-bit decoders
  dot       Algorithm 1 (Dot_HAC), Algorithm 2 (Dot_sHAC), Algorithm 3 (ParDot)
            taken step by step, plus the dense definition Y = X.W in fp64
  bounds    Fact 1, Corollary 1, Eq. (2), Fact 2, Corollary 2, Eq. (3), the
            sHAC-vs-HAC sparsity crossover, psi_CSC and the index-map occupancy
  cnative   ctypes wrapper of oracle/c/oracle.c: the same encoders and
            Algorithms 1-3 in plain C, for sizes where Python loops are too slow

Readings of the paper that the oracle fixes (the paper is silent or garbled):
  * W is n x m; an input vector x has n entries; the result has m entries;
    a batch X is B x n with one input vector per row and Y = X.W is B x m
    (the shapes printed in Algorithms 1-3 are inconsistent with each other).
  * b = 32: the stream is an array of 32-bit unsigned words; the first bit of
    the stream is the most significant bit of word 0.
  * The alphabet is the set of fp32 values that occur in W (HAC: the value 0
    included when it occurs; sHAC: non-zero values only).  Symbols are
    numbered with 0 first (if present) and the other values in ascending
    numeric order.  -0.0 is stored as +0.0; NaN / Inf are rejected.
  * Any optimal prefix code is a valid Huffman code; what is unique is the
    total cost sum(f_i * l_i).  A one-symbol alphabet gets the 1-bit code "0".
  * Decoders stop on the symbol count (n*m for HAC, q for sHAC), never on the
    end of the bits, so the zero padding of the last word is never decoded.
  * Algorithm 2 leaves Y[j] = 0 for every empty column, leading and trailing
    ones included.

Pins (tests/ with `-m "not gpu"`): the paper's Examples 1 and 2, brute-force
optimal code lengths on tiny alphabets, Kraft equality and prefix-freeness,
the entropy sandwich H <= avg <= H+1, equiprobable 2^j alphabets, bit-exact
round trips, scipy's CSC arrays and product, numpy's dense fp64 product,
identity batches, linearity, and the space bounds listed above.

unified.py writes out the single dictionary shared by all layers of a network
(Sect. V-H) on top of `formats`, and a chain of layers X -> act(X.W + b) in fp64
with a forward error bound; its readings and pins are in that module's header.

gapcode.py holds an extension that is not in the paper (sHAC whose row indices
are replaced by Golomb-Rice coded gaps); its definition and its own pins are in
that module's header.
"""
