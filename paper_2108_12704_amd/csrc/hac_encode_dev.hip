// GPU-side encoder: builds a HAC or sHAC blob (arXiv 2108.12704 Sect. IV-B / IV-C) from a matrix
// that already lives in device memory, byte for byte the blob hac_encode / shac_encode would build
// on the host.
//
// The steps of the host encoder, split between device and host:
//   1. device  histogram of the distinct fp32 values (a hash table keyed by bit pattern, privatised
//              in LDS per block), and the number of non-zeros and the last non-zero row of every
//              (row segment, column); the occupied slots of the table are gathered into a list,
//              and a thread per column walks its segments for the row after the last non-zero
//              above each;
//   2. host    alphabet in value order, Huffman lengths, canonical code, decode tables (all of
//              the size of the alphabet);
//   3. device  code bits of every (row segment, column); with Rice-coded row gaps also the gap
//              bits for every parameter k = 0..15, per (segment, column) and in total; then the
//              bits and non-zeros of every column (the Rice parameter, picked on the host from
//              the 16 totals, says which gap bits count);
//   4. host    chunk size, prefix sums over the columns (first stream bit, CSC position, first
//              chunk of every column), section offsets, header;
//      device  a thread per column walks its segments again: first stream bit / CSC position of
//              every segment, and where the non-zero before it ended;
//   5. device  one thread per (row segment, column) walks its rows and writes codewords (and
//              row-index fields or gap codewords) with atomic ORs into the zeroed stream, and the
//              chunk entries.
// A thread owns one column of a segment of rows (1024 on large matrices, down to 32 on small ones, so
// that there are threads enough to fill the chip), so the 64 lanes of a wave read 64
// neighbouring columns of one row: coalesced reads of the row-major matrix in all three passes;
// the per-column walks read the (segment, column) arrays the same way.
// What crosses the bus is of the size of the alphabet and of the number of columns, never of the
// matrix.  The call synchronises the stream twice before its final wait (steps 2 and 4 need the
// device's results), three times with Rice-coded gaps.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "hac_hostlib.h"

namespace {

using namespace hac_internal;

constexpr uint32_t kHashSlots = 1u << 17;          // distinct values <= 65536 keep the load below 1/2
constexpr uint32_t kSegRowsMax = 1024, kSegRowsMin = 32;

// Rows per segment: 1024 on a large matrix, fewer on a small one, so that there are about 128 K
// (segment, column) threads to fill the chip; a power of two, and at most 65535 segments (grid rows).
__host__ inline uint32_t seg_rows_for(uint64_t n, uint64_t m)
{
    const uint64_t want = (n * m + 131071) / 131072;
    uint32_t r = kSegRowsMin;
    while (r < kSegRowsMax && (r < want || (n + r - 1) / r > 65535)) r <<= 1;
    return r;
}
constexpr uint32_t kLocalSlots = 1024;
constexpr uint32_t kFlagNonFinite = 1u, kFlagTableFull = 2u;

__host__ __device__ inline uint32_t mix32(uint32_t k)
{
    k ^= k >> 16; k *= 0x7feb352du; k ^= k >> 15; k *= 0x846ca68bu; k ^= k >> 16;
    return k;
}

__global__ void fill_zero_kernel(uint32_t* p, uint64_t count)
{
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) p[i] = 0u;
}

__device__ void table_add(uint32_t* keys, uint32_t* cnts, uint32_t* flags, uint32_t key, uint32_t add)
{
    uint32_t h = mix32(key) & (kHashSlots - 1);
    for (uint32_t probe = 0; probe < kHashSlots; ++probe) {
        const uint32_t old = atomicCAS(&keys[h], 0u, key);
        if (old == 0u || old == key) { atomicAdd(&cnts[h], add); return; }
        h = (h + 1) & (kHashSlots - 1);
    }
    atomicOr(flags, kFlagTableFull);
}

// Rows r0 .. r1 - 1 of column j, in order: eight loads are issued before the first value is used, so
// that a thread has eight rows in flight instead of one (the walk itself is sequential).
template <class F>
__device__ __forceinline__ void for_rows(const float* __restrict__ W, uint64_t ldw, uint32_t j, uint32_t r0, uint32_t r1, F f)
{
    uint32_t r = r0;
    for (; r + 8 <= r1; r += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = W[(uint64_t)(r + u) * ldw + j];
#pragma unroll
        for (int u = 0; u < 8; ++u) f(r + u, v[u]);
    }
    for (; r < r1; ++r) f(r, W[(uint64_t)r * ldw + j]);
}

// step 1
__global__ void __launch_bounds__(256)
enc_scan_kernel(const float* __restrict__ W, uint32_t n, uint32_t m, uint64_t ldw, uint32_t seg_rows,
                uint32_t* keys, uint32_t* cnts, uint32_t* seg_nnz, uint32_t* seg_last, uint32_t* flags)
{
    __shared__ uint32_t lk[kLocalSlots], lc[kLocalSlots];
    for (uint32_t i = threadIdx.x; i < kLocalSlots; i += 256) { lk[i] = 0u; lc[i] = 0u; }
    __syncthreads();
    const uint32_t j = blockIdx.x * 256 + threadIdx.x, seg = blockIdx.y;
    const uint32_t r0 = seg * seg_rows, r1 = r0 + seg_rows < n ? r0 + seg_rows : n;
    uint32_t count = 0, last = 0xffffffffu;
    if (j < m) {
        for_rows(W, ldw, j, r0, r1, [&](uint32_t r, float v) {
            if (v == 0.0f) return;                                   // +0.0 and -0.0 are the null entry
            if (!isfinite(v)) { atomicOr(flags, kFlagNonFinite); return; }
            ++count; last = r;
            const uint32_t key = __float_as_uint(v);
            uint32_t h = mix32(key) & (kLocalSlots - 1);
            bool done = false;
            for (uint32_t probe = 0; probe < 64 && !done; ++probe) {
                const uint32_t old = atomicCAS(&lk[h], 0u, key);
                if (old == 0u || old == key) { atomicAdd(&lc[h], 1u); done = true; }
                h = (h + 1) & (kLocalSlots - 1);
            }
            if (!done) table_add(keys, cnts, flags, key, 1u);        // the block's table is crowded
        });
        seg_nnz[(uint64_t)seg * m + j] = count;
        seg_last[(uint64_t)seg * m + j] = last;
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < kLocalSlots; i += 256)
        if (lk[i]) table_add(keys, cnts, flags, lk[i], lc[i]);
}

__device__ __forceinline__ uint32_t symbol_of(const uint32_t* __restrict__ keys, const uint32_t* __restrict__ slot_sym,
                                              uint32_t key)
{
    uint32_t h = mix32(key) & (kHashSlots - 1);
    for (uint32_t probe = 0; probe < kHashSlots; ++probe) {         // the key is in the table: step 1 put it there
        if (keys[h] == key) return slot_sym[h];
        h = (h + 1) & (kHashSlots - 1);
    }
    return 0u;
}

// Rows r0 .. r1 - 1 of column j with each non-zero's symbol (+ shift), code length and, when
// `codes` is given, codeword.  The lookups of eight rows travel together: first the eight
// values, then their eight hash probes, their symbols, their lengths and codewords -- five trips
// to memory per eight rows instead of five per non-zero (some lane of a wave holds a non-zero in
// almost every row, so the whole wave pays for each trip).
// NZ_ONLY: f sees the non-zero rows only (in order).  They pass through a queue of the thread's own
// in LDS (queue[(8 entries x 3 words) x 256 threads]), so that a wave runs f as often as its
// fullest lane has non-zeros among the eight rows, not once for every row in which any lane has one.
template <bool NZ_ONLY, class F>
__device__ __forceinline__ void for_rows_coded(const float* __restrict__ W, uint64_t ldw, uint32_t j, uint32_t r0, uint32_t r1,
                                               const uint32_t* __restrict__ keys, const uint32_t* __restrict__ slot_sym,
                                               uint32_t shift, const uint8_t* __restrict__ lens,
                                               const uint32_t* __restrict__ codes, uint32_t* queue, F f)
{
    uint32_t r = r0;
    for (; r + 8 <= r1; r += 8) {
        float v[8];
        uint32_t h[8], got[8], sym[8], len[8], code[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = W[(uint64_t)(r + u) * ldw + j];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t key = __float_as_uint(v[u]);
            h[u] = mix32(key) & (kHashSlots - 1);
            got[u] = v[u] != 0.0f ? keys[h[u]] : key;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {                                // the key is in the table: step 1 put it there
            const uint32_t key = __float_as_uint(v[u]);
            for (uint32_t probe = 0; got[u] != key && probe < kHashSlots; ++probe) {
                h[u] = (h[u] + 1) & (kHashSlots - 1);
                got[u] = keys[h[u]];
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) sym[u] = v[u] != 0.0f ? slot_sym[h[u]] + shift : 0u;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            len[u] = v[u] != 0.0f ? lens[sym[u]] : 0u;
            code[u] = (codes && v[u] != 0.0f) ? codes[sym[u]] : 0u;
        }
        // All of the above has arrived before the first row is applied: f may issue stores and atomics,
        // and a wait for a load that was issued before them would wait for them too (one counter).
        __builtin_amdgcn_s_waitcnt(0x0f70);                          // vmcnt(0), the other counters untouched
        if constexpr (NZ_ONLY) {
            uint32_t* q = queue + threadIdx.x;
            uint32_t cnt = 0;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (v[u] != 0.0f) {
                    q[(cnt * 3 + 0) * 256] = r + u; q[(cnt * 3 + 1) * 256] = len[u]; q[(cnt * 3 + 2) * 256] = code[u];
                    ++cnt;
                }
            }
            for (uint32_t i = 0; i < cnt; ++i) f(q[(i * 3 + 0) * 256], 1.0f, 0u, q[(i * 3 + 1) * 256], q[(i * 3 + 2) * 256]);
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) f(r + u, v[u], sym[u], len[u], code[u]);
        }
    }
    for (; r < r1; ++r) {
        const float v = W[(uint64_t)r * ldw + j];
        uint32_t sym = 0, len = 0, code = 0;
        if (v != 0.0f) {
            sym = symbol_of(keys, slot_sym, __float_as_uint(v)) + shift;
            len = lens[sym];
            if (codes) code = codes[sym];
        }
        if (!NZ_ONLY || v != 0.0f) f(r, v, sym, len, code);
    }
}

__device__ __forceinline__ uint32_t rice_len(uint32_t d, uint32_t k)
{
    const uint32_t q = d >> k;
    return q < kRiceEscape ? q + 1 + k : kRiceEscape + 1 + 32;
}

// step 3.  gap_bits (Rice-coded gaps only, else nullptr): [k][segment][column] bits of the gap
// codewords for k = 0..15; gap_total: their 16 sums over the matrix.
__global__ void __launch_bounds__(256)
enc_bits_kernel(const float* __restrict__ W, uint32_t n, uint32_t m, uint64_t ldw,
                const uint32_t* __restrict__ keys, const uint32_t* __restrict__ slot_sym,
                const uint8_t* __restrict__ lens, uint32_t* seg_codebits,
                const uint32_t* __restrict__ seg_prev_row1, uint32_t* gap_bits, unsigned long long* gap_total,
                uint64_t seg_cols, uint32_t seg_rows)
{
    const uint32_t j = blockIdx.x * 256 + threadIdx.x, seg = blockIdx.y;
    const uint32_t r0 = seg * seg_rows, r1 = r0 + seg_rows < n ? r0 + seg_rows : n;
    const uint64_t at = (uint64_t)seg * m + j;
    uint32_t bits = 0;
    uint32_t g[kRiceKMax + 1];
#pragma unroll
    for (uint32_t k = 0; k <= kRiceKMax; ++k) g[k] = 0;
    if (j < m) {
        uint32_t next = gap_bits ? seg_prev_row1[at] : 0u;           // the row the next gap counts from
        for_rows_coded<false>(W, ldw, j, r0, r1, keys, slot_sym, 0u, lens, nullptr, nullptr,
                              [&](uint32_t r, float v, uint32_t, uint32_t len, uint32_t) {
            if (v == 0.0f) return;
            bits += len;
            if (gap_bits) {
                const uint32_t d = r - next;
#pragma unroll
                for (uint32_t k = 0; k <= kRiceKMax; ++k) g[k] += rice_len(d, k);
                next = r + 1;
            }
        });
        seg_codebits[at] = bits;
    }
    if (!gap_bits) return;
#pragma unroll
    for (uint32_t k = 0; k <= kRiceKMax; ++k) {
        if (j < m) gap_bits[(uint64_t)k * seg_cols + at] = g[k];
        unsigned long long t = g[k];                                  // lanes past m hold 0
        for (int off = 32; off >= 1; off >>= 1) t += __shfl_down(t, off, 64);
        if ((threadIdx.x & 63) == 0 && t) atomicAdd(&gap_total[k], t);
    }
}

// `len` bits of `code` (right-justified), MSB first, at stream bit `bit`; the words start zeroed
__device__ __forceinline__ void put_bits(uint32_t* words, uint64_t bit, uint32_t code, uint32_t len)
{
    const uint64_t w = bit >> 5;
    const uint32_t off = (uint32_t)(bit & 31);
    const uint64_t v = (uint64_t)code << (64 - len - off);          // 1 <= len <= 32, off <= 31
    const uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
    if (hi) atomicOr(&words[w], hi);
    if (lo) atomicOr(&words[w + 1], lo);
}

struct EmitArgs {
    const float* W; uint32_t n, m; uint64_t ldw;
    const uint32_t* keys; const uint32_t* slot_sym; const uint32_t* codes; const uint8_t* lens;
    const uint32_t* seg_bit0; const uint32_t* seg_pos0; const uint32_t* seg_prev_end; const uint32_t* seg_prev_row1;
    const uint32_t* col_bit; const uint32_t* col_pos; const uint32_t* col_chunk;
    uint32_t* stream; void* ent; uint32_t* ri;
    uint32_t shac, has_zero, zcode, zlen, chunk, ent_bits, row_bits, ri_bits;
    uint32_t rice, rice_k;                                              // sHAC with Rice-coded gaps in the stream
    uint32_t seg_rows;
};

// step 5
__global__ void __launch_bounds__(256) enc_emit_kernel(EmitArgs a)
{
    __shared__ uint32_t queue[8 * 3 * 256];
    const uint32_t j = blockIdx.x * 256 + threadIdx.x, seg = blockIdx.y;
    if (j >= a.m) return;
    const uint32_t r0 = seg * a.seg_rows, r1 = r0 + a.seg_rows < a.n ? r0 + a.seg_rows : a.n;
    const uint64_t at = (uint64_t)seg * a.m + j;
    uint32_t bit = a.seg_bit0[at], pos = a.seg_pos0[at];
    uint32_t pend = a.seg_prev_end[at], prow = a.seg_prev_row1[at];   // HAC: where the non-zero before this one ended
    const uint32_t cbit0 = a.col_bit[j], cpos0 = a.col_pos[j], cchunk0 = a.col_chunk[j];
    const uint32_t chunk = hac_internal::chunk_of_column(a.chunk, a.col_pos[j + 1] - cpos0);   // of this column
    const uint32_t shift = (!a.shac && a.has_zero) ? 1u : 0u;          // HAC numbers 0.0 as symbol 0
    auto on_nonzero = [&](uint32_t r, uint32_t len, uint32_t code) {
        const uint32_t q = pos - cpos0;
        if (q % chunk == 0) {
            const uint32_t g = cchunk0 + q / chunk;
            if (a.rice) {
                // the chunk starts at its first gap codeword; the gap counts from the row after the non-zero before
                const uint32_t rel = bit - cbit0;
                if (a.ent_bits == 32) static_cast<uint32_t*>(a.ent)[g] = (rel << a.row_bits) | prow;
                else { static_cast<uint32_t*>(a.ent)[2 * (uint64_t)g] = prow; static_cast<uint32_t*>(a.ent)[2 * (uint64_t)g + 1] = rel; }
            } else if (a.shac) {
                const uint32_t rel = bit - cbit0;
                if (a.ent_bits == 16) static_cast<uint16_t*>(a.ent)[g] = (uint16_t)rel;
                else static_cast<uint32_t*>(a.ent)[g] = rel;
            } else {
                const uint32_t rel = pend - cbit0;
                if (a.ent_bits == 32) static_cast<uint32_t*>(a.ent)[g] = (rel << a.row_bits) | prow;
                else { static_cast<uint32_t*>(a.ent)[2 * (uint64_t)g] = prow; static_cast<uint32_t*>(a.ent)[2 * (uint64_t)g + 1] = rel; }
            }
        }
        if (a.rice) {
            const uint32_t d = r - prow, k = a.rice_k, qq = d >> k;
            if (qq < kRiceEscape) {
                put_bits(a.stream, (uint64_t)bit + qq, (1u << k) | (d & ((1u << k) - 1u)), k + 1);
                bit += qq + 1 + k;
            } else {
                put_bits(a.stream, (uint64_t)bit + kRiceEscape, 1u, 1);
                put_bits(a.stream, (uint64_t)bit + kRiceEscape + 1, d, 32);
                bit += kRiceEscape + 1 + 32;
            }
        }
        put_bits(a.stream, bit, code, len);
        bit += len;
        pend = bit; prow = r + 1;
        if (a.shac && !a.rice) put_bits(a.ri, (uint64_t)pos * a.ri_bits, r, a.ri_bits);
        ++pos;
    };
    if (a.shac || a.zcode == 0) {
        // zeros write nothing (sHAC has none in its stream; an all-zero codeword is what the cleared
        // stream already holds): only the non-zeros are visited, a run of zeros just moves `bit`
        uint32_t next_row = r0;
        for_rows_coded<true>(a.W, a.ldw, j, r0, r1, a.keys, a.slot_sym, shift, a.lens, a.codes, queue,
                             [&](uint32_t r, float, uint32_t, uint32_t len, uint32_t code) {
            if (!a.shac) bit += (r - next_row) * a.zlen;
            next_row = r + 1;
            on_nonzero(r, len, code);
        });
    } else {
        for_rows_coded<false>(a.W, a.ldw, j, r0, r1, a.keys, a.slot_sym, shift, a.lens, a.codes, nullptr,
                              [&](uint32_t r, float v, uint32_t, uint32_t len, uint32_t code) {
            if (v == 0.0f) {
                put_bits(a.stream, bit, a.zcode, a.zlen);
                bit += a.zlen;
                return;
            }
            on_nonzero(r, len, code);
        });
    }
}

// step 1, second part: the occupied slots of the table as a list of (key, count, slot), in no
// particular order (the host sorts by value); *n_list counts them, entries past `cap` are dropped
// (the host then sees n_list > cap and gives up: more than 65536 distinct values)
__global__ void __launch_bounds__(256)
enc_gather_kernel(const uint32_t* __restrict__ keys, const uint32_t* __restrict__ cnts, uint32_t* list, uint32_t cap, uint32_t* n_list)
{
    const uint32_t h = blockIdx.x * 256 + threadIdx.x;
    if (h >= kHashSlots) return;
    const uint32_t key = keys[h];
    if (!key) return;
    const uint32_t i = atomicAdd(n_list, 1u);
    if (i < cap) { list[3 * (uint64_t)i] = key; list[3 * (uint64_t)i + 1] = cnts[h]; list[3 * (uint64_t)i + 2] = h; }
}

// the row after the last non-zero above every segment (0 at a column's top); a thread per column
__global__ void __launch_bounds__(256)
enc_prev_row_kernel(const uint32_t* __restrict__ seg_nnz, const uint32_t* __restrict__ seg_last, uint32_t S, uint32_t m,
                    uint32_t* __restrict__ seg_prev_row1)
{
    const uint32_t j = blockIdx.x * 256 + threadIdx.x;
    if (j >= m) return;
    uint32_t prev = 0;
    for (uint32_t s = 0; s < S; ++s) {
        const uint64_t at = (uint64_t)s * m + j;
        seg_prev_row1[at] = prev;
        if (seg_nnz[at]) prev = seg_last[at] + 1;
    }
}

// step 2 -> 3: slot_sym[slot of list entry i] = sym[i] (index among the non-zero values)
__global__ void __launch_bounds__(256)
enc_slot_sym_kernel(const uint32_t* __restrict__ list, const uint32_t* __restrict__ sym, uint32_t count, uint32_t* __restrict__ slot_sym)
{
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < count) slot_sym[list[3 * (uint64_t)i + 2]] = sym[i];
}

struct SegBits {
    const uint32_t* seg_nnz; const uint32_t* seg_codebits; const uint32_t* seg_gapbits;   // gap bits of the chosen k, or nullptr
    uint32_t n, m, seg_rows, zlen, shac;
    // stream bits of segment s of the column at index `at`
    __device__ __forceinline__ uint64_t bits(uint32_t s, uint64_t at) const {
        const uint64_t r0 = (uint64_t)s * seg_rows, r1 = r0 + seg_rows < n ? r0 + seg_rows : n;
        return (uint64_t)seg_codebits[at] + (shac ? 0ull : (r1 - r0 - seg_nnz[at]) * zlen) + (seg_gapbits ? seg_gapbits[at] : 0u);
    }
};

// step 3, second part: non-zeros and stream bits of every column
__global__ void __launch_bounds__(256)
enc_col_sums_kernel(SegBits sb, uint32_t S, uint32_t* __restrict__ col_nnz, unsigned long long* __restrict__ col_bits)
{
    const uint32_t j = blockIdx.x * 256 + threadIdx.x;
    if (j >= sb.m) return;
    uint32_t nnz = 0;
    unsigned long long bits = 0;
    for (uint32_t s = 0; s < S; ++s) {
        const uint64_t at = (uint64_t)s * sb.m + j;
        nnz += sb.seg_nnz[at];
        bits += sb.bits(s, at);
    }
    col_nnz[j] = nnz; col_bits[j] = bits;
}

// step 4, device part: running state per column over its segments
__global__ void __launch_bounds__(256)
enc_seg_walk_kernel(SegBits sb, uint32_t S, const uint32_t* __restrict__ seg_last,
                    const uint32_t* __restrict__ col_bit, const uint32_t* __restrict__ col_pos,
                    uint32_t* __restrict__ seg_bit0, uint32_t* __restrict__ seg_pos0, uint32_t* __restrict__ seg_prev_end)
{
    const uint32_t j = blockIdx.x * 256 + threadIdx.x;
    if (j >= sb.m) return;
    uint64_t cur_bit = col_bit[j], cur_pos = col_pos[j], cur_end = col_bit[j];
    for (uint32_t s = 0; s < S; ++s) {
        const uint64_t at = (uint64_t)s * sb.m + j;
        const uint64_t r0 = (uint64_t)s * sb.seg_rows, r1 = r0 + sb.seg_rows < sb.n ? r0 + sb.seg_rows : sb.n;
        seg_bit0[at] = (uint32_t)cur_bit; seg_pos0[at] = (uint32_t)cur_pos; seg_prev_end[at] = (uint32_t)cur_end;
        const uint64_t cnt = sb.seg_nnz[at], seg_bits = sb.bits(s, at);
        if (cnt) {
            const uint64_t trailing = r1 - 1 - seg_last[at];                 // zeros after the segment's last non-zero
            cur_end = cur_bit + seg_bits - (sb.shac ? 0ull : trailing * sb.zlen);
        }
        cur_bit += seg_bits; cur_pos += cnt;
    }
}

constexpr uint32_t kListCap = 65536 + 64;          // one more than the largest alphabet is enough to see "too many"

struct WsLayout {
    size_t keys, cnts, flags, seg_nnz, seg_codebits, seg_last, seg_bit0, seg_pos0, seg_prev_end, seg_prev_row1,
           slot_sym, codes, lens, gap_bits, list, sym, col_nnz, col_bits, total;
};

WsLayout ws_layout(uint64_t n, uint64_t m)
{
    const uint64_t seg_rows = seg_rows_for(n, m), S = (n + seg_rows - 1) / seg_rows;
    WsLayout L;
    size_t c = 0;
    auto take = [&](size_t bytes) { const size_t o = c; c = (c + bytes + 255) / 256 * 256; return o; };
    L.keys = take(4ull * kHashSlots); L.cnts = take(4ull * kHashSlots); L.flags = take(256);
    L.seg_nnz = take(4 * S * m); L.seg_last = take(4 * S * m); L.seg_codebits = take(4 * S * m);   // keys .. seg_last: one copy back
    L.seg_bit0 = take(4 * S * m); L.seg_pos0 = take(4 * S * m); L.seg_prev_end = take(4 * S * m); L.seg_prev_row1 = take(4 * S * m);
    L.slot_sym = take(4ull * kHashSlots); L.codes = take(4ull * 65537); L.lens = take(65537);
    L.gap_bits = take(4 * S * m * (kRiceKMax + 1));                  // used with Rice-coded gaps only
    L.list = take(12ull * kListCap); L.sym = take(4ull * kListCap);
    L.col_nnz = take(4 * m); L.col_bits = take(8 * m);
    L.total = c;
    return L;
}

int hip_fail(hipError_t e) { hac_internal::set_last_hip_error((int)e); return HAC_EHIP; }

} // namespace

extern "C" size_t hac_encode_dev_workspace_bytes(int64_t n, int64_t m)
{
    if (n < 1 || m < 1 || n > 0x7fffffffll || m > 0x7fffffffll) return 0;
    return ws_layout((uint64_t)n, (uint64_t)m).total;
}

extern "C" int hac_encode_dev(uint32_t format, const float* d_W, int64_t n, int64_t m, int64_t ldw,
                              const hac_opts_t* opts, void* d_blob, size_t blob_capacity, hac_desc_t* desc,
                              void* d_ws, size_t ws_bytes, hac_stream_t stream_)
{
    if (!d_W || !desc || !d_ws) return HAC_EINVAL;
    if (format != HAC_FORMAT_HAC && format != HAC_FORMAT_SHAC) return HAC_EINVAL;
    if (n < 1 || m < 1 || ldw < m) return HAC_EINVAL;
    if (n > 0x7fffffffll || m > 0x7fffffffll) return HAC_ERANGE;
    const uint32_t seg_rows = seg_rows_for((uint64_t)n, (uint64_t)m);
    if ((n + seg_rows - 1) / seg_rows > 65535) return HAC_ERANGE;       // one grid row per segment of rows
    int rc = check_opts(opts);
    if (rc) return rc;
    if (opts && opts->chunk_rows) return HAC_EINVAL;                   // the row index is built by the host encoders only
    const bool shac = format == HAC_FORMAT_SHAC;
    const bool rice = opts && opts->ri_coding == HAC_RI_RICE;
    if (rice && (!shac || opts->ri_bits)) return HAC_EINVAL;          // as the host encoders
    const uint32_t need_bits = std::max<uint32_t>(ceil_log2((uint64_t)n), 1);
    uint32_t ri_bits = 0;
    if (shac && !rice) {
        ri_bits = opts && opts->ri_bits ? opts->ri_bits : need_bits;
        if (ri_bits < need_bits || ri_bits > 32) return HAC_EINVAL;
    }
    if (reinterpret_cast<uintptr_t>(d_ws) % 256 || (d_blob && reinterpret_cast<uintptr_t>(d_blob) % 256)) return HAC_EINVAL;
    const WsLayout L = ws_layout((uint64_t)n, (uint64_t)m);
    if (ws_bytes < L.total) return HAC_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    hac_internal::set_last_hip_error(0);
    uint8_t* ws = static_cast<uint8_t*>(d_ws);
    auto dptr = [&](size_t off) { return reinterpret_cast<uint32_t*>(ws + off); };
    const uint32_t S = (uint32_t)(((uint64_t)n + seg_rows - 1) / seg_rows);
    const size_t SM = (size_t)S * (size_t)m;
    const dim3 grid((uint32_t)((m + 255) / 256), S);
    hipError_t e;
    try {
        const dim3 cgrid((uint32_t)((m + 255) / 256));               // a thread per column
        // ---- step 1 ----
        uint32_t* d_flags = dptr(L.flags);                           // [0] flags, [1] length of the list, +64 bytes: gap totals
        uint32_t* d_n_list = d_flags + 1;
        hipLaunchKernelGGL(fill_zero_kernel, dim3(512), dim3(256), 0, stream, dptr(L.keys), (uint64_t)(L.seg_nnz - L.keys) / 4);
        hipLaunchKernelGGL(enc_scan_kernel, grid, dim3(256), 0, stream, d_W, (uint32_t)n, (uint32_t)m, (uint64_t)ldw, seg_rows,
                           dptr(L.keys), dptr(L.cnts), dptr(L.seg_nnz), dptr(L.seg_last), d_flags);
        hipLaunchKernelGGL(enc_gather_kernel, dim3(kHashSlots / 256), dim3(256), 0, stream, dptr(L.keys), dptr(L.cnts),
                           dptr(L.list), kListCap, d_n_list);
        hipLaunchKernelGGL(enc_prev_row_kernel, cgrid, dim3(256), 0, stream, dptr(L.seg_nnz), dptr(L.seg_last), S, (uint32_t)m,
                           dptr(L.seg_prev_row1));
        if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e);
        // flags and the length of the list first (they sit side by side), then as much of the list
        // as is in use; a small alphabet arrives with the first copy
        constexpr uint32_t kFirst = 1024;
        std::vector<uint32_t> list(3 * (size_t)kFirst);
        uint32_t head2[2] = { 0, 0 };
        if ((e = hipMemcpyAsync(head2, d_flags, 8, hipMemcpyDeviceToHost, stream)) != hipSuccess) return hip_fail(e);
        if ((e = hipMemcpyAsync(list.data(), dptr(L.list), 12 * (size_t)kFirst, hipMemcpyDeviceToHost, stream)) != hipSuccess) return hip_fail(e);
        if ((e = hipStreamSynchronize(stream)) != hipSuccess) return hip_fail(e);
        const uint32_t flags = head2[0], n_list = head2[1];
        if (flags & kFlagNonFinite) return HAC_EINVAL;
        if (flags & kFlagTableFull) return HAC_ERANGE;
        if (n_list > 65536) return HAC_ERANGE;
        if (n_list > kFirst) {
            list.resize(3 * (size_t)n_list);
            if ((e = hipMemcpyAsync(list.data(), dptr(L.list), 12 * (size_t)n_list, hipMemcpyDeviceToHost, stream)) != hipSuccess) return hip_fail(e);
            if ((e = hipStreamSynchronize(stream)) != hipSuccess) return hip_fail(e);
        }

        // ---- step 2 ----
        struct Val { float v; uint32_t at; uint64_t f; };             // at: position in the list
        std::vector<Val> vals(n_list);
        uint64_t nnz = 0;
        for (uint32_t i = 0; i < n_list; ++i) {
            std::memcpy(&vals[i].v, &list[3 * (size_t)i], 4);
            vals[i].at = i; vals[i].f = list[3 * (size_t)i + 1];
            nnz += vals[i].f;
        }
        if (nnz > 0xfffffff0ull) return HAC_ERANGE;
        std::sort(vals.begin(), vals.end(), [](const Val& a, const Val& b) { return a.v < b.v; });
        const uint64_t zeros = (uint64_t)n * (uint64_t)m - nnz;
        const bool has_zero = !shac && zeros > 0;
        const uint32_t shift = has_zero ? 1u : 0u;
        std::vector<float> codebook;
        std::vector<uint64_t> freq;
        if (has_zero) { codebook.push_back(0.0f); freq.push_back(zeros); }
        for (const Val& x : vals) { codebook.push_back(x.v); freq.push_back(x.f); }
        std::vector<uint8_t> len; uint32_t lmax = 0;
        if (!huffman_lengths(freq, len, lmax)) return HAC_ERANGE;
        CodeTables t; canonical_codes(len, t);
        uint64_t total_bits = 0;
        for (size_t i = 0; i < freq.size(); ++i) total_bits += freq[i] * len[i];
        if (total_bits > 0xfffffff0ull) return HAC_ERANGE;
        const uint32_t lut_bits = pick_lut_bits(opts, lmax);
        if (lut_bits < 1 || lut_bits > 12) return HAC_EINVAL;
        std::vector<uint32_t> lut; build_lut(len, t, lut_bits, lut);
        const uint32_t zlen = has_zero ? len[0] : 0, zcode = has_zero ? t.code[0] : 0;

        // the device looks lengths up by "index among the non-zero values" in step 3 and by symbol in step 5
        std::vector<uint32_t> sym_of_entry(std::max<size_t>(n_list, 1), 0);
        for (size_t i = 0; i < vals.size(); ++i) sym_of_entry[vals[i].at] = (uint32_t)i;
        std::vector<uint8_t> nz_len(vals.size());
        for (size_t i = 0; i < vals.size(); ++i) nz_len[i] = len[i + shift];
        if (n_list) {
            if ((e = hipMemcpyAsync(dptr(L.sym), sym_of_entry.data(), 4ull * n_list, hipMemcpyHostToDevice, stream)) != hipSuccess) return hip_fail(e);
            if ((e = hipMemcpyAsync(ws + L.lens, nz_len.data(), nz_len.size(), hipMemcpyHostToDevice, stream)) != hipSuccess) return hip_fail(e);
            hipLaunchKernelGGL(enc_slot_sym_kernel, dim3((n_list + 255) / 256), dim3(256), 0, stream, dptr(L.list), dptr(L.sym), n_list,
                               dptr(L.slot_sym));
        }

        // ---- step 3 ----
        unsigned long long* d_gap_total = reinterpret_cast<unsigned long long*>(ws + L.flags + 64);   // zeroed with the flags
        hipLaunchKernelGGL(enc_bits_kernel, grid, dim3(256), 0, stream, d_W, (uint32_t)n, (uint32_t)m, (uint64_t)ldw,
                           dptr(L.keys), dptr(L.slot_sym), ws + L.lens, dptr(L.seg_codebits), dptr(L.seg_prev_row1),
                           rice ? dptr(L.gap_bits) : static_cast<uint32_t*>(nullptr), d_gap_total, (uint64_t)SM, seg_rows);
        if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e);
        // the Rice parameter: fewest gap bits, the smaller k on ties
        uint32_t rice_k = 0; uint64_t gap_bits = 0;
        if (rice) {
            unsigned long long gap_total[kRiceKMax + 1] = { 0 };
            if ((e = hipMemcpyAsync(gap_total, d_gap_total, sizeof gap_total, hipMemcpyDeviceToHost, stream)) != hipSuccess) return hip_fail(e);
            if ((e = hipStreamSynchronize(stream)) != hipSuccess) return hip_fail(e);
            gap_bits = ~0ull;
            for (uint32_t k = 0; k <= kRiceKMax; ++k) if (gap_total[k] < gap_bits) { gap_bits = gap_total[k]; rice_k = k; }
            if (nnz == 0) { gap_bits = 0; rice_k = 0; }
            total_bits += gap_bits;
            if (total_bits > 0xfffffff0ull) return HAC_ERANGE;
        }
        SegBits sb;
        sb.seg_nnz = dptr(L.seg_nnz); sb.seg_codebits = dptr(L.seg_codebits);
        sb.seg_gapbits = rice ? dptr(L.gap_bits) + (size_t)rice_k * SM : nullptr;
        sb.n = (uint32_t)n; sb.m = (uint32_t)m; sb.seg_rows = seg_rows; sb.zlen = zlen; sb.shac = shac ? 1u : 0u;
        unsigned long long* d_col_bits = reinterpret_cast<unsigned long long*>(ws + L.col_bits);
        hipLaunchKernelGGL(enc_col_sums_kernel, cgrid, dim3(256), 0, stream, sb, S, dptr(L.col_nnz), d_col_bits);
        if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e);
        std::vector<uint32_t> col_nnz((size_t)m);
        std::vector<unsigned long long> col_bits((size_t)m);
        if ((e = hipMemcpyAsync(col_nnz.data(), dptr(L.col_nnz), 4 * (size_t)m, hipMemcpyDeviceToHost, stream)) != hipSuccess) return hip_fail(e);
        if ((e = hipMemcpyAsync(col_bits.data(), d_col_bits, 8 * (size_t)m, hipMemcpyDeviceToHost, stream)) != hipSuccess) return hip_fail(e);
        if ((e = hipStreamSynchronize(stream)) != hipSuccess) return hip_fail(e);

        // ---- step 4 ----
        uint64_t max_col_nnz = 0, max_col_bits = 0;
        for (int64_t j = 0; j < m; ++j) {
            max_col_nnz = std::max<uint64_t>(max_col_nnz, col_nnz[(size_t)j]);
            max_col_bits = std::max<uint64_t>(max_col_bits, col_bits[(size_t)j]);
        }
        const uint32_t Cn = pick_chunk(opts, max_col_nnz);
        // the three per-column arrays sit side by side in the blob (256-byte aligned sections): one
        // host buffer with the same spacing, one copy
        const size_t col_stride = (4 * ((size_t)m + 1) + 255) / 256 * 256 / 4;       // words from one array to the next
        std::vector<uint32_t> col_arrays(3 * col_stride, 0);
        uint32_t* col_chunk = col_arrays.data();
        uint32_t* col_pos = col_chunk + col_stride;
        uint32_t* col_bit = col_pos + col_stride;
        uint64_t bit = 0, pos = 0, chunks = 0;
        for (int64_t j = 0; j < m; ++j) {
            col_bit[(size_t)j] = (uint32_t)bit; col_pos[(size_t)j] = (uint32_t)pos; col_chunk[(size_t)j] = (uint32_t)chunks;
            bit += col_bits[(size_t)j]; pos += col_nnz[(size_t)j];
            const uint32_t cj = chunk_of_column(Cn, col_nnz[(size_t)j]);
            chunks += (col_nnz[(size_t)j] + cj - 1) / cj;
        }
        col_bit[(size_t)m] = (uint32_t)bit; col_pos[(size_t)m] = (uint32_t)pos; col_chunk[(size_t)m] = (uint32_t)chunks;
        if (bit != total_bits || pos != nnz) return HAC_EFORMAT;
        if (chunks > 0xfffffff0ull) return HAC_ERANGE;

        hac_desc_t d;
        std::memset(&d, 0, sizeof d);
        d.magic = kMagic; d.version = kVersion; d.format = format; d.header_bytes = 256;
        d.n = (uint64_t)n; d.m = (uint64_t)m; d.nnz = nnz; d.total_bits = total_bits; d.n_words = (total_bits + 31) / 32;
        d.k_sym = (uint32_t)codebook.size(); d.lmax = lmax; d.lut_bits = lut_bits;
        d.chunk = Cn; d.n_chunks = chunks; d.max_col_bits = max_col_bits; d.max_col_nnz = max_col_nnz;
        if (rice) {
            const uint32_t brel_bits = std::max<uint32_t>(ceil_log2(max_col_bits + 1), 1);
            d.ent_bits = need_bits + brel_bits <= 32 ? 32 : 64;
            d.row_bits = d.ent_bits == 32 ? need_bits : 0;
            d.ri_coding = HAC_RI_RICE; d.rice_k = rice_k; d.gap_bits = gap_bits;
        } else if (shac) {
            d.ri_bits = ri_bits;
            d.ent_bits = max_col_bits < 65536 ? 16 : 32;
            if (nnz * (uint64_t)ri_bits > 0xfffffff0ull * 32ull) return HAC_ERANGE;
        } else {
            d.has_zero = has_zero ? 1 : 0;
            d.zero_len = (has_zero && zcode == 0) ? zlen : 0;
            const uint32_t brel_bits = std::max<uint32_t>(ceil_log2(max_col_bits + 1), 1);
            d.ent_bits = need_bits + brel_bits <= 32 ? 32 : 64;
            d.row_bits = d.ent_bits == 32 ? need_bits : 0;
        }
        place_sections(d);
        *desc = d;
        if (!d_blob || blob_capacity < d.blob_bytes) return HAC_EWORKSPACE;         // desc->blob_bytes says how much

        // head of the blob (header, tables, per-column arrays) is assembled here and copied over
        const size_t head_bytes = (size_t)d.off_stream;
        std::vector<uint8_t> head(head_bytes, 0);
        std::memcpy(head.data(), &d, sizeof d);
        write_tables(head.data(), d, codebook, len, t, lut);
        uint8_t* blob = static_cast<uint8_t*>(d_blob);
        hipLaunchKernelGGL(fill_zero_kernel, dim3(1024), dim3(256), 0, stream, reinterpret_cast<uint32_t*>(blob + d.off_stream),
                           (uint64_t)(d.blob_bytes - d.off_stream) / 4);
        if ((e = hipMemcpyAsync(blob, head.data(), head_bytes, hipMemcpyHostToDevice, stream)) != hipSuccess) return hip_fail(e);
        if (d.off_col_pos - d.off_col_chunk != 4 * col_stride || d.off_col_bit - d.off_col_pos != 4 * col_stride) return HAC_EFORMAT;
        if ((e = hipMemcpyAsync(blob + d.off_col_chunk, col_chunk, 4 * (2 * col_stride + (size_t)m + 1), hipMemcpyHostToDevice, stream)) != hipSuccess) return hip_fail(e);
        hipLaunchKernelGGL(enc_seg_walk_kernel, cgrid, dim3(256), 0, stream, sb, S, dptr(L.seg_last),
                           reinterpret_cast<const uint32_t*>(blob + d.off_col_bit), reinterpret_cast<const uint32_t*>(blob + d.off_col_pos),
                           dptr(L.seg_bit0), dptr(L.seg_pos0), dptr(L.seg_prev_end));
        // step 5 looks codes and lengths up by symbol
        if (!t.code.empty() && (e = hipMemcpyAsync(dptr(L.codes), t.code.data(), 4 * t.code.size(), hipMemcpyHostToDevice, stream)) != hipSuccess) return hip_fail(e);
        if (!len.empty() && (e = hipMemcpyAsync(ws + L.lens, len.data(), len.size(), hipMemcpyHostToDevice, stream)) != hipSuccess) return hip_fail(e);

        // ---- step 5 ----
        EmitArgs a;
        a.W = d_W; a.n = (uint32_t)n; a.m = (uint32_t)m; a.ldw = (uint64_t)ldw;
        a.keys = dptr(L.keys); a.slot_sym = dptr(L.slot_sym); a.codes = dptr(L.codes); a.lens = ws + L.lens;
        a.seg_bit0 = dptr(L.seg_bit0); a.seg_pos0 = dptr(L.seg_pos0); a.seg_prev_end = dptr(L.seg_prev_end); a.seg_prev_row1 = dptr(L.seg_prev_row1);
        a.col_bit = reinterpret_cast<const uint32_t*>(blob + d.off_col_bit);
        a.col_pos = reinterpret_cast<const uint32_t*>(blob + d.off_col_pos);
        a.col_chunk = reinterpret_cast<const uint32_t*>(blob + d.off_col_chunk);
        a.stream = reinterpret_cast<uint32_t*>(blob + d.off_stream);
        a.ent = blob + d.off_chunk_ent;
        a.ri = (shac && !rice) ? reinterpret_cast<uint32_t*>(blob + d.off_ri) : nullptr;
        a.rice = rice ? 1u : 0u; a.rice_k = rice_k;
        a.seg_rows = seg_rows;
        a.shac = shac ? 1u : 0u; a.has_zero = has_zero ? 1u : 0u; a.zcode = zcode; a.zlen = zlen;
        a.chunk = Cn; a.ent_bits = d.ent_bits; a.row_bits = d.row_bits; a.ri_bits = ri_bits;
        hipLaunchKernelGGL(enc_emit_kernel, grid, dim3(256), 0, stream, a);
        if ((e = hipGetLastError()) != hipSuccess) return hip_fail(e);
        // the host vectors above feed asynchronous copies: they must outlive them
        if ((e = hipStreamSynchronize(stream)) != hipSuccess) return hip_fail(e);
        return HAC_OK;
    } catch (const std::bad_alloc&) {
        return HAC_ENOMEM;
    }
}
