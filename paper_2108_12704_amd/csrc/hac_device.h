// Decode primitives of libhac's kernels (gfx950): the blob as the device sees it, word sources
// (global memory or a copy staged in LDS), the decode tables in LDS, one codeword, and one lane's
// walk through a chunk of a HAC stream (arXiv 2108.12704 Sect. IV-B), an sHAC stream (Sect. IV-C)
// or an sHAC stream with Rice-coded row gaps.  Included by hac_kernels.hip only.
#ifndef HAC_DEVICE_H
#define HAC_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kWave = 64;
constexpr uint32_t kCodebookLdsMax = 1024;   // symbols whose values are staged in LDS

typedef __attribute__((address_space(3))) const uint32_t lds_cu32;
typedef __attribute__((address_space(3))) const float lds_cf32;

struct DevBlob {
    const float* codebook;
    const uint32_t* canon;      // first_code[33], count[33], first_index[33]
    const uint32_t* symsort;
    const uint32_t* lut;
    const uint32_t* stream;
    const uint32_t* colchunk;   // m + 1
    const uint32_t* colpos;     // m + 1 (sHAC: cb)
    const uint32_t* colbit;     // m + 1
    const void* ent;            // chunk entries
    const uint32_t* ri;         // sHAC
    uint32_t n, m, nnz, k_sym, lmax, lut_bits, has_zero, zero_len, chunk, ri_bits, ent_bits, row_bits, n_chunks;
    uint32_t rice, rice_k;      // sHAC whose row gaps are Rice-coded in front of each value's codeword
};

// (relative bit offset, first row) of chunk g
// request_entry only loads; entry_fields takes the loaded bits apart.  A kernel that has other
// loads to issue calls the two apart, so that no wait sits between its loads.
__device__ __forceinline__ uint2 request_entry(const DevBlob& d, uint32_t g)
{
    uint2 raw = make_uint2(0u, 0u);
    if (d.ent_bits == 32) raw.x = static_cast<const uint32_t*>(d.ent)[g];
    else if (d.ent_bits == 16) raw.x = static_cast<const uint16_t*>(d.ent)[g];
    else raw = static_cast<const uint2*>(d.ent)[g];
    return raw;
}

__device__ __forceinline__ void entry_fields(const DevBlob& d, const uint2& raw, uint32_t& rel, uint32_t& row)
{
    if (d.ent_bits == 32) {
        rel = raw.x >> d.row_bits;                   // sHAC: row_bits = 0
        row = raw.x & ((1u << d.row_bits) - 1u);
    } else if (d.ent_bits == 16) {
        rel = raw.x; row = 0;
    } else {
        row = raw.x; rel = raw.y;
    }
}

__device__ __forceinline__ void load_entry(const DevBlob& d, uint32_t g, uint32_t& rel, uint32_t& row)
{
    entry_fields(d, request_entry(d, g), rel, row);
}

// ---------------------------------------------------------------------------
// word sources: the blob's stream / ri words in global memory, or a copy staged
// in LDS that starts at word `wbase`
// ---------------------------------------------------------------------------
template <bool LDS>
struct WordSrc {
    const uint32_t* w;
    uint32_t wbase;
    __device__ __forceinline__ uint32_t word(uint32_t i) const {
        if (LDS) return ((lds_cu32*)w)[i - wbase];
        return w[i];
    }
    // bits [bp, bp + 32), left-aligned
    __device__ __forceinline__ uint32_t peek32(uint32_t bp) const {
        const uint32_t wi = bp >> 5, off = bp & 31;
        const uint32_t w0 = word(wi), w1 = word(wi + 1);
        return off ? __builtin_amdgcn_alignbit(w0, w1, 32 - off) : w0;
    }
    // a `bits`-wide field (1..32) that starts at bit position bp
    __device__ __forceinline__ uint32_t field(uint64_t bp, uint32_t bits) const {
        const uint32_t wi = (uint32_t)(bp >> 5), off = (uint32_t)(bp & 31);
        const uint32_t w0 = word(wi), w1 = word(wi + 1);
        const uint32_t top = off ? __builtin_amdgcn_alignbit(w0, w1, 32 - off) : w0;
        return top >> (32 - bits);
    }
    // The staged copy only.  Bits [rel, rel + 32) with rel counted from the copy's first word and
    // handed over as rel - 1: the pair of words is then taken one word early when rel is a multiple
    // of 32, the funnel shift (which takes its amount modulo 32) by -rel = ~(rel - 1) is right in
    // every case, and nothing is selected.  At rel == 0 the word in front of the copy is read and
    // not used: every kernel keeps its tables (or other staged words) there.
    __device__ __forceinline__ uint32_t peek32_rm1(int32_t rm1) const {
        static_assert(LDS, "positions relative to the staged copy");
        lds_cu32* sw = (lds_cu32*)w;
        const int32_t q = rm1 >> 5;
        return __builtin_amdgcn_alignbit(sw[q], sw[q + 1], ~(uint32_t)rm1);
    }
    __device__ __forceinline__ uint32_t field_rel(uint32_t rel, uint32_t bits) const {
        return peek32_rm1((int32_t)rel - 1) >> (32 - bits);
    }
};

// Decode tables of one block in LDS.  Layout (uint32 words):
//   lut2[2^lut_bits][2] | canon[99] (+1 pad) | codebook[k4] | symsort[k4]     k4 = k_sym rounded up to 4
// lut2 pairs the blob's first-level entry with the shared value of its symbol, so a short
// codeword costs one 64-bit LDS read.  codebook / symsort sit in LDS only when
// k_sym <= kCodebookLdsMax; otherwise the (rare) long codewords read them from the blob.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) const u32x2 lds_cu2;

struct Tables {
    const uint2* lut2;          // LDS
    const uint32_t* canon;      // LDS
    const float* cb;            // LDS when small, else the blob's copy
    const uint32_t* symsort;    // likewise
    bool small;                 // k_sym <= kCodebookLdsMax (uniform)
};

// Code longer than the first-level table: canonical search by length.
// Returns {(symbol << 6) | length, value bits}.
__device__ __noinline__ uint2 decode_long(const uint32_t* canon_, const uint32_t* symsort, const float* cb, bool small,
                                          uint32_t top, uint32_t lut_bits, uint32_t lmax)
{
    lds_cu32* canon = (lds_cu32*)canon_;
    for (uint32_t l = lut_bits + 1; l <= lmax; ++l) {
        const uint32_t code = top >> (32 - l);
        const uint32_t rel = code - canon[l];
        if (rel < canon[33 + l]) {
            const uint32_t idx = canon[66 + l] + rel;
            const uint32_t sy = small ? ((lds_cu32*)symsort)[idx] : symsort[idx];
            const float v = small ? ((lds_cf32*)cb)[sy] : cb[sy];
            return make_uint2((sy << 6) | l, __float_as_uint(v));
        }
    }
    return make_uint2(lmax ? lmax : 1, 0u);   // unreachable for a validated blob; still makes progress
}

struct Decoded { uint32_t sym, len; float val; };

__device__ __forceinline__ Decoded decode_symbol(const DevBlob& d, const Tables& t, uint32_t top)
{
    const u32x2 raw = ((lds_cu2*)t.lut2)[top >> (32 - d.lut_bits)];
    uint2 e = make_uint2(raw.x, raw.y);
    if ((e.x & 63u) == 0) e = decode_long(t.canon, t.symsort, t.cb, t.small, top, d.lut_bits, d.lmax);
    Decoded r;
    r.len = e.x & 63u; r.sym = e.x >> 6; r.val = __uint_as_float(e.y);
    return r;
}

__device__ __forceinline__ uint32_t table_words_dev(const DevBlob& d)
{
    const uint32_t k4 = (d.k_sym + 3u) & ~3u;
    return ((2u << d.lut_bits) + 100u + (d.k_sym <= kCodebookLdsMax ? 2u * k4 : 0u) + 3u) & ~3u;
}

// All threads of the block copy the tables; the caller synchronises afterwards.
//
// The copy is split in three so that every trip to memory carries as many loads as possible and a
// kernel can put its own loads beside them: request_tables issues everything that depends on
// nothing (first-level entries, canonical table, codebook, symbol order), request_table_values the
// shared values of the first-level entries (they depend on the entries), store_tables writes LDS.
// A loop of load / store pairs would pay one trip per turn and per table instead.  Loads of the
// first kTabTurns turns of every loop are issued from clamped, valid indices on every thread;
// what a small block or a long table leaves over is copied the plain way.
constexpr int kTabTurns = 4;                        // (the asm statement in store_tables names four values)
struct TableRegs { uint32_t e[kTabTurns], v[kTabTurns]; uint32_t canon, cb, sort; };

__device__ __forceinline__ TableRegs request_tables(const DevBlob& d)
{
    TableRegs r;
    const uint32_t nl = 1u << d.lut_bits;
#pragma unroll
    for (int k = 0; k < kTabTurns; ++k) {
        const uint32_t i = threadIdx.x + k * blockDim.x;
        r.e[k] = d.lut[i < nl ? i : nl - 1u];
        r.v[k] = 0u;
    }
    r.canon = d.canon[threadIdx.x < 99u ? threadIdx.x : 98u];
    // no branch around a load: the number of loads in flight is then the same on every path, and a
    // later wait for these can leave younger loads travelling.  Without symbols (an empty address
    // map) the canonical table stands in as a valid address.
    const uint32_t* cbp = d.k_sym ? reinterpret_cast<const uint32_t*>(d.codebook) : d.canon;
    const uint32_t* sop = d.k_sym ? d.symsort : d.canon;
    const uint32_t last = d.k_sym ? d.k_sym - 1u : 0u;
    const uint32_t i = threadIdx.x < last ? threadIdx.x : last;
    r.cb = cbp[i];
    r.sort = sop[i];
    return r;
}

__device__ __forceinline__ void request_table_values(const DevBlob& d, TableRegs& r)
{
    const uint32_t* cbp = d.k_sym ? reinterpret_cast<const uint32_t*>(d.codebook) : d.canon;
#pragma unroll
    for (int k = 0; k < kTabTurns; ++k) r.v[k] = cbp[(r.e[k] & 63u) ? r.e[k] >> 6 : 0u];
}

__device__ __forceinline__ Tables store_tables(const DevBlob& d, uint32_t* smem, TableRegs& r)
{
    const uint32_t nl = 1u << d.lut_bits;
    const uint32_t k4 = (d.k_sym + 3u) & ~3u;
    uint2* s_lut2 = reinterpret_cast<uint2*>(smem);
    uint32_t* s_canon = smem + 2 * nl;
    float* s_cb = reinterpret_cast<float*>(s_canon + 100);
    uint32_t* s_sort = reinterpret_cast<uint32_t*>(s_cb) + k4;
    // The values pass through an empty asm statement first: their loads then stay where they were
    // issued (the compiler would otherwise move a load down beside the guarded store that uses it,
    // behind every load issued since).
    static_assert(kTabTurns == 4, "the asm statement below names four values");
    asm volatile("" : "+v"(r.v[0]), "+v"(r.v[1]), "+v"(r.v[2]), "+v"(r.v[3]));
#pragma unroll
    for (int k = 0; k < kTabTurns; ++k) {
        const uint32_t i = threadIdx.x + k * blockDim.x;
        if (i < nl) s_lut2[i] = make_uint2(r.e[k], (r.e[k] & 63u) ? r.v[k] : 0u);
    }
    for (uint32_t i = threadIdx.x + kTabTurns * blockDim.x; i < nl; i += blockDim.x) {
        const uint32_t e = d.lut[i];
        s_lut2[i] = make_uint2(e, (e & 63u) ? __float_as_uint(d.codebook[e >> 6]) : 0u);
    }
    if (threadIdx.x < 99u) s_canon[threadIdx.x] = r.canon;
    for (uint32_t i = threadIdx.x + blockDim.x; i < 99u; i += blockDim.x) s_canon[i] = d.canon[i];
    Tables t;
    t.lut2 = s_lut2; t.canon = s_canon; t.small = d.k_sym <= kCodebookLdsMax;
    if (t.small) {
        if (threadIdx.x < d.k_sym) { s_cb[threadIdx.x] = __uint_as_float(r.cb); s_sort[threadIdx.x] = r.sort; }
        for (uint32_t i = threadIdx.x + blockDim.x; i < d.k_sym; i += blockDim.x) { s_cb[i] = d.codebook[i]; s_sort[i] = d.symsort[i]; }
        t.cb = s_cb; t.symsort = s_sort;
    } else {
        t.cb = d.codebook; t.symsort = d.symsort;
    }
    return t;
}

__device__ __forceinline__ Tables load_tables(const DevBlob& d, uint32_t* smem)
{
    TableRegs r = request_tables(d);
    request_table_values(d, r);
    return store_tables(d, smem, r);
}

// ---------------------------------------------------------------------------
// one lane's progress through one chunk
// ---------------------------------------------------------------------------
struct ChunkState {
    uint32_t bp;      // next stream bit
    uint32_t row;     // HAC: row of the next symbol
    uint32_t wpos;    // CSC position of the next non-zero this lane will emit
    uint32_t wend;    // one past the chunk's last non-zero
};

// HAC: emit non-zeros until wpos reaches `limit` (<= wend).  Zeros only move `row`.
// When the zero symbol's codeword is the single bit 0, a run of zeros is a run of
// 0 bits and is skipped with a count-leading-zeros.
template <class Src, class Emit>
__device__ __forceinline__ void hac_advance(const DevBlob& d, const Tables& tb, const Src& src,
                                            ChunkState& st, uint32_t limit, Emit emit)
{
    const bool zfast = d.zero_len == 1;
    while (st.wpos < limit) {
        uint32_t top = src.peek32(st.bp);
        if (zfast) {
            if (top == 0) {                                            // a non-zero follows, so the run ends
                st.bp += 32; st.row += 32;
                st.wpos = st.row > d.n ? limit : st.wpos;              // ... unless the stream is damaged: end the walk
                continue;
            }
            const uint32_t z = (uint32_t)__builtin_clz(top);
            if (z) {
                st.bp += z; st.row += z;
                top = z + d.lmax <= 32 ? top << z : src.peek32(st.bp);
            }
        }
        const Decoded q = decode_symbol(d, tb, top);
        st.bp += q.len;
        if (d.has_zero && q.sym == 0) {
            st.row++;
            st.wpos = st.row > d.n ? limit : st.wpos;                  // a damaged stream: end the walk
            continue;
        }
        emit(st.wpos, st.row, q.sym, q.val);
        st.row++; st.wpos++;
    }
}

// HAC, zero symbol = the single bit 0, words staged in LDS.  One pass of the loop per
// non-zero: 128 stream bits are fetched at once, a count-leading-zeros over the first
// 64 skips the zero run, and the codeword is taken from the same fetch.  Only a run
// of 64 or more zeros takes an extra pass (which steps over 96 bits when they are all zero:
// the lanes of a wave walk independently, and the wave runs as long as its slowest lane).
// The position is kept relative to the staged copy, less one (see WordSrc::peek32_rm1): three
// funnel shifts give the 96 bits, no 64-bit shift and no select on the bit offset.
__device__ __forceinline__ uint32_t leading_zeros_raw(uint32_t x)        // 0xffffffff for x == 0, as the instruction counts
{
    uint32_t r;
    asm("v_ffbh_u32 %0, %1" : "=v"(r) : "v"(x));
    return r;
}

template <class Emit>
__device__ __forceinline__ void hac_advance_zrun(const DevBlob& d, const Tables& tb, const WordSrc<true>& src,
                                                 ChunkState& st, uint32_t limit, Emit emit)
{
    lds_cu32* sw = (lds_cu32*)src.w;
    int32_t rm1 = (int32_t)(st.bp - (src.wbase << 5)) - 1;
    while (st.wpos < limit) {
        const int32_t q = rm1 >> 5;
        const uint32_t s = ~(uint32_t)rm1;
        const uint32_t w0 = sw[q], w1 = sw[q + 1], w2 = sw[q + 2], w3 = sw[q + 3];
        const uint32_t hi = __builtin_amdgcn_alignbit(w0, w1, s);
        const uint32_t mid = __builtin_amdgcn_alignbit(w1, w2, s);
        const uint32_t lo = __builtin_amdgcn_alignbit(w2, w3, s);
        if ((hi | mid) == 0) {                                             // a non-zero follows, so the run ends
            const uint32_t skip = lo ? 64u : 96u;                          // all 96 fetched bits may be zeros
            rm1 += (int32_t)skip; st.row += skip;
            st.wpos = st.row > d.n ? limit : st.wpos;                      // ... unless the stream is damaged: end the walk
            continue;
        }
        // hi == 0 counts as 0xffffffff and loses against 32 + (zeros of mid); mid == 0 with hi != 0 wraps to
        // 31, which is never below the zeros of hi
        const uint32_t zh = leading_zeros_raw(hi), zm = leading_zeros_raw(mid) + 32u;
        const uint32_t z = zh < zm ? zh : zm;
        const uint32_t x0 = z < 32u ? hi : mid, x1 = z < 32u ? mid : lo;
        const uint32_t zz = z & 31u;
        const uint32_t top = (x0 << zz) | ((x1 >> 1) >> (zz ^ 31u));
        const Decoded sy = decode_symbol(d, tb, top);
        st.row += z;
        rm1 += (int32_t)(z + sy.len);
        emit(st.wpos, st.row, sy.sym, sy.val);
        st.row++; st.wpos++;
    }
    st.bp = (uint32_t)(rm1 + 1) + (src.wbase << 5);
}

// sHAC: every symbol is a non-zero.
template <class Src, class Emit>
__device__ __forceinline__ void shac_advance(const DevBlob& d, const Tables& tb, const Src& src,
                                             ChunkState& st, uint32_t limit, Emit emit)
{
    while (st.wpos < limit) {
        const Decoded q = decode_symbol(d, tb, src.peek32(st.bp));
        st.bp += q.len;
        emit(st.wpos, 0u, q.sym, q.val);
        st.wpos++;
    }
}

// The same over the staged copy: one funnel shift per codeword.
template <class Emit>
__device__ __forceinline__ void shac_advance(const DevBlob& d, const Tables& tb, const WordSrc<true>& src,
                                             ChunkState& st, uint32_t limit, Emit emit)
{
    int32_t rm1 = (int32_t)(st.bp - (src.wbase << 5)) - 1;
    while (st.wpos < limit) {
        const Decoded sy = decode_symbol(d, tb, src.peek32_rm1(rm1));
        rm1 += (int32_t)sy.len;
        emit(st.wpos, 0u, sy.sym, sy.val);
        st.wpos++;
    }
    st.bp = (uint32_t)(rm1 + 1) + (src.wbase << 5);
}

// sHAC with Rice-coded row gaps: gap codeword, then the value's codeword.  Gap d with
// q = d >> k: q zeros, a one, k low bits of d; from q = 31 on: 31 zeros, a one, d in 32 bits.
// st.row is the row the next gap counts from.  Words staged in LDS: one fetch of 128 bits
// serves the unary part (count-leading-zeros), the remainder and the value's codeword.
template <class Emit>
__device__ __forceinline__ void gap_advance(const DevBlob& d, const Tables& tb, const WordSrc<true>& src,
                                            ChunkState& st, uint32_t limit, Emit emit)
{
    lds_cu32* sw = (lds_cu32*)src.w;
    const uint32_t k = d.rice_k;
    while (st.wpos < limit) {
        const uint32_t wi = (st.bp >> 5) - src.wbase, off = st.bp & 31;
        const uint32_t w0 = sw[wi], w1 = sw[wi + 1], w2 = sw[wi + 2], w3 = sw[wi + 3];
        const uint32_t hi = (uint32_t)(((((uint64_t)w0 << 32) | w1) << off) >> 32);
        const uint32_t mid = (uint32_t)(((((uint64_t)w1 << 32) | w2) << off) >> 32);
        const uint32_t lo = (uint32_t)(((((uint64_t)w2 << 32) | w3) << off) >> 32);
        const uint32_t z = hi ? (uint32_t)__builtin_clz(hi) : 31u;        // a valid stream has a one within 32 bits
        const uint32_t s1 = z + 1;                                        // 1..32
        const uint32_t p0 = (uint32_t)(((((uint64_t)hi << 32) | mid) << s1) >> 32);
        const uint32_t p1 = (uint32_t)(((((uint64_t)mid << 32) | lo) << s1) >> 32);
        uint32_t gapv, top, used;
        if (z < 31) {
            const uint64_t w = (((uint64_t)p0 << 32) | p1) << k;          // k <= 15
            gapv = (z << k) | (uint32_t)(((uint64_t)p0 << k) >> 32);
            top = (uint32_t)(w >> 32);
            used = s1 + k;
        } else {
            gapv = p0; top = p1; used = s1 + 32;
        }
        const Decoded q = decode_symbol(d, tb, top);
        const uint32_t row = st.row + gapv;
        st.bp += used + q.len;
        st.row = row + 1;
        emit(st.wpos, row, q.sym, q.val);
        st.wpos++;
    }
}

// The same from any word source, one field at a time (streams too long to stage, and the
// test-only decode kernel).
template <class Src, class Emit>
__device__ __forceinline__ void gap_advance_slow(const DevBlob& d, const Tables& tb, const Src& src,
                                                 ChunkState& st, uint32_t limit, Emit emit)
{
    const uint32_t k = d.rice_k;
    while (st.wpos < limit) {
        const uint32_t hi = src.peek32(st.bp);
        const uint32_t z = hi ? (uint32_t)__builtin_clz(hi) : 31u;
        st.bp += z + 1;
        uint32_t gapv;
        if (z < 31) {
            gapv = (z << k) | (k ? src.peek32(st.bp) >> (32 - k) : 0u);
            st.bp += k;
        } else {
            gapv = src.peek32(st.bp);
            st.bp += 32;
        }
        const Decoded q = decode_symbol(d, tb, src.peek32(st.bp));
        st.bp += q.len;
        const uint32_t row = st.row + gapv;
        st.row = row + 1;
        emit(st.wpos, row, q.sym, q.val);
        st.wpos++;
    }
}

// column that owns chunk g: largest j with colchunk[j] <= g (global memory search)
__device__ __forceinline__ uint32_t column_of_chunk(const DevBlob& d, uint32_t g)
{
    uint32_t lo = 0, hi = d.m;               // invariant: colchunk[lo] <= g < colchunk[hi]
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (d.colchunk[mid] <= g) lo = mid; else hi = mid;
    }
    return lo;
}

} // namespace

#endif
