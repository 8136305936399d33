// Device side of libhac for gfx950 (MI355X): decode-and-accumulate kernels for
// HAC (arXiv 2108.12704 Sect. IV-B, Algorithm 1) and sHAC (Sect. IV-C,
// Algorithm 2) blobs, Y = X.W for a batch (Algorithm 3's result, with the
// stream decoded once per launch instead of once per row of X).
//
// Work split.  The stream is serial by nature; the chunk index stored beside
// it gives every chunk (HAC: `chunk` rows of one column; sHAC: `chunk`
// non-zeros of one column) its starting bit, so one lane decodes one chunk.
// A wavefront owns a few whole columns of W:
//   decode phase: its 64 lanes decode the columns' chunks side by side and
//                 leave (row, value) pairs, in CSC order, in a per-wave LDS list;
//   FMA phase   : the lanes turn into batch lanes: the wave walks the list
//                 and lane b accumulates x[b][row] * value from the
//                 feature-major copy of X (one coalesced row segment per
//                 non-zero).  A column's sum is complete inside one wave, so
//                 Y is written once, without atomics, in a fixed order.
// B = 1 skips the list: every lane multiplies as it decodes, x sits in LDS,
// and a fixed-shape butterfly adds the lanes of a column.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/hac.h"

namespace {

constexpr int kWave = 64;
constexpr uint32_t kCodebookLdsMax = 1024;   // symbols whose values are staged in LDS

struct DevBlob {
    const float* codebook;
    const uint32_t* canon;      // first_code[33], count[33], first_index[33]
    const uint32_t* symsort;
    const uint32_t* lut;
    const uint32_t* stream;
    const uint32_t* cbit;
    const uint32_t* cpos;       // HAC
    const uint32_t* colchunk;   // sHAC
    const uint32_t* cb;         // sHAC
    const uint32_t* ri;         // sHAC
    uint32_t n, m, nnz, k_sym, lmax, lut_bits, has_zero, zero_len, chunk, ri_bits, cpc, n_chunks;
};

// ---------------------------------------------------------------------------
// bit reader: a 96-bit sliding register window over an MSB-first uint32 stream
// ---------------------------------------------------------------------------
struct BitReader {
    const uint32_t* w;
    uint32_t widx;
    uint32_t a, b, c;

    __device__ __forceinline__ void seek(const uint32_t* words, uint32_t bp) {
        w = words;
        widx = bp >> 5;
        a = w[widx]; b = w[widx + 1]; c = w[widx + 2];
    }
    // bits [bp, bp + 64) left-aligned; bp never moves backwards
    __device__ __forceinline__ uint64_t window(uint32_t bp) {
        const uint32_t wi = bp >> 5;
        if (wi != widx) {
            if (wi == widx + 1) { a = b; b = c; c = w[wi + 2]; }
            else { a = w[wi]; b = w[wi + 1]; c = w[wi + 2]; }
            widx = wi;
        }
        const uint32_t off = bp & 31;
        const uint64_t hi = ((uint64_t)a << 32) | b;
        return off ? ((hi << off) | (uint64_t)(c >> (32 - off))) : hi;
    }
};

// Code longer than the first-level table: canonical search by length.
__device__ __noinline__ uint32_t decode_long(const DevBlob& d, uint32_t top, uint32_t& len)
{
    for (uint32_t l = d.lut_bits + 1; l <= d.lmax; ++l) {
        const uint32_t code = top >> (32 - l);
        const uint32_t rel = code - d.canon[l];
        if (rel < d.canon[33 + l]) { len = l; return d.symsort[d.canon[66 + l] + rel]; }
    }
    len = d.lmax ? d.lmax : 1;      // unreachable for a validated blob; still makes progress
    return 0;
}

__device__ __forceinline__ uint32_t decode_symbol(const DevBlob& d, const uint32_t* s_lut,
                                                  uint32_t top, uint32_t& len)
{
    const uint32_t e = s_lut[top >> (32 - d.lut_bits)];
    len = e & 63u;
    if (len) return e >> 6;
    return decode_long(d, top, len);
}

__device__ __forceinline__ uint32_t ri_field(const uint32_t* ri, uint32_t p, uint32_t bits)
{
    const uint64_t bp = (uint64_t)p * bits;
    const uint32_t wi = (uint32_t)(bp >> 5), off = (uint32_t)(bp & 31);
    const uint64_t two = ((uint64_t)ri[wi] << 32) | ri[wi + 1];
    return (uint32_t)((two << off) >> (64 - bits));
}

// ---------------------------------------------------------------------------
// one lane's progress through one chunk
// ---------------------------------------------------------------------------
struct ChunkState {
    BitReader rd;
    uint32_t bp;      // next stream bit
    uint32_t row;     // HAC: row of the next symbol
    uint32_t wpos;    // CSC position of the next non-zero this lane will emit
    uint32_t wend;    // one past the chunk's last non-zero
};

// HAC: emit non-zeros until wpos reaches `limit` (<= wend).  Zeros only move `row`.
template <class Emit>
__device__ __forceinline__ void hac_advance(const DevBlob& d, const uint32_t* s_lut,
                                            ChunkState& st, uint32_t limit, Emit emit)
{
    const bool zfast = d.zero_len == 1;
    while (st.wpos < limit) {
        uint64_t win = st.rd.window(st.bp);
        if (zfast) {
            const uint32_t z = win ? (uint32_t)__builtin_clzll(win) : 64u;   // a non-zero follows, so the run ends
            st.bp += z; st.row += z;
            if (z > 32) continue;                     // fewer than 32 valid bits left in the window
            win <<= z;
        }
        uint32_t len;
        const uint32_t s = decode_symbol(d, s_lut, (uint32_t)(win >> 32), len);
        st.bp += len;
        if (d.has_zero && s == 0) { st.row++; continue; }
        emit(st.wpos, st.row, s);
        st.row++; st.wpos++;
    }
}

// sHAC: every symbol is a non-zero; the row comes from the packed ri fields.
template <class Emit>
__device__ __forceinline__ void shac_advance(const DevBlob& d, const uint32_t* s_lut,
                                             ChunkState& st, uint32_t limit, Emit emit)
{
    while (st.wpos < limit) {
        const uint64_t win = st.rd.window(st.bp);
        uint32_t len;
        const uint32_t s = decode_symbol(d, s_lut, (uint32_t)(win >> 32), len);
        st.bp += len;
        emit(st.wpos, ri_field(d.ri, st.wpos, d.ri_bits), s);
        st.wpos++;
    }
}

__device__ __forceinline__ void hac_open(const DevBlob& d, uint32_t g, ChunkState& st)
{
    st.bp = d.cbit[g];
    st.row = (g % d.cpc) * d.chunk;
    st.wpos = d.cpos[g];
    st.wend = d.cpos[g + 1];
    if (st.wpos < st.wend) st.rd.seek(d.stream, st.bp);
}

// column that owns sHAC chunk g, searched in [c0, c1)
__device__ __forceinline__ uint32_t shac_col_of(const DevBlob& d, uint32_t g, uint32_t c0, uint32_t c1)
{
    uint32_t lo = c0, hi = c1;              // invariant: colchunk[lo] <= g < colchunk[hi]
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (d.colchunk[mid] <= g) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ void shac_open(const DevBlob& d, uint32_t g, uint32_t col, ChunkState& st)
{
    st.bp = d.cbit[g];
    st.row = 0;
    st.wpos = d.cb[col] + (g - d.colchunk[col]) * d.chunk;
    const uint32_t cend = d.cb[col + 1];
    st.wend = st.wpos + d.chunk < cend ? st.wpos + d.chunk : cend;
    st.rd.seek(d.stream, st.bp);
}

__device__ __forceinline__ void load_tables(const DevBlob& d, uint32_t* s_lut, float* s_cb)
{
    const uint32_t nl = 1u << d.lut_bits;
    for (uint32_t i = threadIdx.x; i < nl; i += blockDim.x) s_lut[i] = d.lut[i];
    if (d.k_sym <= kCodebookLdsMax)
        for (uint32_t i = threadIdx.x; i < d.k_sym; i += blockDim.x) s_cb[i] = d.codebook[i];
}

__device__ __forceinline__ float value_of(const DevBlob& d, const float* s_cb, uint32_t s)
{
    return d.k_sym <= kCodebookLdsMax ? s_cb[s] : d.codebook[s];
}

// XCD-aware block order: hardware deals consecutive block ids round-robin to the
// 8 XCDs; this gives every XCD (hence every L2) one contiguous range of columns.
__device__ __forceinline__ uint32_t logical_block(uint32_t nblocks_padded)
{
    const uint32_t per = nblocks_padded >> 3;
    return (blockIdx.x & 7u) * per + (blockIdx.x >> 3);
}

// ---------------------------------------------------------------------------
// TEST-ONLY decode kernels
// ---------------------------------------------------------------------------
__global__ void fill_u32_kernel(uint32_t* p, uint64_t count, uint32_t v)
{
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) p[i] = v;
}

__global__ void __launch_bounds__(256)
hac_decode_kernel(DevBlob d, float* W, int32_t* sym)
{
    extern __shared__ uint32_t smem[];
    uint32_t* s_lut = smem;
    float* s_cb = reinterpret_cast<float*>(smem + (1u << d.lut_bits));
    load_tables(d, s_lut, s_cb);
    __syncthreads();
    const uint32_t g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= d.n_chunks) return;
    const uint32_t col = g / d.cpc;
    ChunkState st;
    hac_open(d, g, st);
    hac_advance(d, s_lut, st, st.wend, [&](uint32_t, uint32_t row, uint32_t s) {
        if (sym) sym[(uint64_t)col * d.n + row] = (int32_t)s;
        if (W) W[(uint64_t)row * d.m + col] = value_of(d, s_cb, s);
    });
}

__global__ void __launch_bounds__(256)
shac_decode_kernel(DevBlob d, float* nz, int32_t* sym, int32_t* row_out, int32_t* col_out)
{
    extern __shared__ uint32_t smem[];
    uint32_t* s_lut = smem;
    float* s_cb = reinterpret_cast<float*>(smem + (1u << d.lut_bits));
    load_tables(d, s_lut, s_cb);
    __syncthreads();
    const uint32_t g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= d.n_chunks) return;
    const uint32_t col = shac_col_of(d, g, 0, d.m);
    ChunkState st;
    shac_open(d, g, col, st);
    shac_advance(d, s_lut, st, st.wend, [&](uint32_t p, uint32_t row, uint32_t s) {
        if (sym) sym[p] = (int32_t)s;
        if (nz) nz[p] = value_of(d, s_cb, s);
        if (row_out) row_out[p] = (int32_t)row;
        if (col_out) col_out[p] = (int32_t)col;
    });
}

// ---------------------------------------------------------------------------
// X (B x n, row-major) -> XT (n x Bp, feature-major), zero padded for b >= B
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
transpose_pad_kernel(const float* __restrict__ X, uint32_t B, uint32_t n, uint64_t ldx,
                     float* __restrict__ XT, uint32_t Bp)
{
    __shared__ float tile[32][33];
    const uint32_t tx = threadIdx.x & 31, ty = threadIdx.x >> 5;       // 32 x 8
    const uint32_t r0 = blockIdx.x * 32, b0 = blockIdx.y * 32;
    for (uint32_t k = 0; k < 32; k += 8) {
        const uint32_t b = b0 + ty + k, r = r0 + tx;
        tile[ty + k][tx] = (b < B && r < n) ? X[(uint64_t)b * ldx + r] : 0.0f;
    }
    __syncthreads();
    for (uint32_t k = 0; k < 32; k += 8) {
        const uint32_t r = r0 + ty + k, b = b0 + tx;
        if (r < n && b < Bp) XT[(uint64_t)r * Bp + b] = tile[tx][ty + k];
    }
}

// ---------------------------------------------------------------------------
// B = 1: every lane multiplies as it decodes
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

template <bool SHAC, bool X_LDS>
__global__ void __launch_bounds__(1024)
dot_b1_kernel(DevBlob d, const float* __restrict__ x, float* __restrict__ y,
              uint32_t cpw, uint32_t nblocks)
{
    extern __shared__ uint32_t smem[];
    uint32_t* s_lut = smem;
    float* s_cb = reinterpret_cast<float*>(smem + (1u << d.lut_bits));
    float* s_x = s_cb + (d.k_sym <= kCodebookLdsMax ? ((d.k_sym + 3u) & ~3u) : 0u);
    load_tables(d, s_lut, s_cb);
    if (X_LDS)
        for (uint32_t i = threadIdx.x; i < d.n; i += blockDim.x) s_x[i] = x[i];
    __syncthreads();
    const uint32_t lb = logical_block(gridDim.x);
    if (lb >= nblocks) return;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = lb * (blockDim.x / kWave) + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t c0 = wave * cpw;
    if (c0 >= d.m) return;
    const uint32_t c1 = c0 + cpw < d.m ? c0 + cpw : d.m;
    const uint32_t g0 = SHAC ? d.colchunk[c0] : c0 * d.cpc;
    const uint32_t g1 = SHAC ? d.colchunk[c1] : c1 * d.cpc;
    float colsum = 0.0f;                                    // lane l keeps the sum of column c0 + l
    for (uint32_t gb = g0; gb < g1; gb += kWave) {
        const uint32_t g = gb + lane;
        float part = 0.0f;
        uint32_t col = 0xffffffffu;
        if (g < g1) {
            ChunkState st;
            if (SHAC) { col = shac_col_of(d, g, c0, c1); shac_open(d, g, col, st); }
            else { col = g / d.cpc; hac_open(d, g, st); }
            auto emit = [&](uint32_t, uint32_t row, uint32_t s) {
                const float xv = X_LDS ? s_x[row] : x[row];
                part = fmaf(xv, value_of(d, s_cb, s), part);
            };
            if (SHAC) shac_advance(d, s_lut, st, st.wend, emit);
            else hac_advance(d, s_lut, st, st.wend, emit);
        }
        // chunk ids ascend with the lane, so the columns present form a range
        const uint32_t last = (g1 - gb < (uint32_t)kWave ? g1 - gb : (uint32_t)kWave) - 1;
        const uint32_t cmin = __shfl(col, 0, kWave), cmax = __shfl(col, (int)last, kWave);
        for (uint32_t cc = cmin; cc <= cmax; ++cc) {
            const float r = wave_sum(col == cc ? part : 0.0f);
            if (lane == cc - c0) colsum += r;
        }
    }
    if (lane < c1 - c0) y[c0 + lane] = colsum;
}

// ---------------------------------------------------------------------------
// batch kernel: decode into a per-wave LDS list, then batch lanes accumulate
// ---------------------------------------------------------------------------
template <int NB> struct VecLoad;
template <> struct VecLoad<1> { static __device__ __forceinline__ void ld(const float* p, float* v) { v[0] = *p; } };
template <> struct VecLoad<2> { static __device__ __forceinline__ void ld(const float* p, float* v) { const float2 t = *reinterpret_cast<const float2*>(p); v[0] = t.x; v[1] = t.y; } };
template <> struct VecLoad<4> { static __device__ __forceinline__ void ld(const float* p, float* v) { const float4 t = *reinterpret_cast<const float4*>(p); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; } };

// gw: lanes per group (power of two, gw * NB = batch columns handled per pass);
// 64 / gw groups walk the list interleaved and are added together at a column's end.
template <bool SHAC, int NB>
__global__ void __launch_bounds__(256)
dot_batch_kernel(DevBlob d, const float* __restrict__ XT, uint32_t Bp, uint32_t B,
                 float* __restrict__ Y, uint64_t ldy, uint32_t cpw, uint32_t gw,
                 uint32_t list_cap, uint32_t nblocks)
{
    extern __shared__ uint32_t smem[];
    uint32_t* s_lut = smem;
    float* s_cb = reinterpret_cast<float*>(smem + (1u << d.lut_bits));
    uint2* s_lists = reinterpret_cast<uint2*>(s_cb + (d.k_sym <= kCodebookLdsMax ? ((d.k_sym + 3u) & ~3u) : 0u));
    load_tables(d, s_lut, s_cb);
    __syncthreads();
    const uint32_t lb = logical_block(gridDim.x);
    if (lb >= nblocks) return;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wib = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    uint2* list = s_lists + (uint64_t)wib * list_cap;
    const uint32_t wave = lb * (blockDim.x / kWave) + wib;
    const uint32_t c0 = wave * cpw;
    if (c0 >= d.m) return;
    const uint32_t c1 = c0 + cpw < d.m ? c0 + cpw : d.m;
    const uint32_t g1 = SHAC ? d.colchunk[c1] : c1 * d.cpc;
    const uint32_t posbase = SHAC ? d.cb[c0] : d.cpos[c0 * d.cpc];
    const uint32_t posend = SHAC ? d.cb[c1] : d.cpos[c1 * d.cpc];

    const uint32_t ng = kWave / gw;                 // groups
    const uint32_t grp = lane / gw, lig = lane % gw;
    const uint32_t boff = blockIdx.y * 256u + lig * NB;   // first batch column of this lane
    const float* xt = XT + boff;

    // decode state of this lane
    uint32_t g = (SHAC ? d.colchunk[c0] : c0 * d.cpc) + lane;
    bool have = false;
    ChunkState st;
    auto open_next = [&]() {
        have = false;
        while (g < g1) {
            if (SHAC) shac_open(d, g, shac_col_of(d, g, c0, c1), st); else hac_open(d, g, st);
            if (st.wpos < st.wend) { have = true; return; }
            g += kWave;                              // chunk without non-zeros
        }
    };
    open_next();

    float acc[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) acc[i] = 0.0f;
    uint32_t cc = c0;                                // column being accumulated (wave-uniform)

    auto flush = [&]() {
        // add the groups together in a fixed order, then group 0 stores Y[b][cc]
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            float v = acc[i];
            for (uint32_t off = 32; off >= gw; off >>= 1) v += __shfl_xor(v, (int)off, kWave);
            const uint32_t b = boff + i;
            if (grp == 0 && b < B) Y[(uint64_t)b * ldy + cc] = v;
            acc[i] = 0.0f;
        }
    };

    for (uint32_t winbase = posbase; winbase < posend; winbase += list_cap) {
        const uint32_t winend = winbase + list_cap < posend ? winbase + list_cap : posend;
        // ---- decode phase ----
        while (have) {
            const uint32_t lim = st.wend < winend ? st.wend : winend;
            auto emit = [&](uint32_t p, uint32_t row, uint32_t s) {
                list[p - winbase] = make_uint2(row, __float_as_uint(value_of(d, s_cb, s)));
            };
            if (SHAC) shac_advance(d, s_lut, st, lim, emit); else hac_advance(d, s_lut, st, lim, emit);
            if (st.wpos == st.wend) { g += kWave; open_next(); }
            else break;                              // the window is full for this lane
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // ---- FMA phase ----
        uint32_t t = winbase;
        while (cc < c1) {
            const uint32_t pe = SHAC ? d.cb[cc + 1] : d.cpos[(cc + 1) * d.cpc];
            const uint32_t hi = pe < winend ? pe : winend;
#pragma unroll 4
            for (uint32_t u = t + grp; u < hi; u += ng) {
                const uint2 e = list[u - winbase];
                float xv[NB];
                VecLoad<NB>::ld(xt + (uint64_t)e.x * Bp, xv);
                const float wv = __uint_as_float(e.y);
#pragma unroll
                for (int i = 0; i < NB; ++i) acc[i] = fmaf(xv[i], wv, acc[i]);
            }
            t = hi;
            if (pe <= winend) { flush(); ++cc; }
            else break;                              // column continues in the next window
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    while (cc < c1) { flush(); ++cc; }               // trailing columns without non-zeros
}

// ---------------------------------------------------------------------------
// host-side launch helpers
// ---------------------------------------------------------------------------
thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) { g_last_hip_error = (int)e; return HAC_EHIP; }

int make_dev(const hac_desc_t* desc, const void* d_blob, uint32_t format, DevBlob& d)
{
    if (!desc || !d_blob) return HAC_EINVAL;
    if (desc->magic != 0x31434148u || desc->version != 1 || desc->format != format) return HAC_EINVAL;
    if (reinterpret_cast<uintptr_t>(d_blob) % 256) return HAC_EINVAL;
    if (desc->lut_bits < 1 || desc->lut_bits > 12 || desc->lmax > 32) return HAC_EINVAL;
    if (desc->n > 0x7fffffffull || desc->m > 0x7fffffffull || desc->nnz > 0xfffffff0ull ||
        desc->n_chunks > 0xfffffff0ull) return HAC_EINVAL;
    const uint8_t* b = static_cast<const uint8_t*>(d_blob);
    d.codebook = reinterpret_cast<const float*>(b + desc->off_codebook);
    d.canon = reinterpret_cast<const uint32_t*>(b + desc->off_canon);
    d.symsort = reinterpret_cast<const uint32_t*>(b + desc->off_symsort);
    d.lut = reinterpret_cast<const uint32_t*>(b + desc->off_lut);
    d.stream = reinterpret_cast<const uint32_t*>(b + desc->off_stream);
    d.cbit = reinterpret_cast<const uint32_t*>(b + desc->off_chunk_bit);
    d.cpos = format == HAC_FORMAT_HAC ? reinterpret_cast<const uint32_t*>(b + desc->off_chunk_pos) : nullptr;
    d.colchunk = format == HAC_FORMAT_SHAC ? reinterpret_cast<const uint32_t*>(b + desc->off_col_chunk) : nullptr;
    d.cb = format == HAC_FORMAT_SHAC ? reinterpret_cast<const uint32_t*>(b + desc->off_cb) : nullptr;
    d.ri = format == HAC_FORMAT_SHAC ? reinterpret_cast<const uint32_t*>(b + desc->off_ri) : nullptr;
    d.n = (uint32_t)desc->n; d.m = (uint32_t)desc->m; d.nnz = (uint32_t)desc->nnz;
    d.k_sym = desc->k_sym; d.lmax = desc->lmax; d.lut_bits = desc->lut_bits;
    d.has_zero = desc->has_zero; d.zero_len = desc->zero_len; d.chunk = desc->chunk;
    d.ri_bits = desc->ri_bits; d.cpc = desc->chunks_per_col; d.n_chunks = (uint32_t)desc->n_chunks;
    return HAC_OK;
}

uint32_t table_words(const DevBlob& d)
{
    return (1u << d.lut_bits) + (d.k_sym <= kCodebookLdsMax ? ((d.k_sym + 3u) & ~3u) : 0u);
}

struct BatchShape { uint32_t gw, nb, Bp, tiles; };

BatchShape batch_shape(int64_t B)
{
    BatchShape s;
    if (B <= 64) { uint32_t g = 1; while (g < (uint32_t)B) g <<= 1; s.gw = g; s.nb = 1; s.Bp = g; s.tiles = 1; }
    else if (B <= 128) { s.gw = 64; s.nb = 2; s.Bp = 128; s.tiles = 1; }
    else { s.gw = 64; s.nb = 4; s.Bp = (uint32_t)((B + 255) / 256 * 256); s.tiles = s.Bp / 256; }
    return s;
}

constexpr size_t kLdsLimit = 160 * 1024;

uint32_t default_cpw(const hac_desc_t* desc)
{
    const double chunks_per_col = (double)desc->n_chunks / (double)desc->m;
    uint32_t cpw = 1;
    if (chunks_per_col < 64.0) cpw = (uint32_t)(64.0 / (chunks_per_col > 1.0 ? chunks_per_col : 1.0));
    if (cpw < 1) cpw = 1;
    if (cpw > 16) cpw = 16;
    while (cpw > 1 && desc->m / cpw < 2048) cpw >>= 1;       // keep enough wavefronts in flight
    return cpw;
}

int dot_impl(uint32_t format, const hac_desc_t* desc, const void* d_blob,
             const float* d_X, int64_t B, int64_t ldx, float* d_Y, int64_t ldy,
             void* d_ws, size_t ws_bytes, const hac_launch_t* launch, hac_stream_t stream_)
{
    DevBlob d;
    int rc = make_dev(desc, d_blob, format, d);
    if (rc) return rc;
    if (B < 0 || B > 0x7fffffffll) return HAC_EINVAL;
    if (B == 0) return HAC_OK;
    if (!d_X || !d_Y || ldx < (int64_t)desc->n || ldy < (int64_t)desc->m) return HAC_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    uint32_t cpw = default_cpw(desc), wpb = 0, list_cap = 1024, variant = 0;
    if (launch) {
        if (launch->cols_per_wave > 64 || launch->waves_per_block > 16) return HAC_EINVAL;
        if (launch->cols_per_wave) cpw = launch->cols_per_wave;
        wpb = launch->waves_per_block;
        variant = launch->variant;
        if (launch->reserved[0]) list_cap = launch->reserved[0];
        if (list_cap < 64 || list_cap > 4096) return HAC_EINVAL;
    }
    const uint32_t nwaves = (d.m + cpw - 1) / cpw;
    const bool shac = format == HAC_FORMAT_SHAC;
    g_last_hip_error = 0;

    if (B == 1 && variant != 2) {
        if (!wpb) wpb = 16;
        const size_t base = 4ull * table_words(d);
        const bool x_lds = base + 4ull * d.n <= kLdsLimit - 1024 && variant != 1;
        const size_t lds = base + (x_lds ? 4ull * d.n : 0);
        const uint32_t nblocks = (nwaves + wpb - 1) / wpb;
        const uint32_t grid = (nblocks + 7) / 8 * 8;
        void (*k)(DevBlob, const float*, float*, uint32_t, uint32_t) =
            shac ? (x_lds ? dot_b1_kernel<true, true> : dot_b1_kernel<true, false>)
                 : (x_lds ? dot_b1_kernel<false, true> : dot_b1_kernel<false, false>);
        if (lds > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return hip_fail(e);
        }
        hipLaunchKernelGGL(k, dim3(grid), dim3(wpb * kWave), lds, stream, d, d_X, d_Y, cpw, nblocks);
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? HAC_OK : hip_fail(e);
    }

    const BatchShape bs = batch_shape(B);
    const size_t need = 4ull * d.n * bs.Bp;
    if (!d_ws || ws_bytes < need) return HAC_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(d_ws) % 256) return HAC_EINVAL;
    float* XT = static_cast<float*>(d_ws);
    {
        dim3 grid((d.n + 31) / 32, (bs.Bp + 31) / 32);
        hipLaunchKernelGGL(transpose_pad_kernel, grid, dim3(256), 0, stream,
                           d_X, (uint32_t)B, d.n, (uint64_t)ldx, XT, bs.Bp);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
    }
    if (!wpb) wpb = 4;
    if (wpb > 4) wpb = 4;                                   // the kernel is bounded to 256 threads
    const size_t lds = 4ull * table_words(d) + 8ull * list_cap * wpb;
    if (lds > kLdsLimit) return HAC_EINVAL;
    const uint32_t nblocks = (nwaves + wpb - 1) / wpb;
    const uint32_t grid = (nblocks + 7) / 8 * 8;
    typedef void (*kern_t)(DevBlob, const float*, uint32_t, uint32_t, float*, uint64_t,
                           uint32_t, uint32_t, uint32_t, uint32_t);
    kern_t k;
    if (bs.nb == 1) k = shac ? dot_batch_kernel<true, 1> : dot_batch_kernel<false, 1>;
    else if (bs.nb == 2) k = shac ? dot_batch_kernel<true, 2> : dot_batch_kernel<false, 2>;
    else k = shac ? dot_batch_kernel<true, 4> : dot_batch_kernel<false, 4>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return hip_fail(e);
    }
    hipLaunchKernelGGL(k, dim3(grid, bs.tiles), dim3(wpb * kWave), lds, stream,
                       d, XT, bs.Bp, (uint32_t)B, d_Y, (uint64_t)ldy, cpw, bs.gw, list_cap, nblocks);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? HAC_OK : hip_fail(e);
}

} // namespace

extern "C" size_t hac_workspace_bytes(const hac_desc_t* desc, int64_t B)
{
    if (!desc || B <= 0) return 0;
    const BatchShape bs = batch_shape(B);
    return (size_t)4 * (size_t)desc->n * bs.Bp;             // B = 1 does not use it, but a variant may
}

extern "C" int hac_dot(const hac_desc_t* desc, const void* d_blob, const float* d_X, int64_t B, int64_t ldx,
                       float* d_Y, int64_t ldy, void* d_ws, size_t ws_bytes,
                       const hac_launch_t* launch, hac_stream_t stream)
{
    return dot_impl(HAC_FORMAT_HAC, desc, d_blob, d_X, B, ldx, d_Y, ldy, d_ws, ws_bytes, launch, stream);
}

extern "C" int shac_dot(const hac_desc_t* desc, const void* d_blob, const float* d_X, int64_t B, int64_t ldx,
                        float* d_Y, int64_t ldy, void* d_ws, size_t ws_bytes,
                        const hac_launch_t* launch, hac_stream_t stream)
{
    return dot_impl(HAC_FORMAT_SHAC, desc, d_blob, d_X, B, ldx, d_Y, ldy, d_ws, ws_bytes, launch, stream);
}

extern "C" int hac_decode_dev(const hac_desc_t* desc, const void* d_blob, float* d_W, int32_t* d_sym,
                              hac_stream_t stream_)
{
    DevBlob d;
    int rc = make_dev(desc, d_blob, HAC_FORMAT_HAC, d);
    if (rc) return rc;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    g_last_hip_error = 0;
    const uint64_t nm = (uint64_t)d.n * d.m;
    // zero entries are exactly those the index says hold no non-zero: pre-fill with symbol 0 / +0.0
    if (d_W) hipLaunchKernelGGL(fill_u32_kernel, dim3(1024), dim3(256), 0, stream, reinterpret_cast<uint32_t*>(d_W), nm, 0u);
    if (d_sym) hipLaunchKernelGGL(fill_u32_kernel, dim3(1024), dim3(256), 0, stream, reinterpret_cast<uint32_t*>(d_sym), nm, 0u);
    const size_t lds = 4ull * table_words(d);
    const uint32_t grid = (d.n_chunks + 255) / 256;
    if (grid) hipLaunchKernelGGL(hac_decode_kernel, dim3(grid), dim3(256), lds, stream, d, d_W, d_sym);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? HAC_OK : hip_fail(e);
}

extern "C" int shac_decode_dev(const hac_desc_t* desc, const void* d_blob, float* d_nz, int32_t* d_sym,
                               int32_t* d_row, int32_t* d_col, hac_stream_t stream_)
{
    DevBlob d;
    int rc = make_dev(desc, d_blob, HAC_FORMAT_SHAC, d);
    if (rc) return rc;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    g_last_hip_error = 0;
    const size_t lds = 4ull * table_words(d);
    const uint32_t grid = (d.n_chunks + 255) / 256;
    if (grid) hipLaunchKernelGGL(shac_decode_kernel, dim3(grid), dim3(256), lds, stream, d, d_nz, d_sym, d_row, d_col);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? HAC_OK : hip_fail(e);
}

extern "C" int hac_last_hip_error(void) { return g_last_hip_error; }
