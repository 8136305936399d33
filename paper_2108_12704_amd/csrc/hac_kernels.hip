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

// Optional phase timing (build with -DHAC_PHASE_TIMING): lane 0 of each wave of the batch
// kernel stores the shader clock at phase boundaries; hac_debug_phases() copies them out.
#ifdef HAC_PHASE_TIMING
__device__ unsigned long long g_phase[16384 * 8];
#define HAC_MARK(k) do { if (lane == 0 && wave < 16384) g_phase[wave * 8 + (k)] = wall_clock64(); } while (0)
#else
#define HAC_MARK(k) do { } while (0)
#endif

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
// bit reader: a 96-bit sliding register window over an MSB-first uint32 stream.
// The words come either from global memory (word index = stream index) or from
// a copy staged in LDS that starts at stream word `wbase`.
// ---------------------------------------------------------------------------
typedef __attribute__((address_space(3))) const uint32_t lds_cu32;

template <bool LDS>
struct BitReader {
    const uint32_t* w;
    uint32_t wbase;
    uint32_t widx;
    uint32_t a, b, c;

    __device__ __forceinline__ uint32_t word(uint32_t i) const {
        if (LDS) return ((lds_cu32*)w)[i - wbase];
        return w[i];
    }
    __device__ __forceinline__ void seek(const uint32_t* words, uint32_t base, uint32_t bp) {
        w = words; wbase = base;
        widx = bp >> 5;
        a = word(widx); b = word(widx + 1); c = word(widx + 2);
    }
    // bits [bp, bp + 64) left-aligned; bp never moves backwards
    __device__ __forceinline__ uint64_t window(uint32_t bp) {
        const uint32_t wi = bp >> 5;
        if (wi != widx) {
            if (wi == widx + 1) { a = b; b = c; c = word(wi + 2); }
            else { a = word(wi); b = word(wi + 1); c = word(wi + 2); }
            widx = wi;
        }
        const uint32_t off = bp & 31;
        const uint64_t hi = ((uint64_t)a << 32) | b;
        return off ? ((hi << off) | (uint64_t)(c >> (32 - off))) : hi;
    }
};

// Decode tables of one block in LDS.  Layout (uint32 words):
//   lut[2^lut_bits] | canon[99] (+1 pad) | codebook[k4] | symsort[k4]     k4 = k_sym rounded up to 4
// The last two only when k_sym <= kCodebookLdsMax; otherwise they are read from the blob.
struct Tables {
    const uint32_t* lut;        // LDS
    const uint32_t* canon;      // LDS: first_code[33], count[33], first_index[33]
    const float* cb;            // LDS when small, else the blob's copy
    const uint32_t* symsort;    // likewise
    bool small;                 // k_sym <= kCodebookLdsMax (uniform)
};

// Code longer than the first-level table: canonical search by length.
// Returns (symbol << 6) | length.
__device__ __noinline__ uint32_t decode_long(const uint32_t* canon_, const uint32_t* symsort, bool small,
                                             uint32_t top, uint32_t lut_bits, uint32_t lmax)
{
    lds_cu32* canon = (lds_cu32*)canon_;
    for (uint32_t l = lut_bits + 1; l <= lmax; ++l) {
        const uint32_t code = top >> (32 - l);
        const uint32_t rel = code - canon[l];
        if (rel < canon[33 + l]) {
            const uint32_t idx = canon[66 + l] + rel;
            const uint32_t sy = small ? ((lds_cu32*)symsort)[idx] : symsort[idx];
            return (sy << 6) | l;
        }
    }
    return lmax ? lmax : 1;          // unreachable for a validated blob; still makes progress (symbol 0)
}

__device__ __forceinline__ uint32_t decode_symbol(const DevBlob& d, const Tables& t,
                                                  uint32_t top, uint32_t& len)
{
    uint32_t e = ((lds_cu32*)t.lut)[top >> (32 - d.lut_bits)];
    if ((e & 63u) == 0) e = decode_long(t.canon, t.symsort, t.small, top, d.lut_bits, d.lmax);
    len = e & 63u;
    return e >> 6;
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
    uint32_t bp;      // next stream bit
    uint32_t row;     // HAC: row of the next symbol
    uint32_t wpos;    // CSC position of the next non-zero this lane will emit
    uint32_t wend;    // one past the chunk's last non-zero
};

// HAC: emit non-zeros until wpos reaches `limit` (<= wend).  Zeros only move `row`.
template <class Reader, class Emit>
__device__ __forceinline__ void hac_advance(const DevBlob& d, const Tables& tb, Reader& rd,
                                            ChunkState& st, uint32_t limit, Emit emit)
{
    const bool zfast = d.zero_len == 1;
    while (st.wpos < limit) {
        uint64_t win = rd.window(st.bp);
        if (zfast) {
            const uint32_t z = win ? (uint32_t)__builtin_clzll(win) : 64u;   // a non-zero follows, so the run ends
            st.bp += z; st.row += z;
            if (z > 32) continue;                     // fewer than 32 valid bits left in the window
            win <<= z;
        }
        uint32_t len;
        const uint32_t s = decode_symbol(d, tb, (uint32_t)(win >> 32), len);
        st.bp += len;
        if (d.has_zero && s == 0) { st.row++; continue; }
        emit(st.wpos, st.row, s);
        st.row++; st.wpos++;
    }
}

// sHAC: every symbol is a non-zero; the row comes from the packed ri fields.
template <bool WANT_ROW, class Reader, class Emit>
__device__ __forceinline__ void shac_advance(const DevBlob& d, const Tables& tb, Reader& rd,
                                             ChunkState& st, uint32_t limit, Emit emit)
{
    while (st.wpos < limit) {
        const uint64_t win = rd.window(st.bp);
        uint32_t len;
        const uint32_t s = decode_symbol(d, tb, (uint32_t)(win >> 32), len);
        st.bp += len;
        emit(st.wpos, WANT_ROW ? ri_field(d.ri, st.wpos, d.ri_bits) : 0u, s);
        st.wpos++;
    }
}

__device__ __forceinline__ void hac_open(const DevBlob& d, uint32_t g, ChunkState& st, BitReader<false>& rd)
{
    st.bp = d.cbit[g];
    st.row = (g % d.cpc) * d.chunk;
    st.wpos = d.cpos[g];
    st.wend = d.cpos[g + 1];
    if (st.wpos < st.wend) rd.seek(d.stream, 0, st.bp);
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

__device__ __forceinline__ void shac_open(const DevBlob& d, uint32_t g, uint32_t col, ChunkState& st,
                                          BitReader<false>& rd)
{
    st.bp = d.cbit[g];
    st.row = 0;
    st.wpos = d.cb[col] + (g - d.colchunk[col]) * d.chunk;
    const uint32_t cend = d.cb[col + 1];
    st.wend = st.wpos + d.chunk < cend ? st.wpos + d.chunk : cend;
    rd.seek(d.stream, 0, st.bp);
}

__device__ __forceinline__ uint32_t table_words_dev(const DevBlob& d)
{
    const uint32_t k4 = (d.k_sym + 3u) & ~3u;
    return ((1u << d.lut_bits) + 100u + (d.k_sym <= kCodebookLdsMax ? 2u * k4 : 0u) + 3u) & ~3u;
}

// All threads of the block copy the tables; the caller synchronises afterwards.
__device__ __forceinline__ Tables load_tables(const DevBlob& d, uint32_t* smem)
{
    const uint32_t nl = 1u << d.lut_bits;
    const uint32_t k4 = (d.k_sym + 3u) & ~3u;
    uint32_t* s_lut = smem;
    uint32_t* s_canon = smem + nl;
    float* s_cb = reinterpret_cast<float*>(s_canon + 100);
    uint32_t* s_sort = reinterpret_cast<uint32_t*>(s_cb) + k4;
    for (uint32_t i = threadIdx.x; i < nl; i += blockDim.x) s_lut[i] = d.lut[i];
    for (uint32_t i = threadIdx.x; i < 99u; i += blockDim.x) s_canon[i] = d.canon[i];
    Tables t;
    t.lut = s_lut; t.canon = s_canon; t.small = d.k_sym <= kCodebookLdsMax;
    if (d.k_sym <= kCodebookLdsMax) {
        for (uint32_t i = threadIdx.x; i < d.k_sym; i += blockDim.x) { s_cb[i] = d.codebook[i]; s_sort[i] = d.symsort[i]; }
        t.cb = s_cb; t.symsort = s_sort;
    } else {
        t.cb = d.codebook; t.symsort = d.symsort;
    }
    return t;
}

typedef __attribute__((address_space(3))) const float lds_cf32;
__device__ __forceinline__ float value_of(const Tables& t, uint32_t s)
{
    return t.small ? ((lds_cf32*)t.cb)[s] : t.cb[s];
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
    const Tables tb = load_tables(d, smem);
    __syncthreads();
    const uint32_t g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= d.n_chunks) return;
    const uint32_t col = g / d.cpc;
    ChunkState st;
    BitReader<false> rd;
    hac_open(d, g, st, rd);
    hac_advance(d, tb, rd, st, st.wend, [&](uint32_t, uint32_t row, uint32_t s) {
        if (sym) sym[(uint64_t)col * d.n + row] = (int32_t)s;
        if (W) W[(uint64_t)row * d.m + col] = value_of(tb, s);
    });
}

__global__ void __launch_bounds__(256)
shac_decode_kernel(DevBlob d, float* nz, int32_t* sym, int32_t* row_out, int32_t* col_out)
{
    extern __shared__ uint32_t smem[];
    const Tables tb = load_tables(d, smem);
    __syncthreads();
    const uint32_t g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= d.n_chunks) return;
    const uint32_t col = shac_col_of(d, g, 0, d.m);
    ChunkState st;
    BitReader<false> rd;
    shac_open(d, g, col, st, rd);
    shac_advance<true>(d, tb, rd, st, st.wend, [&](uint32_t p, uint32_t row, uint32_t s) {
        if (sym) sym[p] = (int32_t)s;
        if (nz) nz[p] = value_of(tb, s);
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
    const Tables tb = load_tables(d, smem);
    float* s_x = reinterpret_cast<float*>(smem + table_words_dev(d));
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
            BitReader<false> rd;
            if (SHAC) { col = shac_col_of(d, g, c0, c1); shac_open(d, g, col, st, rd); }
            else { col = g / d.cpc; hac_open(d, g, st, rd); }
            auto emit = [&](uint32_t, uint32_t row, uint32_t s) {
                const float xv = X_LDS ? s_x[row] : x[row];
                part = fmaf(xv, value_of(tb, s), part);
            };
            if (SHAC) shac_advance<true>(d, tb, rd, st, st.wend, emit);
            else hac_advance(d, tb, rd, st, st.wend, emit);
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

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// FMA phase building blocks.  A lane group takes every ng-th list entry; the
// loads of kPipe entries are issued together before the first multiply, so that
// many row fetches are in flight per wave.  UNI: one group spans the wave, an entry
// is wave-uniform and travels in scalar registers.

template <int NB, int kPipe>
struct EntryGroup {
    uint2 e[kPipe];
    float x[kPipe][NB];
};

template <int NB, bool UNI, int kPipe>
__device__ __forceinline__ void group_load(EntryGroup<NB, kPipe>& G, const uint2* list, uint32_t idx, uint32_t ng,
                                           const float* xt, uint32_t Bp)
{
#pragma unroll
    for (int k = 0; k < kPipe; ++k) {
        G.e[k] = list[idx + k * ng];
        if (UNI) { G.e[k].x = __builtin_amdgcn_readfirstlane(G.e[k].x); G.e[k].y = __builtin_amdgcn_readfirstlane(G.e[k].y); }
    }
#pragma unroll
    for (int k = 0; k < kPipe; ++k) VecLoad<NB>::ld(xt + (uint64_t)G.e[k].x * Bp, G.x[k]);
}

template <int NB, int kPipe>
__device__ __forceinline__ void group_fma(const EntryGroup<NB, kPipe>& G, float (&acc)[NB])
{
#pragma unroll
    for (int k = 0; k < kPipe; ++k) {
        const float wv = __uint_as_float(G.e[k].y);
#pragma unroll
        for (int i = 0; i < NB; ++i) acc[i] = fmaf(G.x[k][i], wv, acc[i]);
    }
}

// Accumulate list entries with CSC positions [lo, hi) (list index = position - winbase).
template <int NB, bool UNI, int kPipe>
__device__ __forceinline__ void fma_entries(const uint2* list, uint32_t winbase, uint32_t lo, uint32_t hi,
                                            uint32_t ng, uint32_t grp, const float* xt, uint32_t Bp,
                                            float (&acc)[NB])
{
    const uint32_t first = lo + grp;
    const uint32_t count = first < hi ? (hi - first + ng - 1) / ng : 0u;     // entries of this lane group
    const uint32_t full = count / kPipe;
    uint32_t idx = first - winbase;
    const uint32_t step = kPipe * ng;
    for (uint32_t i = 0; i < full; ++i, idx += step) {
        EntryGroup<NB, kPipe> G;
        group_load<NB, UNI, kPipe>(G, list, idx, ng, xt, Bp);
        group_fma<NB, kPipe>(G, acc);
    }
    // last, partial group: entries past the end read entry `idx` again and are not added
    const uint32_t rest = count - full * kPipe;
    if (rest) {
        EntryGroup<NB, kPipe> G;
#pragma unroll
        for (int k = 0; k < kPipe; ++k) {
            G.e[k] = list[idx + ((uint32_t)k < rest ? k * ng : 0u)];
            if (UNI) { G.e[k].x = __builtin_amdgcn_readfirstlane(G.e[k].x); G.e[k].y = __builtin_amdgcn_readfirstlane(G.e[k].y); }
        }
#pragma unroll
        for (int k = 0; k < kPipe; ++k) VecLoad<NB>::ld(xt + (uint64_t)G.e[k].x * Bp, G.x[k]);
#pragma unroll
        for (int k = 0; k < kPipe; ++k) {
            if ((uint32_t)k < rest) {
                const float wv = __uint_as_float(G.e[k].y);
#pragma unroll
                for (int i = 0; i < NB; ++i) acc[i] = fmaf(G.x[k][i], wv, acc[i]);
            }
        }
    }
}

// Index entries of one lane's chunk.
struct LaneChunk {
    uint32_t bp, bit1;      // first stream bit of the chunk, first bit after it
    uint32_t wpos, wend;    // CSC positions of its non-zeros
    uint32_t row;           // HAC: first row
};

// Lane `lane` takes chunk gb + lane (if below g1).  sHAC: colchunk_l / cbeg_l hold
// colchunk[c0 + l] and cb[c0 + l] of lane l (l <= ncols); all lanes must call this together.
template <bool SHAC>
__device__ __forceinline__ LaneChunk load_lane_chunk(const DevBlob& d, uint32_t gb, uint32_t g1, uint32_t lane,
                                                     uint32_t ncols, uint32_t colchunk_l, uint32_t cbeg_l)
{
    LaneChunk c;
    c.bp = c.bit1 = c.wpos = c.wend = c.row = 0;
    const uint32_t g = gb + lane;
    const bool active = g < g1;
    if (active) { c.bp = d.cbit[g]; c.bit1 = d.cbit[g + 1]; }
    if (SHAC) {
        uint32_t rel = 0;                                    // column of chunk g, relative to c0
        for (uint32_t k = 1; k < ncols; ++k) rel += (uint32_t)__shfl((int)colchunk_l, (int)k, kWave) <= g ? 1u : 0u;
        const uint32_t cc0 = (uint32_t)__shfl((int)colchunk_l, (int)rel, kWave);
        const uint32_t p0 = (uint32_t)__shfl((int)cbeg_l, (int)rel, kWave);
        const uint32_t p1 = (uint32_t)__shfl((int)cbeg_l, (int)rel + 1, kWave);
        if (active) {
            c.wpos = p0 + (g - cc0) * d.chunk;
            c.wend = c.wpos + d.chunk < p1 ? c.wpos + d.chunk : p1;
        }
    } else if (active) {
        c.wpos = d.cpos[g];
        c.wend = d.cpos[g + 1];
        c.row = (g % d.cpc) * d.chunk;
    }
    return c;
}

// gw: lanes per group (power of two, gw * NB = batch columns handled per pass);
// 64 / gw groups walk the list interleaved and are added together at a column's end.
template <int NB, bool UNI> struct BatchTraits {
    static constexpr int kPipe = (NB == 4 && !UNI) ? 8 : 16;        // row fetches in flight per lane group
    static constexpr int kMaxThreads = 1024;
};

template <bool SHAC, int NB, bool UNI>
__global__ void __launch_bounds__((BatchTraits<NB, UNI>::kMaxThreads))
dot_batch_kernel(DevBlob d, const float* __restrict__ XT, uint32_t Bp, uint32_t B,
                 float* __restrict__ Y, uint64_t ldy, uint32_t cpw, uint32_t gw,
                 uint32_t list_cap, uint32_t sbuf_words, uint32_t nblocks)
{
    extern __shared__ uint32_t smem[];
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wib = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t lb = logical_block(gridDim.x);
    const uint32_t wave = lb * (blockDim.x / kWave) + wib;
    const uint32_t c0 = wave * cpw;
    const bool live = lb < nblocks && c0 < d.m;
    HAC_MARK(0);
    uint32_t c1 = 0, ncols = 0, gfirst = 0, g1 = 0;
    uint32_t colend_l = 0, colchunk_l = 0, cbeg_l = 0;
    LaneChunk nxt;
    nxt.bp = nxt.bit1 = nxt.wpos = nxt.wend = nxt.row = 0;
    // The index of the first batch of chunks is requested before the decode tables,
    // so that both round trips to memory overlap.
    if (live) {
        c1 = c0 + cpw < d.m ? c0 + cpw : d.m;
        ncols = c1 - c0;
        if (SHAC) {
            if (lane <= ncols) { colchunk_l = d.colchunk[c0 + lane]; cbeg_l = d.cb[c0 + lane]; }
            gfirst = (uint32_t)__shfl((int)colchunk_l, 0, kWave);
            g1 = (uint32_t)__shfl((int)colchunk_l, (int)ncols, kWave);
        } else {
            gfirst = c0 * d.cpc;
            g1 = c1 * d.cpc;
            if (lane < ncols) colend_l = d.cpos[(c0 + lane + 1) * d.cpc];
        }
        nxt = load_lane_chunk<SHAC>(d, gfirst, g1, lane, ncols, colchunk_l, cbeg_l);
    }
    const Tables tb = load_tables(d, smem);
    __syncthreads();
    if (!live) return;
    HAC_MARK(1);

    uint32_t* sbuf = smem + table_words_dev(d) + (uint64_t)wib * (sbuf_words + 2 * list_cap);   // staged stream
    uint2* list = reinterpret_cast<uint2*>(sbuf + sbuf_words);                                  // (row, value)
    const uint32_t ng = kWave / gw;
    const uint32_t grp = lane / gw, lig = lane % gw;
    const uint32_t boff = blockIdx.y * 256u + lig * NB;      // first batch column of this lane
    const float* xt = XT + boff;

    float acc[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) acc[i] = 0.0f;
    uint32_t cc = c0;                                        // column being accumulated (wave-uniform)
    uint32_t t = 0;                                          // next CSC position to consume
    bool t_set = false;

    auto flush = [&]() {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            float v = acc[i];
            for (uint32_t off = 32; off >= gw; off >>= 1) v += __shfl_xor(v, (int)off, kWave);
            const uint32_t b = boff + i;
            if (grp == 0 && b < B) Y[(uint64_t)b * ldy + cc] = v;
            acc[i] = 0.0f;
        }
    };

    for (uint32_t gb = gfirst; gb < g1; gb += kWave) {
        const uint32_t nact = g1 - gb < (uint32_t)kWave ? g1 - gb : (uint32_t)kWave;
        const bool active = lane < nact;
        const LaneChunk cur = nxt;
        if (gb + kWave < g1) nxt = load_lane_chunk<SHAC>(d, gb + kWave, g1, lane, ncols, colchunk_l, cbeg_l);
        ChunkState st;
        st.bp = cur.bp; st.row = cur.row; st.wpos = cur.wpos; st.wend = cur.wend;
        const uint32_t blo = (uint32_t)__shfl((int)cur.bp, 0, kWave);
        const uint32_t bhi = (uint32_t)__shfl((int)cur.bit1, (int)(nact - 1), kWave);
        const uint32_t pbeg = (uint32_t)__shfl((int)cur.wpos, 0, kWave);
        const uint32_t pend = (uint32_t)__shfl((int)cur.wend, (int)(nact - 1), kWave);
        if (pbeg == pend) continue;                          // these chunks hold zeros only
        if (!t_set) { t = pbeg; t_set = true; }
        // ---- stage the stream words of these chunks in LDS (coalesced 128-bit loads) ----
        const uint32_t wlo = (blo >> 5) & ~3u;
        const uint32_t nw = ((bhi >> 5) + 3) - wlo + 1;      // the reader looks two words past the current one
        const bool staged = nw <= sbuf_words;
        if (staged) {
            const uint4* src = reinterpret_cast<const uint4*>(d.stream + wlo);
            uint4* dst = reinterpret_cast<uint4*>(sbuf);
            for (uint32_t i = lane; i * 4 < nw; i += kWave) dst[i] = src[i];
        }
        wave_sync();
        HAC_MARK(2);
        bool opened = false;
        BitReader<true> rl;
        BitReader<false> rg;
        for (uint32_t winbase = pbeg; winbase < pend; winbase += list_cap) {
            const uint32_t winend = winbase + list_cap < pend ? winbase + list_cap : pend;
            // ---- decode phase: lanes = chunks ----
            const uint32_t lim = st.wend < winend ? st.wend : winend;
            if (active && st.wpos < lim) {
                auto emit = [&](uint32_t p, uint32_t row, uint32_t s) {
                    if (SHAC) list[p - winbase].y = __float_as_uint(value_of(tb, s));
                    else list[p - winbase] = make_uint2(row, __float_as_uint(value_of(tb, s)));
                };
                if (staged) {
                    if (!opened) { rl.seek(sbuf, wlo, st.bp); opened = true; }
                    if (SHAC) shac_advance<false>(d, tb, rl, st, lim, emit); else hac_advance(d, tb, rl, st, lim, emit);
                } else {
                    if (!opened) { rg.seek(d.stream, 0, st.bp); opened = true; }
                    if (SHAC) shac_advance<false>(d, tb, rg, st, lim, emit); else hac_advance(d, tb, rg, st, lim, emit);
                }
            }
            HAC_MARK(3);
            if (SHAC) {
                // row indices: fixed-width fields, unpacked by all lanes side by side
                for (uint32_t p = winbase + lane; p < winend; p += kWave)
                    list[p - winbase].x = ri_field(d.ri, p, d.ri_bits);
            }
            wave_sync();
            HAC_MARK(4);
            // ---- FMA phase: lanes = batch ----
            while (cc < c1) {
                const uint32_t pe = SHAC ? (uint32_t)__shfl((int)cbeg_l, (int)(cc - c0 + 1), kWave)
                                         : (uint32_t)__shfl((int)colend_l, (int)(cc - c0), kWave);
                const uint32_t hi = pe < winend ? pe : winend;
                if (t < hi) fma_entries<NB, UNI, BatchTraits<NB, UNI>::kPipe>(list, winbase, t, hi, ng, grp, xt, Bp, acc);
                t = hi > t ? hi : t;
                if (pe <= winend) { flush(); ++cc; }
                else break;                                  // column continues in the next window
            }
            wave_sync();
            HAC_MARK(5);
        }
    }
    while (cc < c1) { flush(); ++cc; }                       // trailing columns without non-zeros
    HAC_MARK(6);
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
    const uint32_t k4 = (d.k_sym + 3u) & ~3u;
    return ((1u << d.lut_bits) + 100u + (d.k_sym <= kCodebookLdsMax ? 2u * k4 : 0u) + 3u) & ~3u;
}

struct BatchShape { uint32_t gw, nb, Bp, tiles; };

// Bp: padded batch width of the feature-major copy; a wave pass covers gw * nb
// batch columns (at most 256); wider batches take several passes (grid.y).
BatchShape batch_shape(int64_t B)
{
    BatchShape s;
    uint32_t p = 1;
    while (p < (uint32_t)(B < 256 ? B : 256)) p <<= 1;
    s.nb = p < 4 ? p : 4;
    s.gw = p / s.nb;
    if (B <= 256) { s.Bp = p; s.tiles = 1; }
    else { s.Bp = (uint32_t)((B + 255) / 256 * 256); s.tiles = s.Bp / 256; }
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

uint32_t round_up(uint32_t v, uint32_t q) { return (v + q - 1) / q * q; }

typedef void (*batch_kern_t)(DevBlob, const float*, uint32_t, uint32_t, float*, uint64_t,
                             uint32_t, uint32_t, uint32_t, uint32_t, uint32_t);

template <bool SHAC>
batch_kern_t pick_batch_kernel(uint32_t nb, bool uni)
{
    if (nb == 1) return uni ? dot_batch_kernel<SHAC, 1, true> : dot_batch_kernel<SHAC, 1, false>;
    if (nb == 2) return uni ? dot_batch_kernel<SHAC, 2, true> : dot_batch_kernel<SHAC, 2, false>;
    return uni ? dot_batch_kernel<SHAC, 4, true> : dot_batch_kernel<SHAC, 4, false>;
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
    uint32_t cpw = default_cpw(desc), wpb = 0, list_cap = 0, sbuf_words = 0, variant = 0;
    bool reuse_xt = false;
    if (launch) {
        if (launch->cols_per_wave > 32 || launch->waves_per_block > 16) return HAC_EINVAL;
        if (launch->cols_per_wave) cpw = launch->cols_per_wave;
        wpb = launch->waves_per_block;
        variant = launch->variant & 0xffu;
        reuse_xt = (launch->variant & HAC_LAUNCH_REUSE_XT) != 0;
        if (launch->variant & ~(0xffu | HAC_LAUNCH_REUSE_XT)) return HAC_EINVAL;
        list_cap = launch->reserved[0];
        sbuf_words = launch->reserved[1];
        if (list_cap && (list_cap < 64 || list_cap > 4096)) return HAC_EINVAL;
        if (sbuf_words && (sbuf_words < 16 || sbuf_words > 8192 || sbuf_words % 4)) return HAC_EINVAL;
        if (launch->reserved[2] || launch->reserved[3] || launch->reserved[4]) return HAC_EINVAL;
    }
    const uint32_t nwaves = (d.m + cpw - 1) / cpw;
    const bool shac = format == HAC_FORMAT_SHAC;
    g_last_hip_error = 0;

    if (B == 1 && variant == 1) {
        if (!wpb) wpb = 16;
        const size_t base = 4ull * table_words(d);
        const bool x_lds = base + 4ull * d.n <= kLdsLimit - 1024;
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
    const float* XT = d_X;                                   // B = 1: X is its own feature-major copy
    if (B > 1) {
        const size_t need = 4ull * d.n * bs.Bp;
        if (!d_ws || ws_bytes < need) return HAC_EWORKSPACE;
        if (reinterpret_cast<uintptr_t>(d_ws) % 256) return HAC_EINVAL;
        float* xt = static_cast<float*>(d_ws);
        XT = xt;
        if (!reuse_xt) {
            dim3 grid((d.n + 31) / 32, (bs.Bp + 31) / 32);
            hipLaunchKernelGGL(transpose_pad_kernel, grid, dim3(256), 0, stream,
                               d_X, (uint32_t)B, d.n, (uint64_t)ldx, xt, bs.Bp);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return hip_fail(e);
        }
    }
    // per-wave LDS: stream words of one batch of 64 chunks, and the list of its non-zeros
    {
        const double cpcol = (double)desc->n_chunks / (double)desc->m;
        double cols = cpcol > 0.0 ? 64.0 / cpcol : (double)cpw;
        if (cols > (double)cpw) cols = (double)cpw;
        if (!sbuf_words) {
            const double est = ((double)desc->max_col_bits / 32.0 + 1.0) * cols + 8.0;
            sbuf_words = round_up((uint32_t)(est < 4096.0 ? est : 4096.0), 64);
            if (sbuf_words > 4096) sbuf_words = 4096;
        }
        if (!list_cap) {
            const double est = (double)desc->max_col_nnz * cols;
            list_cap = round_up((uint32_t)(est < 2048.0 ? (est > 1.0 ? est : 1.0) : 2048.0), 64);
        }
    }
    const size_t per_wave = 4ull * sbuf_words + 8ull * list_cap;
    if (!wpb) {
        // as many wavefronts per CU as LDS allows (at most 16), in blocks that share one copy of the tables
        const size_t tbl = 4ull * table_words(d);
        uint32_t best_waves = 0;
        for (uint32_t w = 16; w >= 1; w >>= 1) {
            const size_t blk = tbl + w * per_wave;
            if (blk > kLdsLimit) continue;
            uint32_t waves = (uint32_t)(kLdsLimit / blk) * w;
            if (waves > 16) waves = 16;
            if (waves > best_waves) { best_waves = waves; wpb = w; }
        }
        if (!wpb) wpb = 1;
    }
    const size_t lds = 4ull * table_words(d) + (size_t)wpb * per_wave;
    if (lds > kLdsLimit) return HAC_EINVAL;
    const uint32_t nblocks = (nwaves + wpb - 1) / wpb;
    const uint32_t grid = (nblocks + 7) / 8 * 8;
    const bool uni = bs.gw == 64;
    batch_kern_t k = shac ? pick_batch_kernel<true>(bs.nb, uni) : pick_batch_kernel<false>(bs.nb, uni);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return hip_fail(e);
    }
    hipLaunchKernelGGL(k, dim3(grid, bs.tiles), dim3(wpb * kWave), lds, stream,
                       d, XT, bs.Bp, (uint32_t)B, d_Y, (uint64_t)ldy, cpw, bs.gw, list_cap, sbuf_words, nblocks);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? HAC_OK : hip_fail(e);
}

} // namespace

extern "C" size_t hac_workspace_bytes(const hac_desc_t* desc, int64_t B)
{
    if (!desc || B <= 0) return 0;
    if (B == 1) return 0;                                    // a single row is its own feature-major copy
    const BatchShape bs = batch_shape(B);
    return (size_t)4 * (size_t)desc->n * bs.Bp;
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

#ifdef HAC_PHASE_TIMING
extern "C" int hac_debug_phases(unsigned long long* out, size_t count)
{
    if (count > 16384 * 8) count = 16384 * 8;
    return hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase), count * sizeof(unsigned long long)) == hipSuccess ? 0 : -5;
}
#endif
