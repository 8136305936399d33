// Device side of libhac for gfx950 (MI355X): decode-and-accumulate kernels for
// HAC (arXiv 2108.12704 Sect. IV-B, Algorithm 1) and sHAC (Sect. IV-C,
// Algorithm 2) blobs, Y = X.W for a batch (Algorithm 3's result, with the
// stream decoded once per launch instead of once per row of X).
//
// Work split.  The stream is serial by nature; the index stored beside it
// gives every chunk (a fixed number of consecutive non-zeros of one column) its
// starting bit, so one lane decodes one chunk and all lanes of a wavefront do
// the same amount of work.  A wavefront owns a few whole columns of W:
//   staging     : the columns' stream words (and, for sHAC, their packed row
//                 indices) are copied to LDS with coalesced 128-bit loads;
//   decode phase: the 64 lanes decode the columns' chunks side by side from
//                 LDS and leave (row, value) pairs, in CSC order, in a
//                 per-wave LDS list;
//   FMA phase   : the lanes turn into batch lanes: the wave walks the list
//                 and lane b accumulates x[b][row] * value from the
//                 feature-major copy of X (one coalesced row segment per
//                 non-zero, many fetches in flight).  A column's sum is
//                 complete inside one wave, so Y is written once, without
//                 atomics, in a fixed order.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <atomic>
#include <cstdarg>
#include <cstdio>

#include "../../include/hac.h"
#include "hac_internal.h"
#include "hac_hostlib.h"
#include "hac_device.h"

// Optional phase timing (build with -DHAC_PHASE_TIMING): lane 0 of each wave of the dot
// kernels stores a 100 MHz clock at phase boundaries; hac_debug_phases() copies them out.
#ifdef HAC_PHASE_TIMING
__device__ unsigned long long g_phase[16384 * 8];
#define HAC_MARK(k) do { if (lane == 0 && wave < 16384) g_phase[wave * 8 + (k)] = wall_clock64(); } while (0)
#else
#define HAC_MARK(k) do { } while (0)
#endif

namespace {

// XCD-aware block order: hardware deals consecutive block ids round-robin to the
// 8 XCDs; this gives every XCD (hence every L2) one contiguous range of columns.
__device__ __forceinline__ uint32_t logical_block(uint32_t nblocks_padded)
{
    const uint32_t per = nblocks_padded >> 3;
    return (blockIdx.x & 7u) * per + (blockIdx.x >> 3);
}

// ---------------------------------------------------------------------------
// TEST-ONLY decode kernels: one lane per chunk, words read from global memory
// ---------------------------------------------------------------------------
__global__ void fill_u32_kernel(uint32_t* p, uint64_t count, uint32_t v)
{
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) p[i] = v;
}

template <bool SHAC>
__global__ void __launch_bounds__(256)
decode_kernel(DevBlob d, float* vals, int32_t* sym, int32_t* row_out, int32_t* col_out)
{
    extern __shared__ uint32_t smem[];
    const Tables tb = load_tables(d, smem);
    __syncthreads();
    const uint32_t g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= d.n_chunks) return;
    const uint32_t col = column_of_chunk(d, g);
    uint32_t rel, row0;
    load_entry(d, g, rel, row0);
    ChunkState st;
    st.bp = d.colbit[col] + rel;
    st.row = row0;
    const uint32_t cend = d.colpos[col + 1];
    const uint32_t chunk = hac_internal::chunk_of_column(d.chunk, cend - d.colpos[col]);
    st.wpos = d.colpos[col] + (g - d.colchunk[col]) * chunk;
    st.wend = st.wpos + chunk < cend ? st.wpos + chunk : cend;
    WordSrc<false> src = { d.stream, 0 };
    if (SHAC && d.rice) {
        gap_advance_slow(d, tb, src, st, st.wend, [&](uint32_t p, uint32_t row, uint32_t s, float v) {
            if (sym) sym[p] = (int32_t)s;
            if (vals) vals[p] = v;
            if (row_out) row_out[p] = (int32_t)row;
            if (col_out) col_out[p] = (int32_t)col;
        });
    } else if (SHAC) {
        WordSrc<false> rsrc = { d.ri, 0 };
        shac_advance(d, tb, src, st, st.wend, [&](uint32_t p, uint32_t, uint32_t s, float v) {
            if (sym) sym[p] = (int32_t)s;
            if (vals) vals[p] = v;
            if (row_out) row_out[p] = (int32_t)rsrc.field((uint64_t)p * d.ri_bits, d.ri_bits);
            if (col_out) col_out[p] = (int32_t)col;
        });
    } else {
        // vals: dense n x m row-major; sym: dense, column order (both pre-filled with zeros)
        hac_advance(d, tb, src, st, st.wend, [&](uint32_t, uint32_t row, uint32_t s, float v) {
            if (sym) sym[(uint64_t)col * d.n + row] = (int32_t)s;
            if (vals) vals[(uint64_t)row * d.m + col] = v;
        });
    }
}

// Dense route, step 1: write the pointer of every non-zero into an index map (n rows of
// `pitch` pointers, pre-filled with 0).  HAC: pointer = symbol (0.0 is symbol 0 when it
// occurs); sHAC, whose alphabet has no 0.0: pointer = symbol + 1.  One lane per chunk.
// Copy n4 16-byte pieces from global memory to LDS with all threads of the block, four loads per
// thread in flight: the loads of a turn are issued from clamped indices before the first store
// (the values pass through an empty asm statement, or the compiler pairs every load with its
// guarded store again and waits in between).
__device__ __forceinline__ void block_copy_u4(uint4* dst, const uint4* src, uint32_t n4)
{
    for (uint32_t base = 0; base < n4; base += 4 * blockDim.x) {
        uint4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t i = base + threadIdx.x + k * blockDim.x;
            v[k] = src[i < n4 ? i : n4 - 1u];
        }
        asm volatile("" : "+v"(v[0].x), "+v"(v[0].y), "+v"(v[0].z), "+v"(v[0].w), "+v"(v[1].x), "+v"(v[1].y), "+v"(v[1].z), "+v"(v[1].w),
                          "+v"(v[2].x), "+v"(v[2].y), "+v"(v[2].z), "+v"(v[2].w), "+v"(v[3].x), "+v"(v[3].y), "+v"(v[3].z), "+v"(v[3].w));
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t i = base + threadIdx.x + k * blockDim.x;
            if (i < n4) dst[i] = v[k];
        }
    }
}

template <typename IdxT>
__global__ void __launch_bounds__(256)
decode_to_index_kernel(DevBlob d, IdxT* idx, uint64_t pitch, uint32_t shac, uint32_t s_words, uint32_t r_words,
                       uint32_t c_words)
{
    extern __shared__ uint32_t smem[];
    __shared__ uint32_t range[4];                       // the block's stream words [0], [1) and CSC positions [2], [3)
    TableRegs tr = request_tables(d);
    uint32_t* sstage = smem + table_words_dev(d);       // s_words: the stream words of the block's chunks
    uint32_t* rstage = sstage + s_words;                // r_words: their ri fields (sHAC with fields)
    uint32_t* cstage = rstage + r_words;                // c_words: colchunk[0 .. m], or nothing when it is too long
    const uint32_t g0 = blockIdx.x * blockDim.x, g = g0 + threadIdx.x;
    const uint32_t glast = g0 + blockDim.x - 1 < d.n_chunks - 1 ? g0 + blockDim.x - 1 : d.n_chunks - 1;
    const bool live = g < d.n_chunks;
    // this chunk's index entry, and for the block's last chunk the entry after it (the end of the
    // block's stream range): requested with the tables
    uint2 ent_raw = make_uint2(0u, 0u), ent_next = make_uint2(0u, 0u);
    if (live) ent_raw = request_entry(d, g);
    if (g == glast && glast + 1 < d.n_chunks) ent_next = request_entry(d, glast + 1);
    request_table_values(d, tr);
    // which column owns a chunk: a binary search over colchunk, from a copy in LDS when it fits
    // (a dozen dependent reads per lane, tens of cycles each instead of hundreds); colchunk sits
    // in a 256-byte aligned section with room behind its m + 1 words
    if (c_words) block_copy_u4(reinterpret_cast<uint4*>(cstage), reinterpret_cast<const uint4*>(d.colchunk), (d.m + 4) >> 2);
    const Tables tb = store_tables(d, smem, tr);
    if (c_words) __syncthreads();
    auto owner = [&](uint32_t chunk) -> uint32_t {
        if (!c_words) return column_of_chunk(d, chunk);
        uint32_t lo = 0, hi = d.m;                       // invariant: colchunk[lo] <= chunk < colchunk[hi]
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (((lds_cu32*)cstage)[mid] <= chunk) lo = mid; else hi = mid;
        }
        return lo;
    };
    uint32_t col = 0;
    ChunkState st = { 0, 0, 0, 0 };
    if (live) {
        col = owner(g);
        uint32_t rel, row0;
        entry_fields(d, ent_raw, rel, row0);
        st.bp = d.colbit[col] + rel;
        st.row = row0;
        const uint32_t cend = d.colpos[col + 1];
        const uint32_t chunk = hac_internal::chunk_of_column(d.chunk, cend - d.colpos[col]);
        st.wpos = d.colpos[col] + (g - d.colchunk[col]) * chunk;
        st.wend = st.wpos + chunk < cend ? st.wpos + chunk : cend;
    }
    // The chunks of a block follow one another in the stream: from the first one's start to the
    // start of the chunk after the last one (or the end of the stream) is one contiguous range.
    if (threadIdx.x == 0) { range[0] = st.bp >> 5; range[2] = st.wpos; }
    if (g == glast) {
        uint32_t endbit = d.colbit[d.m];
        if (glast + 1 < d.n_chunks) {
            uint32_t rel2, row2;
            entry_fields(d, ent_next, rel2, row2);
            endbit = d.colbit[owner(glast + 1)] + rel2;
        }
        range[1] = (endbit + 31) >> 5;
        range[3] = st.wend;
    }
    __syncthreads();                                    // tables and range complete
    // Stage the range in LDS when it fits (a lane's walk is a chain of dependent reads: tens of
    // cycles each from LDS, hundreds from L2 with 64 lanes on 64 different lines); else read the blob.
    const uint32_t wlo = range[0] & ~3u;
    const uint32_t nw = range[1] >= wlo ? range[1] - wlo + 8 : 0xffffffffu;     // 128-bit windows read past the last bit
    const uint64_t rlo_bit = (uint64_t)range[2] * d.ri_bits, rhi_bit = (uint64_t)range[3] * d.ri_bits;
    const uint32_t rwlo = (uint32_t)(rlo_bit >> 5) & ~3u;
    const bool fields = shac && !d.rice;
    const uint32_t rnw = fields ? (uint32_t)((rhi_bit + 31) >> 5) - rwlo + 4 : 0;
    const bool staged = nw <= s_words && rnw <= r_words && range[3] >= range[2];
    if (staged) {
        block_copy_u4(reinterpret_cast<uint4*>(sstage), reinterpret_cast<const uint4*>(d.stream + wlo), (nw + 3) >> 2);
        if (fields) block_copy_u4(reinterpret_cast<uint4*>(rstage), reinterpret_cast<const uint4*>(d.ri + rwlo), (rnw + 3) >> 2);
    }
    __syncthreads();
    if (!live) return;
    auto walk = [&](auto src, auto rsrc) {
        if (shac && d.rice) {
            gap_advance_slow(d, tb, src, st, st.wend, [&](uint32_t, uint32_t row, uint32_t s, float) {
                idx[(uint64_t)row * pitch + col] = (IdxT)(s + 1);
            });
        } else if (shac) {
            shac_advance(d, tb, src, st, st.wend, [&](uint32_t p, uint32_t, uint32_t s, float) {
                const uint32_t row = rsrc.field((uint64_t)p * d.ri_bits, d.ri_bits);
                idx[(uint64_t)row * pitch + col] = (IdxT)(s + 1);
            });
        } else {
            hac_advance(d, tb, src, st, st.wend, [&](uint32_t, uint32_t row, uint32_t s, float) {
                idx[(uint64_t)row * pitch + col] = (IdxT)s;
            });
        }
    };
    if (staged) walk(WordSrc<true>{ sstage, wlo }, WordSrc<true>{ rstage, rwlo });
    else walk(WordSrc<false>{ d.stream, 0 }, WordSrc<false>{ d.ri, 0 });
}

// ---------------------------------------------------------------------------
// X (B x n, row-major) -> XT, feature-major in panels of `wp` batch columns:
// XT[(b / wp) * n * wp + r * wp + b % wp] = X[b][r], zero for B <= b < Bp.
// One pass of the batch kernel reads one panel: rows of wp floats, contiguous.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
transpose_pad_kernel(const float* __restrict__ X, uint32_t B, uint32_t n, uint64_t ldx,
                     float* __restrict__ XT, uint32_t Bp, uint32_t wp)
{
    __shared__ float tile[32][33];
    const uint32_t tx = threadIdx.x & 31, ty = threadIdx.x >> 5;       // 32 x 8
    const uint32_t r0 = blockIdx.x * 32, b0 = blockIdx.y * 32;
    float v[4];                                        // clamped addresses: four loads in flight, zeros put in afterwards
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) {
        const uint32_t b = b0 + ty + 8 * k, r = r0 + tx;
        v[k] = X[(uint64_t)(b < B ? b : B - 1) * ldx + (r < n ? r : n - 1)];
    }
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) {
        const uint32_t b = b0 + ty + 8 * k, r = r0 + tx;
        tile[ty + 8 * k][tx] = (b < B && r < n) ? v[k] : 0.0f;
    }
    __syncthreads();
    for (uint32_t k = 0; k < 32; k += 8) {
        const uint32_t r = r0 + ty + k, b = b0 + tx;
        if (r < n && b < Bp) XT[(uint64_t)(b / wp) * n * wp + (uint64_t)r * wp + (b % wp)] = tile[tx][ty + k];
    }
}

// Same re-layout for panels of exactly 32 batch columns: a block turns 32 batch rows x 128
// features into one contiguous 16 KB piece of a panel.  With X 16-byte aligned (vec = 1) the
// reads are 128-bit (512 bytes per batch row) and so are the writes.
__global__ void __launch_bounds__(256)
transpose_panel32_kernel(const float* __restrict__ X, uint32_t B, uint32_t n, uint64_t ldx,
                         float* __restrict__ XT, uint32_t vec)
{
    __shared__ float tile[32][129];
    const uint32_t r0 = blockIdx.x * 128, b0 = blockIdx.y * 32;
    // All loads of a thread are issued before the first is used: rows past B and features past n
    // are read from a clamped, valid address and replaced by zero afterwards (a guarded load would
    // be compiled into load / wait / store turns, one trip to memory each).
    if (vec && r0 + 128 <= n) {
        float4 v[4];
#pragma unroll
        for (uint32_t i = 0; i < 4; ++i) {
            const uint32_t idx = threadIdx.x + 256 * i;          // float4 index: 32 rows x 32 quads
            const uint32_t b = b0 + (idx >> 5), q = idx & 31;
            v[i] = *reinterpret_cast<const float4*>(X + (uint64_t)(b < B ? b : B - 1) * ldx + r0 + 4 * q);
        }
#pragma unroll
        for (uint32_t i = 0; i < 4; ++i) {
            const uint32_t idx = threadIdx.x + 256 * i;
            const uint32_t b = idx >> 5, q = idx & 31;
            const bool ok = b0 + b < B;
            tile[b][4 * q + 0] = ok ? v[i].x : 0.0f; tile[b][4 * q + 1] = ok ? v[i].y : 0.0f;
            tile[b][4 * q + 2] = ok ? v[i].z : 0.0f; tile[b][4 * q + 3] = ok ? v[i].w : 0.0f;
        }
    } else {
        float v[16];
#pragma unroll
        for (uint32_t i = 0; i < 16; ++i) {
            const uint32_t idx = threadIdx.x + 256 * i;
            const uint32_t b = b0 + (idx >> 7), r = r0 + (idx & 127);
            v[i] = X[(uint64_t)(b < B ? b : B - 1) * ldx + (r < n ? r : n - 1)];
        }
#pragma unroll
        for (uint32_t i = 0; i < 16; ++i) {
            const uint32_t idx = threadIdx.x + 256 * i;
            const uint32_t b = idx >> 7, r = idx & 127;
            tile[b][r] = (b0 + b < B && r0 + r < n) ? v[i] : 0.0f;
        }
    }
    __syncthreads();
    float* out = XT + (uint64_t)blockIdx.y * n * 32 + (uint64_t)r0 * 32;
#pragma unroll
    for (uint32_t i = 0; i < 4; ++i) {
        const uint32_t idx = threadIdx.x + 256 * i;              // float4 index: 128 features x 8 quads of batch
        const uint32_t r = idx >> 3, bq = (idx & 7) * 4;
        if (r0 + r < n) {
            const float4 v = make_float4(tile[bq][r], tile[bq + 1][r], tile[bq + 2][r], tile[bq + 3][r]);
            *reinterpret_cast<float4*>(out + (uint64_t)r * 32 + bq) = v;
        }
    }
}

// ---------------------------------------------------------------------------
// batch kernel
// ---------------------------------------------------------------------------
template <int NB> struct VecLoad;
template <> struct VecLoad<1> { static __device__ __forceinline__ void ld(const float* p, float* v) { v[0] = *p; } };
template <> struct VecLoad<2> { static __device__ __forceinline__ void ld(const float* p, float* v) { const float2 t = *reinterpret_cast<const float2*>(p); v[0] = t.x; v[1] = t.y; } };
template <> struct VecLoad<4> { static __device__ __forceinline__ void ld(const float* p, float* v) { const float4 t = *reinterpret_cast<const float4*>(p); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; } };

// the same from a copy of X in LDS
template <int NB> struct VecLoadLds {
    static __device__ __forceinline__ void ld(lds_cf32* p, float* v) {
#pragma unroll
        for (int i = 0; i < NB; ++i) v[i] = p[i];
    }
};

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// What happens to a finished sum before it is stored: + bias[column], max(., 0), and where it
// goes.  yt = nullptr: Y[b * ldy + column].  yt set: the feature-major layout the next layer of
// a chain reads as its XT, panels of wp batch columns, yt[(b / wp) * m * wp + column * wp + b % wp],
// with 0 in the padded batch columns.
struct Epilogue {
    const float* bias;
    float* yt;
    uint32_t relu;
};

__device__ __forceinline__ float epilogue_apply(const Epilogue& e, float v, uint32_t col)
{
    if (e.bias) v += e.bias[col];
    if (e.relu) v = fmaxf(v, 0.0f);
    return v;
}

// FMA phase building blocks.  A lane group takes every ng-th list entry; the
// loads of kPipe entries are issued together before the first multiply, so that
// many row fetches are in flight per wave.
template <int NB, int kPipe>
struct EntryGroup {
    uint2 e[kPipe];
    float x[kPipe][NB];
};

// Accumulate list entries with CSC positions [lo, hi) (list index = position - winbase).
template <int NB, int kPipe>
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
#pragma unroll
        for (int k = 0; k < kPipe; ++k) G.e[k] = list[idx + k * ng];
#pragma unroll
        for (int k = 0; k < kPipe; ++k) VecLoad<NB>::ld(xt + (uint64_t)G.e[k].x * Bp, G.x[k]);
#pragma unroll
        for (int k = 0; k < kPipe; ++k) {
            const float wv = __uint_as_float(G.e[k].y);
#pragma unroll
            for (int i2 = 0; i2 < NB; ++i2) acc[i2] = fmaf(G.x[k][i2], wv, acc[i2]);
        }
    }
    // last, partial group: only the entries that exist are fetched (a lane that is switched off asks
    // the memory path for nothing; a repeated fetch of some valid row would cost it a line like any other)
    const uint32_t rest = count - full * kPipe;
    if (rest) {
        EntryGroup<NB, kPipe> G;
#pragma unroll
        for (int k = 0; k < kPipe; ++k) {
            G.e[k] = make_uint2(0u, 0u);
#pragma unroll
            for (int i2 = 0; i2 < NB; ++i2) G.x[k][i2] = 0.0f;
        }
#pragma unroll
        for (int k = 0; k < kPipe; ++k) if ((uint32_t)k < rest) G.e[k] = list[idx + k * ng];
#pragma unroll
        for (int k = 0; k < kPipe; ++k) if ((uint32_t)k < rest) VecLoad<NB>::ld(xt + (uint64_t)G.e[k].x * Bp, G.x[k]);
#pragma unroll
        for (int k = 0; k < kPipe; ++k) {
            const float wv = __uint_as_float(G.e[k].y);          // 0.0 for an entry that does not exist
#pragma unroll
            for (int i2 = 0; i2 < NB; ++i2) acc[i2] = fmaf(G.x[k][i2], wv, acc[i2]);
        }
    }
}

template <int NB> struct BatchTraits {
    static constexpr int kPipe = NB == 4 ? 10 : 16;                 // row fetches in flight per lane group
    static constexpr int kMaxThreads = 1024;
};

// The loaded values pass through an empty asm statement: all the loads above it are issued before
// the first wait, and none of them is moved down into the guarded store that uses it (the compiler
// would otherwise turn load, load, ..., store, store, ... back into load / wait / store turns).
#define HAC_PIN_U4(q) "+v"((q).x), "+v"((q).y), "+v"((q).z), "+v"((q).w)
__device__ __forceinline__ void pin_loads(uint4 (&a)[4])
{
    asm volatile("" : HAC_PIN_U4(a[0]), HAC_PIN_U4(a[1]), HAC_PIN_U4(a[2]), HAC_PIN_U4(a[3]));
}

// Copy words [wlo, wlo + nw) of `src` (wlo and nw multiples of 4, nw >= 4) to LDS with 128-bit
// loads, four per lane in flight (4 KB per wave and trip to memory): the loads of a turn are issued
// from clamped indices before the first is stored.  Starts at 16-byte piece `first`.
__device__ __forceinline__ void stage_words(uint32_t* dst, const uint32_t* src, uint32_t wlo, uint32_t nw, uint32_t lane,
                                            uint32_t first = 0)
{
    const uint4* s4 = reinterpret_cast<const uint4*>(src + wlo);
    uint4* d4 = reinterpret_cast<uint4*>(dst);
    const uint32_t n4 = nw >> 2;
    for (uint32_t base = first; base < n4; base += 4 * kWave) {
        uint4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t i = base + lane + k * kWave;
            v[k] = s4[i < n4 ? i : n4 - 1u];
        }
        pin_loads(v);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t i = base + lane + k * kWave;
            if (i < n4) d4[i] = v[k];
        }
    }
}

// A wave's stream words and, with RI, its ri words, in two steps: request_stage issues the loads of
// the first turn(s) of the copies, finish_stage stores them and copies what is left.  In between a
// kernel can finish other work whose loads are older (the decode tables and the block's barrier
// behind them) while these travel.  First trip: 4 KB of a HAC stream (a column of the largest
// layer here has 3.5 KB); with ri words, 1 KB of the stream and 1 KB of ri (the codewords of the
// non-zeros alone are short).  Every load instruction of a wave occupies the address path for its
// 64 lanes whatever they ask for, so turns that are rarely needed are left to the second step.
// `staged` false (nothing to stage, or more than fits): the loads are still issued, from `safe`
// (16 valid, aligned bytes), so that the number of loads in flight does not depend on the path.
template <bool RI> struct StageRegs { static constexpr int kTurns = RI ? 1 : 4; uint4 s[4], r; };

template <bool RI>
__device__ __forceinline__ void request_stage(StageRegs<RI>& q, bool staged, const uint32_t* safe,
                                              const uint32_t* stream, uint32_t swlo, uint32_t snw,
                                              const uint32_t* ri, uint32_t rwlo, uint32_t rnw, uint32_t lane)
{
    const uint4* s4 = reinterpret_cast<const uint4*>(staged ? stream + swlo : safe);
    const uint32_t sn4 = staged ? snw >> 2 : 1u, rn4 = staged ? rnw >> 2 : 1u;
#pragma unroll
    for (int k = 0; k < StageRegs<RI>::kTurns; ++k) {
        const uint32_t i = lane + k * kWave;
        q.s[k] = s4[i < sn4 ? i : sn4 - 1u];
    }
    if constexpr (RI) {
        const uint4* r4 = reinterpret_cast<const uint4*>(staged ? ri + rwlo : safe);
        q.r = r4[lane < rn4 ? lane : rn4 - 1u];
    }
}

template <bool RI>
__device__ __forceinline__ void finish_stage(StageRegs<RI>& q, uint32_t* sdst, const uint32_t* stream, uint32_t swlo, uint32_t snw,
                                             uint32_t* rdst, const uint32_t* ri, uint32_t rwlo, uint32_t rnw, uint32_t lane)
{
    const uint32_t sn4 = snw >> 2, rn4 = rnw >> 2;
    if constexpr (RI) asm volatile("" : HAC_PIN_U4(q.s[0]), HAC_PIN_U4(q.r));
    else pin_loads(q.s);
#pragma unroll
    for (int k = 0; k < StageRegs<RI>::kTurns; ++k) {
        const uint32_t i = lane + k * kWave;
        if (i < sn4) reinterpret_cast<uint4*>(sdst)[i] = q.s[k];
    }
    if constexpr (RI) {
        if (lane < rn4) reinterpret_cast<uint4*>(rdst)[lane] = q.r;
    }
    stage_words(sdst, stream, swlo, snw, lane, StageRegs<RI>::kTurns * kWave);
    if constexpr (RI) stage_words(rdst, ri, rwlo, rnw, lane, kWave);
}

// Barrier of the block that orders LDS only: loads from global memory stay in flight across it.
__device__ __forceinline__ void block_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// gw: lanes per group (power of two); a pass over the list covers gw * NB batch
// columns, and npass passes cover this block's share of the batch.  Passes keep
// the part of the feature-major X that a pass touches small enough to stay in
// L2 while all wavefronts of an XCD gather from it.  64 / gw groups walk the
// list interleaved and are added together at a column's end.  part_words: LDS
// words per wave for partial sums of a column that does not fit one list window
// (npass * 64 * NB, or 0 when the launch guarantees that no column is split).
// MP: several passes (npass > 1); the single-pass variant has no pass loop and no barrier.
// EPI: the epilogue (bias, max(., 0), feature-major output) is compiled in; a plain product runs
// the variant without it, which needs fewer registers (the single-pass kernel would spill one).
template <bool SHAC, int NB, bool MP, bool EPI>
__global__ void __launch_bounds__((BatchTraits<NB>::kMaxThreads))
dot_batch_kernel(DevBlob d, const float* __restrict__ XT, uint32_t Bp, uint32_t B,
                 float* __restrict__ Y, uint64_t ldy, uint32_t cpw, uint32_t gw, uint32_t npass,
                 uint32_t list_cap, uint32_t sbuf_words, uint32_t part_words, uint32_t nblocks,
                 uint32_t sync_passes, Epilogue epi)
{
    extern __shared__ uint32_t smem[];
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wib = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    // Work items are (batch tile, column block) pairs, tile-major; every XCD takes one contiguous
    // range of them, so the feature-major panels of one tile are fetched into few L2s only.
    const uint32_t item = logical_block(gridDim.x);
    const uint32_t tile = item / nblocks;
    const uint32_t lb = item - tile * nblocks;
    const uint32_t wave = lb * (blockDim.x / kWave) + wib;
    const uint32_t c0 = wave * cpw;
    const uint32_t tile_b = gw * NB * npass;                 // batch columns per block
    if (tile * tile_b >= B) return;                          // padding of the grid, or a tile of padding only
    // passes that hold at least one real batch row: the last tile (or a batch that is not a power
    // of two) ends before the block's npass panels do
    const uint32_t rows_here = B - tile * tile_b < tile_b ? B - tile * tile_b : tile_b;
    const uint32_t live_passes = MP ? (rows_here + gw * NB - 1) / (gw * NB) : 1u;
    const bool live = c0 < d.m;
    HAC_MARK(0);
    // Per-column index of this wave's columns: lane l keeps column c0 + l (l <= ncols).
    // Requested before the decode tables so that both trips to memory overlap.
    uint32_t ncols = 0, cchunk_l = 0, cpos_l = 0, cbit_l = 0;
    if (live) {
        const uint32_t cend = c0 + cpw < d.m ? c0 + cpw : d.m;
        ncols = cend - c0;
        if (lane <= ncols) {
            cchunk_l = d.colchunk[c0 + lane];
            cpos_l = d.colpos[c0 + lane];
            cbit_l = d.colbit[c0 + lane];
        }
    }
    // Two trips to memory before the first codeword is decoded: (1) the column index above and
    // what the tables need first, (2) chunk entries, stream (and ri) words and the values of the
    // first-level table.  One barrier then covers the tables and the staged words.
    TableRegs tr = request_tables(d);
    const uint32_t c1 = c0 + ncols;
    const uint32_t gfirst = (uint32_t)__shfl((int)cchunk_l, 0, kWave);
    const uint32_t g1 = (uint32_t)__shfl((int)cchunk_l, (int)ncols, kWave);
    const uint32_t posbase = (uint32_t)__shfl((int)cpos_l, 0, kWave);
    const uint32_t posend = (uint32_t)__shfl((int)cpos_l, (int)ncols, kWave);
    const uint32_t bit_lo = (uint32_t)__shfl((int)cbit_l, 0, kWave);
    const uint32_t bit_hi = (uint32_t)__shfl((int)cbit_l, (int)ncols, kWave);

    uint32_t* sbuf = smem + table_words_dev(d) + (uint64_t)wib * (sbuf_words + 2 * list_cap + part_words);   // staged words
    uint2* list = reinterpret_cast<uint2*>(sbuf + sbuf_words);                                  // (row, value)
    float* part = reinterpret_cast<float*>(sbuf + sbuf_words + 2 * list_cap);                   // [pass][NB][lane]

    // ---- stage this wave's stream words (and ri words) in LDS ----
    const uint32_t swlo = (bit_lo >> 5) & ~3u;
    const uint32_t snw = (((bit_hi >> 5) + 4) - swlo + 4) & ~3u;        // the decoder reads three words past the current one
    const uint64_t rb_lo = (uint64_t)posbase * d.ri_bits, rb_hi = (uint64_t)posend * d.ri_bits;
    const uint32_t rwlo = (uint32_t)(rb_lo >> 5) & ~3u;
    const uint32_t rnw = SHAC ? ((((uint32_t)(rb_hi >> 5) + 2) - rwlo + 4) & ~3u) : 0u;
    const bool staged = posend > posbase && snw + rnw <= sbuf_words;
    // index entries of the first batch of chunks (requested together with the staging loads)
    uint2 ent_raw = make_uint2(0u, 0u);
    if (gfirst + lane < g1) ent_raw = request_entry(d, gfirst + lane);
    request_table_values(d, tr);
    StageRegs<SHAC> sq;
    request_stage<SHAC>(sq, staged, d.canon, d.stream, swlo, snw, d.ri, rwlo, rnw, lane);
    const Tables tb = store_tables(d, smem, tr);
    block_sync_lds();                                        // the tables; the staged words are still on their way
    if (!live) {
        // sync_passes: every wave of the block meets at a barrier once per pass (see accumulate)
        if (MP && sync_passes) for (uint32_t p = 1; p < live_passes; ++p) __syncthreads();
        return;
    }
    HAC_MARK(1);
    if (staged) finish_stage<SHAC>(sq, sbuf, d.stream, swlo, snw, sbuf + snw, d.ri, rwlo, rnw, lane);
    wave_sync();
    HAC_MARK(2);
    const WordSrc<true> s_lds = { sbuf, swlo };
    const WordSrc<false> s_glb = { d.stream, 0 };
    const WordSrc<true> r_lds = { sbuf + snw, rwlo };
    const WordSrc<false> r_glb = { d.ri, 0 };
    const uint32_t ri_rel0 = (uint32_t)(rb_lo - 32ull * rwlo);          // bit of CSC position posbase in the staged ri words

    const uint32_t ng = kWave / gw;
    const uint32_t grp = lane / gw, lig = lane % gw;
    const uint32_t pass_w = gw * NB;                          // batch columns per pass = width of one panel of XT
    const uint64_t panel = (uint64_t)d.n * pass_w;            // floats per panel
    const uint32_t boff = tile * tile_b + lig * NB;           // first batch column of this lane, pass 0
    const float* xt = XT + (uint64_t)tile * npass * panel + lig * NB;
    uint32_t cc = c0;                                        // column being accumulated (wave-uniform)
    uint32_t t = posbase;                                    // next CSC position to consume

    // Consume list entries [t, hi) of column cc in every pass.  `carried`: earlier windows already
    // hold partial sums of this column in `part`; `last`: the column ends here, so the sums are
    // reduced over the lane groups and stored, else they are parked in `part`.
    auto accumulate = [&](uint32_t winbase, uint32_t hi, bool carried, bool last) {
        const uint32_t passes = live_passes;
        for (uint32_t p = 0; p < passes; ++p) {
            // Keeping the block's waves on the same pass keeps the panels of XT they gather from few
            // enough to stay in L2.  Only set when every wave calls this exactly once (one column per
            // wave, no column split over windows).  The first pass starts without waiting: a wave
            // that has decoded its column early gathers while the others still decode.
            if (MP && sync_passes && p > 0) __syncthreads();
            float a[NB];
#pragma unroll
            for (int i = 0; i < NB; ++i) a[i] = (carried && part_words) ? part[(p * NB + i) * kWave + lane] : 0.0f;
            // (the single-pass kernel with the epilogue compiled in keeps one fetch fewer in flight: with ten it spills)
            constexpr int kPipe = BatchTraits<NB>::kPipe - ((EPI && !MP && NB == 4) ? 1 : 0);
            if (t < hi) fma_entries<NB, kPipe>(list, winbase, t, hi, ng, grp, xt + p * panel, pass_w, a);
            if (last) {
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    float v = a[i];
                    for (uint32_t off = 32; off >= gw; off >>= 1) v += __shfl_xor(v, (int)off, kWave);
                    const uint32_t b = boff + p * pass_w + i;
                    if (grp == 0) {
                        if constexpr (EPI) {
                            if (epi.yt)
                                epi.yt[((uint64_t)(b / pass_w) * d.m + cc) * pass_w + (b % pass_w)] =
                                    b < B ? epilogue_apply(epi, v, cc) : 0.0f;
                            else if (b < B) Y[(uint64_t)b * ldy + cc] = epilogue_apply(epi, v, cc);
                        } else {
                            if (b < B) Y[(uint64_t)b * ldy + cc] = v;
                        }
                    }
                }
            } else if (part_words) {                       // always true here: the host sizes `part` whenever a split can occur
#pragma unroll
                for (int i = 0; i < NB; ++i) part[(p * NB + i) * kWave + lane] = a[i];
            }
        }
    };

    for (uint32_t gb = gfirst; gb < g1; gb += kWave) {
        const uint32_t nact = g1 - gb < (uint32_t)kWave ? g1 - gb : (uint32_t)kWave;
        const bool active = lane < nact;
        const uint32_t g = gb + lane;
        // column of chunk g, relative to c0: number of columns l >= 1 whose first chunk is <= g
        uint32_t rel = 0;
        for (uint32_t k = 1; k < ncols; ++k) rel += (uint32_t)__shfl((int)cchunk_l, (int)k, kWave) <= g ? 1u : 0u;
        const uint32_t col_chunk0 = (uint32_t)__shfl((int)cchunk_l, (int)rel, kWave);
        const uint32_t col_pos0 = (uint32_t)__shfl((int)cpos_l, (int)rel, kWave);
        const uint32_t col_pos1 = (uint32_t)__shfl((int)cpos_l, (int)rel + 1, kWave);
        const uint32_t col_bit0 = (uint32_t)__shfl((int)cbit_l, (int)rel, kWave);
        ChunkState st;
        uint32_t ent_rel, ent_row;
        entry_fields(d, ent_raw, ent_rel, ent_row);
        st.bp = col_bit0 + ent_rel;
        st.row = ent_row;
        const uint32_t chunk = hac_internal::chunk_of_column(d.chunk, col_pos1 - col_pos0);
        st.wpos = col_pos0 + (g - col_chunk0) * chunk;
        st.wend = st.wpos + chunk < col_pos1 ? st.wpos + chunk : col_pos1;
        if (!active) { st.wpos = 0; st.wend = 0; }
        const uint32_t pbeg = (uint32_t)__shfl((int)st.wpos, 0, kWave);
        const uint32_t pend = (uint32_t)__shfl((int)st.wend, (int)(nact - 1), kWave);
        // entries of the next batch travel while this one is decoded
        if (gb + kWave + lane < g1) ent_raw = request_entry(d, gb + kWave + lane);

        for (uint32_t winbase = pbeg; winbase < pend; winbase += list_cap) {
            const uint32_t winend = winbase + list_cap < pend ? winbase + list_cap : pend;
            // ---- decode phase: lanes = chunks ----
            const uint32_t lim = st.wend < winend ? st.wend : winend;
            if (active && st.wpos < lim) {
                auto emit = [&](uint32_t p, uint32_t row, uint32_t, float v) {
                    if (SHAC) list[p - winbase].y = __float_as_uint(v);
                    else list[p - winbase] = make_uint2(row, __float_as_uint(v));
                };
                if (staged) {
                    if (SHAC) shac_advance(d, tb, s_lds, st, lim, emit);
                    else if (d.rice) gap_advance(d, tb, s_lds, st, lim, emit);
                    else if (d.zero_len == 1) hac_advance_zrun(d, tb, s_lds, st, lim, emit);
                    else hac_advance(d, tb, s_lds, st, lim, emit);
                } else {
                    if (SHAC) shac_advance(d, tb, s_glb, st, lim, emit);
                    else if (d.rice) gap_advance_slow(d, tb, s_glb, st, lim, emit);
                    else hac_advance(d, tb, s_glb, st, lim, emit);
                }
            }
            HAC_MARK(3);
            if (SHAC) {
                // row indices: fixed-width fields, unpacked by all lanes side by side
                for (uint32_t p = winbase + lane; p < winend; p += kWave) {
                    list[p - winbase].x = staged ? r_lds.field_rel(__umul24(p - posbase, d.ri_bits) + ri_rel0, d.ri_bits)
                                                 : r_glb.field((uint64_t)p * d.ri_bits, d.ri_bits);
                }
            }
            wave_sync();
            HAC_MARK(4);
            // ---- FMA phase: lanes = batch ----
            while (cc < c1) {
                const uint32_t ps = (uint32_t)__shfl((int)cpos_l, (int)(cc - c0), kWave);
                const uint32_t pe = (uint32_t)__shfl((int)cpos_l, (int)(cc - c0 + 1), kWave);
                const uint32_t hi = pe < winend ? pe : winend;
                const bool last = pe <= winend;
                if (last || t < hi) accumulate(winbase, hi, t > ps, last);
                t = hi > t ? hi : t;
                if (last) ++cc;
                else break;                                  // column continues in the next window
            }
            wave_sync();
            HAC_MARK(5);
        }
    }
    while (cc < c1) {                                        // trailing columns without non-zeros
        const uint32_t ps = (uint32_t)__shfl((int)cpos_l, (int)(cc - c0), kWave);
        accumulate(t, t, t > ps, true);
        ++cc;
    }
    HAC_MARK(6);
}

// ---------------------------------------------------------------------------
// small-batch kernel (at most 4 rows of X)
// ---------------------------------------------------------------------------
// With so few batch columns there is nothing to share between lanes, so a lane
// multiplies the non-zeros it decodes itself: the fetch of X for one non-zero
// travels while the next codeword is decoded, and no list is written.  XT holds
// NB floats per row of W (B = 1: X itself).  Lane sums are added over the lanes
// of a column with a segmented shuffle reduction (columns own contiguous lanes),
// then over chunk batches in LDS (colsum), always in the same order.
//
// XLDS: XT is X itself (B x n, row-major, leading dimension ldx) and every block first copies it,
// feature-major with NB floats per row of W, into LDS behind the tables (x_words words): no
// re-layout launch, and the rows of X are then fetched from LDS.  For X of at most ~128 KB.
template <bool SHAC, int NB, bool XLDS>
__global__ void __launch_bounds__(1024)
dot_small_kernel(DevBlob d, const float* __restrict__ XT, uint32_t B, uint64_t ldx, uint32_t x_words,
                 float* __restrict__ Y, uint64_t ldy,
                 uint32_t cpw, uint32_t sbuf_words, uint32_t sum_words, uint32_t nblocks, Epilogue epi)
{
    extern __shared__ uint32_t smem[];
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wib = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t lb = logical_block(gridDim.x);
    const uint32_t wave = lb * (blockDim.x / kWave) + wib;
    const uint32_t c0 = wave * cpw;
    const bool live = lb < nblocks && c0 < d.m;
    HAC_MARK(0);
    uint32_t ncols = 0, cchunk_l = 0, cpos_l = 0, cbit_l = 0;
    if (live) {
        const uint32_t cend = c0 + cpw < d.m ? c0 + cpw : d.m;
        ncols = cend - c0;
        if (lane <= ncols) {
            cchunk_l = d.colchunk[c0 + lane];
            cpos_l = d.colpos[c0 + lane];
            cbit_l = d.colbit[c0 + lane];
        }
    }
    // two trips to memory before the first codeword is decoded, as in the batch kernel
    TableRegs tr = request_tables(d);
    float* xs = reinterpret_cast<float*>(smem + table_words_dev(d));      // XLDS: [row of W][NB]
    if (XLDS) {
        // a thread takes whole rows of W: NB coalesced reads (one per batch row), one contiguous store
        for (uint32_t r = threadIdx.x; r < d.n; r += blockDim.x) {
            float v[NB];
#pragma unroll
            for (int i = 0; i < NB; ++i) v[i] = (uint32_t)i < B ? XT[(uint64_t)i * ldx + r] : 0.0f;
#pragma unroll
            for (int i = 0; i < NB; ++i) xs[(uint64_t)r * NB + i] = v[i];
        }
    }
    const uint32_t gfirst = (uint32_t)__shfl((int)cchunk_l, 0, kWave);
    const uint32_t g1 = (uint32_t)__shfl((int)cchunk_l, (int)ncols, kWave);
    const uint32_t posbase = (uint32_t)__shfl((int)cpos_l, 0, kWave);
    const uint32_t posend = (uint32_t)__shfl((int)cpos_l, (int)ncols, kWave);
    const uint32_t bit_lo = (uint32_t)__shfl((int)cbit_l, 0, kWave);
    const uint32_t bit_hi = (uint32_t)__shfl((int)cbit_l, (int)ncols, kWave);

    uint32_t* sbuf = smem + table_words_dev(d) + (XLDS ? x_words : 0u) + (uint64_t)wib * (sbuf_words + sum_words);
    float* colsum = reinterpret_cast<float*>(sbuf + sbuf_words);          // [column][NB]
    lds_cf32* xs_lds = (lds_cf32*)xs;

    const uint32_t swlo = (bit_lo >> 5) & ~3u;
    const uint32_t snw = (((bit_hi >> 5) + 4) - swlo + 4) & ~3u;
    const uint64_t rb_lo = (uint64_t)posbase * d.ri_bits, rb_hi = (uint64_t)posend * d.ri_bits;
    const uint32_t rwlo = (uint32_t)(rb_lo >> 5) & ~3u;
    const uint32_t rnw = SHAC ? ((((uint32_t)(rb_hi >> 5) + 2) - rwlo + 4) & ~3u) : 0u;
    const bool staged = posend > posbase && snw + rnw <= sbuf_words;
    uint2 ent_raw = make_uint2(0u, 0u);
    if (gfirst + lane < g1) ent_raw = request_entry(d, gfirst + lane);
    request_table_values(d, tr);
    StageRegs<SHAC> sq;
    request_stage<SHAC>(sq, staged, d.canon, d.stream, swlo, snw, d.ri, rwlo, rnw, lane);
    const Tables tb = store_tables(d, smem, tr);
    for (uint32_t i = lane; i < ncols * NB; i += kWave) colsum[i] = 0.0f;
    if (XLDS) __syncthreads();                               // the block's copy of X came through plain loads
    else block_sync_lds();                                   // the tables; the staged words are still on their way
    if (!live) return;
    HAC_MARK(1);
    if (staged) finish_stage<SHAC>(sq, sbuf, d.stream, swlo, snw, sbuf + snw, d.ri, rwlo, rnw, lane);
    wave_sync();
    HAC_MARK(2);
    const WordSrc<true> s_lds = { sbuf, swlo };
    const WordSrc<false> s_glb = { d.stream, 0 };
    const WordSrc<true> r_lds = { sbuf + snw, rwlo };
    const WordSrc<false> r_glb = { d.ri, 0 };
    const uint32_t ri_rel0 = (uint32_t)(rb_lo - 32ull * rwlo);          // bit of CSC position posbase in the staged ri words

    for (uint32_t gb = gfirst; gb < g1; gb += kWave) {
        const uint32_t nact = g1 - gb < (uint32_t)kWave ? g1 - gb : (uint32_t)kWave;
        const bool active = lane < nact;
        const uint32_t g = gb + lane;
        uint32_t rel = 0;
        for (uint32_t k = 1; k < ncols; ++k) rel += (uint32_t)__shfl((int)cchunk_l, (int)k, kWave) <= g ? 1u : 0u;
        const uint32_t col_chunk0 = (uint32_t)__shfl((int)cchunk_l, (int)rel, kWave);
        const uint32_t col_pos0 = (uint32_t)__shfl((int)cpos_l, (int)rel, kWave);
        const uint32_t col_pos1 = (uint32_t)__shfl((int)cpos_l, (int)rel + 1, kWave);
        const uint32_t col_bit0 = (uint32_t)__shfl((int)cbit_l, (int)rel, kWave);
        ChunkState st;
        uint32_t ent_rel, ent_row;
        entry_fields(d, ent_raw, ent_rel, ent_row);
        st.bp = col_bit0 + ent_rel;
        st.row = ent_row;
        const uint32_t chunk = hac_internal::chunk_of_column(d.chunk, col_pos1 - col_pos0);
        st.wpos = col_pos0 + (g - col_chunk0) * chunk;
        st.wend = st.wpos + chunk < col_pos1 ? st.wpos + chunk : col_pos1;
        if (!active) { st.wpos = 0; st.wend = 0; }
        if (gb + kWave + lane < g1) ent_raw = request_entry(d, gb + kWave + lane);

        // a[] += pv * px[] is applied when the next non-zero has been decoded, just before px is
        // fetched again, so the fetch of X for one non-zero travels during a whole decode step
        float a[NB], px[NB], pv = 0.0f;
#pragma unroll
        for (int i = 0; i < NB; ++i) { a[i] = 0.0f; px[i] = 0.0f; }
        if (active) {
            auto emit = [&](uint32_t p, uint32_t row, uint32_t, float v) {
                if (SHAC) {
                    if (staged) row = r_lds.field_rel(__umul24(p - posbase, d.ri_bits) + ri_rel0, d.ri_bits);
                    else row = r_glb.field((uint64_t)p * d.ri_bits, d.ri_bits);
                }
#pragma unroll
                for (int i = 0; i < NB; ++i) a[i] = fmaf(px[i], pv, a[i]);
                if constexpr (XLDS) VecLoadLds<NB>::ld(xs_lds + row * NB, px);
                else VecLoad<NB>::ld(XT + (uint64_t)row * NB, px);
                pv = v;
            };
            if (staged) {
                if (SHAC) shac_advance(d, tb, s_lds, st, st.wend, emit);
                else if (d.rice) gap_advance(d, tb, s_lds, st, st.wend, emit);
                else if (d.zero_len == 1) hac_advance_zrun(d, tb, s_lds, st, st.wend, emit);
                else hac_advance(d, tb, s_lds, st, st.wend, emit);
            } else {
                if (SHAC) shac_advance(d, tb, s_glb, st, st.wend, emit);
                else if (d.rice) gap_advance_slow(d, tb, s_glb, st, st.wend, emit);
                else hac_advance(d, tb, s_glb, st, st.wend, emit);
            }
        }
        HAC_MARK(3);
        const uint32_t key = active ? rel : 0xffffffffu;
        const uint32_t key_up = (uint32_t)__shfl_up((int)key, 1, kWave);
        const bool head = active && (lane == 0 || key_up != key);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            float v = fmaf(px[i], pv, a[i]);
            for (uint32_t off = 1; off < (uint32_t)kWave; off <<= 1) {
                const float o = __shfl_down(v, off, kWave);
                const uint32_t ko = (uint32_t)__shfl_down((int)key, off, kWave);
                if (lane + off < (uint32_t)kWave && ko == key) v += o;
            }
            if (head) colsum[rel * NB + i] += v;
        }
        wave_sync();                                         // the next batch may continue the same column
        HAC_MARK(4);
    }
    for (uint32_t j = lane; j < ncols; j += kWave) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            if (epi.yt) epi.yt[(uint64_t)(c0 + j) * NB + i] = (uint32_t)i < B ? epilogue_apply(epi, colsum[j * NB + i], c0 + j) : 0.0f;
            else if ((uint32_t)i < B) Y[(uint64_t)i * ldy + c0 + j] = epilogue_apply(epi, colsum[j * NB + i], c0 + j);
        }
    }
    HAC_MARK(5);
    HAC_MARK(6);
}

// ---------------------------------------------------------------------------
// host-side launch helpers
// ---------------------------------------------------------------------------
thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) { g_last_hip_error = (int)e; return HAC_EHIP; }

// What the planning calls need of a header before they divide by its fields (the device calls
// check more, in make_dev and im_dot_impl).
bool desc_plausible(const hac_desc_t* d)
{
    if (!d || d->magic != 0x31434148u || d->version != 2) return false;
    if (d->format != HAC_FORMAT_HAC && d->format != HAC_FORMAT_SHAC && d->format != HAC_FORMAT_IM) return false;
    if (d->n < 1 || d->m < 1 || d->n > 0x7fffffffull || d->m > 0x7fffffffull) return false;
    if (d->format != HAC_FORMAT_IM && (hac_internal::chunk_base(d->chunk) < 1 || hac_internal::chunk_base(d->chunk) > 65536 || d->lut_bits < 1 || d->lut_bits > 12)) return false;
    return true;
}

int make_dev(const hac_desc_t* desc, const void* d_blob, uint32_t format, DevBlob& d)
{
    if (!desc || !d_blob || !desc_plausible(desc)) return HAC_EINVAL;
    if (desc->magic != 0x31434148u || desc->version != 2 || desc->format != format) return HAC_EINVAL;
    if (reinterpret_cast<uintptr_t>(d_blob) % 256) return HAC_EINVAL;
    if (desc->lut_bits < 1 || desc->lut_bits > 12 || desc->lmax > 32) return HAC_EINVAL;
    if (desc->n > 0x7fffffffull || desc->m > 0x7fffffffull || desc->nnz > 0xfffffff0ull ||
        desc->n_chunks > 0xfffffff0ull || hac_internal::chunk_base(desc->chunk) < 1 || hac_internal::chunk_base(desc->chunk) > 65536) return HAC_EINVAL;
    if (desc->ent_bits != 16 && desc->ent_bits != 32 && desc->ent_bits != 64) return HAC_EINVAL;
    if (desc->row_bits > 31 || desc->ri_bits > 32) return HAC_EINVAL;
    const bool rice = format == HAC_FORMAT_SHAC && desc->ri_coding == HAC_RI_RICE;
    if (desc->ri_coding > HAC_RI_RICE || (format == HAC_FORMAT_HAC && desc->ri_coding)) return HAC_EINVAL;
    if (rice && (desc->rice_k > 15 || desc->ri_bits || desc->ent_bits == 16)) return HAC_EINVAL;
    if (format == HAC_FORMAT_SHAC && !rice && (desc->ri_bits < 1 || desc->ent_bits == 64)) return HAC_EINVAL;
    const uint8_t* b = static_cast<const uint8_t*>(d_blob);
    d.codebook = reinterpret_cast<const float*>(b + desc->off_codebook);
    d.canon = reinterpret_cast<const uint32_t*>(b + desc->off_canon);
    d.symsort = reinterpret_cast<const uint32_t*>(b + desc->off_symsort);
    d.lut = reinterpret_cast<const uint32_t*>(b + desc->off_lut);
    d.stream = reinterpret_cast<const uint32_t*>(b + desc->off_stream);
    d.colchunk = reinterpret_cast<const uint32_t*>(b + desc->off_col_chunk);
    d.colpos = reinterpret_cast<const uint32_t*>(b + desc->off_col_pos);
    d.colbit = reinterpret_cast<const uint32_t*>(b + desc->off_col_bit);
    d.ent = b + desc->off_chunk_ent;
    d.ri = (format == HAC_FORMAT_SHAC && !rice) ? reinterpret_cast<const uint32_t*>(b + desc->off_ri) : nullptr;
    d.rice = rice ? 1u : 0u; d.rice_k = desc->rice_k;
    d.n = (uint32_t)desc->n; d.m = (uint32_t)desc->m; d.nnz = (uint32_t)desc->nnz;
    d.k_sym = desc->k_sym; d.lmax = desc->lmax; d.lut_bits = desc->lut_bits;
    d.has_zero = desc->has_zero; d.zero_len = desc->zero_len; d.chunk = desc->chunk;
    d.ri_bits = desc->ri_bits; d.ent_bits = desc->ent_bits; d.row_bits = desc->row_bits;
    d.n_chunks = (uint32_t)desc->n_chunks;
    return HAC_OK;
}

uint32_t table_words(const DevBlob& d)
{
    const uint32_t k4 = (d.k_sym + 3u) & ~3u;
    return ((2u << d.lut_bits) + 100u + (d.k_sym <= kCodebookLdsMax ? 2u * k4 : 0u) + 3u) & ~3u;
}

struct BatchShape { uint32_t gw, nb, npass, Bp, tiles; };

// Bp: padded batch width of the feature-major copy (a power of two up to 256, else a
// multiple of 256).  One pass covers gw * nb batch columns (a pass over 32 touches
// n * 128 bytes of the copy); a block runs the passes of one tile of tile_b batch
// columns; Bp / tile_b tiles cover the batch.
BatchShape batch_shape(int64_t B, uint32_t pass_w, uint32_t tile_b)
{
    BatchShape s;
    uint32_t p = 1;
    while (p < (uint32_t)(B < 256 ? B : 256)) p <<= 1;
    s.Bp = B <= 256 ? p : (uint32_t)((B + 255) / 256 * 256);
    uint32_t t = p < tile_b ? p : tile_b;                    // batch columns per block, a power of two
    uint32_t w = t < pass_w ? t : pass_w;                    // batch columns per pass
    s.nb = w < 4 ? w : 4;
    s.gw = w / s.nb;
    s.npass = t / w;
    s.tiles = s.Bp / t;
    return s;
}

constexpr size_t kLdsLimit = 160 * 1024;
constexpr uint32_t kDefaultTile = 256;

uint32_t round_up(uint32_t v, uint32_t q) { return (v + q - 1) / q * q; }

// columns per wavefront: fill the 64 decode lanes, but keep enough wavefronts in flight
uint32_t default_cpw(const hac_desc_t* desc)
{
    const double chunks_per_col = (double)desc->n_chunks / (double)desc->m;
    uint32_t cpw = 1;
    if (chunks_per_col < 64.0) cpw = (uint32_t)(64.0 / (chunks_per_col > 1.0 ? chunks_per_col : 1.0));
    if (cpw < 1) cpw = 1;
    if (cpw > 16) cpw = 16;
    while (cpw > 1 && desc->m / cpw < 2048) cpw >>= 1;
    return cpw;
}

// Dense route (decode to an index map, then fp32 MFMA tiles) or sparse route (vector FMAs per
// non-zero)?  Decided from rough time estimates, with constants measured on an MI355X:
//   sparse: every non-zero gathers 4 bytes per batch column (at least 32) through the vector
//           memory path, about 22 TB/s over the whole chip and 140 GB/s per busy CU (a block covers
//           16 columns of W and up to 256 batch columns), plus the re-layout of X and ~12 us;
//   dense : ~35 non-zeros per ns to decode into the index map, then the contraction at about
//           95 TFLOP/s, but never faster than its serial K loop (3 us per step of 32 per round of
//           512 work items), plus the pass that adds the K splits.
struct DenseRoute { bool use; uint32_t idx_bits; uint64_t pitch; size_t idx_bytes, bytes; };

DenseRoute dense_route(const hac_desc_t* desc, int64_t B, const hac_launch_t* launch)
{
    DenseRoute r = { false, 0, 0, 0, 0 };
    const uint64_t k_tot = (uint64_t)desc->k_sym + (desc->format == HAC_FORMAT_SHAC ? 1 : 0);
    if (k_tot > 65536 || B < 1) return r;
    r.idx_bits = k_tot <= 256 ? 8 : 16;
    r.pitch = (desc->m + 15) / 16 * 16;
    r.idx_bytes = (size_t)((desc->n * r.pitch * (r.idx_bits / 8) + 255) / 256 * 256);
    const hac_internal::GemmPlan plan = hac_internal::plan_index_gemm((uint32_t)B, (uint32_t)desc->n, (uint32_t)desc->m);
    r.bytes = r.idx_bytes + ((plan.part_bytes + 255) / 256 * 256);
    const uint32_t force = launch ? launch->variant & (HAC_LAUNCH_SPARSE_ROUTE | HAC_LAUNCH_DENSE_ROUTE) : 0u;
    if (force == HAC_LAUNCH_DENSE_ROUTE) { r.use = true; return r; }
    if (force == HAC_LAUNCH_SPARSE_ROUTE || B < 32) return r;
    const double nnz = (double)desc->nnz, n = (double)desc->n, m = (double)desc->m, b = (double)B;
    const double bp = (double)((B + 31) / 32 * 32);
    const double blocks = ((m + 15.0) / 16.0) * (double)((B + 255) / 256);
    const double busy = blocks < 256.0 ? blocks : 256.0;
    const double rate = busy * 140e3 < 22e6 ? busy * 140e3 : 22e6;             // bytes per us
    const double sparse_us = 12.0 + nnz * bp * 4.0 / rate + b * n * 8.0 / 3e6;
    const double items = (double)plan.tiles * plan.splits;
    const double rounds = (double)(uint64_t)((items + 511.0) / 512.0);
    const double flops_us = 2.0 * b * n * m / 9.5e7, serial_us = plan.steps_per_split * 3.0 * rounds;
    const double dense_us = 10.0 + nnz / 35e3 + (flops_us > serial_us ? flops_us : serial_us) + (double)plan.part_bytes / 2e6;
    r.use = dense_us < sparse_us;
    return r;
}

} // namespace

#include "hac_rows.h"

namespace {

size_t table_bytes_of(const hac_desc_t* desc)
{
    const uint32_t k4 = (desc->k_sym + 3u) & ~3u;
    return 4ull * (((2u << desc->lut_bits) + 100u + (desc->k_sym <= kCodebookLdsMax ? 2u * k4 : 0u) + 3u) & ~3u);
}

typedef void (*batch_kern_t)(DevBlob, const float*, uint32_t, uint32_t, float*, uint64_t,
                             uint32_t, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t, Epilogue);

// How a layer of a chain is wired (hac_forward); all zero for a plain dot call.
//   xt_in : the input is already feature-major (written by the layer before): no re-layout
//   yt_out: write the result feature-major for the layer after (sparse route only)
//   bias, relu: applied to every finished sum
struct ChainIO {
    const float* xt_in;
    float* yt_out;
    const float* bias;
    uint32_t relu;
};

__global__ void __launch_bounds__(256)
bias_act_kernel(float* __restrict__ Y, uint32_t B, uint32_t m, uint64_t ldy, const float* __restrict__ bias, uint32_t relu)
{
    const uint64_t total = (uint64_t)B * m;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t b = (uint32_t)(i / m), c = (uint32_t)(i - (uint64_t)b * m);
        float v = Y[(uint64_t)b * ldy + c];
        if (bias) v += bias[c];
        if (relu) v = fmaxf(v, 0.0f);
        Y[(uint64_t)b * ldy + c] = v;
    }
}

void launch_bias_act(float* d_Y, uint32_t B, uint32_t m, uint64_t ldy, const float* bias, uint32_t relu, hipStream_t stream)
{
    if (!bias && !relu) return;
    const uint64_t total = (uint64_t)B * m;
    const uint32_t grid = (uint32_t)std::min<uint64_t>((total + 255) / 256, 4096);
    hipLaunchKernelGGL(bias_act_kernel, dim3(grid), dim3(256), 0, stream, d_Y, B, m, ldy, bias, relu);
}

template <bool SHAC, bool EPI>
batch_kern_t pick_batch_kernel(uint32_t nb, bool multipass)
{
    if (nb == 1) return dot_batch_kernel<SHAC, 1, false, EPI>;
    if (nb == 2) return dot_batch_kernel<SHAC, 2, false, EPI>;
    return multipass ? dot_batch_kernel<SHAC, 4, true, EPI> : dot_batch_kernel<SHAC, 4, false, EPI>;
}

// per-wave LDS words for the stream (and ri) words of a wave's columns
uint32_t default_staging_words(const hac_desc_t* desc, uint32_t cpw)
{
    const bool ri_fields = desc->format == HAC_FORMAT_SHAC && desc->ri_coding == HAC_RI_FIELDS;
    double est = ((double)desc->max_col_bits / 32.0 + 2.0) * cpw + 16.0;
    if (ri_fields) est += ((double)desc->max_col_nnz * desc->ri_bits / 32.0 + 2.0) * cpw + 12.0;
    return round_up((uint32_t)(est < 8192.0 ? est : 8192.0), 16);
}

// Batches of 2 to 8 rows and a short X (at most 32 KB once padded to a power of two of rows):
// every block keeps its own feature-major copy of X in LDS, so there is no re-layout launch and
// no workspace.  Measured on 512 x 4096 layers: 7-8 us against 9-10 (4 rows), 10 against 13-14
// (8 rows); with X of 64 KB or more the copies and the lost occupancy cost more than the launch
// (4096 x 4096, 8 rows: 25 against 17 us), and 8 rows with more than half a million non-zeros are
// better off with the list kernel.
struct XldsPlan { bool use; uint32_t nb, wpb, x_words; size_t lds; };

XldsPlan xlds_plan(const hac_desc_t* desc, int64_t B, const hac_launch_t* launch)
{
    XldsPlan p = { false, 0, 0, 0, 0 };
    if (B < 2 || B > 8 || desc->format == HAC_FORMAT_IM) return p;
    uint32_t cpw = default_cpw(desc), wpb = 0, sbuf_words = 0;
    if (launch) {
        if (launch->variant & (HAC_LAUNCH_NO_X_LDS | HAC_LAUNCH_LIST_KERNEL | HAC_LAUNCH_REUSE_XT | HAC_LAUNCH_DENSE_ROUTE)) return p;
        if (launch->cols_per_wave) cpw = launch->cols_per_wave;
        wpb = launch->waves_per_block;
        sbuf_words = launch->staging_words;
    }
    if (!sbuf_words) sbuf_words = default_staging_words(desc, cpw);
    p.nb = B <= 2 ? 2u : B <= 4 ? 4u : 8u;
    if (desc->n * p.nb > 8192) return p;
    if (p.nb == 8 && desc->nnz > (1u << 19)) return p;
    p.x_words = round_up((uint32_t)desc->n * p.nb, 4);
    const uint32_t k4 = (desc->k_sym + 3u) & ~3u;
    const size_t tbl = 4ull * (((2u << desc->lut_bits) + 100u + (desc->k_sym <= kCodebookLdsMax ? 2u * k4 : 0u) + 3u) & ~3u);
    const size_t per_wave = 4ull * (sbuf_words + round_up(cpw * p.nb, 4));
    const size_t fixed = tbl + 4ull * p.x_words;
    const uint32_t nwaves = (uint32_t)((desc->m + cpw - 1) / cpw);
    if (!wpb) {
        for (wpb = 16; wpb > 4 && fixed + wpb * per_wave > kLdsLimit; wpb >>= 1) {}
        while (wpb > 4 && (nwaves + wpb - 1) / wpb < 256) wpb >>= 1;
    }
    p.wpb = wpb;
    p.lds = fixed + (size_t)wpb * per_wave;
    p.use = p.lds <= kLdsLimit;
    return p;
}

int dot_impl(uint32_t format, const hac_desc_t* desc, const void* d_blob,
             const float* d_X, int64_t B, int64_t ldx, float* d_Y, int64_t ldy,
             void* d_ws, size_t ws_bytes, const hac_launch_t* launch, hac_stream_t stream_,
             const ChainIO* io = nullptr)
{
    DevBlob d;
    int rc = make_dev(desc, d_blob, format, d);
    if (rc) return rc;
    if (B < 0 || B > 0x7fffffffll) return HAC_EINVAL;
    if (B == 0) return HAC_OK;
    const ChainIO none = { nullptr, nullptr, nullptr, 0u };
    if (!io) { io = &none; hac_internal::note_reset(); }
    using hac_internal::note_kernel;
    const char* const tf[2] = { "false", "true" };
    if (!io->xt_in && (!d_X || ldx < (int64_t)desc->n)) return HAC_EINVAL;
    if (!io->yt_out && (!d_Y || ldy < (int64_t)desc->m)) return HAC_EINVAL;
    const Epilogue epi = { io->bias, io->yt_out, io->relu };
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    uint32_t cpw = default_cpw(desc), wpb = 0, list_cap = 0, sbuf_words = 0, pass_w = 32, tile_b = kDefaultTile;
    bool reuse_xt = false, list_kernel = false;
    if (launch) {
        if (launch->cols_per_wave > 32 || launch->waves_per_block > 16) return HAC_EINVAL;
        if (launch->cols_per_wave) cpw = launch->cols_per_wave;
        wpb = launch->waves_per_block;
        reuse_xt = (launch->variant & HAC_LAUNCH_REUSE_XT) != 0;
        list_kernel = (launch->variant & HAC_LAUNCH_LIST_KERNEL) != 0;
        const uint32_t routes = HAC_LAUNCH_SPARSE_ROUTE | HAC_LAUNCH_DENSE_ROUTE;
        const uint32_t rowsk = HAC_LAUNCH_ROWS_KERNEL | HAC_LAUNCH_NO_ROWS_KERNEL;
        if (launch->variant & ~(HAC_LAUNCH_REUSE_XT | HAC_LAUNCH_LIST_KERNEL | HAC_LAUNCH_NO_X_LDS | routes | rowsk)) return HAC_EINVAL;
        if ((launch->variant & routes) == routes || (launch->variant & rowsk) == rowsk) return HAC_EINVAL;
        if (launch->sessions_per_block > 65536) return HAC_EINVAL;
        list_cap = launch->list_entries;
        sbuf_words = launch->staging_words;
        if (list_cap && (list_cap < 64 || list_cap > 4096)) return HAC_EINVAL;
        if (sbuf_words && (sbuf_words < 16 || sbuf_words > 16384 || sbuf_words % 4)) return HAC_EINVAL;
        if (launch->pass_width) pass_w = launch->pass_width;
        if (pass_w != 32 && pass_w != 64 && pass_w != 128 && pass_w != 256) return HAC_EINVAL;
        if (launch->free_running > 1) return HAC_EINVAL;
        if (launch->tile_width) tile_b = launch->tile_width;
        if (tile_b != 32 && tile_b != 64 && tile_b != 128 && tile_b != 256) return HAC_EINVAL;
        if (tile_b < pass_w) return HAC_EINVAL;
    }
    const uint32_t nwaves = (d.m + cpw - 1) / cpw;
    const bool shac = format == HAC_FORMAT_SHAC && !d.rice;   // Rice-coded gaps decode like a HAC stream: no ri words
    g_last_hip_error = 0;

    const DenseRoute dr = dense_route(desc, B, launch);
    if (launch && (launch->variant & HAC_LAUNCH_DENSE_ROUTE) && !dr.use) return HAC_EINVAL;   // too many symbols
    if (dr.use) {
        if (io->xt_in || io->yt_out) return HAC_EINVAL;       // the dense route reads and writes row-major
        if (!d_ws || ws_bytes < dr.bytes) return HAC_EWORKSPACE;
        if (reinterpret_cast<uintptr_t>(d_ws) % 256) return HAC_EINVAL;
        // 1. all pointers 0, 2. the pointer of every non-zero, 3. tiles on the matrix cores
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1024), dim3(256), 0, stream, static_cast<uint32_t*>(d_ws),
                           (uint64_t)(dr.idx_bytes / 4), 0u);
        note_kernel("fill_u32_kernel");
        note_kernel("decode_to_index_kernel<unsigned %s>", dr.idx_bits == 8 ? "char" : "short");
        // LDS beside the tables: room for the stream words (and ri fields) of a block's chunks
        const uint32_t s_words = 6144, r_words = (format == HAC_FORMAT_SHAC && !d.rice) ? 6144u : 0u;
        const uint32_t c_words = d.m + 1 <= 8192 ? round_up(d.m + 1, 4) : 0u;       // colchunk, for the owner search
        const size_t lds = 4ull * (table_words(d) + s_words + r_words + c_words);
        const uint32_t grid = (d.n_chunks + 255) / 256;
        const uint32_t is_shac = format == HAC_FORMAT_SHAC ? 1u : 0u;
        if (grid) {
            if (lds > 64 * 1024) {
                const void* f = dr.idx_bits == 8 ? reinterpret_cast<const void*>(decode_to_index_kernel<uint8_t>)
                                                 : reinterpret_cast<const void*>(decode_to_index_kernel<uint16_t>);
                hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                if (e != hipSuccess) return hip_fail(e);
            }
            if (dr.idx_bits == 8)
                hipLaunchKernelGGL(decode_to_index_kernel<uint8_t>, dim3(grid), dim3(256), lds, stream, d,
                                   static_cast<uint8_t*>(d_ws), dr.pitch, is_shac, s_words, r_words, c_words);
            else
                hipLaunchKernelGGL(decode_to_index_kernel<uint16_t>, dim3(grid), dim3(256), lds, stream, d,
                                   static_cast<uint16_t*>(d_ws), dr.pitch, is_shac, s_words, r_words, c_words);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
        float* part = reinterpret_cast<float*>(static_cast<uint8_t*>(d_ws) + dr.idx_bytes);
        e = hac_internal::launch_index_gemm(d_X, (uint64_t)ldx, (uint32_t)B, d_ws, dr.idx_bits, dr.pitch, d.codebook,
                                            d.k_sym, is_shac, d.n, d.m, d_Y, (uint64_t)ldy, part, stream);
        if (e != hipSuccess) return hip_fail(e);
        launch_bias_act(d_Y, (uint32_t)B, d.m, (uint64_t)ldy, io->bias, io->relu, stream);
        e = hipGetLastError();
        return e == hipSuccess ? HAC_OK : hip_fail(e);
    }
    const bool plain = !io->xt_in && !io->yt_out && !io->bias && !io->relu;
    const RowsPlan rk = plain ? plan_rows(desc, B, launch, table_bytes_of(desc)) : RowsPlan{};
    if (launch && (launch->variant & HAC_LAUNCH_ROWS_KERNEL) && !rk.use) return HAC_EINVAL;   // no row index, or it does not fit
    if (rk.use) {
        if (rk.part_bytes) {
            if (!d_ws || ws_bytes < rk.part_bytes) return HAC_EWORKSPACE;
            if (reinterpret_cast<uintptr_t>(d_ws) % 256) return HAC_EINVAL;
        }
        RowsParams rp = rk.rp;
        rp.rent = static_cast<const uint8_t*>(d_blob) + desc->off_row_ent;
        rp.vecx = (reinterpret_cast<uintptr_t>(d_X) % 16 == 0 && ldx % 4 == 0) ? 1u : 0u;
        auto k = shac ? dot_rows_kernel<true> : dot_rows_kernel<false>;
        if (rk.lds > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)rk.lds);
            if (e != hipSuccess) return hip_fail(e);
        }
        float* part = static_cast<float*>(d_ws);
        hipLaunchKernelGGL(k, dim3(rk.grid), dim3(kRowsWaves * 64), rk.lds, stream, d, rp, d_X, (uint64_t)ldx, (uint32_t)B,
                           part, d_Y, (uint64_t)ldy);
        note_kernel("dot_rows_kernel<%s>", tf[shac]);
        if (rp.nparts > 1) {
            hipLaunchKernelGGL(rows_reduce_kernel, dim3((d.m + 15) / 16, rp.tiles), dim3(256), 0, stream,
                               part, rp.nparts, d.m, (uint32_t)B, d_Y, (uint64_t)ldy);
            note_kernel("rows_reduce_kernel");
        }
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? HAC_OK : hip_fail(e);
    }
    const XldsPlan xp = io->xt_in ? XldsPlan{ false, 0, 0, 0, 0 } : xlds_plan(desc, B, launch);
    if (xp.use) {
        // 2 to 8 batch rows and a short X: the block's own copy of X in LDS, lanes multiply what they decode
        if (!sbuf_words) sbuf_words = default_staging_words(desc, cpw);
        const uint32_t sum_words = round_up(cpw * xp.nb, 4);
        const uint32_t nblocks = (nwaves + xp.wpb - 1) / xp.wpb;
        const uint32_t grid = (nblocks + 7) / 8 * 8;
        typedef void (*xlds_kern_t)(DevBlob, const float*, uint32_t, uint64_t, uint32_t, float*, uint64_t,
                                    uint32_t, uint32_t, uint32_t, uint32_t, Epilogue);
        xlds_kern_t k;
        if (xp.nb == 2) k = shac ? dot_small_kernel<true, 2, true> : dot_small_kernel<false, 2, true>;
        else if (xp.nb == 4) k = shac ? dot_small_kernel<true, 4, true> : dot_small_kernel<false, 4, true>;
        else k = shac ? dot_small_kernel<true, 8, true> : dot_small_kernel<false, 8, true>;
        if (xp.lds > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)xp.lds);
            if (e != hipSuccess) return hip_fail(e);
        }
        hipLaunchKernelGGL(k, dim3(grid), dim3(xp.wpb * kWave), xp.lds, stream,
                           d, d_X, (uint32_t)B, (uint64_t)ldx, xp.x_words, d_Y, (uint64_t)ldy, cpw, sbuf_words, sum_words, nblocks, epi);
        note_kernel("dot_small_kernel<%s, %u, true>", tf[shac], xp.nb);
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? HAC_OK : hip_fail(e);
    }
    const BatchShape bs = batch_shape(B, pass_w, tile_b);
    const float* XT = io->xt_in ? io->xt_in : d_X;           // B = 1: X is its own feature-major copy
    if (B > 1 && !io->xt_in) {
        const size_t need = 4ull * d.n * bs.Bp;
        if (!d_ws || ws_bytes < need) return HAC_EWORKSPACE;
        if (reinterpret_cast<uintptr_t>(d_ws) % 256) return HAC_EINVAL;
        float* xt = static_cast<float*>(d_ws);
        XT = xt;
        if (!reuse_xt) {
            if (bs.gw * bs.nb == 32) {
                dim3 grid((d.n + 127) / 128, (uint32_t)((B + 31) / 32));     // panels of padding only are never read
                const uint32_t vec = (reinterpret_cast<uintptr_t>(d_X) % 16 == 0 && ldx % 4 == 0) ? 1u : 0u;
                hipLaunchKernelGGL(transpose_panel32_kernel, grid, dim3(256), 0, stream,
                                   d_X, (uint32_t)B, d.n, (uint64_t)ldx, xt, vec);
                note_kernel("transpose_panel32_kernel");
            } else {
                dim3 grid((d.n + 31) / 32, (bs.Bp + 31) / 32);
                hipLaunchKernelGGL(transpose_pad_kernel, grid, dim3(256), 0, stream,
                                   d_X, (uint32_t)B, d.n, (uint64_t)ldx, xt, bs.Bp, bs.gw * bs.nb);
                note_kernel("transpose_pad_kernel");
            }
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return hip_fail(e);
        }
    }
    // per-wave LDS: the stream (and ri) words of the wave's columns, and the list of one batch's non-zeros
    if (!sbuf_words) sbuf_words = default_staging_words(desc, cpw);
    if (!list_cap) {
        double est = (double)desc->max_col_nnz * cpw;
        // (with chunk sizes per column a column has at most 64 chunks: a batch then never holds more than the longest column)
        const double one_batch = (desc->chunk & hac_internal::kChunkPerColumn) ? (double)desc->max_col_nnz * cpw
                                                                               : 64.0 * desc->chunk;
        if (est > one_batch) est = one_batch;
        list_cap = round_up((uint32_t)(est < 2048.0 ? (est > 1.0 ? est : 1.0) : 2048.0), 64);
    }
    if (bs.gw == 1 && bs.npass == 1 && !list_kernel) {
        // at most 4 batch columns: lanes multiply what they decode, no list
        const uint32_t sum_words = round_up(cpw * bs.nb, 4);
        const size_t per_wave_s = 4ull * (sbuf_words + sum_words);
        const size_t tbl = 4ull * table_words(d);
        if (!wpb) {
            // blocks of 4 waves: the barrier behind the tables then waits for 4 waves instead of 16
            // (the largest layer here at B = 1: 15.7 -> 15.2 us, address map 11.8 -> 11.3 us)
            for (wpb = 4; wpb > 1 && tbl + wpb * per_wave_s > kLdsLimit; wpb >>= 1) {}
            // a narrow matrix: smaller blocks, so that they reach more of the 256 CUs
            while (wpb > 4 && (nwaves + wpb - 1) / wpb < 256) wpb >>= 1;
        }
        const size_t lds = tbl + (size_t)wpb * per_wave_s;
        if (lds > kLdsLimit) return HAC_EINVAL;
        const uint32_t nblocks = (nwaves + wpb - 1) / wpb;
        const uint32_t grid = (nblocks + 7) / 8 * 8;
        typedef void (*small_kern_t)(DevBlob, const float*, uint32_t, uint64_t, uint32_t, float*, uint64_t,
                                     uint32_t, uint32_t, uint32_t, uint32_t, Epilogue);
        small_kern_t k;
        if (bs.nb == 1) k = shac ? dot_small_kernel<true, 1, false> : dot_small_kernel<false, 1, false>;
        else if (bs.nb == 2) k = shac ? dot_small_kernel<true, 2, false> : dot_small_kernel<false, 2, false>;
        else k = shac ? dot_small_kernel<true, 4, false> : dot_small_kernel<false, 4, false>;
        if (lds > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return hip_fail(e);
        }
        hipLaunchKernelGGL(k, dim3(grid), dim3(wpb * kWave), lds, stream,
                           d, XT, (uint32_t)B, (uint64_t)0, 0u, d_Y, (uint64_t)ldy, cpw, sbuf_words, sum_words, nblocks, epi);
        note_kernel("dot_small_kernel<%s, %u, false>", tf[shac], bs.nb);
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? HAC_OK : hip_fail(e);
    }
    // a column that exceeds the list window (or the 64 chunks of one batch) parks partial sums in LDS
    // (no split is possible when all chunks of a wave fit one batch of 64 and all its non-zeros one window)
    // most chunks in one column (with chunk sizes per column: never more than 64)
    const uint32_t chunk_least = hac_internal::chunk_base(desc->chunk);
    uint64_t col_chunks = (desc->max_col_nnz + chunk_least - 1) / chunk_least;
    if ((desc->chunk & hac_internal::kChunkPerColumn) && col_chunks > 64) col_chunks = 64;
    const bool may_split = (uint64_t)cpw * col_chunks > 64 || (uint64_t)cpw * desc->max_col_nnz > list_cap;
    const uint32_t part_words = may_split ? bs.npass * bs.nb * 64u : 0u;
    const size_t per_wave = 4ull * sbuf_words + 8ull * list_cap + 4ull * part_words;
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
        // a single pass has no barrier between passes to keep in step: two blocks of 8 waves per CU
        // do slightly better than one of 16 (22.4 against 23.0 us at B = 32), the multi-pass kernel
        // does worse with them (107.3 against 103.6 us at B = 256)
        if (bs.npass == 1 && wpb == 16 && (uint32_t)(kLdsLimit / (tbl + 8 * per_wave)) * 8 >= best_waves) wpb = 8;
        // a narrow matrix: smaller blocks, so that they reach more of the 256 CUs (each CU gathers
        // through its own vector memory path; measured on a 4096 x 1000 layer at B = 64: 27 -> 17 us)
        while (wpb > 4 && (uint64_t)((nwaves + wpb - 1) / wpb) * bs.tiles < 256) wpb >>= 1;
    }
    const size_t lds = 4ull * table_words(d) + (size_t)wpb * per_wave;
    if (lds > kLdsLimit) return HAC_EINVAL;
    uint32_t sync_passes = (bs.npass > 1 && cpw == 1 && !may_split) ? 1u : 0u;
    if (launch && launch->free_running == 1) sync_passes = 0;           // measurement aid: free-running passes
    const uint32_t nblocks = (nwaves + wpb - 1) / wpb;
    const uint64_t items = (uint64_t)nblocks * bs.tiles;
    if (items > 0x7ffffff0ull) return HAC_EINVAL;
    const uint32_t grid = (uint32_t)((items + 7) / 8 * 8);
    const bool with_epilogue = io->bias || io->relu || io->yt_out;
    batch_kern_t k = with_epilogue
        ? (shac ? pick_batch_kernel<true, true>(bs.nb, bs.npass > 1) : pick_batch_kernel<false, true>(bs.nb, bs.npass > 1))
        : (shac ? pick_batch_kernel<true, false>(bs.nb, bs.npass > 1) : pick_batch_kernel<false, false>(bs.nb, bs.npass > 1));
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return hip_fail(e);
    }
    hipLaunchKernelGGL(k, dim3(grid), dim3(wpb * kWave), lds, stream,
                       d, XT, bs.Bp, (uint32_t)B, d_Y, (uint64_t)ldy, cpw, bs.gw, bs.npass, list_cap, sbuf_words, part_words, nblocks,
                       sync_passes, epi);
    note_kernel("dot_batch_kernel<%s, %u, %s, %s>", tf[shac], bs.nb, tf[bs.nb == 4 && bs.npass > 1], tf[with_epilogue]);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? HAC_OK : hip_fail(e);
}

} // namespace

extern "C" size_t hac_workspace_bytes_for(const hac_desc_t* desc, int64_t B, const hac_launch_t* launch)
{
    if (!desc_plausible(desc) || B <= 0 || B > 0x7fffffffll) return 0;
    if (desc->format == HAC_FORMAT_IM)
        return hac_internal::plan_index_gemm((uint32_t)B, (uint32_t)desc->n, (uint32_t)desc->m).part_bytes;
    const DenseRoute dr = dense_route(desc, B, launch);
    if (dr.use) return dr.bytes;
    const RowsPlan rk = plan_rows(desc, B, launch, table_bytes_of(desc));
    if (rk.use) return rk.part_bytes;
    if (B == 1) return 0;                                    // a single row is its own feature-major copy
    if (xlds_plan(desc, B, launch).use) return 0;            // X is copied into LDS by every block
    const BatchShape bs = batch_shape(B, 32, kDefaultTile);
    return (size_t)4 * (size_t)desc->n * bs.Bp;
}

extern "C" int hac_dot_route(const hac_desc_t* desc, int64_t B, const hac_launch_t* launch)
{
    if (!desc_plausible(desc) || B < 0 || B > 0x7fffffffll || desc->format == HAC_FORMAT_IM) return HAC_EINVAL;
    return dense_route(desc, B, launch).use ? HAC_ROUTE_DENSE : HAC_ROUTE_SPARSE;
}

namespace {

int im_dot_impl(const hac_desc_t* desc, const void* d_blob, const float* d_X, int64_t B, int64_t ldx,
                float* d_Y, int64_t ldy, void* d_ws, size_t ws_bytes, hac_stream_t stream,
                const float* bias, uint32_t relu)
{
    if (!desc || !d_blob || !desc_plausible(desc)) return HAC_EINVAL;
    if (desc->format != HAC_FORMAT_IM) return HAC_EINVAL;
    if (reinterpret_cast<uintptr_t>(d_blob) % 256) return HAC_EINVAL;
    if (desc->n > 0x7fffffffull || desc->m > 0x7fffffffull) return HAC_EINVAL;
    if ((desc->ent_bits != 8 && desc->ent_bits != 16) || desc->k_sym < 1 || desc->k_sym > 65536) return HAC_EINVAL;
    if (desc->idx_pitch != (desc->m + 15) / 16 * 16 || desc->off_stream % 256 || desc->off_codebook % 256) return HAC_EINVAL;
    if (B < 0 || B > 0x7fffffffll) return HAC_EINVAL;
    if (B == 0) return HAC_OK;
    if (!d_X || !d_Y || ldx < (int64_t)desc->n || ldy < (int64_t)desc->m) return HAC_EINVAL;
    g_last_hip_error = 0;
    if (!bias && !relu) hac_internal::note_reset();
    const size_t need = hac_internal::plan_index_gemm((uint32_t)B, (uint32_t)desc->n, (uint32_t)desc->m).part_bytes;
    if (need && (!d_ws || ws_bytes < need)) return HAC_EWORKSPACE;
    if (need && reinterpret_cast<uintptr_t>(d_ws) % 256) return HAC_EINVAL;
    const uint8_t* b = static_cast<const uint8_t*>(d_blob);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    hipError_t e = hac_internal::launch_index_gemm(d_X, (uint64_t)ldx, (uint32_t)B, b + desc->off_stream, desc->ent_bits,
                                                   desc->idx_pitch, reinterpret_cast<const float*>(b + desc->off_codebook),
                                                   desc->k_sym, 0u, (uint32_t)desc->n, (uint32_t)desc->m, d_Y,
                                                   (uint64_t)ldy, static_cast<float*>(d_ws), hs);
    if (e != hipSuccess) return hip_fail(e);
    launch_bias_act(d_Y, (uint32_t)B, (uint32_t)desc->m, (uint64_t)ldy, bias, relu, hs);
    e = hipGetLastError();
    return e == hipSuccess ? HAC_OK : hip_fail(e);
}

// ---- chain of layers -------------------------------------------------------------------
// Between two layers that both take the sparse route the activations stay feature-major (the
// layout the FMA phase gathers from), so only the chain's input is re-laid out; a layer on the
// dense route (or an index map) reads and writes row-major.
struct ChainPlan {
    uint32_t Bp;
    size_t act_bytes;            // one activation buffer (there are two)
    size_t scratch_bytes;        // the largest per-layer workspace
    bool sparse[256];            // kMaxChain entries: the layer takes the sparse route
    bool wants_xt[256];          // ... and gathers from a feature-major copy of its input in global memory
};
constexpr uint32_t kMaxChain = 256;

bool layer_sparse(const hac_desc_t* desc, int64_t B)
{
    return desc->format != HAC_FORMAT_IM && !dense_route(desc, B, nullptr).use;
}

int plan_chain(const hac_layer_t* layers, uint32_t L, int64_t B, ChainPlan& P)
{
    if (!layers || L < 1 || L > kMaxChain || B < 0 || B > 0x7fffffffll) return HAC_EINVAL;
    P.Bp = B ? batch_shape(B, 32, kDefaultTile).Bp : 0;
    P.act_bytes = 0; P.scratch_bytes = 0;
    for (uint32_t l = 0; l < L; ++l) {
        const hac_desc_t* d = layers[l].desc;
        if (!d || !layers[l].d_blob || layers[l].activation > HAC_ACT_RELU || layers[l].reserved) return HAC_EINVAL;
        if (d->magic != 0x31434148u || d->version != 2) return HAC_EINVAL;
        if (d->format != HAC_FORMAT_HAC && d->format != HAC_FORMAT_SHAC && d->format != HAC_FORMAT_IM) return HAC_EINVAL;
        if (!desc_plausible(d)) return HAC_EINVAL;
        if (l && d->n != layers[l - 1].desc->m) return HAC_EINVAL;
    }
    if (!B) return HAC_OK;
    for (uint32_t l = 0; l < L; ++l) {
        const hac_desc_t* d = layers[l].desc;
        P.sparse[l] = layer_sparse(d, B);
        P.wants_xt[l] = P.sparse[l] && !xlds_plan(d, B, nullptr).use;
        if (l + 1 < L) P.act_bytes = std::max<size_t>(P.act_bytes, (size_t)4 * P.Bp * (size_t)d->m);
    }
    P.act_bytes = (P.act_bytes + 255) / 256 * 256;
    for (uint32_t l = 0; l < L; ++l) {
        const bool fed = l && P.sparse[l - 1] && P.wants_xt[l];      // input arrives feature-major
        const size_t need = fed ? 0 : hac_workspace_bytes_for(layers[l].desc, B, nullptr);
        P.scratch_bytes = std::max(P.scratch_bytes, (need + 255) / 256 * 256);
    }
    return HAC_OK;
}

} // namespace

extern "C" int im_dot(const hac_desc_t* desc, const void* d_blob, const float* d_X, int64_t B, int64_t ldx,
                      float* d_Y, int64_t ldy, void* d_ws, size_t ws_bytes,
                      const hac_launch_t* launch, hac_stream_t stream)
{
    if (launch) return HAC_EINVAL;
    return im_dot_impl(desc, d_blob, d_X, B, ldx, d_Y, ldy, d_ws, ws_bytes, stream, nullptr, 0u);
}

extern "C" size_t hac_forward_workspace_bytes(const hac_layer_t* layers, uint32_t n_layers, int64_t B)
{
    ChainPlan P;
    if (plan_chain(layers, n_layers, B, P) != HAC_OK || !B) return 0;
    return (n_layers > 1 ? 2 * P.act_bytes : 0) + P.scratch_bytes;
}

extern "C" int hac_forward(const hac_layer_t* layers, uint32_t n_layers, const float* d_X, int64_t B, int64_t ldx,
                           float* d_Y, int64_t ldy, void* d_ws, size_t ws_bytes, hac_stream_t stream)
{
    ChainPlan P;
    int rc = plan_chain(layers, n_layers, B, P);
    if (rc) return rc;
    if (B == 0) return HAC_OK;
    if (!d_X || !d_Y || ldx < (int64_t)layers[0].desc->n || ldy < (int64_t)layers[n_layers - 1].desc->m) return HAC_EINVAL;
    const size_t need = (n_layers > 1 ? 2 * P.act_bytes : 0) + P.scratch_bytes;
    if (need && (!d_ws || ws_bytes < need)) return HAC_EWORKSPACE;
    if (need && reinterpret_cast<uintptr_t>(d_ws) % 256) return HAC_EINVAL;
    uint8_t* ws = static_cast<uint8_t*>(d_ws);
    float* act[2] = { reinterpret_cast<float*>(ws), reinterpret_cast<float*>(ws + P.act_bytes) };
    void* scratch = P.scratch_bytes ? ws + (n_layers > 1 ? 2 * P.act_bytes : 0) : nullptr;
    for (uint32_t l = 0; l < n_layers; ++l) {
        const hac_layer_t& ly = layers[l];
        const hac_desc_t* d = ly.desc;
        const bool fed = l && P.sparse[l - 1] && P.wants_xt[l];
        const bool feeds = l + 1 < n_layers && P.sparse[l] && P.wants_xt[l + 1];
        const float* in = l ? act[(l - 1) & 1] : d_X;
        const int64_t ld_in = l ? (int64_t)d->n : ldx;
        float* out = l + 1 < n_layers ? act[l & 1] : d_Y;
        const int64_t ld_out = l + 1 < n_layers ? (int64_t)d->m : ldy;
        const uint32_t relu = ly.activation == HAC_ACT_RELU ? 1u : 0u;
        if (d->format == HAC_FORMAT_IM) {
            rc = im_dot_impl(d, ly.d_blob, in, B, ld_in, out, ld_out, scratch, P.scratch_bytes, stream, ly.d_bias, relu);
        } else {
            const ChainIO io = { fed ? in : nullptr, feeds ? out : nullptr, ly.d_bias, relu };
            rc = dot_impl(d->format, d, ly.d_blob, in, B, ld_in, out, ld_out, scratch, P.scratch_bytes, nullptr, stream, &io);
        }
        if (rc) return rc;
    }
    return HAC_OK;
}

extern "C" size_t hac_workspace_bytes(const hac_desc_t* desc, int64_t B)
{
    if (!desc || B <= 0) return 0;
    return hac_workspace_bytes_for(desc, B, nullptr);
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

// ---- a dot call for callers that cannot allocate ------------------------------------------
// The workspace of hac_dot / shac_dot (the feature-major copy of X, or the dense route's index
// map and partial sums) lives in this file-scope device array instead of caller memory.  Every
// GPU holds its own copy of the array at its own address: host code asks the runtime for that
// address once per device and passes it on like any other workspace pointer; the array's name
// itself is never handed to a kernel.
constexpr size_t kStaticWsBytes = HAC_NOALLOC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Address of `scratch` on the current device (looked up on the first call there, then kept).
int static_workspace(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return HAC_EINVAL;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e != hipSuccess ? e : hipErrorInvalidSymbol);
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // two threads racing here store the same address
    }
    *out = p;
    return HAC_OK;
}
} // namespace

extern "C" int hac_dot_noalloc(const hac_desc_t* desc, const void* d_blob, const float* d_X, int64_t B, int64_t ldx,
                               float* d_Y, int64_t ldy, const hac_launch_t* launch, hac_stream_t stream)
{
    if (!desc_plausible(desc) || (desc->format != HAC_FORMAT_HAC && desc->format != HAC_FORMAT_SHAC)) return HAC_EINVAL;
    if (B < 0 || B > 0x7fffffffll) return HAC_EINVAL;
    const size_t need = hac_workspace_bytes_for(desc, B, launch);
    if (need > kStaticWsBytes) return HAC_EWORKSPACE;
    void* ws = nullptr;
    if (need) {
        const int rc = static_workspace(&ws);
        if (rc) return rc;
    }
    return dot_impl(desc->format, desc, d_blob, d_X, B, ldx, d_Y, ldy, ws, need ? kStaticWsBytes : 0, launch, stream);
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
    if (grid) hipLaunchKernelGGL(decode_kernel<false>, dim3(grid), dim3(256), lds, stream, d, d_W, d_sym,
                                 static_cast<int32_t*>(nullptr), static_cast<int32_t*>(nullptr));
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
    if (grid) hipLaunchKernelGGL(decode_kernel<true>, dim3(grid), dim3(256), lds, stream, d, d_nz, d_sym, d_row, d_col);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? HAC_OK : hip_fail(e);
}

extern "C" int hac_last_hip_error(void) { return g_last_hip_error; }

namespace { thread_local char g_kernels[512]; thread_local size_t g_kernels_len = 0; }

void hac_internal::note_reset() { g_kernels[0] = 0; g_kernels_len = 0; }

void hac_internal::note_kernel(const char* fmt, ...)
{
    if (g_kernels_len + 4 >= sizeof g_kernels) return;
    if (g_kernels_len) { memcpy(g_kernels + g_kernels_len, "; ", 3); g_kernels_len += 2; }
    va_list ap;
    va_start(ap, fmt);
    const int w = vsnprintf(g_kernels + g_kernels_len, sizeof g_kernels - g_kernels_len, fmt, ap);
    va_end(ap);
    if (w > 0) g_kernels_len = std::min(sizeof g_kernels - 1, g_kernels_len + (size_t)w);
}

extern "C" const char* hac_last_kernels(void) { return g_kernels; }

void hac_internal::set_last_hip_error(int e) { g_last_hip_error = e; }

#ifdef HAC_PHASE_TIMING
extern "C" int hac_debug_phases(unsigned long long* out, size_t count)
{
    if (count > 16384 * 8) count = 16384 * 8;
    return hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase), count * sizeof(unsigned long long)) == hipSuccess ? 0 : -5;
}
#endif
