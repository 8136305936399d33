// Dense-tile product for an index-mapped matrix on gfx950 (MI355X):
//     Y[b][j] = sum_i X[b][i] * c[Pi[i][j]]
// (arXiv 2108.12704 Sect. III-C1: representatives in a vector c, pointers to them
// in the index map Pi; the form the paper uses for layers that are quantized but
// hardly pruned, where the product really is a dense contraction).
//
// The pointers are what is read from memory (1 or 2 bytes per weight); a tile of
// them is turned into fp32 through a copy of c in LDS and multiplied on the
// matrix cores with v_mfma_f32_32x32x2_f32 (fp32 in, fp32 accumulate, so the
// result keeps the accuracy of the vector path).
//
// Tiling: a block of 4 wavefronts owns 32 RT batch rows x 128 columns of Y
// (RT = 2..8, chosen per launch so that the tiles fill the 256 CUs evenly) and
// walks K = n in steps of 32; wavefront w owns the 32 columns [32 w, 32 w + 32)
// of the tile and all its rows, as RT MFMA tiles (16 RT accumulator registers).
// LDS holds the X tile row-major (a batch row's 32 k values side by side, rows 36
// floats apart) and the decoded W tile k-major (32 consecutive columns of one k);
// both are double buffered, the next tile's global loads are issued before the
// MFMA loop of the current one and stored during its second half.
// Lane layout of the instruction (checked on the device): A operand lane l holds
// A[i = l % 32][k = l / 32], B operand lane l holds B[k = l / 32][j = l % 32],
// accumulator register v of lane l is D[(v % 4) + 8 (v / 4) + 4 (l / 32)][l % 32].
// The order of k inside a step is free as long as both operands agree: matrix
// instruction kk of a step multiplies k = kk (lanes 0..31) and k = 16 + kk (lanes
// 32..63), so a lane's 16 A values of a step are 16 consecutive floats of its row:
// four 128-bit LDS reads instead of sixteen 32-bit ones, and the thread that
// fetched four consecutive k of a row from X stores them with one 128-bit write.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hac_internal.h"

namespace {

constexpr int BN = 128, BK = 32;
constexpr int LDB = BN + 4;                        // LDS row pitch of the W tile (floats)
constexpr int LDA = BK + 4;                        // LDS row pitch of the X tile: 36 floats, so that 16 lanes'
                                                   // 128-bit accesses to 16 rows fall on 64 different banks
constexpr int kMinRT = 2, kMaxRT = 8;              // row tiles of 32 per block
constexpr uint32_t kLutLdsMax = 4096;              // representatives kept in LDS

typedef float f32x16 __attribute__((ext_vector_type(16)));

template <typename IdxT> struct IdxRegs;
template <> struct IdxRegs<uint8_t> { uint4 v[1]; };
template <> struct IdxRegs<uint16_t> { uint4 v[2]; };

__device__ __forceinline__ uint32_t logical_tile(uint32_t tiles_padded)
{
    // consecutive logical tiles on one XCD: the column tiles of a row tile share X rows in that L2
    const uint32_t per = tiles_padded >> 3;
    return (blockIdx.x & 7u) * per + (blockIdx.x >> 3);
}

template <typename IdxT, bool LUT_LDS, int RT, bool XVEC>
__global__ void __launch_bounds__(256)
index_gemm_kernel(const float* __restrict__ X, uint64_t ldx, uint32_t B,
                  const IdxT* __restrict__ idx, uint64_t pitch,          // pitch in elements, a multiple of 16
                  const float* __restrict__ codebook, uint32_t k_sym, uint32_t zero_first,
                  uint32_t n, uint32_t m, float* __restrict__ Y, uint64_t ldy,
                  uint32_t tiles_n, uint32_t tiles, uint32_t x_vec,
                  uint32_t splits, uint32_t steps_per_split, float* __restrict__ part)
{
    constexpr int BM = 32 * RT;
    extern __shared__ float lds[];
    float* As = lds;                                   // [2][BM][LDA]
    float* Bs = lds + 2 * BM * LDA;                    // [2][BK][LDB]
    float* lut = Bs + 2 * BK * LDB;                    // [k_sym + zero_first] when LUT_LDS
    // work item = (tile, K split); with more than one split a block writes its partial tile to
    // part[split][B][m] and a second kernel adds the splits in order
    const uint32_t item = logical_tile(gridDim.x);
    if (item >= tiles * splits) return;
    const uint32_t tile = item / splits, split = item - tile * splits;
    const uint32_t tm = tile / tiles_n, tn = tile - tm * tiles_n;
    const uint32_t m0 = tm * BM, n0 = tn * BN;
    const uint32_t t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const uint32_t l32 = lane & 31, half = lane >> 5;

    // pointer -> value table: entry 0 is 0.0 when the pointers were written with an offset of one
    const uint32_t k_tot = k_sym + zero_first;
    if (LUT_LDS) {
        for (uint32_t i = t; i < k_tot; i += 256)
            lut[i] = (zero_first && i == 0) ? 0.0f : codebook[i - zero_first];
    }
    auto value_of = [&](uint32_t p) -> float {
        if (LUT_LDS) return lut[p];
        return (zero_first && p == 0) ? 0.0f : codebook[p - zero_first];
    };

    // global -> register staging of one K step; two sets, so that a tile's loads are issued two
    // steps before the tile is needed (one whole step before its stores to LDS begin)
    struct Stage { float4 ra[RT]; IdxRegs<IdxT> rb; };
    const uint32_t a_row = t >> 3, a_kq = t & 7;       // rows a_row + 32 r, k = 4 a_kq .. 4 a_kq + 3
    const uint32_t b_k = t >> 3, b_seg = t & 7;        // idx row b_k, columns 16 b_seg .. 16 b_seg + 15
    // Rows past B and index columns past the pitch are read from a clamped, valid address: a K
    // step that lies wholly inside n then issues the same loads on every path, and the wait before
    // a tile's stores can leave the younger tile's loads in flight.  A row past B multiplies a copy
    // of row B - 1; rows of the product are independent and those are never stored.  Only the
    // last, partial K step takes the guarded path.
    const float* xrow[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        const uint32_t row = m0 + a_row + 32 * r;
        xrow[r] = X + (uint64_t)(row < B ? row : B - 1) * ldx + 4 * a_kq;
    }
    const bool col_ok = n0 + 16 * b_seg < pitch;
    const IdxT* icol = idx + (col_ok ? n0 + 16 * b_seg : 0);
    constexpr int NV = sizeof(IdxT) == 1 ? 1 : 2;
    // a K step that lies wholly inside n: the same loads on every path
    auto load_full = [&](uint32_t k0, Stage& st) {
        if (XVEC) {
#pragma unroll
            for (int r = 0; r < RT; ++r) st.ra[r] = *reinterpret_cast<const float4*>(xrow[r] + k0);
        } else {
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const float* p = xrow[r] + k0;
                st.ra[r] = make_float4(p[0], p[1], p[2], p[3]);
            }
        }
        const uint4* p = reinterpret_cast<const uint4*>(icol + (uint64_t)(k0 + b_k) * pitch);
#pragma unroll
        for (int q = 0; q < NV; ++q) st.rb.v[q] = p[q];
    };
    // the last, partial K step: guarded element by element
    auto load_tail = [&](uint32_t k0, Stage& st) {
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            const uint32_t k = k0 + 4 * a_kq;
            const float* p = xrow[r] + k0;
            float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (k < n) v.x = p[0];
            if (k + 1 < n) v.y = p[1];
            if (k + 2 < n) v.z = p[2];
            if (k + 3 < n) v.w = p[3];
            st.ra[r] = v;
        }
#pragma unroll
        for (int q = 0; q < NV; ++q) st.rb.v[q] = make_uint4(0, 0, 0, 0);
        if (k0 + b_k < n) {
            const uint4* p = reinterpret_cast<const uint4*>(icol + (uint64_t)(k0 + b_k) * pitch);
#pragma unroll
            for (int q = 0; q < NV; ++q) st.rb.v[q] = p[q];
        }
    };
    // registers -> LDS in pieces, so that the work can be spread over the MFMA loop
    auto store_a = [&](uint32_t buf, int r, const Stage& st) {          // rows a_row + 32 r of the X tile
        float* a = As + buf * BM * LDA + (a_row + 32 * r) * LDA + 4 * a_kq;
        *reinterpret_cast<float4*>(a) = make_float4(st.ra[r].x, st.ra[r].y, st.ra[r].z, st.ra[r].w);
    };
    // pointers -> values (columns 16 b_seg + 4 q .. + 3 of the W tile), then values -> LDS: two steps,
    // so that the table lookups can be issued some matrix instructions before their results are stored
    auto lookup_b = [&](int q, const Stage& st) -> float4 {
        float4 o;
        if constexpr (sizeof(IdxT) == 1) {
            const uint32_t u = q == 0 ? st.rb.v[0].x : q == 1 ? st.rb.v[0].y : q == 2 ? st.rb.v[0].z : st.rb.v[0].w;
            o.x = value_of(u & 255u); o.y = value_of((u >> 8) & 255u);
            o.z = value_of((u >> 16) & 255u); o.w = value_of(u >> 24);
        } else {
            const uint4 v = st.rb.v[q >> 1];
            const uint32_t u0 = (q & 1) ? v.z : v.x, u1 = (q & 1) ? v.w : v.y;
            o.x = value_of(u0 & 65535u); o.y = value_of(u0 >> 16);
            o.z = value_of(u1 & 65535u); o.w = value_of(u1 >> 16);
        }
        return o;
    };
    auto store_b = [&](uint32_t buf, int q, const float4& o) {
        float* b = Bs + buf * BK * LDB + b_k * LDB + 16 * b_seg;
        *reinterpret_cast<float4*>(b + 4 * q) = o;
    };

    f32x16 acc[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;

    const uint32_t all_steps = (n + BK - 1) / BK;
    const uint32_t kt0 = split * steps_per_split;
    const uint32_t ksteps = kt0 + steps_per_split < all_steps ? kt0 + steps_per_split : all_steps;   // one past the last

    // Multiply the tile in LDS buffer `buf`; with STORE, meanwhile move the tile held in `st` to the
    // other buffer (nobody reads it during this step), a piece at a time between the matrix
    // instructions.
    auto multiply = [&](uint32_t buf, bool store, const Stage& st) {
        const float* a = As + buf * BM * LDA + l32 * LDA + 16 * half;
        const float* b = Bs + buf * BK * LDB + wave * 32 + l32 + 16 * half * LDB;
        // a quarter step's operands (4 k per lane) are fetched from LDS before the matrix
        // instructions of the quarter before issue
        float4 av[RT];
        float bv[4];
        float4 wv[4];                                  // the next W tile's values between lookup and store
#pragma unroll
        for (int q = 0; q < 4; ++q) wv[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
        for (int i = 0; i < RT; ++i) av[i] = *reinterpret_cast<const float4*>(a + 32 * i * LDA);
#pragma unroll
        for (int j = 0; j < 4; ++j) bv[j] = b[j * LDB];
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            float4 nav[RT];
            float nbv[4];
#pragma unroll
            for (int i = 0; i < RT; ++i) nav[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
            for (int j = 0; j < 4; ++j) nbv[j] = 0.0f;
            if (qd + 1 < 4) {
#pragma unroll
                for (int i = 0; i < RT; ++i) nav[i] = *reinterpret_cast<const float4*>(a + 32 * i * LDA + 4 * (qd + 1));
#pragma unroll
                for (int j = 0; j < 4; ++j) nbv[j] = b[(4 * (qd + 1) + j) * LDB];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int kk = 4 * qd + j;
                __builtin_amdgcn_sched_barrier(0);     // keep the LDS reads ahead of the matrix instructions
#pragma unroll
                for (int i = 0; i < RT; ++i) {
                    const float ak = j == 0 ? av[i].x : j == 1 ? av[i].y : j == 2 ? av[i].z : av[i].w;
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(ak, bv[j], acc[i], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (store) {
                    if (kk >= 2 && kk - 2 < RT) store_a(buf ^ 1, kk - 2, st);
                    if (kk >= 6 && kk < 10) wv[kk - 6] = lookup_b(kk - 6, st);
                    if (kk >= 8 && kk < 12) store_b(buf ^ 1, kk - 8, wv[kk - 8]);
                }
            }
#pragma unroll
            for (int i = 0; i < RT; ++i) av[i] = nav[i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = nbv[j];
        }
    };
    auto store_all = [&](uint32_t buf, const Stage& st) {
#pragma unroll
        for (int r = 0; r < RT; ++r) store_a(buf, r, st);
#pragma unroll
        for (int q = 0; q < 4; ++q) store_b(buf, q, lookup_b(q, st));
    };

    // Full K steps [kt0, kfull) are pipelined: while tile kt is multiplied, tile kt + 1 (requested a
    // step earlier) moves to LDS and tile kt + 2 is requested.  A partial last step follows on its own.
    const uint32_t nfull = n / BK;
    const uint32_t kfull = ksteps < nfull ? ksteps : nfull;
    Stage s0, s1;
    __syncthreads();                                   // the table is complete before the first lookup
    if (kt0 < kfull) {
        load_full(kt0 * BK, s0);
        if (kt0 + 1 < kfull) load_full((kt0 + 1) * BK, s1);
        store_all(kt0 & 1, s0);
        __syncthreads();
        for (uint32_t kt = kt0; kt < kfull; kt += 2) {
            if (kt + 2 < kfull) load_full((kt + 2) * BK, s0);
            multiply(kt & 1, kt + 1 < kfull, s1);
            __syncthreads();
            if (kt + 1 < kfull) {
                if (kt + 3 < kfull) load_full((kt + 3) * BK, s1);
                multiply((kt + 1) & 1, kt + 2 < kfull, s0);
                __syncthreads();
            }
        }
    }
    if (kfull < ksteps && kfull >= kt0) {              // the partial step (n is not a multiple of 32)
        load_tail(kfull * BK, s0);
        store_all(kfull & 1, s0);
        __syncthreads();
        multiply(kfull & 1, false, s0);
    }

    const uint32_t col = n0 + wave * 32 + l32;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t row = m0 + i * 32 + (v & 3) + 8 * (v >> 2) + 4 * half;
            if (row < B && col < m) {
                if (splits == 1) Y[(uint64_t)row * ldy + col] = acc[i][v];
                else part[((uint64_t)split * B + row) * m + col] = acc[i][v];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Small batches (at most 32 rows of X, in groups of 8 along the grid's y): nothing much for the
// matrix cores to do; the index map is read straight through, once per group of 8 batch rows
// (from L2 after the first), and every pointer is used for the group's rows.  A block of 256
// threads owns 256 columns and a range of rows of W: thread (c, g) walks the rows g, g + 4, ...
// of the range for the four columns 4c .. 4c + 3 (one 4- or 8-byte load per row; a wavefront
// reads 256 neighbouring pointers of one row), with the range's X values in LDS (one broadcast
// read per row) and the representatives in LDS.  The four row groups of a block are added in
// LDS, the row ranges by splitk_reduce_kernel: a fixed order.
// ---------------------------------------------------------------------------
constexpr int SB_NB = 8, SB_COLS = 256, SB_GROUPS = 4;     // widest layout: 64 column lanes x 4 row groups
constexpr uint32_t kSmallMaxRows = 1024;           // rows of W per block (32 KB of X in LDS)

template <typename IdxT> struct Ptr4;
template <> struct Ptr4<uint8_t> {
    static __device__ __forceinline__ void ld(const uint8_t* p, uint32_t* out) {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(p);
        out[0] = w & 255u; out[1] = (w >> 8) & 255u; out[2] = (w >> 16) & 255u; out[3] = w >> 24;
    }
};
template <> struct Ptr4<uint16_t> {
    static __device__ __forceinline__ void ld(const uint16_t* p, uint32_t* out) {
        const uint2 w = *reinterpret_cast<const uint2*>(p);
        out[0] = w.x & 65535u; out[1] = w.x >> 16; out[2] = w.y & 65535u; out[3] = w.y >> 16;
    }
};

template <typename IdxT, bool LUT_LDS, bool WIDE>
__global__ void __launch_bounds__(256)
index_small_kernel(const float* __restrict__ X, uint64_t ldx, uint32_t B,
                   const IdxT* __restrict__ idx, uint64_t pitch,
                   const float* __restrict__ codebook, uint32_t k_sym, uint32_t zero_first,
                   uint32_t n, uint32_t m, uint32_t rows_per_split, uint32_t tiles_m, uint32_t splits,
                   uint32_t cl_log2_arg, float* __restrict__ Y, uint64_t ldy, float* __restrict__ part)
{
    const uint32_t cl_log2 = WIDE ? 6u : cl_log2_arg;              // the widest layout with compile-time shapes
    // 2^cl_log2 column lanes (4 columns each) x 256 / 2^cl_log2 row groups: 64 x 4 for a map of 129
    // columns or more, fewer lanes and more row groups for a narrow one, so that its rows are spread
    // over the block's threads instead of leaving most of them idle
    const uint32_t cl = 1u << cl_log2, cols = 4u << cl_log2, groups = 256u >> cl_log2;
    extern __shared__ float lds[];
    float* xs = lds;                                               // [rows_per_split][SB_NB]
    float* red = xs + (size_t)rows_per_split * SB_NB;              // [groups][SB_NB][cols]: 8192 floats in every layout
    float* lut = red + SB_GROUPS * SB_NB * SB_COLS;                // [k_sym + zero_first] when LUT_LDS
    const uint32_t tile = blockIdx.x % tiles_m, split = blockIdx.x / tiles_m;
    const uint32_t b0 = blockIdx.y * SB_NB;                        // this block's batch rows b0 .. b0 + 7
    const uint32_t nb = B - b0 < (uint32_t)SB_NB ? B - b0 : (uint32_t)SB_NB;
    const uint32_t c = threadIdx.x & (cl - 1), g = threadIdx.x >> cl_log2;
    const uint32_t j = tile * cols + 4 * c;                        // first of this thread's four columns
    const uint32_t r0 = split * rows_per_split;
    const uint32_t rows = r0 < n ? (n - r0 < rows_per_split ? n - r0 : rows_per_split) : 0u;
    const uint32_t k_tot = k_sym + zero_first;
    if (LUT_LDS) {
        for (uint32_t i = threadIdx.x; i < k_tot; i += 256)
            lut[i] = (zero_first && i == 0) ? 0.0f : codebook[i - zero_first];
    }
    // a thread stages whole rows: SB_NB coalesced reads (one per batch row), one contiguous store
    for (uint32_t i = threadIdx.x; i < rows; i += 256) {
        float v[SB_NB];
#pragma unroll
        for (int b = 0; b < SB_NB; ++b) v[b] = (uint32_t)b < nb ? X[(uint64_t)(b0 + b) * ldx + r0 + i] : 0.0f;
#pragma unroll
        for (int b = 0; b < SB_NB; ++b) xs[(size_t)i * SB_NB + b] = v[b];
    }
    __syncthreads();
    auto value_of = [&](uint32_t p) -> float {
        if (LUT_LDS) return lut[p];
        return (zero_first && p == 0) ? 0.0f : codebook[p - zero_first];
    };
    float acc[4][SB_NB];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int b = 0; b < SB_NB; ++b) acc[u][b] = 0.0f;
    // the pitch is a multiple of 16 and j of 4: four pointers from j on lie inside the row; those of
    // columns past m are padding (pointer 0) and their sums are never stored
    if (j < pitch) {
        const IdxT* col = idx + (uint64_t)r0 * pitch + j;
        auto row_step = [&](uint32_t i, const uint32_t* p) {
            const float* xr = xs + (size_t)i * SB_NB;
            float x[SB_NB];
#pragma unroll
            for (int b = 0; b < SB_NB; ++b) x[b] = xr[b];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float w = value_of(p[u]);
#pragma unroll
                for (int b = 0; b < SB_NB; ++b) acc[u][b] = fmaf(w, x[b], acc[u][b]);
            }
        };
        uint32_t i = g;
        // four rows at a time: their pointers are requested together, so that a thread with few
        // rows does not pay one trip to memory per row
        for (; i + 3 * groups < rows; i += 4 * groups) {
            uint32_t p[4][4];
#pragma unroll
            for (int q = 0; q < 4; ++q) Ptr4<IdxT>::ld(col + (uint64_t)(i + q * groups) * pitch, p[q]);
#pragma unroll
            for (int q = 0; q < 4; ++q) row_step(i + q * groups, p[q]);
        }
        for (; i < rows; i += groups) {
            uint32_t p[4];
            Ptr4<IdxT>::ld(col + (uint64_t)i * pitch, p);
            row_step(i, p);
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int b = 0; b < SB_NB; ++b) red[(g * SB_NB + b) * cols + 4 * c + u] = acc[u][b];
    __syncthreads();
    // every (batch row, column) of the block: its row groups added in order, the outputs dealt to
    // the threads (256 columns x 8 rows in the widest layout, 16 x 8 with 64 row groups in the narrowest)
    for (uint32_t o = threadIdx.x; o < cols * nb; o += 256) {
        const uint32_t jl = o & (cols - 1), b = o >> (cl_log2 + 2);
        const uint32_t jc = tile * cols + jl;
        if (jc >= m) continue;
        float v = red[b * cols + jl];
        for (uint32_t q = 1; q < groups; ++q) v += red[(q * SB_NB + b) * cols + jl];
        if (splits == 1) Y[(uint64_t)(b0 + b) * ldy + jc] = v;
        else part[((uint64_t)split * B + b0 + b) * m + jc] = v;
    }
}

// Y = part[0] + part[1] + ... in that order (bitwise reproducible).
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const float* __restrict__ part, uint32_t splits, uint32_t B, uint32_t m,
                     float* __restrict__ Y, uint64_t ldy)
{
    const uint64_t total = (uint64_t)B * m;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        float v = part[i];
        uint32_t s = 1;
        for (; s + 3 < splits; s += 4) {                   // four loads in flight, added in order
            const float a = part[(uint64_t)s * total + i], b = part[(uint64_t)(s + 1) * total + i];
            const float c = part[(uint64_t)(s + 2) * total + i], d = part[(uint64_t)(s + 3) * total + i];
            v += a; v += b; v += c; v += d;
        }
        for (; s < splits; ++s) v += part[(uint64_t)s * total + i];
        const uint64_t row = i / m;
        Y[row * ldy + (i - row * m)] = v;
    }
}

} // namespace

namespace hac_internal {

static size_t index_gemm_lds_bytes(uint32_t k_tot, int rt)
{
    return sizeof(float) * (2 * 32 * rt * LDA + 2 * BK * LDB + (k_tot <= kLutLdsMax ? k_tot : 0));
}

GemmPlan plan_index_gemm(uint32_t B, uint32_t n, uint32_t m)
{
    GemmPlan p;
    p.small = B <= 4u * SB_NB;
    if (p.small) {
        // blocks of 256 columns x a range of rows: about 512 blocks, at most 32 ranges (the pass that
        // adds them walks them one after the other) unless the rows of a range would not fit LDS
        // column lanes per row group: 64 (256 columns a block) from 129 columns on, else the power of
        // two that covers the map, at least 4 (p.rt carries its logarithm in this mode)
        uint32_t cl_log2 = 6;
        if (m <= 128) { cl_log2 = 2; while ((4u << cl_log2) < m) ++cl_log2; }
        const uint32_t tiles_m = (m + (4u << cl_log2) - 1) / (4u << cl_log2);
        const uint32_t groups = (B + SB_NB - 1) / SB_NB;
        uint32_t splits = (512 + tiles_m * groups - 1) / (tiles_m * groups);
        const uint32_t most = (n + 31) / 32, least = (n + kSmallMaxRows - 1) / kSmallMaxRows;
        if (splits > 32) splits = 32;
        if (splits > most) splits = most;
        if (splits < least) splits = least;
        if (splits < 1) splits = 1;
        p.steps_per_split = ((n + splits - 1) / splits + 3) / 4 * 4;          // rows per block
        p.splits = (n + p.steps_per_split - 1) / p.steps_per_split;
        p.steps = n; p.rt = cl_log2; p.tiles = tiles_m;
        p.part_bytes = p.splits > 1 ? (size_t)p.splits * B * m * sizeof(float) : 0;
        return p;
    }
    const uint64_t tiles_n = (m + BN - 1) / BN;
    const uint32_t steps = (n + BK - 1) / BK;
    // Row tiles per block: the time of a launch goes like (rounds of tiles over the CUs) x (rows per
    // tile); blocks of up to 4 row tiles fit a CU two at a time and then share its matrix pipes.
    // Pick the shape with the fewest padded rows per CU, the larger tile on ties (less re-reading
    // of the index map).
    int best_rt = kMinRT;
    double best_cost = 1e300;
    for (int rt = kMinRT; rt <= kMaxRT; ++rt) {
        const uint64_t tiles = (uint64_t)((B + 32 * rt - 1) / (32 * rt)) * tiles_n;
        const uint64_t slots = rt <= 4 ? 512 : 256;
        const uint64_t rounds = (tiles + slots - 1) / slots;
        const double cost = (double)rounds * rt * (rt <= 4 ? 2.0 : 1.0);
        if (cost <= best_cost) { best_cost = cost; best_rt = rt; }
    }
    p.rt = (uint32_t)best_rt;
    const uint64_t tiles = (uint64_t)((B + 32 * best_rt - 1) / (32 * best_rt)) * tiles_n;
    // a tile's K loop is serial (about 3 us per step of 32): with tiles for at most half of the
    // CUs, K is split until there are about two work items per CU, keeping at least 8 steps per split
    uint32_t splits = 1;
    if (tiles <= 128) {
        splits = (uint32_t)((512 + tiles - 1) / tiles);
        const uint32_t most = steps / 8 ? steps / 8 : 1;
        if (splits > most) splits = most;
        if (splits > 32) splits = 32;
    }
    p.steps_per_split = (steps + splits - 1) / splits;
    p.splits = (steps + p.steps_per_split - 1) / p.steps_per_split;       // no empty split
    p.part_bytes = p.splits > 1 ? (size_t)p.splits * B * m * sizeof(float) : 0;
    p.tiles = tiles;
    p.steps = steps;
    return p;
}

namespace {

typedef void (*gemm_kern_t)(const float*, uint64_t, uint32_t, const void*, uint64_t, const float*, uint32_t, uint32_t,
                            uint32_t, uint32_t, float*, uint64_t, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t, float*);

template <typename IdxT, bool LUT_LDS, int RT>
void launch_one(dim3 grid, size_t lds, hipStream_t stream, hipError_t& err,
                const float* d_X, uint64_t ldx, uint32_t B, const void* d_idx, uint64_t pitch, const float* d_codebook,
                uint32_t k_sym, uint32_t zero_first, uint32_t n, uint32_t m, float* d_Y, uint64_t ldy, uint32_t tiles_n,
                uint32_t tiles, uint32_t x_vec, uint32_t splits, uint32_t steps_per_split, float* d_part)
{
    auto k = x_vec ? index_gemm_kernel<IdxT, LUT_LDS, RT, true> : index_gemm_kernel<IdxT, LUT_LDS, RT, false>;
    if (lds > 64 * 1024) {
        err = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (err != hipSuccess) return;
    }
    hipLaunchKernelGGL(k, grid, dim3(256), lds, stream, d_X, ldx, B, static_cast<const IdxT*>(d_idx), pitch, d_codebook,
                       k_sym, zero_first, n, m, d_Y, ldy, tiles_n, tiles, x_vec, splits, steps_per_split, d_part);
    note_kernel("index_gemm_kernel<unsigned %s, %s, %d, %s>", sizeof(IdxT) == 1 ? "char" : "short", LUT_LDS ? "true" : "false", RT,
                x_vec ? "true" : "false");
    err = hipGetLastError();
}

template <typename IdxT, bool LUT_LDS, typename... Args>
void launch_rt(uint32_t rt, Args&&... args)
{
    switch (rt) {
    case 2: launch_one<IdxT, LUT_LDS, 2>(args...); break;
    case 3: launch_one<IdxT, LUT_LDS, 3>(args...); break;
    case 4: launch_one<IdxT, LUT_LDS, 4>(args...); break;
    case 5: launch_one<IdxT, LUT_LDS, 5>(args...); break;
    case 6: launch_one<IdxT, LUT_LDS, 6>(args...); break;
    case 7: launch_one<IdxT, LUT_LDS, 7>(args...); break;
    default: launch_one<IdxT, LUT_LDS, 8>(args...); break;
    }
}

} // namespace

hipError_t launch_index_gemm(const float* d_X, uint64_t ldx, uint32_t B, const void* d_idx, uint32_t idx_bits,
                             uint64_t pitch, const float* d_codebook, uint32_t k_sym, uint32_t zero_first,
                             uint32_t n, uint32_t m, float* d_Y, uint64_t ldy, float* d_part, hipStream_t stream)
{
    const uint32_t tiles_n = (m + BN - 1) / BN;
    const GemmPlan plan = plan_index_gemm(B, n, m);
    if (plan.small) {
        if (plan.splits > 1 && !d_part) return hipErrorInvalidValue;
        if (idx_bits != 8 && idx_bits != 16) return hipErrorInvalidValue;
        const uint64_t blocks = plan.tiles * plan.splits;
        if (blocks > 0x7ffffff0ull) return hipErrorInvalidValue;
        const uint32_t k_tot = k_sym + zero_first;
        const bool lut_lds = k_tot <= kLutLdsMax;
        const size_t lds = sizeof(float) * ((size_t)plan.steps_per_split * SB_NB + SB_GROUPS * SB_NB * SB_COLS + (lut_lds ? k_tot : 0));
        if (lds > 160 * 1024) return hipErrorInvalidValue;           // (the plan keeps a range at kSmallMaxRows rows: 32 + 64 + 16 KB at most)
        const dim3 grid((uint32_t)blocks, (B + SB_NB - 1) / SB_NB);
        // (the rows of a range, the partial sums of the row groups and the table can exceed the 64 KB a
        // kernel gets without asking)
        hipError_t attr = hipSuccess;
        auto launch_small = [&](auto kern, auto idxp) {
            if (lds > 64 * 1024) {
                attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                if (attr != hipSuccess) return;
            }
            hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, d_X, ldx, B,
                               idxp, pitch, d_codebook, k_sym, zero_first, n, m,
                               plan.steps_per_split, (uint32_t)plan.tiles, plan.splits, plan.rt, d_Y, ldy, d_part);
            note_kernel("index_small_kernel<unsigned %s, %s, %s>", idx_bits == 8 ? "char" : "short", lut_lds ? "true" : "false",
                        plan.rt == 6 ? "true" : "false");
        };
        const bool narrow = plan.rt == 6;
        const uint8_t* i8 = static_cast<const uint8_t*>(d_idx);
        const uint16_t* i16 = static_cast<const uint16_t*>(d_idx);
        if (idx_bits == 8) {
            if (lut_lds) { if (narrow) launch_small(index_small_kernel<uint8_t, true, true>, i8); else launch_small(index_small_kernel<uint8_t, true, false>, i8); }
            else { if (narrow) launch_small(index_small_kernel<uint8_t, false, true>, i8); else launch_small(index_small_kernel<uint8_t, false, false>, i8); }
        } else {
            if (lut_lds) { if (narrow) launch_small(index_small_kernel<uint16_t, true, true>, i16); else launch_small(index_small_kernel<uint16_t, true, false>, i16); }
            else { if (narrow) launch_small(index_small_kernel<uint16_t, false, true>, i16); else launch_small(index_small_kernel<uint16_t, false, false>, i16); }
        }
        if (attr != hipSuccess) return attr;
        hipError_t e = hipGetLastError();
        if (e != hipSuccess || plan.splits == 1) return e;
        const uint64_t total = (uint64_t)B * m;
        const uint32_t rgrid = (uint32_t)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3(rgrid), dim3(256), 0, stream, d_part, plan.splits, B, m, d_Y, ldy);
        note_kernel("splitk_reduce_kernel");
        return hipGetLastError();
    }
    const uint64_t items64 = plan.tiles * plan.splits;
    if (items64 > 0x7ffffff0ull) return hipErrorInvalidValue;
    if (plan.splits > 1 && !d_part) return hipErrorInvalidValue;
    if (idx_bits != 8 && idx_bits != 16) return hipErrorInvalidValue;
    const uint32_t tiles = (uint32_t)plan.tiles;
    const dim3 grid(((uint32_t)items64 + 7) / 8 * 8);
    const uint32_t k_tot = k_sym + zero_first;
    const bool lut_lds = k_tot <= kLutLdsMax;
    const size_t lds = index_gemm_lds_bytes(k_tot, (int)plan.rt);
    const uint32_t x_vec = (reinterpret_cast<uintptr_t>(d_X) % 16 == 0 && ldx % 4 == 0) ? 1u : 0u;
    hipError_t e = hipSuccess;
    if (idx_bits == 8) {
        if (lut_lds) launch_rt<uint8_t, true>(plan.rt, grid, lds, stream, e, d_X, ldx, B, d_idx, pitch, d_codebook, k_sym, zero_first,
                                              n, m, d_Y, ldy, tiles_n, tiles, x_vec, plan.splits, plan.steps_per_split, d_part);
        else launch_rt<uint8_t, false>(plan.rt, grid, lds, stream, e, d_X, ldx, B, d_idx, pitch, d_codebook, k_sym, zero_first,
                                       n, m, d_Y, ldy, tiles_n, tiles, x_vec, plan.splits, plan.steps_per_split, d_part);
    } else {
        if (lut_lds) launch_rt<uint16_t, true>(plan.rt, grid, lds, stream, e, d_X, ldx, B, d_idx, pitch, d_codebook, k_sym, zero_first,
                                               n, m, d_Y, ldy, tiles_n, tiles, x_vec, plan.splits, plan.steps_per_split, d_part);
        else launch_rt<uint16_t, false>(plan.rt, grid, lds, stream, e, d_X, ldx, B, d_idx, pitch, d_codebook, k_sym, zero_first,
                                        n, m, d_Y, ldy, tiles_n, tiles, x_vec, plan.splits, plan.steps_per_split, d_part);
    }
    if (e != hipSuccess || plan.splits == 1) return e;
    const uint64_t total = (uint64_t)B * m;
    const uint32_t rgrid = (uint32_t)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(rgrid), dim3(256), 0, stream, d_part, plan.splits, B, m, d_Y, ldy);
    note_kernel("splitk_reduce_kernel");
    return hipGetLastError();
}

} // namespace hac_internal
