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
// Tiling: a block of 4 wavefronts owns 128 batch rows x 128 columns of Y and walks
// K = n in steps of 32; wavefront (wm, wn) owns a 64 x 64 quarter as 2 x 2 MFMA
// tiles (64 accumulator registers).  LDS holds the X tile k-major (lanes read 32
// consecutive batch rows of one k) and the decoded W tile k-major (32 consecutive
// columns of one k); both are double buffered, the next tile's global loads are
// issued before the MFMA loop of the current one and stored after it.
// Lane layout of the instruction (checked on the device): A operand lane l holds
// A[i = l % 32][k = l / 32], B operand lane l holds B[k = l / 32][j = l % 32],
// accumulator register v of lane l is D[(v % 4) + 8 (v / 4) + 4 (l / 32)][l % 32].
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hac_internal.h"

namespace {

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDA = BM + 4, LDB = BN + 4;          // LDS row pitches (floats)
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

template <typename IdxT, bool LUT_LDS>
__global__ void __launch_bounds__(256)
index_gemm_kernel(const float* __restrict__ X, uint64_t ldx, uint32_t B,
                  const IdxT* __restrict__ idx, uint64_t pitch,          // pitch in elements, a multiple of 16
                  const float* __restrict__ codebook, uint32_t k_sym, uint32_t zero_first,
                  uint32_t n, uint32_t m, float* __restrict__ Y, uint64_t ldy,
                  uint32_t tiles_n, uint32_t tiles, uint32_t x_vec,
                  uint32_t splits, uint32_t steps_per_split, float* __restrict__ part)
{
    extern __shared__ float lds[];
    float* As = lds;                                   // [2][BK][LDA]
    float* Bs = lds + 2 * BK * LDA;                    // [2][BK][LDB]
    float* lut = Bs + 2 * BK * LDB;                    // [k_sym + zero_first] when LUT_LDS
    // work item = (tile, K split); with more than one split a block writes its partial tile to
    // part[split][B][m] and a second kernel adds the splits in order
    const uint32_t item = logical_tile(gridDim.x);
    if (item >= tiles * splits) return;
    const uint32_t tile = item / splits, split = item - tile * splits;
    const uint32_t tm = tile / tiles_n, tn = tile - tm * tiles_n;
    const uint32_t m0 = tm * BM, n0 = tn * BN;
    const uint32_t t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const uint32_t wm = wave >> 1, wn = wave & 1;
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

    // global -> register staging of one K step
    const uint32_t a_row = t >> 3, a_kq = t & 7;       // rows a_row + 32 r, k = 4 a_kq .. 4 a_kq + 3
    const uint32_t b_k = t >> 3, b_seg = t & 7;        // idx row b_k, columns 16 b_seg .. 16 b_seg + 15
    float4 ra[4];
    IdxRegs<IdxT> rb;
    auto load_global = [&](uint32_t k0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t row = m0 + a_row + 32 * r, k = k0 + 4 * a_kq;
            float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (row < B) {
                const float* p = X + (uint64_t)row * ldx + k;
                if (x_vec && k + 3 < n) v = *reinterpret_cast<const float4*>(p);
                else {
                    if (k < n) v.x = p[0];
                    if (k + 1 < n) v.y = p[1];
                    if (k + 2 < n) v.z = p[2];
                    if (k + 3 < n) v.w = p[3];
                }
            }
            ra[r] = v;
        }
        const uint32_t k = k0 + b_k, c = n0 + 16 * b_seg;
        constexpr int NV = sizeof(IdxT) == 1 ? 1 : 2;
#pragma unroll
        for (int q = 0; q < NV; ++q) rb.v[q] = make_uint4(0, 0, 0, 0);
        if (k < n && c < pitch) {
            const uint4* p = reinterpret_cast<const uint4*>(idx + (uint64_t)k * pitch + c);
#pragma unroll
            for (int q = 0; q < NV; ++q) rb.v[q] = p[q];
        }
    };
    // registers -> LDS in four quarters (q = 0..3), so that the work can be spread over the MFMA loop
    auto store_quarter = [&](uint32_t buf, int q) {
        float* a = As + buf * BK * LDA;
        const uint32_t row = a_row + 32 * q;
        a[(4 * a_kq + 0) * LDA + row] = ra[q].x;
        a[(4 * a_kq + 1) * LDA + row] = ra[q].y;
        a[(4 * a_kq + 2) * LDA + row] = ra[q].z;
        a[(4 * a_kq + 3) * LDA + row] = ra[q].w;
        float* b = Bs + buf * BK * LDB + b_k * LDB + 16 * b_seg;
        float4 o;
        if constexpr (sizeof(IdxT) == 1) {
            const uint32_t u = q == 0 ? rb.v[0].x : q == 1 ? rb.v[0].y : q == 2 ? rb.v[0].z : rb.v[0].w;
            o.x = value_of(u & 255u); o.y = value_of((u >> 8) & 255u);
            o.z = value_of((u >> 16) & 255u); o.w = value_of(u >> 24);
        } else {
            const uint4 v = rb.v[q >> 1];
            const uint32_t u0 = (q & 1) ? v.z : v.x, u1 = (q & 1) ? v.w : v.y;
            o.x = value_of(u0 & 65535u); o.y = value_of(u0 >> 16);
            o.z = value_of(u1 & 65535u); o.w = value_of(u1 >> 16);
        }
        *reinterpret_cast<float4*>(b + 4 * q) = o;
    };
    auto store_lds = [&](uint32_t buf) {
#pragma unroll
        for (int q = 0; q < 4; ++q) store_quarter(buf, q);
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const uint32_t all_steps = (n + BK - 1) / BK;
    const uint32_t kt0 = split * steps_per_split;
    const uint32_t ksteps = kt0 + steps_per_split < all_steps ? kt0 + steps_per_split : all_steps;   // one past the last
    load_global(kt0 * BK);
    __syncthreads();                                   // the table is complete before the first lookup
    store_lds(kt0 & 1);
    __syncthreads();
    for (uint32_t kt = kt0; kt < ksteps; ++kt) {
        const uint32_t buf = kt & 1;
        if (kt + 1 < ksteps) load_global((kt + 1) * BK);
        const float* a = As + buf * BK * LDA + wm * 64 + l32 + half * LDA;
        const float* b = Bs + buf * BK * LDB + wn * 64 + l32 + half * LDB;
        // operands of step kk + 1 are fetched from LDS before the matrix instructions of step kk issue
        float a0 = a[0], a1 = a[32], b0 = b[0], b1 = b[32];
#pragma unroll
        for (int kk = 0; kk < BK / 2; ++kk) {
            float na0 = 0.0f, na1 = 0.0f, nb0 = 0.0f, nb1 = 0.0f;
            if (kk + 1 < BK / 2) {
                na0 = a[(2 * kk + 2) * LDA]; na1 = a[(2 * kk + 2) * LDA + 32];
                nb0 = b[(2 * kk + 2) * LDB]; nb1 = b[(2 * kk + 2) * LDB + 32];
            }
            __builtin_amdgcn_sched_barrier(0);         // keep these LDS reads ahead of the matrix instructions
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
            // the next tile goes to the other buffer (nobody reads it during this step), a quarter at a
            // time between the matrix instructions, late in the step so that its global loads have landed
            if (kk >= 9 && (kk & 1) == 1 && kt + 1 < ksteps) store_quarter(buf ^ 1, (kk - 9) >> 1);
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t col = n0 + wn * 64 + j * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t row = m0 + wm * 64 + i * 32 + (v & 3) + 8 * (v >> 2) + 4 * half;
                if (row < B && col < m) {
                    if (splits == 1) Y[(uint64_t)row * ldy + col] = acc[i][j][v];
                    else part[((uint64_t)split * B + row) * m + col] = acc[i][j][v];
                }
            }
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
        for (uint32_t s = 1; s < splits; ++s) v += part[(uint64_t)s * total + i];
        const uint64_t row = i / m;
        Y[row * ldy + (i - row * m)] = v;
    }
}

} // namespace

namespace hac_internal {

static size_t index_gemm_lds_bytes(uint32_t k_tot)
{
    return sizeof(float) * (2 * BK * LDA + 2 * BK * LDB + (k_tot <= kLutLdsMax ? k_tot : 0));
}

GemmPlan plan_index_gemm(uint32_t B, uint32_t n, uint32_t m)
{
    GemmPlan p;
    const uint64_t tiles = (uint64_t)((B + BM - 1) / BM) * ((m + BN - 1) / BN);
    const uint32_t steps = (n + BK - 1) / BK;
    // a tile's K loop is serial (about 3 us per step of 32): with fewer tiles than CUs, K is split
    // until there are about two work items per CU, keeping at least 8 steps per split
    uint32_t splits = 1;
    if (tiles < 256) {
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

hipError_t launch_index_gemm(const float* d_X, uint64_t ldx, uint32_t B, const void* d_idx, uint32_t idx_bits,
                             uint64_t pitch, const float* d_codebook, uint32_t k_sym, uint32_t zero_first,
                             uint32_t n, uint32_t m, float* d_Y, uint64_t ldy, float* d_part, hipStream_t stream)
{
    const uint32_t tiles_n = (m + BN - 1) / BN;
    const GemmPlan plan = plan_index_gemm(B, n, m);
    const uint64_t items64 = plan.tiles * plan.splits;
    if (items64 > 0x7ffffff0ull) return hipErrorInvalidValue;
    if (plan.splits > 1 && !d_part) return hipErrorInvalidValue;
    const uint32_t tiles = (uint32_t)plan.tiles;
    const uint32_t grid = ((uint32_t)items64 + 7) / 8 * 8;
    const uint32_t k_tot = k_sym + zero_first;
    const bool lut_lds = k_tot <= kLutLdsMax;
    const size_t lds = index_gemm_lds_bytes(k_tot);
    const uint32_t x_vec = (reinterpret_cast<uintptr_t>(d_X) % 16 == 0 && ldx % 4 == 0) ? 1u : 0u;
    typedef void (*kern8_t)(const float*, uint64_t, uint32_t, const uint8_t*, uint64_t, const float*, uint32_t, uint32_t,
                            uint32_t, uint32_t, float*, uint64_t, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t, float*);
    typedef void (*kern16_t)(const float*, uint64_t, uint32_t, const uint16_t*, uint64_t, const float*, uint32_t, uint32_t,
                             uint32_t, uint32_t, float*, uint64_t, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t, float*);
    if (idx_bits == 8) {
        kern8_t k = lut_lds ? index_gemm_kernel<uint8_t, true> : index_gemm_kernel<uint8_t, false>;
        if (lds > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(k, dim3(grid), dim3(256), lds, stream, d_X, ldx, B, static_cast<const uint8_t*>(d_idx), pitch,
                           d_codebook, k_sym, zero_first, n, m, d_Y, ldy, tiles_n, tiles, x_vec,
                           plan.splits, plan.steps_per_split, d_part);
    } else if (idx_bits == 16) {
        kern16_t k = lut_lds ? index_gemm_kernel<uint16_t, true> : index_gemm_kernel<uint16_t, false>;
        if (lds > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(k, dim3(grid), dim3(256), lds, stream, d_X, ldx, B, static_cast<const uint16_t*>(d_idx), pitch,
                           d_codebook, k_sym, zero_first, n, m, d_Y, ldy, tiles_n, tiles, x_vec,
                           plan.splits, plan.steps_per_split, d_part);
    } else {
        return hipErrorInvalidValue;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || plan.splits == 1) return e;
    const uint64_t total = (uint64_t)B * m;
    const uint32_t rgrid = (uint32_t)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(rgrid), dim3(256), 0, stream, d_part, plan.splits, B, m, d_Y, ldy);
    return hipGetLastError();
}

} // namespace hac_internal
