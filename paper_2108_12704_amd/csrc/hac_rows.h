// Row-blocked batch kernel of libhac (gfx950): Y = X.W for batches of more than 128 rows, with
// the rows of X held in LDS instead of being gathered from L2 once per non-zero.
//
// Work split.  A block of 16 wavefronts owns 256 columns of W (16 per wavefront), up to 256 batch
// rows, and a range of rows of W; the row index of the blob (hac_desc_t.chunk_rows) cuts every
// column at the same rows, so the block can start decoding each of its columns at the top of its
// range.  The range is worked off in sessions of 4 index entries:
//   decode : lane (column, entry) decodes the non-zeros of its piece of the column (HAC,
//            Algorithm 1's walk; sHAC, Algorithm 2's with ri unpacked) into a per-wave list in
//            LDS, (offset of the row of X in LDS, shared value) per non-zero, column after column,
//            rows ascending; counts per (slab of rows, column) are kept beside it;
//   multiply: the session's rows of X pass through LDS slab by slab (R rows x 256 batch columns,
//            two buffers).  All threads of the block load a slab from row-major X with 128-bit
//            loads and store it transposed; a row of X then is 1 KB of LDS, 16 bytes per lane.
//            Per slab a wavefront walks its 16 columns; per non-zero: one broadcast read of the
//            list entry, one 128-bit read of the lane's 4 batch columns, 4 FMAs into the column's
//            4 accumulator registers.  The accumulators of all 16 columns stay in registers for
//            the whole range.
// Blocks that share a column group but own different row ranges write partial sums, which a small
// second kernel adds in a fixed order (bitwise reproducible, no atomics).
//
// LDS rows are 1040 bytes apart: with the lanes of a wavefront holding 16 batch rows x 4 row
// quads of a slab, the four 32-bit stores of a transposed quad fall into 64 different banks.
#ifndef HAC_ROWS_H
#define HAC_ROWS_H

namespace {

constexpr int kRowsWaves = 16;               // wavefronts per block
constexpr int kRowsCpw = 16;                 // columns of W per wavefront
constexpr uint32_t kRowsLpc = 4;             // lanes (entries of the row index) per column
constexpr uint32_t kRowsBatch = 256;         // batch rows per block
constexpr uint32_t kSlabPitch = 1040;        // bytes from one row of X to the next in LDS
constexpr uint32_t kSlabPitchW = kSlabPitch / 4;
constexpr int kSlabLoads = 4;                // 128-bit loads per thread, batch row and slab: R <= 64

struct RowsParams {
    const void* rent;                        // row index
    uint32_t chunk_rows, nq, rent_bits, rpos_bits;
    uint32_t R;                              // rows per slab, a multiple of 4, <= 64
    uint32_t magicR;                         // floor(2^32 / R) + 1
    uint32_t nrb;                            // slabs per session: ceil(4 * chunk_rows / R)
    uint32_t list_cap;                       // list entries per wavefront
    uint32_t stage_words;                    // words per wavefront for staged stream / ri words (inside the slab buffers)
    uint32_t S;                              // sessions: ceil(nq / 4)
    uint32_t T;                              // sessions per block
    uint32_t nparts;                         // row ranges: ceil(S / T)
    uint32_t ncg;                            // column groups of 256
    uint32_t tiles;                          // batch tiles of 256
    uint32_t vecx;                           // rows of X are 16-byte aligned
};

__device__ __forceinline__ void rows_entry(const RowsParams& rp, uint64_t e, uint32_t& rel_bit, uint32_t& rel_pos)
{
    if (rp.rent_bits == 32) {
        const uint32_t v = static_cast<const uint32_t*>(rp.rent)[e];
        rel_bit = v >> rp.rpos_bits;
        rel_pos = v & ((1u << rp.rpos_bits) - 1u);
    } else {
        const uint2 v = static_cast<const uint2*>(rp.rent)[e];
        rel_pos = v.x; rel_bit = v.y;
    }
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, uint32_t lane)
{
#pragma unroll
    for (uint32_t off = 1; off < (uint32_t)kWave; off <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)v, off, kWave);
        if (lane >= off) v += o;
    }
    return v;
}

struct SlabRegs { float4 v[1][kSlabLoads]; };

// The calling thread's share of one slab of X: batch row bl of the block's tile, row
// quads qsub, qsub + 4, ...  Rows past `rend` and batch rows past B read as zero.  A slab that
// lies inside the session and an X whose rows are 16-byte aligned take the first path: every load
// is issued, from a clamped address, before any is looked at.
__device__ __forceinline__ void slab_request(SlabRegs& s, const float* __restrict__ X, uint64_t ldx, uint32_t B, uint32_t bglob,
                                             uint32_t r0, uint32_t rend, uint32_t R, uint32_t qsub, uint32_t Q, uint32_t vecx)
{
    if (vecx && r0 + R <= rend) {
#pragma unroll
        for (int h = 0; h < 1; ++h) {
            const uint32_t b = bglob + 128u * h;
            const float* row = X + (uint64_t)(b < B ? b : B - 1u) * ldx + r0;
#pragma unroll
            for (int u = 0; u < kSlabLoads; ++u) {
                const uint32_t q = qsub + 4u * u;
                if (4u * u < Q) s.v[h][u] = *reinterpret_cast<const float4*>(row + 4u * (q < Q ? q : Q - 1u));   // (uniform)
            }
        }
#pragma unroll
        for (int h = 0; h < 1; ++h) {
            if (bglob + 128u * h >= B) {
#pragma unroll
                for (int u = 0; u < kSlabLoads; ++u) s.v[h][u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
        }
        return;
    }
#pragma unroll
    for (int h = 0; h < 1; ++h) {
        const uint32_t b = bglob + 128u * h;
#pragma unroll
        for (int u = 0; u < kSlabLoads; ++u) {
            const uint32_t q = qsub + 4u * u;
            const uint32_t r = r0 + 4u * q;
            float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (b < B && q < Q && r < rend) {
                const float* p = X + (uint64_t)b * ldx + r;
                v.x = p[0];
                if (r + 1 < rend) v.y = p[1];
                if (r + 2 < rend) v.z = p[2];
                if (r + 3 < rend) v.w = p[3];
            }
            s.v[h][u] = v;
        }
    }
}

__device__ __forceinline__ void slab_store(const SlabRegs& s, float* ring, uint32_t buf, uint32_t R, uint32_t bl, uint32_t qsub, uint32_t Q)
{
#pragma unroll
    for (int h = 0; h < 1; ++h) {
#pragma unroll
        for (int u = 0; u < kSlabLoads; ++u) {
            const uint32_t q = qsub + 4u * u;
            if (q < Q) {
                float* p = ring + (buf * R + 4u * q) * kSlabPitchW + bl + 128u * h;
                p[0] = s.v[h][u].x; p[kSlabPitchW] = s.v[h][u].y; p[2 * kSlabPitchW] = s.v[h][u].z; p[3 * kSlabPitchW] = s.v[h][u].w;
            }
        }
    }
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const f32x4 lds_cf4;
typedef __attribute__((address_space(3))) const char lds_cchar;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) const u32x2 lds_cu2v;


template <bool SHAC>
__global__ void __launch_bounds__(kRowsWaves * 64)
dot_rows_kernel(DevBlob d, RowsParams rp, const float* __restrict__ X, uint64_t ldx, uint32_t B,
                float* __restrict__ part, float* __restrict__ Y, uint64_t ldy)
{
    extern __shared__ uint32_t smem[];
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wib = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    // work items are (batch tile, row range, column group), column groups fastest: an XCD (one L2)
    // gets a contiguous range of items, hence few row ranges, and fetches their rows of X once
    const uint32_t item = logical_block(gridDim.x);
    if (item >= rp.tiles * rp.nparts * rp.ncg) return;
    const uint32_t tile = item / (rp.nparts * rp.ncg);
    const uint32_t rem = item - tile * rp.nparts * rp.ncg;
    const uint32_t pidx = rem / rp.ncg, g = rem - pidx * rp.ncg;
    const uint32_t col0 = (g * kRowsWaves + wib) * kRowsCpw;
    const uint32_t ci = lane >> 2, sub = lane & 3;
#ifdef HAC_PHASE_TIMING
    const uint32_t wave = blockIdx.x * kRowsWaves + wib;
    unsigned long long t_wait = 0, t_store = 0;
#endif
    HAC_MARK(0);

    // LDS: tables | lists | counts | slab buffers (also the staging area of the decode phase)
    TableRegs tr = request_tables(d);
    request_table_values(d, tr);
    uint32_t* p_lists = smem + table_words_dev(d);
    uint2* list = reinterpret_cast<uint2*>(p_lists) + (uint64_t)wib * rp.list_cap;
    uint32_t* cnt = p_lists + 2u * kRowsWaves * rp.list_cap + wib * rp.nrb * 4u;       // [slab][16 columns], one byte each
    float* ring = reinterpret_cast<float*>(p_lists + 2u * kRowsWaves * rp.list_cap + kRowsWaves * rp.nrb * 4u);
    uint32_t* sbuf = reinterpret_cast<uint32_t*>(ring) + wib * rp.stage_words;
    const Tables tb = store_tables(d, smem, tr);

    // the thread's share of a slab of X
    const uint32_t bl = wib * 16u + (lane & 15u), qsub = (lane >> 4) & 3u;
    const uint32_t bglob = tile * kRowsBatch + bl;
    const uint32_t Q = rp.R >> 2;
    const uint32_t lane16 = lane * 16u;
    lds_cchar* ringc = (lds_cchar*)ring;                            // the slab buffers, addressed in bytes
    lds_cu2v* listl = (lds_cu2v*)list;

    uint32_t touched = 0;                                            // keeps the early touches of X alive; never stored
    float acc[kRowsCpw][4];
#pragma unroll
    for (int c = 0; c < kRowsCpw; ++c) { acc[c][0] = 0.0f; acc[c][1] = 0.0f; acc[c][2] = 0.0f; acc[c][3] = 0.0f; }

    for (uint32_t t = 0; t < rp.T; ++t) {
        const uint32_t sess = pidx * rp.T + t;
        if (sess >= rp.S) break;
        const uint32_t q0 = sess * kRowsLpc;
        const uint32_t row0 = q0 * rp.chunk_rows;
        const uint32_t rend = row0 + kRowsLpc * rp.chunk_rows < d.n ? row0 + kRowsLpc * rp.chunk_rows : d.n;
        const uint32_t nrb = (rend - row0 + rp.R - 1) / rp.R;
        // The session's rows of X are touched once, early, by the blocks that share them (the column
        // groups of this row range sit on one XCD): each takes a share of the rows, one 128-byte line
        // per load, so that the slab loads of the multiply phase find them in L2.
        {
            const uint32_t span = rend - row0;
            const uint32_t share = ((span + rp.ncg - 1) / rp.ncg + 31u) & ~31u;
            const uint32_t rs = row0 + g * share;
            const uint32_t pieces = share >> 5;
            for (uint32_t i = threadIdx.x; i < kRowsBatch * pieces; i += blockDim.x) {
                const uint32_t b = i / pieces, r = rs + (i - b * pieces) * 32u;
                if (tile * kRowsBatch + b < B && r < rend) touched ^= __float_as_uint(X[(uint64_t)(tile * kRowsBatch + b) * ldx + r]);
            }
        }
        // the first slab travels while the session is decoded
        SlabRegs xs;
        slab_request(xs, X, ldx, B, bglob, row0, rend, rp.R, qsub, Q, rp.vecx);
        // every wavefront is done with the slab buffers of the session before (and, the first time,
        // the tables are complete)
        __syncthreads();
        HAC_MARK(1);
        for (uint32_t i = lane; i < rp.nrb * 4u; i += kWave) cnt[i] = 0u;

        // per-column cursors into the list, two 16-bit cursors per register (uniform values)
        uint32_t curp[kRowsCpw / 2];
        uint32_t hbase = 0;                                          // list entries of the halves before this one
#pragma unroll
        for (int h = 0; h < kRowsCpw / 16; ++h) {                   // (one turn: a wavefront decodes its 16 columns side by side)
            // ---- this lane's piece: entry q of column col ----
            const uint32_t col = col0 + 16u * h + ci;
            const bool col_ok = col < d.m;
            uint32_t colbit = 0, colpos = 0;
            if (col_ok) { colbit = d.colbit[col]; colpos = d.colpos[col]; }
            const uint32_t q = q0 + sub;
            const bool piece = col_ok && q < rp.nq;
            const uint32_t qe = q0 + kRowsLpc < rp.nq ? q0 + kRowsLpc : rp.nq;      // entry where the column's session ends
            uint32_t bit0 = 0, pos0 = 0, bit1 = 0, pos1 = 0, bite = 0, pose = 0, bits0 = 0, poss0 = 0;
            if (col_ok) {
                const uint64_t e = (uint64_t)col * (rp.nq + 1);
                rows_entry(rp, e + q0, bits0, poss0);                                // where the column's session begins
                rows_entry(rp, e + qe, bite, pose);
                if (piece) { rows_entry(rp, e + q, bit0, pos0); rows_entry(rp, e + q + 1, bit1, pos1); }
            }
            uint32_t ncnt = piece ? pos1 - pos0 : 0u;
            const uint32_t incl = wave_incl_scan(ncnt, lane);
            uint32_t base = hbase + incl - ncnt;
            if (hbase + incl > rp.list_cap) { ncnt = 0; base = 0; }  // never for a blob the encoders wrote (max_tile_nnz)
#pragma unroll
            for (int c = 0; c < 16; c += 2) {
                const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)base, 4 * c);
                const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)base, 4 * c + 4);
                curp[8 * h + c / 2] = lo | (hi << 16);
            }
            hbase += (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);

            // ---- stage the columns' stream words (and ri words) of the session ----
            const uint32_t bit_lo = colbit + bits0, bit_hi = colbit + bite;
            const uint32_t swlo = (bit_lo >> 5) & ~3u;
            const uint32_t snw = col_ok ? ((((bit_hi >> 5) + 4) - swlo + 4) & ~3u) : 0u;
            const uint64_t rb_lo = (uint64_t)(colpos + poss0) * d.ri_bits, rb_hi = (uint64_t)(colpos + pose) * d.ri_bits;
            const uint32_t rwlo = (uint32_t)(rb_lo >> 5) & ~3u;
            const uint32_t rnw = (SHAC && col_ok) ? ((((uint32_t)(rb_hi >> 5) + 2) - rwlo + 4) & ~3u) : 0u;
            const uint32_t mine = sub == 0 ? snw + rnw : 0u;
            const uint32_t sincl = wave_incl_scan(mine, lane);
            const uint32_t soff = (uint32_t)__shfl((int)(sincl - mine), (int)(ci * 4u), kWave);   // words before this column's segment
            const uint32_t stotal = (uint32_t)__shfl((int)sincl, kWave - 1, kWave);
            const bool staged = stotal <= rp.stage_words;
            wave_sync();                                            // the half before is done with the staging area
            if (staged) {
                const uint4* s4 = reinterpret_cast<const uint4*>(d.stream + swlo);
                uint4* d4 = reinterpret_cast<uint4*>(sbuf + soff);
                for (uint32_t i = sub; i < (snw >> 2); i += 4) d4[i] = s4[i];
                if (SHAC) {
                    const uint4* r4 = reinterpret_cast<const uint4*>(d.ri + rwlo);
                    uint4* e4 = reinterpret_cast<uint4*>(sbuf + soff + snw);
                    for (uint32_t i = sub; i < (rnw >> 2); i += 4) e4[i] = r4[i];
                }
            }
            wave_sync();
            if (h == 0) HAC_MARK(2);

            // ---- decode: lanes = pieces of columns ----
            ChunkState st;
            st.bp = colbit + bit0;
            st.row = q * rp.chunk_rows;
            st.wpos = base;
            st.wend = base + ncnt;
            const uint32_t cshift = 8u * (ci & 3u), cword = 4u * h + (ci >> 2);
            const WordSrc<true> r_lds = { sbuf + soff + snw, rwlo };
            const WordSrc<false> r_glb = { d.ri, 0 };
            const uint32_t ri_rel0 = (uint32_t)(rb_lo - 32ull * rwlo);   // bit of the session's first row index in the staged words
            const uint32_t gpos0 = colpos + pos0;                     // CSC position of the piece's first non-zero
            auto emit = [&](uint32_t p, uint32_t row, uint32_t, float v) {
                if (SHAC) {
                    if (staged) row = r_lds.field_rel(__umul24(pos0 - poss0 + (p - base), d.ri_bits) + ri_rel0, d.ri_bits);
                    else row = r_glb.field((uint64_t)(gpos0 + (p - base)) * d.ri_bits, d.ri_bits);
                }
                uint32_t rr = row - row0;
                rr = rr < rend - row0 ? rr : 0u;                      // (a damaged stream: stay inside the buffers)
                uint32_t k = __umulhi(rr, rp.magicR);
                if (k * rp.R > rr) --k;
                const uint32_t rl = rr - k * rp.R;
                list[p] = make_uint2(((k & 1u) * rp.R + rl) * kSlabPitch, __float_as_uint(v));
                atomicAdd(&cnt[k * 4u + cword], 1u << cshift);
            };
            if (st.wpos < st.wend) {
                if (staged) {
                    const WordSrc<true> s_lds = { sbuf + soff, swlo };
                    if (SHAC) shac_advance(d, tb, s_lds, st, st.wend, emit);
                    else if (d.zero_len == 1) hac_advance_zrun(d, tb, s_lds, st, st.wend, emit);
                    else hac_advance(d, tb, s_lds, st, st.wend, emit);
                } else {
                    const WordSrc<false> s_glb = { d.stream, 0 };
                    if (SHAC) shac_advance(d, tb, s_glb, st, st.wend, emit);
                    else hac_advance(d, tb, s_glb, st, st.wend, emit);
                }
            }
        }
        HAC_MARK(3);
        __syncthreads();                                          // lists and counts complete; the staging area is free
        HAC_MARK(4);

        // ---- multiply: slabs of X through LDS ----
        slab_store(xs, ring, 0u, rp.R, bl, qsub, Q);
        if (nrb > 1) slab_request(xs, X, ldx, B, bglob, row0 + rp.R, rend, rp.R, qsub, Q, rp.vecx);
        __syncthreads();
        for (uint32_t rb = 0; rb < nrb; ++rb) {
            uint32_t cw[kRowsCpw / 4];
            {
                const uint4 c0 = *reinterpret_cast<const uint4*>(cnt + rb * 4u);
                cw[0] = (uint32_t)__builtin_amdgcn_readfirstlane((int)c0.x); cw[1] = (uint32_t)__builtin_amdgcn_readfirstlane((int)c0.y);
                cw[2] = (uint32_t)__builtin_amdgcn_readfirstlane((int)c0.z); cw[3] = (uint32_t)__builtin_amdgcn_readfirstlane((int)c0.w);
            }
            // The 16 columns in turn (all indices are compile-time constants once unrolled); a column
            // without a non-zero in this slab costs three scalar instructions.
#pragma unroll
            for (int c = 0; c < kRowsCpw; ++c) {
                const uint32_t k = (cw[c >> 2] >> (8 * (c & 3))) & 255u;
                if (k) {
                    const uint32_t at = (curp[c >> 1] >> (16 * (c & 1))) & 0xffffu;
                    for (uint32_t i = 0; i < k; ++i) {
                        const u32x2 e = listl[at + i];
                        const f32x4 x = *(lds_cf4*)(ringc + (e.x + lane16));
                        const float w = __uint_as_float(e.y);
                        acc[c][0] = fmaf(x.x, w, acc[c][0]); acc[c][1] = fmaf(x.y, w, acc[c][1]);
                        acc[c][2] = fmaf(x.z, w, acc[c][2]); acc[c][3] = fmaf(x.w, w, acc[c][3]);
                    }
                    curp[c >> 1] += k << (16 * (c & 1));
                }
            }
            if (rb + 1 < nrb) {
#ifdef HAC_PHASE_TIMING
                const unsigned long long ts = wall_clock64();
#endif
                slab_store(xs, ring, (rb + 1) & 1u, rp.R, bl, qsub, Q);
#ifdef HAC_PHASE_TIMING
                __builtin_amdgcn_s_waitcnt(0);
                t_store += wall_clock64() - ts;
#endif
                if (rb + 2 < nrb) slab_request(xs, X, ldx, B, bglob, row0 + (rb + 2) * rp.R, rend, rp.R, qsub, Q, rp.vecx);
#ifdef HAC_PHASE_TIMING
                const unsigned long long tw = wall_clock64();
#endif
                __syncthreads();
#ifdef HAC_PHASE_TIMING
                t_wait += wall_clock64() - tw;
#endif
            }
        }
        HAC_MARK(5);
    }

    // ---- the block's sums: partial sums of its row range, or Y itself when there is one range ----
    if (touched == 0x7fc12345u && rp.T == 0xffffffffu) part[0] = 0.0f;    // (never true: T is at most 65536)
    const uint32_t b4 = tile * kRowsBatch + lane * 4u;
#pragma unroll
    for (int c = 0; c < kRowsCpw; ++c) {
        const uint32_t cc = col0 + c;
        if (cc < d.m) {
            if (rp.nparts > 1) {
                float* o = part + (((uint64_t)tile * rp.nparts + pidx) * d.m + cc) * kRowsBatch + lane * 4u;
                *reinterpret_cast<float4*>(o) = make_float4(acc[c][0], acc[c][1], acc[c][2], acc[c][3]);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) if (b4 + i < B) Y[(uint64_t)(b4 + i) * ldy + cc] = acc[c][i];
            }
        }
    }
    HAC_MARK(6);
#ifdef HAC_PHASE_TIMING
    if (lane == 0 && wave < 16384) g_phase[wave * 8 + 7] = t_wait | (t_store << 32);
#endif
}

// Y[b][col] = sum over the row ranges p of part[tile][p][col][b % 256], added in the order of p.
// A block of 256 threads takes 16 columns of one batch tile.
__global__ void __launch_bounds__(256)
rows_reduce_kernel(const float* __restrict__ part, uint32_t nparts, uint32_t m, uint32_t B,
                   float* __restrict__ Y, uint64_t ldy)
{
    __shared__ float tileT[16][kRowsBatch + 1];
    const uint32_t tile = blockIdx.y, c0 = blockIdx.x * 16u;
    const uint32_t ncol = m - c0 < 16u ? m - c0 : 16u;
    float4 s[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) s[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    const float* base = part + ((uint64_t)tile * nparts * m + c0) * kRowsBatch;
    for (uint32_t p = 0; p < nparts; ++p) {
        const float4* src = reinterpret_cast<const float4*>(base + (uint64_t)p * m * kRowsBatch);
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t f = threadIdx.x + 256u * u;                 // float4 index: 16 columns x 64
            v[u] = (f >> 6) < ncol ? src[f] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) { s[u].x += v[u].x; s[u].y += v[u].y; s[u].z += v[u].z; s[u].w += v[u].w; }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const uint32_t f = threadIdx.x + 256u * u;
        const uint32_t c = f >> 6, b = (f & 63u) * 4u;
        tileT[c][b] = s[u].x; tileT[c][b + 1] = s[u].y; tileT[c][b + 2] = s[u].z; tileT[c][b + 3] = s[u].w;
    }
    __syncthreads();
    const uint32_t b = tile * kRowsBatch + threadIdx.x;
    if (b < B) {
        float* o = Y + (uint64_t)b * ldy + c0;
        for (uint32_t c = 0; c < ncol; ++c) o[c] = tileT[c][threadIdx.x];
    }
}

// ---- host side: does the row-blocked kernel apply, and with which shape --------------------
struct RowsPlan {
    bool use;
    RowsParams rp;
    size_t lds, part_bytes;
    uint32_t grid;
};

// LDS bytes for slabs of R rows
size_t rows_lds_bytes(size_t table_bytes, uint32_t cap, uint32_t chunk_rows, uint32_t R)
{
    const uint32_t nrb = (kRowsLpc * chunk_rows + R - 1) / R;
    return table_bytes + (size_t)kRowsWaves * cap * 8 + (size_t)kRowsWaves * nrb * 16 + 2ull * R * kSlabPitch;
}

RowsPlan plan_rows(const hac_desc_t* desc, int64_t B, const hac_launch_t* launch, size_t table_bytes)
{
    RowsPlan P;
    memset(&P, 0, sizeof P);
    const uint32_t variant = launch ? launch->variant : 0u;
    if (!desc->chunk_rows || desc->format == HAC_FORMAT_IM || desc->ri_coding == HAC_RI_RICE) return P;
    if (variant & HAC_LAUNCH_NO_ROWS_KERNEL) return P;
    if (!(variant & HAC_LAUNCH_ROWS_KERNEL)) return P;                     // measured slower than the column kernels: on request only
    if (desc->max_tile_nnz == 65535 || (desc->rent_bits != 32 && desc->rent_bits != 64) || desc->rpos_bits > 31) return P;
    if (desc->chunk_rows > desc->n || (uint64_t)desc->chunk_rows * kRowsLpc * 64 >= (1ull << 32)) return P;
    RowsParams& rp = P.rp;
    rp.chunk_rows = desc->chunk_rows;
    rp.nq = (uint32_t)((desc->n + desc->chunk_rows - 1) / desc->chunk_rows);
    rp.rent_bits = desc->rent_bits; rp.rpos_bits = desc->rpos_bits;
    rp.list_cap = (((uint32_t)desc->max_tile_nnz + 1u) + 3u) & ~3u;        // one entry more: read, never used, past a wavefront's last
    if (rp.list_cap < 8) rp.list_cap = 8;
    if (rp.list_cap > 65528) return P;                                     // cursors are kept in 16 bits
    uint32_t R = 64;
    const uint32_t span = kRowsLpc * rp.chunk_rows;
    if (R > ((span + 3u) & ~3u)) R = (span + 3u) & ~3u;
    while (R >= 4 && rows_lds_bytes(table_bytes, rp.list_cap, rp.chunk_rows, R) > kLdsLimit) R -= 4;
    if (R < 4) return P;
    rp.R = R;
    rp.magicR = (uint32_t)((1ull << 32) / R) + 1u;
    rp.nrb = (span + R - 1) / R;
    rp.stage_words = (2u * R * kSlabPitchW / kRowsWaves) & ~3u;
    rp.S = (rp.nq + kRowsLpc - 1) / kRowsLpc;
    rp.ncg = (uint32_t)((desc->m + 255) / 256);
    rp.tiles = (uint32_t)((B + kRowsBatch - 1) / kRowsBatch);
    uint32_t T = launch && launch->sessions_per_block ? launch->sessions_per_block : 0u;
    if (!T) {
        // about one block per CU: fewer row ranges mean fewer partial sums to write and add
        const uint64_t blocks1 = (uint64_t)rp.S * rp.ncg * rp.tiles;
        T = (uint32_t)(blocks1 / 256);
        if (T < 1) T = 1;
    }
    if (T > rp.S) T = rp.S;
    rp.T = T;
    rp.nparts = (rp.S + T - 1) / T;
    const uint64_t items = (uint64_t)rp.tiles * rp.nparts * rp.ncg;
    if (items > 0x7ffffff0ull) return P;
    P.grid = (uint32_t)((items + 7) / 8 * 8);
    P.lds = rows_lds_bytes(table_bytes, rp.list_cap, rp.chunk_rows, R);
    P.part_bytes = rp.nparts > 1 ? (size_t)rp.tiles * rp.nparts * desc->m * kRowsBatch * 4 : 0;
    P.use = true;
    return P;
}

} // namespace

#endif
