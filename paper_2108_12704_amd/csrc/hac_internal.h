// Declarations shared by the translation units of libhac (not part of the C ABI).
#ifndef HAC_INTERNAL_H
#define HAC_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace hac_internal {

// How launch_index_gemm splits the work: `tiles` output tiles, each K loop of `steps` steps cut into
// `splits` ranges of steps_per_split; with more than one split the partial tiles go through a buffer
// of part_bytes bytes (splits x B x m floats) and are added in order by a second kernel.
// A block covers 32 * rt batch rows (rt = 2..8) and 128 columns.
// small (at most 32 batch rows): no matrix cores; `tiles` blocks of 4 << rt columns (256 for maps of
// 129 columns or more), the rows of W cut into `splits` ranges of steps_per_split rows, partial sums
// through the same buffer.
struct GemmPlan { uint64_t tiles; uint32_t steps, splits, steps_per_split, rt; size_t part_bytes; bool small; };
GemmPlan plan_index_gemm(uint32_t B, uint32_t n, uint32_t m);

// Y[B x m] = X[B x n] . c[Pi] for an index map Pi of n rows, `pitch` elements apart (a multiple of
// 16), of idx_bits = 8 or 16 bits each.  zero_first = 1: pointer 0 means 0.0 and pointer p > 0 means
// c[p - 1].  All pointers are device pointers; d_idx is 16-byte aligned; d_part holds
// plan_index_gemm(B, n, m).part_bytes bytes (may be NULL when that is 0).  Asynchronous on `stream`.
hipError_t launch_index_gemm(const float* d_X, uint64_t ldx, uint32_t B, const void* d_idx, uint32_t idx_bits,
                             uint64_t pitch, const float* d_codebook, uint32_t k_sym, uint32_t zero_first,
                             uint32_t n, uint32_t m, float* d_Y, uint64_t ldy, float* d_part, hipStream_t stream);

// The kernels the calling thread's most recent dot call launched, by the names a profiler shows
// (see hac_last_kernels): note_reset() at the start of a call, note_kernel() at every launch.
void note_reset();
void note_kernel(const char* fmt, ...) __attribute__((format(printf, 1, 2)));

} // namespace hac_internal

#endif
