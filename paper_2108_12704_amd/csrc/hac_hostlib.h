// Host-side pieces of libhac shared by its translation units (not part of the C ABI).
#ifndef HAC_HOSTLIB_H
#define HAC_HOSTLIB_H

#include <stdint.h>
#include <string.h>

#include <vector>

#include "../../include/hac.h"

namespace hac_internal {

constexpr uint32_t kMagic = 0x31434148u;   // "HAC1"
constexpr uint32_t kVersion = 2;
constexpr uint32_t kNetMagic = 0x4e434148u; // "HACN"
constexpr uint32_t kNetVersion = 1;
constexpr uint64_t kAlign = 256;
constexpr uint64_t kTailPad = 64;          // zero bytes after stream / ri for window over-reads
constexpr uint32_t kRiceEscape = 31;       // quotients from here on: 31 zeros, a one, the gap in 32 bits
constexpr uint32_t kRiceKMax = 15;

inline uint64_t align_up(uint64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline uint32_t float_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

// Huffman code lengths by merging the two least frequent nodes; false when a length exceeds 32.
bool huffman_lengths(const std::vector<uint64_t>& freq, std::vector<uint8_t>& len, uint32_t& lmax);

struct CodeTables {
    std::vector<uint32_t> code;        // canonical codeword per symbol (right-justified)
    std::vector<uint32_t> symsort;     // symbols in (length, symbol) order
    uint32_t first_code[33], count[33], first_index[33];
};
void canonical_codes(const std::vector<uint8_t>& len, CodeTables& t);
void build_lut(const std::vector<uint8_t>& len, const CodeTables& t, uint32_t lut_bits, std::vector<uint32_t>& lut);

uint32_t ceil_log2(uint64_t v);
uint64_t row_index_entries(const hac_desc_t& d);     // m * (nq + 1), or 0 without a row index
uint32_t pick_chunk_rows(const hac_opts_t* opts, uint64_t n, uint64_t m, uint64_t nnz);
uint32_t pick_lut_bits(const hac_opts_t* opts, uint32_t lmax);
uint32_t pick_chunk(const hac_opts_t* opts, uint64_t max_col_nnz);
// hac_desc_t.chunk: the chunk size, or with bit 31 set the smallest chunk size of a blob whose
// columns have chunk sizes of their own: column j is cut into chunks of
// max(smallest, ceil(non-zeros of j / 64)) non-zeros, so that no column has more than 64 chunks
// and a long column fills the 64 lanes of the wavefront that decodes it
constexpr uint32_t kChunkPerColumn = 0x80000000u;
constexpr uint32_t kChunkPerColumnLeast = 4;
#if defined(__HIP__)
#define HAC_HOST_DEVICE __host__ __device__
#else
#define HAC_HOST_DEVICE
#endif
HAC_HOST_DEVICE inline uint32_t chunk_base(uint32_t c) { return c & ~kChunkPerColumn; }
HAC_HOST_DEVICE inline uint32_t chunk_of_column(uint32_t c, uint64_t col_nnz)
{
    const uint32_t base = c & ~kChunkPerColumn;
    if (!(c & kChunkPerColumn)) return base;
    const uint64_t per = (col_nnz + 63) / 64;
    return per > base ? (uint32_t)per : base;
}
int check_opts(const hac_opts_t* opts);
uint32_t rice_length(uint32_t d, uint32_t k);

// Offsets of all sections and blob_bytes, from the counts already in the header
// (place_tables, then place_layer, from the end of the header).
void place_sections(hac_desc_t& d);
void place_tables(hac_desc_t& d, uint64_t& cursor, uint32_t k_values);   // k_values: entries of the value list when above k_sym
void place_layer(hac_desc_t& d, uint64_t& cursor);
int write_tables(uint8_t* base, const hac_desc_t& d, const std::vector<float>& codebook,
                 const std::vector<uint8_t>& len, const CodeTables& t, const std::vector<uint32_t>& lut);

// what hac_last_hip_error() reports (per thread)
void set_last_hip_error(int e);

} // namespace hac_internal

#endif
