// Host side of libhac: encoders, blob validation, size accounting and a
// sequential decoder.  Definitions follow arXiv 2108.12704 Sect. IV-A (CSC),
// IV-B (HAC) and IV-C (sHAC); the chunk index is this library's addition for
// the GPU (the paper's conclusions only suggest per-column offsets).
#include "../../include/hac.h"
#include "hac_hostlib.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <new>
#include <queue>
#include <utility>
#include <vector>

static_assert(sizeof(hac_desc_t) == 256, "blob header must be 256 bytes");
static_assert(sizeof(hac_net_t) == 256, "network header must be 256 bytes");

using namespace hac_internal;

namespace {

// ---- small open-addressing map: fp32 bit pattern -> dense id --------------------
struct ValueMap {
    std::vector<uint32_t> keys;
    std::vector<uint32_t> ids;
    std::vector<uint8_t> used;
    uint32_t mask = 0;
    uint32_t count = 0;

    void init(uint32_t cap_pow2) {
        keys.assign(cap_pow2, 0); ids.assign(cap_pow2, 0); used.assign(cap_pow2, 0);
        mask = cap_pow2 - 1; count = 0;
    }
    static uint32_t hash(uint32_t k) { k ^= k >> 16; k *= 0x7feb352du; k ^= k >> 15; k *= 0x846ca68bu; k ^= k >> 16; return k; }
    void grow() {
        ValueMap bigger; bigger.init((mask + 1) * 2);
        for (uint32_t i = 0; i <= mask; ++i) if (used[i]) bigger.insert(keys[i], ids[i]);
        *this = std::move(bigger);
    }
    void insert(uint32_t key, uint32_t id) {
        uint32_t h = hash(key) & mask;
        while (used[h]) h = (h + 1) & mask;
        used[h] = 1; keys[h] = key; ids[h] = id; ++count;
    }
    // returns id, inserting a fresh one (= current count) when absent
    uint32_t find_or_add(uint32_t key) {
        uint32_t h = hash(key) & mask;
        while (used[h]) { if (keys[h] == key) return ids[h]; h = (h + 1) & mask; }
        if ((count + 1) * 2 > mask + 1) { grow(); return find_or_add(key); }
        used[h] = 1; keys[h] = key; ids[h] = count;
        return count++;
    }
};

} // namespace

namespace hac_internal {

// ---- Huffman code lengths: merge the two least frequent nodes (Huffman 1952) ---
// Ties: lower (weight, node id) first; leaves are numbered by symbol, internal
// nodes after them in creation order.  A one-symbol alphabet gets length 1.
bool huffman_lengths(const std::vector<uint64_t>& freq, std::vector<uint8_t>& len, uint32_t& lmax)
{
    const size_t k = freq.size();
    len.assign(k, 0);
    lmax = 0;
    if (k == 0) return true;
    if (k == 1) { len[0] = 1; lmax = 1; return true; }
    typedef std::pair<uint64_t, uint32_t> node;                  // (weight, id)
    std::priority_queue<node, std::vector<node>, std::greater<node> > pq;
    for (size_t i = 0; i < k; ++i) pq.push(node(freq[i], (uint32_t)i));
    std::vector<uint32_t> parent(2 * k - 1, 0);
    uint32_t next = (uint32_t)k;
    while (pq.size() > 1) {
        node a = pq.top(); pq.pop();
        node b = pq.top(); pq.pop();
        parent[a.second] = next; parent[b.second] = next;
        pq.push(node(a.first + b.first, next));
        ++next;
    }
    const uint32_t root = next - 1;
    std::vector<uint32_t> depth(2 * k - 1, 0);
    for (uint32_t v = root; v-- > 0;) depth[v] = depth[parent[v]] + 1;   // parents have larger ids
    for (size_t i = 0; i < k; ++i) {
        if (depth[i] > 32) return false;
        len[i] = (uint8_t)depth[i];
        lmax = std::max<uint32_t>(lmax, depth[i]);
    }
    return true;
}

void canonical_codes(const std::vector<uint8_t>& len, CodeTables& t)
{
    const size_t k = len.size();
    t.code.assign(k, 0);
    t.symsort.resize(k);
    for (int l = 0; l <= 32; ++l) t.first_code[l] = t.count[l] = t.first_index[l] = 0;
    for (size_t i = 0; i < k; ++i) t.count[len[i]]++;
    uint32_t idx = 0;
    uint64_t c = 0;
    for (int l = 1; l <= 32; ++l) {
        c <<= 1;
        t.first_code[l] = (uint32_t)c;
        t.first_index[l] = idx;
        c += t.count[l];
        idx += t.count[l];
    }
    std::vector<uint32_t> fill(33, 0);
    for (size_t i = 0; i < k; ++i) {                    // ascending symbol within a length
        const uint32_t l = len[i];
        const uint32_t r = fill[l]++;
        t.code[i] = t.first_code[l] + r;
        t.symsort[t.first_index[l] + r] = (uint32_t)i;
    }
}

void build_lut(const std::vector<uint8_t>& len, const CodeTables& t, uint32_t lut_bits,
               std::vector<uint32_t>& lut)
{
    lut.assign((size_t)1 << lut_bits, 0);
    for (size_t s = 0; s < len.size(); ++s) {
        const uint32_t l = len[s];
        if (l > lut_bits) continue;
        const uint32_t lo = t.code[s] << (lut_bits - l);
        const uint32_t span = 1u << (lut_bits - l);
        for (uint32_t e = 0; e < span; ++e) lut[lo + e] = ((uint32_t)s << 6) | l;
    }
}

} // namespace hac_internal

namespace {

// ---- bit writer: MSB-first into uint32 words; the buffer starts zeroed ----------
struct BitWriter {
    uint32_t* words;
    uint64_t bitpos;
    inline void put(uint32_t code, uint32_t len) {
        const uint64_t w = bitpos >> 5;
        const uint32_t off = (uint32_t)(bitpos & 31);
        const uint64_t v = (uint64_t)code << (64 - len - off);   // len <= 32, off <= 31
        words[w] |= (uint32_t)(v >> 32);
        const uint32_t lo = (uint32_t)v;
        if (lo) words[w + 1] |= lo;
        bitpos += len;
    }
    inline void skip(uint64_t bits) { bitpos += bits; }          // run of zero bits
};

// ---- CSC-like intermediate shared by both encoders ------------------------------
struct Scan {
    int64_t n = 0, m = 0;
    std::vector<float> values;         // alphabet of the non-zero values, ascending
    std::vector<uint64_t> freq;        // their counts
    uint64_t zeros = 0;
    std::vector<uint64_t> cb;          // m + 1
    std::vector<uint32_t> ri;          // nnz
    std::vector<uint32_t> sym;         // nnz: index into `values`
};

int scan_matrix(const float* W, int64_t n, int64_t m, int64_t ldw, Scan& s)
{
    s.n = n; s.m = m;
    ValueMap map; map.init(1024);
    std::vector<uint32_t> raw_keys;
    std::vector<uint64_t> colcount((size_t)m, 0);
    uint64_t nnz = 0;
    for (int64_t i = 0; i < n; ++i) {
        const float* row = W + i * ldw;
        for (int64_t j = 0; j < m; ++j) {
            const float v = row[j];
            if (v == 0.0f) continue;                       // +0.0 and -0.0 both count as null
            if (!std::isfinite(v)) return HAC_EINVAL;
            colcount[(size_t)j]++; nnz++;
        }
    }
    if (nnz > 0xfffffff0ull) return HAC_ERANGE;
    s.zeros = (uint64_t)n * (uint64_t)m - nnz;
    s.cb.assign((size_t)m + 1, 0);
    for (int64_t j = 0; j < m; ++j) s.cb[(size_t)j + 1] = s.cb[(size_t)j] + colcount[(size_t)j];
    s.ri.resize((size_t)nnz);
    s.sym.resize((size_t)nnz);
    std::vector<uint64_t> cursor(s.cb.begin(), s.cb.end() - 1);
    std::vector<uint64_t> rawfreq;
    for (int64_t i = 0; i < n; ++i) {                      // ascending i keeps rows sorted per column
        const float* row = W + i * ldw;
        for (int64_t j = 0; j < m; ++j) {
            const float v = row[j];
            if (v == 0.0f) continue;
            const uint32_t id = map.find_or_add(float_bits(v));
            if (id == rawfreq.size()) { rawfreq.push_back(0); raw_keys.push_back(float_bits(v)); }
            rawfreq[id]++;
            const uint64_t p = cursor[(size_t)j]++;
            s.ri[(size_t)p] = (uint32_t)i;
            s.sym[(size_t)p] = id;
        }
    }
    // renumber ids so that values ascend
    const size_t k = rawfreq.size();
    std::vector<uint32_t> order(k);
    for (size_t i = 0; i < k; ++i) order[i] = (uint32_t)i;
    std::vector<float> rawval(k);
    for (size_t i = 0; i < k; ++i) std::memcpy(&rawval[i], &raw_keys[i], 4);
    std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return rawval[a] < rawval[b]; });
    std::vector<uint32_t> rank(k);
    s.values.resize(k); s.freq.resize(k);
    for (size_t r = 0; r < k; ++r) { rank[order[r]] = (uint32_t)r; s.values[r] = rawval[order[r]]; s.freq[r] = rawfreq[order[r]]; }
    for (size_t p = 0; p < s.sym.size(); ++p) s.sym[p] = rank[s.sym[p]];
    return HAC_OK;
}

} // namespace

namespace hac_internal {

uint32_t ceil_log2(uint64_t v) { uint32_t b = 0; while (((uint64_t)1 << b) < v) ++b; return b; }

// entries of the row index: nq + 1 per column, nq = ceil(n / chunk_rows)
uint64_t row_index_entries(const hac_desc_t& d)
{
    return d.chunk_rows ? d.m * ((d.n + d.chunk_rows - 1) / d.chunk_rows + 1) : 0;
}

// Rows per entry of the row index: 0 (none), the caller's value, or about 8 non-zeros per entry.
uint32_t pick_chunk_rows(const hac_opts_t* opts, uint64_t n, uint64_t m, uint64_t nnz)
{
    if (!opts || !opts->chunk_rows) return 0;
    if (opts->chunk_rows != HAC_CHUNK_ROWS_AUTO) return opts->chunk_rows;
    const uint64_t per8 = nnz ? (8 * n * m + nnz - 1) / nnz : n;         // rows that hold 8 non-zeros of a column on average
    uint64_t r = std::max<uint64_t>(per8, 16);
    r = (r + 3) / 4 * 4;
    return (uint32_t)std::min<uint64_t>(r, n);
}

// Section offsets and total size from the counts already in the header.  One order for all
// formats: code tables, stream, per-column arrays, chunk entries, and ri when it is stored as fields.
void place_tables(hac_desc_t& d, uint64_t& cursor, uint32_t k_values)
{
    auto place = [&](uint64_t bytes) { const uint64_t o = align_up(cursor); cursor = o + bytes; return o; };
    d.off_codebook = place(4ull * (k_values > d.k_sym ? k_values : d.k_sym));
    d.off_codelen = place(d.k_sym);
    d.off_canon = place(3 * 33 * 4);
    d.off_symsort = place(4ull * d.k_sym);
    d.off_lut = place(4ull << d.lut_bits);
}

void place_layer(hac_desc_t& d, uint64_t& cursor)
{
    auto place = [&](uint64_t bytes) { const uint64_t o = align_up(cursor); cursor = o + bytes; return o; };
    d.off_stream = place(4 * d.n_words + kTailPad);
    d.off_col_chunk = place(4 * (d.m + 1));
    d.off_col_pos = place(4 * (d.m + 1));
    d.off_col_bit = place(4 * (d.m + 1));
    d.off_chunk_ent = place(d.n_chunks * (d.ent_bits / 8) + 8);
    if (d.format == HAC_FORMAT_SHAC && d.ri_coding == HAC_RI_FIELDS)
        d.off_ri = place(4 * ((d.nnz * d.ri_bits + 31) / 32) + kTailPad);
    if (d.chunk_rows) d.off_row_ent = place(row_index_entries(d) * (d.rent_bits / 8) + 8);
}

void place_sections(hac_desc_t& d)
{
    uint64_t cursor = sizeof(hac_desc_t);
    place_tables(d, cursor, 0);
    place_layer(d, cursor);
    d.blob_bytes = align_up(cursor);
}

// Fills the sections common to all stream formats (tables).
int write_tables(uint8_t* base, const hac_desc_t& d, const std::vector<float>& codebook,
                 const std::vector<uint8_t>& len, const CodeTables& t, const std::vector<uint32_t>& lut)
{
    if (!codebook.empty()) std::memcpy(base + d.off_codebook, codebook.data(), codebook.size() * 4);
    if (!len.empty()) std::memcpy(base + d.off_codelen, len.data(), len.size());
    uint32_t* canon = reinterpret_cast<uint32_t*>(base + d.off_canon);
    std::memcpy(canon, t.first_code, 33 * 4);
    std::memcpy(canon + 33, t.count, 33 * 4);
    std::memcpy(canon + 66, t.first_index, 33 * 4);
    if (!t.symsort.empty()) std::memcpy(base + d.off_symsort, t.symsort.data(), t.symsort.size() * 4);
    std::memcpy(base + d.off_lut, lut.data(), lut.size() * 4);
    return HAC_OK;
}

uint32_t pick_lut_bits(const hac_opts_t* opts, uint32_t lmax)
{
    uint32_t b = opts && opts->lut_bits ? opts->lut_bits : std::min<uint32_t>(std::max<uint32_t>(lmax, 1), 10);
    return b;
}

uint32_t pick_chunk(const hac_opts_t* opts, uint64_t max_col_nnz)
{
    if (opts && opts->chunk_nnz == HAC_CHUNK_PER_COLUMN) return kChunkPerColumn | kChunkPerColumnLeast;
    if (opts && opts->chunk_nnz) return opts->chunk_nnz;
    const uint64_t c = (max_col_nnz + 63) / 64;              // a 64-lane wavefront covers any column
    return (uint32_t)std::min<uint64_t>(std::max<uint64_t>(c, 4), 65536);
}

int check_opts(const hac_opts_t* opts)
{
    if (!opts) return HAC_OK;
    if (opts->lut_bits > 12 || (opts->chunk_nnz > 65536 && opts->chunk_nnz != HAC_CHUNK_PER_COLUMN) ||
        opts->ri_coding > HAC_RI_RICE) return HAC_EINVAL;
    if (opts->chunk_rows && opts->ri_coding == HAC_RI_RICE) return HAC_EINVAL;
    return HAC_OK;
}

uint32_t rice_length(uint32_t d, uint32_t k)
{
    const uint32_t q = d >> k;
    return q < kRiceEscape ? q + 1 + k : kRiceEscape + 1 + 32;
}

} // namespace hac_internal

namespace {

int check_args(const float* W, int64_t n, int64_t m, int64_t ldw, void** blob, size_t* bytes)
{
    if (!W || !blob || !bytes) return HAC_EINVAL;
    if (n < 1 || m < 1 || ldw < m) return HAC_EINVAL;
    if (n > 0x7fffffffll || m > 0x7fffffffll) return HAC_ERANGE;
    return HAC_OK;
}

// Column-wise chunk bookkeeping shared by both encoders.
struct ColumnIndex {
    std::vector<uint32_t> col_chunk, col_pos, col_bit;   // m + 1 each
    uint64_t n_chunks = 0, max_col_nnz = 0;
    void build(const Scan& s, uint32_t chunk) {
        const size_t m = (size_t)s.m;
        col_chunk.assign(m + 1, 0); col_pos.assign(m + 1, 0); col_bit.assign(m + 1, 0);
        n_chunks = 0;
        for (size_t j = 0; j < m; ++j) {
            const uint64_t cnt = s.cb[j + 1] - s.cb[j];
            col_chunk[j] = (uint32_t)n_chunks;
            col_pos[j] = (uint32_t)s.cb[j];
            const uint32_t c = chunk_of_column(chunk, cnt);
            n_chunks += (cnt + c - 1) / c;
        }
        col_chunk[m] = (uint32_t)n_chunks;
        col_pos[m] = (uint32_t)s.cb[m];
    }
};

// ---- Golomb-Rice code of the row gaps (sHAC with ri_coding = HAC_RI_RICE) ----
// gap of CSC position p: rows skipped since the previous non-zero of the column (or its top)
inline uint32_t gap_at(const Scan& s, uint64_t p, uint64_t col_first)
{
    return p == col_first ? s.ri[(size_t)p] : s.ri[(size_t)p] - s.ri[(size_t)p - 1] - 1;
}

uint64_t max_nnz_per_column(const Scan& s)
{
    uint64_t mx = 0;
    for (size_t j = 0; j + 1 < s.cb.size(); ++j) mx = std::max(mx, s.cb[j + 1] - s.cb[j]);
    return mx;
}

// ---- one Huffman dictionary: a layer's own, or the one all layers of a network share ----
struct Dict {
    std::vector<float> codebook;       // 0.0 first when has_zero, then ascending
    std::vector<uint64_t> freq;
    std::vector<uint8_t> len;
    uint32_t lmax = 0, lut_bits = 0;
    CodeTables t;
    std::vector<uint32_t> lut;
    bool has_zero = false;
};

int finish_dict(Dict& D, const hac_opts_t* opts)
{
    if (!huffman_lengths(D.freq, D.len, D.lmax)) return HAC_ERANGE;
    canonical_codes(D.len, D.t);
    D.lut_bits = pick_lut_bits(opts, D.lmax);
    if (D.lut_bits < 1 || D.lut_bits > 12) return HAC_EINVAL;
    build_lut(D.len, D.t, D.lut_bits, D.lut);
    return HAC_OK;
}

// What one layer needs besides the dictionary: the header with every count filled in (offsets
// are placed by the caller), the per-column arrays, and the dictionary symbol of each of the
// layer's own non-zero values.
struct LayerPlan {
    hac_desc_t d;
    ColumnIndex ci;
    std::vector<uint32_t> map;         // index into Scan::values -> dictionary symbol
    LayerPlan() { std::memset(&d, 0, sizeof d); }
};

void plan_common(const Scan& s, const Dict& D, uint32_t format, LayerPlan& P)
{
    hac_desc_t& d = P.d;
    d.magic = kMagic; d.version = kVersion; d.format = format; d.header_bytes = 256;
    d.n = (uint64_t)s.n; d.m = (uint64_t)s.m; d.nnz = s.ri.size();
    d.k_sym = (uint32_t)D.codebook.size(); d.lmax = D.lmax; d.lut_bits = D.lut_bits;
}

// Row index: header fields (entry width, the fullest tile).  Needs n, m, nnz, max_col_bits and
// max_col_nnz in the header.
int plan_row_index(const Scan& s, const hac_opts_t* opts, hac_desc_t& d)
{
    const uint32_t cr = pick_chunk_rows(opts, d.n, d.m, d.nnz);
    if (!cr) return HAC_OK;
    if (d.ri_coding == HAC_RI_RICE) return HAC_EINVAL;
    if (cr > d.n || (cr < d.n && cr % 4)) return HAC_EINVAL;
    const uint64_t nq = (d.n + cr - 1) / cr;
    if (d.m * (nq + 1) > 0x7ffffff0ull) return HAC_ERANGE;
    d.chunk_rows = cr;
    const uint32_t pos_bits = std::max<uint32_t>(ceil_log2(d.max_col_nnz + 1), 1);
    const uint32_t bit_bits = std::max<uint32_t>(ceil_log2(d.max_col_bits + 1), 1);
    d.rent_bits = pos_bits + bit_bits <= 32 ? 32 : 64;
    d.rpos_bits = d.rent_bits == 32 ? (uint8_t)pos_bits : 0;
    // the fullest tile of 16 columns x 4 entries
    uint64_t worst = 0;
    const uint64_t span = 4ull * cr;
    std::vector<uint64_t> tile((size_t)((d.n + span - 1) / span));
    for (uint64_t j0 = 0; j0 < d.m; j0 += 16) {
        std::fill(tile.begin(), tile.end(), 0);
        const uint64_t j1 = std::min<uint64_t>(j0 + 16, d.m);
        for (uint64_t p = s.cb[(size_t)j0]; p < s.cb[(size_t)j1]; ++p) tile[(size_t)(s.ri[(size_t)p] / span)]++;
        for (uint64_t t : tile) worst = std::max(worst, t);
    }
    d.max_tile_nnz = (uint16_t)std::min<uint64_t>(worst, 65535);
    return HAC_OK;
}

// One column's entries of the row index.  rel_bit_of(q): stream bit, relative to the column's first,
// at which the rows >= q * chunk_rows begin; rel_pos: non-zeros of the column above that row.
template <class BitOf>
void write_row_index_column(uint8_t* base, const hac_desc_t& d, const Scan& s, uint64_t j, uint64_t col_bits, BitOf rel_bit_of)
{
    const uint64_t nq = (d.n + d.chunk_rows - 1) / d.chunk_rows;
    uint32_t* ent = reinterpret_cast<uint32_t*>(base + d.off_row_ent);
    const uint64_t p0 = s.cb[(size_t)j], pend = s.cb[(size_t)j + 1];
    uint64_t p = p0;
    for (uint64_t q = 0; q <= nq; ++q) {
        const uint64_t row = q * d.chunk_rows;
        while (p < pend && s.ri[(size_t)p] < row) ++p;
        const uint64_t rel_pos = q == nq ? pend - p0 : p - p0;
        const uint64_t rel_bit = q == nq ? col_bits : rel_bit_of(q, p);
        const uint64_t e = j * (nq + 1) + q;
        if (d.rent_bits == 32) ent[e] = (uint32_t)((rel_bit << d.rpos_bits) | rel_pos);
        else { ent[2 * e] = (uint32_t)rel_pos; ent[2 * e + 1] = (uint32_t)rel_bit; }
    }
}

// HAC (Sect. IV-B): every entry of W, zeros included, gets a codeword.
int plan_hac(const Scan& s, const Dict& D, const hac_opts_t* opts, LayerPlan& P)
{
    const int64_t n = s.n, m = s.m;
    if (s.zeros && !D.has_zero) return HAC_EINVAL;
    const uint32_t zlen = D.has_zero ? D.len[0] : 0, zcode = D.has_zero ? D.t.code[0] : 0;
    uint64_t total_bits = s.zeros * zlen;
    for (size_t i = 0; i < s.freq.size(); ++i) total_bits += s.freq[i] * D.len[P.map[i]];
    if (total_bits > 0xfffffff0ull) return HAC_ERANGE;
    const uint64_t max_col_nnz = max_nnz_per_column(s);
    const uint32_t Cn = pick_chunk(opts, max_col_nnz);
    P.ci.build(s, Cn);
    if (P.ci.n_chunks > 0xfffffff0ull) return HAC_ERANGE;
    uint64_t max_col_bits = 0;
    for (int64_t j = 0; j < m; ++j) {
        uint64_t bits = ((uint64_t)n - (s.cb[(size_t)j + 1] - s.cb[(size_t)j])) * zlen;
        for (uint64_t p = s.cb[(size_t)j]; p < s.cb[(size_t)j + 1]; ++p) bits += D.len[P.map[s.sym[(size_t)p]]];
        max_col_bits = std::max(max_col_bits, bits);
    }
    const uint32_t row_bits = std::max<uint32_t>(ceil_log2((uint64_t)n), 1);
    const uint32_t brel_bits = std::max<uint32_t>(ceil_log2(max_col_bits + 1), 1);
    const uint32_t ent_bits = row_bits + brel_bits <= 32 ? 32 : 64;
    plan_common(s, D, HAC_FORMAT_HAC, P);
    hac_desc_t& d = P.d;
    d.total_bits = total_bits; d.n_words = (total_bits + 31) / 32;
    d.has_zero = D.has_zero;
    d.zero_len = (D.has_zero && zcode == 0) ? zlen : 0;      // canonical: all-zero word <=> a shortest one
    d.chunk = Cn; d.ri_bits = 0;
    d.ent_bits = ent_bits; d.row_bits = ent_bits == 32 ? row_bits : 0; d.n_chunks = P.ci.n_chunks;
    d.max_col_bits = max_col_bits; d.max_col_nnz = max_col_nnz;
    return plan_row_index(s, opts, d);
}

void write_column_arrays(uint8_t* base, const hac_desc_t& d, const ColumnIndex& ci)
{
    const size_t bytes = 4 * ((size_t)d.m + 1);
    std::memcpy(base + d.off_col_chunk, ci.col_chunk.data(), bytes);
    std::memcpy(base + d.off_col_pos, ci.col_pos.data(), bytes);
    std::memcpy(base + d.off_col_bit, ci.col_bit.data(), bytes);
}

int write_hac(uint8_t* base, const Scan& s, const Dict& D, LayerPlan& P)
{
    const hac_desc_t& d = P.d;
    const int64_t n = s.n, m = s.m;
    const uint32_t Cn = d.chunk, ent_bits = d.ent_bits, row_bits = d.row_bits;
    const uint32_t zlen = D.has_zero ? D.len[0] : 0, zcode = D.has_zero ? D.t.code[0] : 0;
    BitWriter bw = { reinterpret_cast<uint32_t*>(base + d.off_stream), 0 };
    uint32_t* ent = reinterpret_cast<uint32_t*>(base + d.off_chunk_ent);
    auto put_zeros = [&](uint64_t count) {
        if (!count) return;
        if (zcode == 0) bw.skip(count * zlen);              // zero bits are already there
        else for (uint64_t r = 0; r < count; ++r) bw.put(zcode, zlen);
    };
    uint64_t chunk = 0;
    std::vector<uint64_t> nz_bit;                            // row index: where each non-zero's codeword starts
    for (int64_t j = 0; j < m; ++j) {
        uint64_t row = 0;                                    // next row to be written
        const uint64_t p0 = s.cb[(size_t)j], pend = s.cb[(size_t)j + 1];
        P.ci.col_bit[(size_t)j] = (uint32_t)bw.bitpos;
        const uint64_t col_bit0 = bw.bitpos;
        if (d.chunk_rows) nz_bit.assign((size_t)(pend - p0), 0);
        const uint32_t cj = chunk_of_column(Cn, pend - p0);
        for (uint64_t p = p0; p < pend; ++p) {
            if ((p - p0) % cj == 0) {                        // a chunk starts before this non-zero's zero run
                const uint64_t rel = bw.bitpos - col_bit0;
                if (ent_bits == 32) ent[chunk] = (uint32_t)((rel << row_bits) | row);
                else { ent[2 * chunk] = (uint32_t)row; ent[2 * chunk + 1] = (uint32_t)rel; }
                ++chunk;
            }
            put_zeros(s.ri[(size_t)p] - row);
            if (d.chunk_rows) nz_bit[(size_t)(p - p0)] = bw.bitpos - col_bit0;
            const uint32_t sy = P.map[s.sym[(size_t)p]];
            bw.put(D.t.code[sy], D.len[sy]);
            row = (uint64_t)s.ri[(size_t)p] + 1;
        }
        put_zeros((uint64_t)n - row);
        if (d.chunk_rows) {
            // the codeword of entry (q * chunk_rows, j): the zeros between it and the next non-zero below
            // (or the column's end) lie in front of that non-zero's codeword (or of the column's end)
            const uint64_t col_bits = bw.bitpos - col_bit0;
            write_row_index_column(base, d, s, (uint64_t)j, col_bits, [&](uint64_t q, uint64_t p) {
                const uint64_t r = q * d.chunk_rows;
                if (p < pend) return nz_bit[(size_t)(p - p0)] - (s.ri[(size_t)p] - r) * zlen;
                return col_bits - ((uint64_t)n - r) * zlen;
            });
        }
    }
    P.ci.col_bit[(size_t)m] = (uint32_t)bw.bitpos;
    write_column_arrays(base, d, P.ci);
    return (chunk != P.ci.n_chunks || bw.bitpos != d.total_bits) ? HAC_EFORMAT : HAC_OK;
}

// sHAC (Sect. IV-C): the non-zeros get codewords; ri is stored as fields, or (the extension)
// as Rice-coded gaps in front of each codeword.
int check_shac_opts(const hac_opts_t* opts, int64_t n, bool& rice, uint32_t& ri_bits)
{
    const uint32_t need_bits = std::max<uint32_t>(ceil_log2((uint64_t)n), 1);
    rice = opts && opts->ri_coding == HAC_RI_RICE;
    if (rice && opts->ri_bits) return HAC_EINVAL;
    ri_bits = opts && opts->ri_bits ? opts->ri_bits : need_bits;
    if (ri_bits < need_bits || ri_bits > 32) return HAC_EINVAL;
    return HAC_OK;
}

int plan_shac(const Scan& s, const Dict& D, const hac_opts_t* opts, LayerPlan& P)
{
    const int64_t n = s.n, m = s.m;
    bool rice; uint32_t ri_bits;
    int rc = check_shac_opts(opts, n, rice, ri_bits);
    if (rc) return rc;
    const uint64_t nnz = s.ri.size();
    uint64_t total_bits = 0;
    for (size_t i = 0; i < s.freq.size(); ++i) total_bits += s.freq[i] * D.len[P.map[i]];
    if (total_bits > 0xfffffff0ull) return HAC_ERANGE;
    const uint64_t max_col_nnz = max_nnz_per_column(s);
    const uint32_t Cn = pick_chunk(opts, max_col_nnz);
    P.ci.build(s, Cn);
    plan_common(s, D, HAC_FORMAT_SHAC, P);
    hac_desc_t& d = P.d;
    d.chunk = Cn; d.n_chunks = P.ci.n_chunks; d.max_col_nnz = max_col_nnz;
    if (rice) {
        uint32_t k = 0; uint64_t gap_bits = ~0ull;
        for (uint32_t kk = 0; kk <= kRiceKMax; ++kk) {
            uint64_t tot = 0;
            for (int64_t j = 0; j < m; ++j)
                for (uint64_t p = s.cb[(size_t)j]; p < s.cb[(size_t)j + 1]; ++p)
                    tot += rice_length(gap_at(s, p, s.cb[(size_t)j]), kk);
            if (tot < gap_bits) { gap_bits = tot; k = kk; }
        }
        if (nnz == 0) gap_bits = 0;
        total_bits += gap_bits;
        if (total_bits > 0xfffffff0ull) return HAC_ERANGE;
        uint64_t max_col_bits = 0;
        for (int64_t j = 0; j < m; ++j) {
            uint64_t bits = 0;
            for (uint64_t p = s.cb[(size_t)j]; p < s.cb[(size_t)j + 1]; ++p)
                bits += D.len[P.map[s.sym[(size_t)p]]] + rice_length(gap_at(s, p, s.cb[(size_t)j]), k);
            max_col_bits = std::max(max_col_bits, bits);
        }
        const uint32_t row_bits = std::max<uint32_t>(ceil_log2((uint64_t)n), 1);
        const uint32_t brel_bits = std::max<uint32_t>(ceil_log2(max_col_bits + 1), 1);
        const uint32_t ent_bits = row_bits + brel_bits <= 32 ? 32 : 64;
        d.ri_bits = 0; d.ent_bits = ent_bits; d.row_bits = ent_bits == 32 ? row_bits : 0;
        d.max_col_bits = max_col_bits;
        d.ri_coding = HAC_RI_RICE; d.rice_k = k; d.gap_bits = gap_bits;
    } else {
        uint64_t max_col_bits = 0;
        for (int64_t j = 0; j < m; ++j) {
            uint64_t bits = 0;
            for (uint64_t p = s.cb[(size_t)j]; p < s.cb[(size_t)j + 1]; ++p) bits += D.len[P.map[s.sym[(size_t)p]]];
            max_col_bits = std::max(max_col_bits, bits);
        }
        if (nnz * (uint64_t)ri_bits > 0xfffffff0ull * 32ull) return HAC_ERANGE;
        d.ri_bits = ri_bits; d.ent_bits = max_col_bits < 65536 ? 16 : 32; d.row_bits = 0;
        d.max_col_bits = max_col_bits;
    }
    d.total_bits = total_bits; d.n_words = (total_bits + 31) / 32;
    return plan_row_index(s, opts, d);
}

int write_shac(uint8_t* base, const Scan& s, const Dict& D, LayerPlan& P)
{
    const hac_desc_t& d = P.d;
    const int64_t m = s.m;
    const uint32_t Cn = d.chunk, ent_bits = d.ent_bits;
    BitWriter bw = { reinterpret_cast<uint32_t*>(base + d.off_stream), 0 };
    uint64_t chunk = 0;
    if (d.ri_coding == HAC_RI_RICE) {
        // ---- gaps in the stream, in front of each value's codeword ----
        const uint32_t k = d.rice_k, row_bits = d.row_bits;
        uint32_t* ent = reinterpret_cast<uint32_t*>(base + d.off_chunk_ent);
        for (int64_t j = 0; j < m; ++j) {
            const uint64_t p0 = s.cb[(size_t)j], pend = s.cb[(size_t)j + 1];
            P.ci.col_bit[(size_t)j] = (uint32_t)bw.bitpos;
            const uint64_t col_bit0 = bw.bitpos;
            const uint32_t cj = chunk_of_column(Cn, pend - p0);
            for (uint64_t p = p0; p < pend; ++p) {
                const uint32_t g = gap_at(s, p, p0);
                if ((p - p0) % cj == 0) {
                    const uint64_t rel = bw.bitpos - col_bit0;
                    const uint64_t row = (uint64_t)s.ri[(size_t)p] - g;      // the row the gap counts from
                    if (ent_bits == 32) ent[chunk] = (uint32_t)((rel << row_bits) | row);
                    else { ent[2 * chunk] = (uint32_t)row; ent[2 * chunk + 1] = (uint32_t)rel; }
                    ++chunk;
                }
                const uint32_t q = g >> k;
                if (q < kRiceEscape) {
                    bw.skip(q);
                    bw.put((1u << k) | (g & ((1u << k) - 1u)), k + 1);
                } else {
                    bw.skip(kRiceEscape);
                    bw.put(1u, 1);
                    bw.put(g, 32);
                }
                const uint32_t sy = P.map[s.sym[(size_t)p]];
                bw.put(D.t.code[sy], D.len[sy]);
            }
        }
    } else {
        BitWriter rw = { reinterpret_cast<uint32_t*>(base + d.off_ri), 0 };
        uint16_t* ent16 = reinterpret_cast<uint16_t*>(base + d.off_chunk_ent);
        uint32_t* ent32 = reinterpret_cast<uint32_t*>(base + d.off_chunk_ent);
        std::vector<uint64_t> nz_bit;
        for (int64_t j = 0; j < m; ++j) {
            const uint64_t p0 = s.cb[(size_t)j], pend = s.cb[(size_t)j + 1];
            P.ci.col_bit[(size_t)j] = (uint32_t)bw.bitpos;
            const uint64_t col_bit0 = bw.bitpos;
            if (d.chunk_rows) nz_bit.assign((size_t)(pend - p0), 0);
            const uint32_t cj = chunk_of_column(Cn, pend - p0);
            for (uint64_t p = p0; p < pend; ++p) {
                if ((p - p0) % cj == 0) {
                    const uint64_t rel = bw.bitpos - col_bit0;
                    if (ent_bits == 16) ent16[chunk] = (uint16_t)rel; else ent32[chunk] = (uint32_t)rel;
                    ++chunk;
                }
                if (d.chunk_rows) nz_bit[(size_t)(p - p0)] = bw.bitpos - col_bit0;
                const uint32_t sy = P.map[s.sym[(size_t)p]];
                bw.put(D.t.code[sy], D.len[sy]);
                rw.put(s.ri[(size_t)p], d.ri_bits);
            }
            if (d.chunk_rows) {
                const uint64_t col_bits = bw.bitpos - col_bit0;
                write_row_index_column(base, d, s, (uint64_t)j, col_bits, [&](uint64_t, uint64_t p) {
                    return p < pend ? nz_bit[(size_t)(p - p0)] : col_bits;
                });
            }
        }
    }
    P.ci.col_bit[(size_t)m] = (uint32_t)bw.bitpos;
    write_column_arrays(base, d, P.ci);
    return (chunk != P.ci.n_chunks || bw.bitpos != d.total_bits) ? HAC_EFORMAT : HAC_OK;
}

// A layer's own dictionary: HAC numbers 0.0 as symbol 0 when it occurs; sHAC has no symbol for it.
void own_dict(const Scan& s, bool with_zero, Dict& D, std::vector<uint32_t>& map)
{
    D.has_zero = with_zero && s.zeros > 0;
    if (D.has_zero) { D.codebook.push_back(0.0f); D.freq.push_back(s.zeros); }
    D.codebook.insert(D.codebook.end(), s.values.begin(), s.values.end());
    D.freq.insert(D.freq.end(), s.freq.begin(), s.freq.end());
    const uint32_t shift = D.has_zero ? 1u : 0u;
    map.resize(s.values.size());
    for (size_t i = 0; i < map.size(); ++i) map[i] = (uint32_t)i + shift;
}

// One self-contained blob: header, the layer's own tables, its sections.
int encode_single(uint32_t format, const float* W, int64_t n, int64_t m, int64_t ldw,
                  const hac_opts_t* opts, void** blob, size_t* blob_bytes)
{
    Scan s;
    int rc = scan_matrix(W, n, m, ldw, s);
    if (rc) return rc;
    Dict D; LayerPlan P;
    own_dict(s, format == HAC_FORMAT_HAC, D, P.map);
    if ((rc = finish_dict(D, opts))) return rc;
    rc = format == HAC_FORMAT_HAC ? plan_hac(s, D, opts, P) : plan_shac(s, D, opts, P);
    if (rc) return rc;
    hac_desc_t& d = P.d;
    place_sections(d);
    uint8_t* base = static_cast<uint8_t*>(std::calloc(1, (size_t)d.blob_bytes));
    if (!base) return HAC_ENOMEM;
    std::memcpy(base, &d, sizeof d);
    write_tables(base, d, D.codebook, D.len, D.t, D.lut);
    rc = format == HAC_FORMAT_HAC ? write_hac(base, s, D, P) : write_shac(base, s, D, P);
    if (rc) { std::free(base); return rc; }
    *blob = base; *blob_bytes = (size_t)d.blob_bytes;
    return HAC_OK;
}

} // namespace

// =================================================================================
// HAC encoder (Sect. IV-B)
// =================================================================================
extern "C" int hac_encode(const float* W, int64_t n, int64_t m, int64_t ldw,
                          const hac_opts_t* opts, void** blob, size_t* blob_bytes)
{
    int rc = check_args(W, n, m, ldw, blob, blob_bytes);
    if (rc) return rc;
    *blob = nullptr; *blob_bytes = 0;
    if ((rc = check_opts(opts))) return rc;
    if (opts && opts->ri_coding) return HAC_EINVAL;          // the address map of HAC is the stream itself
    try {
        return encode_single(HAC_FORMAT_HAC, W, n, m, ldw, opts, blob, blob_bytes);
    } catch (const std::bad_alloc&) {
        return HAC_ENOMEM;
    }
}

// =================================================================================
// sHAC encoder (Sect. IV-C)
// =================================================================================
extern "C" int shac_encode(const float* W, int64_t n, int64_t m, int64_t ldw,
                           const hac_opts_t* opts, void** blob, size_t* blob_bytes)
{
    int rc = check_args(W, n, m, ldw, blob, blob_bytes);
    if (rc) return rc;
    *blob = nullptr; *blob_bytes = 0;
    if ((rc = check_opts(opts))) return rc;
    bool rice; uint32_t ri_bits;
    if ((rc = check_shac_opts(opts, n, rice, ri_bits))) return rc;
    try {
        return encode_single(HAC_FORMAT_SHAC, W, n, m, ldw, opts, blob, blob_bytes);
    } catch (const std::bad_alloc&) {
        return HAC_ENOMEM;
    }
}

// =================================================================================
// network blob: all layers written with one shared dictionary (Sect. V-H)
// =================================================================================
extern "C" int hac_net_encode(uint32_t n_layers, const uint32_t* formats, const float* const* W,
                              const int64_t* n, const int64_t* m, const int64_t* ldw,
                              const hac_opts_t* opts, void** blob, size_t* blob_bytes)
{
    if (!blob || !blob_bytes) return HAC_EINVAL;
    *blob = nullptr; *blob_bytes = 0;
    if (!formats || !W || !n || !m || !ldw || n_layers < 1 || n_layers > 65536) return HAC_EINVAL;
    int rc = check_opts(opts);
    if (rc) return rc;
    for (uint32_t l = 0; l < n_layers; ++l) {
        if (formats[l] != HAC_FORMAT_HAC && formats[l] != HAC_FORMAT_SHAC && formats[l] != HAC_FORMAT_IM) return HAC_EINVAL;
        void* dummy_blob; size_t dummy_bytes;
        if ((rc = check_args(W[l], n[l], m[l], ldw[l], &dummy_blob, &dummy_bytes))) return rc;
        if (formats[l] == HAC_FORMAT_SHAC) {
            bool rice; uint32_t ri_bits;
            if ((rc = check_shac_opts(opts, n[l], rice, ri_bits))) return rc;
        }
    }
    try {
        std::vector<Scan> scans(n_layers);
        for (uint32_t l = 0; l < n_layers; ++l)
            if ((rc = scan_matrix(W[l], n[l], m[l], ldw[l], scans[l]))) return rc;
        // the pooled source: what every layer writes into its stream
        std::vector<std::pair<float, uint64_t>> pool;
        uint64_t zeros = 0;
        for (uint32_t l = 0; l < n_layers; ++l) {
            const Scan& s = scans[l];
            if (formats[l] == HAC_FORMAT_IM) continue;        // pointers, no codewords
            if (formats[l] == HAC_FORMAT_HAC) zeros += s.zeros;
            for (size_t i = 0; i < s.values.size(); ++i) pool.emplace_back(s.values[i], s.freq[i]);
        }
        std::sort(pool.begin(), pool.end(), [](const std::pair<float, uint64_t>& a, const std::pair<float, uint64_t>& b) {
            return a.first < b.first;
        });
        Dict D;
        D.has_zero = zeros > 0;
        if (D.has_zero) { D.codebook.push_back(0.0f); D.freq.push_back(zeros); }
        for (size_t i = 0; i < pool.size(); ++i) {
            if (i && pool[i].first == pool[i - 1].first) D.freq.back() += pool[i].second;
            else { D.codebook.push_back(pool[i].first); D.freq.push_back(pool[i].second); }
        }
        if ((rc = finish_dict(D, opts))) return rc;
        const uint32_t first = D.has_zero ? 1u : 0u;
        const uint32_t k_sym = (uint32_t)D.codebook.size();
        auto coded_symbol = [&](float v, uint32_t& sym) {
            const auto it = std::lower_bound(D.codebook.begin() + first, D.codebook.end(), v);
            if (it == D.codebook.end() || *it != v) return false;
            sym = (uint32_t)(it - D.codebook.begin());
            return true;
        };
        // values that only index-map layers hold: behind the shared symbols, 0.0 first, then ascending
        std::vector<float> extras;
        bool extra_zero = false, any_im = false;
        for (uint32_t l = 0; l < n_layers; ++l) {
            if (formats[l] != HAC_FORMAT_IM) continue;
            any_im = true;
            if (scans[l].zeros && !D.has_zero) extra_zero = true;
            uint32_t sym;
            for (float v : scans[l].values) if (!coded_symbol(v, sym)) extras.push_back(v);
        }
        std::sort(extras.begin(), extras.end());
        extras.erase(std::unique(extras.begin(), extras.end()), extras.end());
        if (extra_zero) extras.insert(extras.begin(), 0.0f);
        const uint64_t k_values = (uint64_t)k_sym + extras.size();
        if (any_im && (k_values > 65536 || k_values < 1)) return HAC_ERANGE;
        const uint32_t im_bits = k_values <= 256 ? 8 : 16;
        const uint32_t extra_first = extra_zero ? 1u : 0u;
        auto list_index = [&](float v) {                      // position of a non-zero value in the value list
            uint32_t sym;
            if (coded_symbol(v, sym)) return sym;
            const auto it = std::lower_bound(extras.begin() + extra_first, extras.end(), v);
            return k_sym + (uint32_t)(it - extras.begin());
        };

        std::vector<LayerPlan> plans(n_layers);
        for (uint32_t l = 0; l < n_layers; ++l) {
            const Scan& s = scans[l];
            LayerPlan& P = plans[l];
            P.map.resize(s.values.size());
            if (formats[l] == HAC_FORMAT_IM) {
                for (size_t i = 0; i < s.values.size(); ++i) P.map[i] = list_index(s.values[i]);
                hac_desc_t& d = P.d;
                d.magic = kMagic; d.version = kVersion; d.format = HAC_FORMAT_IM; d.header_bytes = 256;
                d.n = (uint64_t)s.n; d.m = (uint64_t)s.m; d.nnz = s.ri.size();
                d.ent_bits = im_bits; d.k_sym = (uint32_t)k_values;
                d.idx_pitch = ((uint64_t)s.m + 15) / 16 * 16;
                d.total_bits = (uint64_t)im_bits * d.n * d.m;
                if (d.n * d.idx_pitch * (im_bits / 8) > 0xffffffff00ull) return HAC_ERANGE;
                d.dict_shared = 1;
                continue;
            }
            uint32_t sym = 0;
            for (size_t i = 0; i < s.values.size(); ++i) { coded_symbol(s.values[i], sym); P.map[i] = sym; }
            rc = formats[l] == HAC_FORMAT_HAC ? plan_hac(s, D, opts, P) : plan_shac(s, D, opts, P);
            if (rc) return rc;
            P.d.has_zero = D.has_zero;
            P.d.dict_shared = 1;
        }

        hac_net_t net;
        std::memset(&net, 0, sizeof net);
        net.magic = kNetMagic; net.version = kNetVersion; net.header_bytes = 256; net.n_layers = n_layers;
        net.off_layers = sizeof(hac_net_t);
        uint64_t cursor = net.off_layers + (uint64_t)n_layers * sizeof(hac_desc_t);
        hac_desc_t tables;
        std::memset(&tables, 0, sizeof tables);
        tables.k_sym = k_sym; tables.lut_bits = D.lut_bits;
        place_tables(tables, cursor, (uint32_t)k_values);
        net.off_codebook = tables.off_codebook; net.off_codelen = tables.off_codelen; net.off_canon = tables.off_canon;
        net.off_symsort = tables.off_symsort; net.off_lut = tables.off_lut;
        net.k_sym = k_sym; net.lmax = D.lmax; net.lut_bits = D.lut_bits; net.has_zero = D.has_zero;
        net.k_values = (uint32_t)k_values;
        for (uint32_t l = 0; l < n_layers; ++l) {
            hac_desc_t& d = plans[l].d;
            d.off_codebook = tables.off_codebook;
            if (d.format == HAC_FORMAT_IM) {                  // the index map, n rows of idx_pitch pointers
                d.off_stream = align_up(cursor);
                cursor = d.off_stream + d.n * d.idx_pitch * (d.ent_bits / 8) + kTailPad;
                continue;
            }
            d.off_codelen = tables.off_codelen; d.off_canon = tables.off_canon;
            d.off_symsort = tables.off_symsort; d.off_lut = tables.off_lut;
            place_layer(d, cursor);
        }
        net.blob_bytes = align_up(cursor);
        for (uint32_t l = 0; l < n_layers; ++l) plans[l].d.blob_bytes = net.blob_bytes;

        uint8_t* base = static_cast<uint8_t*>(std::calloc(1, (size_t)net.blob_bytes));
        if (!base) return HAC_ENOMEM;
        std::memcpy(base, &net, sizeof net);
        write_tables(base, tables, D.codebook, D.len, D.t, D.lut);
        if (!extras.empty()) std::memcpy(base + net.off_codebook + 4ull * k_sym, extras.data(), 4 * extras.size());
        // pointer of the value 0.0 (index-map layers only): the shared symbol 0, or the first extra
        const uint32_t zero_ptr = D.has_zero ? 0u : k_sym;
        for (uint32_t l = 0; l < n_layers; ++l) {
            std::memcpy(base + net.off_layers + (uint64_t)l * sizeof(hac_desc_t), &plans[l].d, sizeof(hac_desc_t));
            if (formats[l] == HAC_FORMAT_IM) {
                const hac_desc_t& d = plans[l].d;
                const Scan& s = scans[l];
                uint8_t* p8 = base + d.off_stream;
                uint16_t* p16 = reinterpret_cast<uint16_t*>(base + d.off_stream);
                if (zero_ptr)                                 // the map starts as all zero bytes: pointer 0
                    for (uint64_t i = 0; i < d.n; ++i)
                        for (uint64_t j = 0; j < d.m; ++j) {
                            if (d.ent_bits == 8) p8[i * d.idx_pitch + j] = (uint8_t)zero_ptr;
                            else p16[i * d.idx_pitch + j] = (uint16_t)zero_ptr;
                        }
                for (int64_t j = 0; j < s.m; ++j)
                    for (uint64_t p = s.cb[(size_t)j]; p < s.cb[(size_t)j + 1]; ++p) {
                        const uint64_t at = (uint64_t)s.ri[(size_t)p] * d.idx_pitch + (uint64_t)j;
                        const uint32_t v = plans[l].map[s.sym[(size_t)p]];
                        if (d.ent_bits == 8) p8[at] = (uint8_t)v; else p16[at] = (uint16_t)v;
                    }
                continue;
            }
            rc = formats[l] == HAC_FORMAT_HAC ? write_hac(base, scans[l], D, plans[l]) : write_shac(base, scans[l], D, plans[l]);
            if (rc) { std::free(base); return rc; }
        }
        *blob = base; *blob_bytes = (size_t)net.blob_bytes;
        return HAC_OK;
    } catch (const std::bad_alloc&) {
        return HAC_ENOMEM;
    }
}

// =================================================================================
// index map encoder (Sect. III-C1)
// =================================================================================
extern "C" int im_encode(const float* W, int64_t n, int64_t m, int64_t ldw,
                         const hac_opts_t* opts, void** blob, size_t* blob_bytes)
{
    int rc = check_args(W, n, m, ldw, blob, blob_bytes);
    if (rc) return rc;
    *blob = nullptr; *blob_bytes = 0;
    if (opts) return HAC_EINVAL;
    try {
        Scan s;
        rc = scan_matrix(W, n, m, ldw, s);
        if (rc) return rc;
        const bool has_zero = s.zeros > 0;
        const uint64_t k = s.values.size() + (has_zero ? 1 : 0);
        if (k > 65536) return HAC_ERANGE;
        const uint32_t bits = k <= 256 ? 8 : 16;
        const uint64_t pitch = ((uint64_t)m + 15) / 16 * 16;
        if ((uint64_t)n * pitch * (bits / 8) > 0xffffffff00ull) return HAC_ERANGE;
        hac_desc_t d;
        std::memset(&d, 0, sizeof d);
        d.magic = kMagic; d.version = kVersion; d.format = HAC_FORMAT_IM; d.header_bytes = 256;
        d.n = (uint64_t)n; d.m = (uint64_t)m; d.nnz = s.ri.size();
        d.total_bits = (uint64_t)bits * (uint64_t)n * (uint64_t)m;
        d.k_sym = (uint32_t)k; d.has_zero = has_zero; d.ent_bits = bits; d.idx_pitch = pitch;
        d.off_codebook = align_up(sizeof(hac_desc_t));
        d.off_stream = align_up(d.off_codebook + 4 * k);
        d.blob_bytes = align_up(d.off_stream + (uint64_t)n * pitch * (bits / 8) + kTailPad);
        uint8_t* base = static_cast<uint8_t*>(std::calloc(1, (size_t)d.blob_bytes));
        if (!base) return HAC_ENOMEM;
        std::memcpy(base, &d, sizeof d);
        float* cb = reinterpret_cast<float*>(base + d.off_codebook);
        const uint32_t shift = has_zero ? 1u : 0u;
        if (has_zero) cb[0] = 0.0f;
        for (size_t i = 0; i < s.values.size(); ++i) cb[i + shift] = s.values[i];
        uint8_t* p8 = base + d.off_stream;
        uint16_t* p16 = reinterpret_cast<uint16_t*>(base + d.off_stream);
        for (int64_t j = 0; j < m; ++j)
            for (uint64_t p = s.cb[(size_t)j]; p < s.cb[(size_t)j + 1]; ++p) {
                const uint64_t at = (uint64_t)s.ri[(size_t)p] * pitch + (uint64_t)j;
                const uint32_t v = s.sym[(size_t)p] + shift;
                if (bits == 8) p8[at] = (uint8_t)v; else p16[at] = (uint16_t)v;
            }
        *blob = base; *blob_bytes = (size_t)d.blob_bytes;
        return HAC_OK;
    } catch (const std::bad_alloc&) {
        return HAC_ENOMEM;
    }
}

extern "C" void hac_free(void* blob) { std::free(blob); }

// =================================================================================
// validation / description
// =================================================================================
namespace {

bool section_ok(const hac_desc_t& d, uint64_t off, uint64_t bytes, size_t total)
{
    if (off < sizeof(hac_desc_t) || off % kAlign) return false;
    if (bytes > total || off > total - bytes) return false;
    return off + bytes <= d.blob_bytes;
}

// A header against the size of the buffer its offsets count from.  in_net: the header of a layer
// of a network blob, whose k_sym / has_zero are those of the shared dictionary.
int check_desc(const hac_desc_t& d, size_t bytes, bool in_net)
{
    if (d.magic != kMagic || d.version != kVersion || d.header_bytes != 256) return HAC_EFORMAT;
    if (d.dict_shared != (in_net ? 1u : 0u)) return HAC_EFORMAT;

    if (d.format != HAC_FORMAT_HAC && d.format != HAC_FORMAT_SHAC && d.format != HAC_FORMAT_IM) return HAC_EFORMAT;
    if (d.blob_bytes > bytes || d.blob_bytes < sizeof(hac_desc_t)) return HAC_EFORMAT;
    if (d.n < 1 || d.m < 1 || d.n > 0x7fffffffull || d.m > 0x7fffffffull) return HAC_EFORMAT;
    if (!d.chunk_rows && (d.off_row_ent || d.rent_bits || d.rpos_bits || d.max_tile_nnz)) return HAC_EFORMAT;
    if (d.chunk_rows && (d.format == HAC_FORMAT_IM || d.ri_coding == HAC_RI_RICE)) return HAC_EFORMAT;
    if (d.format == HAC_FORMAT_IM) {
        if (d.ent_bits != 8 && d.ent_bits != 16) return HAC_EFORMAT;
        if (d.k_sym < 1 || d.k_sym > (d.ent_bits == 8 ? 256u : 65536u) || d.has_zero > (in_net ? 0u : 1u)) return HAC_EFORMAT;
        if (d.idx_pitch != (d.m + 15) / 16 * 16) return HAC_EFORMAT;
        if (d.nnz > d.n * d.m || d.total_bits != (uint64_t)d.ent_bits * d.n * d.m) return HAC_EFORMAT;
        if (d.n_words || d.lmax || d.lut_bits || d.zero_len || d.chunk || d.ri_bits || d.n_chunks || d.off_codelen ||
            d.off_canon || d.off_symsort || d.off_lut || d.off_col_chunk || d.off_col_pos || d.off_col_bit ||
            d.off_chunk_ent || d.off_ri || d.max_col_bits || d.max_col_nnz || d.row_bits || d.ri_coding || d.rice_k ||
            d.gap_bits) return HAC_EFORMAT;
        const size_t tot = (size_t)d.blob_bytes;
        if (!section_ok(d, d.off_codebook, 4ull * d.k_sym, tot)) return HAC_EFORMAT;
        if (d.n * d.idx_pitch > 0xffffffff00ull) return HAC_EFORMAT;
        if (!section_ok(d, d.off_stream, d.n * d.idx_pitch * (d.ent_bits / 8) + kTailPad, tot)) return HAC_EFORMAT;
        return HAC_OK;
    }
    if (d.idx_pitch) return HAC_EFORMAT;
    if (d.nnz > d.n * d.m || d.nnz > 0xfffffff0ull || d.total_bits > 0xfffffff0ull) return HAC_EFORMAT;
    if (d.n_words != (d.total_bits + 31) / 32) return HAC_EFORMAT;
    if (d.lmax > 32 || d.lut_bits < 1 || d.lut_bits > 12) return HAC_EFORMAT;
    if (!in_net && d.k_sym > d.n * d.m) return HAC_EFORMAT;
    if (in_net ? (d.k_sym == 0 && d.total_bits != 0) : ((d.k_sym == 0) != (d.total_bits == 0))) return HAC_EFORMAT;
    if (d.k_sym > 0 && (d.lmax < 1)) return HAC_EFORMAT;
    if (chunk_base(d.chunk) < 1 || chunk_base(d.chunk) > 65536) return HAC_EFORMAT;
    if (d.ri_coding > HAC_RI_RICE) return HAC_EFORMAT;
    if (d.max_col_bits > d.total_bits || d.max_col_nnz > d.nnz || d.max_col_nnz > d.n) return HAC_EFORMAT;
    const size_t tot = (size_t)d.blob_bytes;
    if (!section_ok(d, d.off_codebook, 4ull * d.k_sym, tot)) return HAC_EFORMAT;
    if (!section_ok(d, d.off_codelen, d.k_sym, tot)) return HAC_EFORMAT;
    if (!section_ok(d, d.off_canon, 3 * 33 * 4, tot)) return HAC_EFORMAT;
    if (!section_ok(d, d.off_symsort, 4ull * d.k_sym, tot)) return HAC_EFORMAT;
    if (!section_ok(d, d.off_lut, 4ull << d.lut_bits, tot)) return HAC_EFORMAT;
    if (!section_ok(d, d.off_stream, 4 * d.n_words + kTailPad, tot)) return HAC_EFORMAT;
    if (!section_ok(d, d.off_col_chunk, 4 * (d.m + 1), tot)) return HAC_EFORMAT;
    if (!section_ok(d, d.off_col_pos, 4 * (d.m + 1), tot)) return HAC_EFORMAT;
    if (!section_ok(d, d.off_col_bit, 4 * (d.m + 1), tot)) return HAC_EFORMAT;
    if (d.n_chunks > d.nnz || d.n_chunks > 0xfffffff0ull) return HAC_EFORMAT;
    if (d.format == HAC_FORMAT_HAC) {
        if (d.ent_bits != 32 && d.ent_bits != 64) return HAC_EFORMAT;
        if (d.has_zero > 1) return HAC_EFORMAT;
        if (in_net ? (d.nnz < d.n * d.m && !d.has_zero) : (d.has_zero != (d.nnz < d.n * d.m ? 1u : 0u))) return HAC_EFORMAT;
        const uint32_t need = std::max<uint32_t>(ceil_log2(d.n), 1);
        if (d.ent_bits == 32) {
            if (d.row_bits != need) return HAC_EFORMAT;
            if (d.row_bits + std::max<uint32_t>(ceil_log2(d.max_col_bits + 1), 1) > 32) return HAC_EFORMAT;
        } else if (d.row_bits != 0) return HAC_EFORMAT;
        if (d.ri_bits || d.ri_coding || d.rice_k || d.gap_bits) return HAC_EFORMAT;
    } else if (d.ri_coding == HAC_RI_RICE) {
        if (d.ent_bits != 32 && d.ent_bits != 64) return HAC_EFORMAT;
        const uint32_t need = std::max<uint32_t>(ceil_log2(d.n), 1);
        if (d.ent_bits == 32) {
            if (d.row_bits != need) return HAC_EFORMAT;
            if (d.row_bits + std::max<uint32_t>(ceil_log2(d.max_col_bits + 1), 1) > 32) return HAC_EFORMAT;
        } else if (d.row_bits != 0) return HAC_EFORMAT;
        if (d.ri_bits || d.off_ri || (d.has_zero && !in_net) || d.has_zero > 1 || d.zero_len) return HAC_EFORMAT;
        if (d.rice_k > kRiceKMax || d.gap_bits > d.total_bits) return HAC_EFORMAT;
        if (d.gap_bits < d.nnz) return HAC_EFORMAT;                      // at least the terminating one per gap
    } else {
        if (d.rice_k || d.gap_bits) return HAC_EFORMAT;
        if (d.ent_bits != 16 && d.ent_bits != 32) return HAC_EFORMAT;
        if (d.ent_bits == 16 && d.max_col_bits >= 65536) return HAC_EFORMAT;
        const uint32_t need = std::max<uint32_t>(ceil_log2(d.n), 1);
        if (d.ri_bits < need || d.ri_bits > 32) return HAC_EFORMAT;
        if ((d.has_zero && !in_net) || d.has_zero > 1 || d.zero_len || d.row_bits) return HAC_EFORMAT;
        if (!section_ok(d, d.off_ri, 4 * ((d.nnz * d.ri_bits + 31) / 32) + kTailPad, tot)) return HAC_EFORMAT;
    }
    if (!section_ok(d, d.off_chunk_ent, d.n_chunks * (d.ent_bits / 8) + 8, tot)) return HAC_EFORMAT;
    if (d.chunk_rows) {
        if (d.chunk_rows > d.n || (d.chunk_rows < d.n && d.chunk_rows % 4)) return HAC_EFORMAT;
        if (d.rent_bits != 32 && d.rent_bits != 64) return HAC_EFORMAT;
        const uint32_t pos_bits = std::max<uint32_t>(ceil_log2(d.max_col_nnz + 1), 1);
        if (d.rent_bits == 32 ? (d.rpos_bits != pos_bits || pos_bits + std::max<uint32_t>(ceil_log2(d.max_col_bits + 1), 1) > 32)
                              : d.rpos_bits != 0) return HAC_EFORMAT;
        const uint64_t nq = (d.n + d.chunk_rows - 1) / d.chunk_rows;
        if (d.m * (nq + 1) > 0x7ffffff0ull) return HAC_EFORMAT;
        if (!section_ok(d, d.off_row_ent, row_index_entries(d) * (d.rent_bits / 8) + 8, tot)) return HAC_EFORMAT;
    }
    return HAC_OK;
}

int check_header(const void* blob, size_t bytes, hac_desc_t& d)
{
    if (!blob) return HAC_EINVAL;
    if (bytes < sizeof(hac_desc_t)) return HAC_EFORMAT;
    std::memcpy(&d, blob, sizeof d);
    return check_desc(d, bytes, false);
}

struct View {
    hac_desc_t d;
    const uint8_t* base;
    const float* codebook; const uint8_t* codelen; const uint32_t* canon; const uint32_t* symsort;
    const uint32_t* lut; const uint32_t* stream;
    const uint32_t* colchunk; const uint32_t* colpos; const uint32_t* colbit;
    const uint8_t* ent; const uint32_t* ri;
    const uint32_t* rent;              // row index, or nullptr

    // entry e of the row index
    void row_entry(uint64_t e, uint64_t& rel_bit, uint64_t& rel_pos) const {
        if (d.rent_bits == 32) { rel_bit = rent[e] >> d.rpos_bits; rel_pos = rent[e] & ((1u << d.rpos_bits) - 1u); }
        else { rel_pos = rent[2 * e]; rel_bit = rent[2 * e + 1]; }
    }

    // (relative bit offset, first row) of chunk g
    void entry(uint64_t g, uint64_t& rel, uint64_t& row) const {
        row = 0;
        if (d.format == HAC_FORMAT_HAC || d.ri_coding == HAC_RI_RICE) {
            const uint32_t* e = reinterpret_cast<const uint32_t*>(ent);
            if (d.ent_bits == 32) { rel = e[g] >> d.row_bits; row = e[g] & ((1u << d.row_bits) - 1u); }
            else { row = e[2 * g]; rel = e[2 * g + 1]; }
        } else {
            rel = d.ent_bits == 16 ? reinterpret_cast<const uint16_t*>(ent)[g]
                                   : reinterpret_cast<const uint32_t*>(ent)[g];
        }
    }
};

void make_view(const void* blob, const hac_desc_t& d, View& v)
{
    v.d = d; v.base = static_cast<const uint8_t*>(blob);
    v.codebook = reinterpret_cast<const float*>(v.base + d.off_codebook);
    v.codelen = v.base + d.off_codelen;
    v.canon = reinterpret_cast<const uint32_t*>(v.base + d.off_canon);
    v.symsort = reinterpret_cast<const uint32_t*>(v.base + d.off_symsort);
    v.lut = reinterpret_cast<const uint32_t*>(v.base + d.off_lut);
    v.stream = reinterpret_cast<const uint32_t*>(v.base + d.off_stream);
    v.colchunk = reinterpret_cast<const uint32_t*>(v.base + d.off_col_chunk);
    v.colpos = reinterpret_cast<const uint32_t*>(v.base + d.off_col_pos);
    v.colbit = reinterpret_cast<const uint32_t*>(v.base + d.off_col_bit);
    v.ent = v.base + d.off_chunk_ent;
    v.ri = (d.format == HAC_FORMAT_SHAC && d.ri_coding == HAC_RI_FIELDS)
               ? reinterpret_cast<const uint32_t*>(v.base + d.off_ri) : nullptr;
    v.rent = d.chunk_rows ? reinterpret_cast<const uint32_t*>(v.base + d.off_row_ent) : nullptr;
}

// code tables must describe a complete canonical prefix code consistent with the lengths
int check_tables(const View& v)
{
    const hac_desc_t& d = v.d;
    if (d.k_sym == 0) return HAC_OK;
    std::vector<uint8_t> len(v.codelen, v.codelen + d.k_sym);
    uint32_t lmax = 0;
    unsigned __int128 kraft = 0;
    for (uint32_t s = 0; s < d.k_sym; ++s) {
        if (len[s] < 1 || len[s] > 32) return HAC_EFORMAT;
        lmax = std::max<uint32_t>(lmax, len[s]);
        kraft += (unsigned __int128)1 << (32 - len[s]);
    }
    if (lmax != d.lmax) return HAC_EFORMAT;
    const unsigned __int128 one = (unsigned __int128)1 << 32;
    if (d.k_sym == 1 ? (len[0] != 1) : (kraft != one)) return HAC_EFORMAT;
    CodeTables t; canonical_codes(len, t);
    if (std::memcmp(v.canon, t.first_code, 33 * 4) || std::memcmp(v.canon + 33, t.count, 33 * 4) ||
        std::memcmp(v.canon + 66, t.first_index, 33 * 4)) return HAC_EFORMAT;
    if (std::memcmp(v.symsort, t.symsort.data(), 4ull * d.k_sym)) return HAC_EFORMAT;
    std::vector<uint32_t> lut; build_lut(len, t, d.lut_bits, lut);
    if (std::memcmp(v.lut, lut.data(), lut.size() * 4)) return HAC_EFORMAT;
    for (uint32_t s = 0; s < d.k_sym; ++s) {
        if (!std::isfinite(v.codebook[s])) return HAC_EFORMAT;
        if (s > (d.has_zero ? 1u : 0u) && !(v.codebook[s - 1] < v.codebook[s])) return HAC_EFORMAT;
    }
    if (d.format == HAC_FORMAT_HAC) {
        if (d.has_zero && float_bits(v.codebook[0]) != 0) return HAC_EFORMAT;
        for (uint32_t s = d.has_zero; s < d.k_sym; ++s) if (v.codebook[s] == 0.0f) return HAC_EFORMAT;
        const uint32_t zl = (d.has_zero && t.code[0] == 0) ? len[0] : 0;
        if (zl != d.zero_len) return HAC_EFORMAT;
    } else {
        // an sHAC layer of a network blob may see the shared dictionary's 0.0 (symbol 0), never uses it
        if (d.has_zero && float_bits(v.codebook[0]) != 0) return HAC_EFORMAT;
        for (uint32_t s = d.has_zero; s < d.k_sym; ++s) if (v.codebook[s] == 0.0f) return HAC_EFORMAT;
    }
    return HAC_OK;
}

// sequential canonical decoder over the stream
struct SeqDecoder {
    const View& v;
    uint64_t bitpos = 0;
    explicit SeqDecoder(const View& vv) : v(vv) {}
    inline uint32_t window() const {
        const uint64_t w = bitpos >> 5; const uint32_t off = (uint32_t)(bitpos & 31);
        const uint64_t two = ((uint64_t)v.stream[w] << 32) | v.stream[w + 1];   // tail padding keeps w+1 in bounds
        return (uint32_t)((two << off) >> 32);
    }
    // Rice-coded gap, or -1 (malformed / past the end)
    inline int64_t next_gap(uint32_t k) {
        if (bitpos >= v.d.total_bits) return -1;
        const uint32_t win = window();
        if (win == 0) return -1;                                  // a one must appear within 32 bits
        const uint32_t z = (uint32_t)__builtin_clz(win);
        bitpos += z + 1;
        const uint32_t bits = z < kRiceEscape ? k : 32;
        if (bitpos + bits > v.d.total_bits) return -1;
        uint64_t val = 0;
        if (bits) { val = window() >> (32 - bits); bitpos += bits; }
        return z < kRiceEscape ? (int64_t)(((uint64_t)z << k) | val) : (int64_t)val;
    }
    // returns symbol or -1 (no codeword matches / past the end)
    inline int64_t next() {
        if (bitpos >= v.d.total_bits) return -1;
        const uint32_t win = window();
        const uint32_t e = v.lut[win >> (32 - v.d.lut_bits)];
        uint32_t l = e & 63, s = e >> 6;
        if (l == 0) {
            bool found = false;
            for (l = v.d.lut_bits + 1; l <= v.d.lmax; ++l) {
                const uint32_t c = win >> (32 - l);
                const uint32_t rel = c - v.canon[l];
                if (rel < v.canon[33 + l]) { s = v.symsort[v.canon[66 + l] + rel]; found = true; break; }
            }
            if (!found) return -1;
        }
        if (bitpos + l > v.d.total_bits) return -1;
        bitpos += l;
        return (int64_t)s;
    }
};

inline uint32_t ri_field(const uint32_t* ri, uint64_t p, uint32_t bits)
{
    const uint64_t bp = p * bits; const uint64_t w = bp >> 5; const uint32_t off = (uint32_t)(bp & 31);
    const uint64_t two = ((uint64_t)ri[w] << 32) | ri[w + 1];
    return (uint32_t)((two << off) >> (64 - bits));
}

int check_index_shallow(const View& v)
{
    const hac_desc_t& d = v.d;
    if (v.colpos[0] != 0 || v.colpos[d.m] != d.nnz) return HAC_EFORMAT;
    if (v.colchunk[0] != 0 || v.colchunk[d.m] != d.n_chunks) return HAC_EFORMAT;
    if (v.colbit[0] != 0 || v.colbit[d.m] != d.total_bits) return HAC_EFORMAT;
    uint64_t max_nnz = 0, max_bits = 0;
    for (uint64_t j = 0; j < d.m; ++j) {
        if (v.colpos[j] > v.colpos[j + 1] || v.colbit[j] > v.colbit[j + 1]) return HAC_EFORMAT;
        const uint64_t cnt = v.colpos[j + 1] - v.colpos[j];
        if (cnt > d.n) return HAC_EFORMAT;
        const uint32_t cj = chunk_of_column(d.chunk, cnt);
        if ((uint64_t)v.colchunk[j + 1] - v.colchunk[j] != (cnt + cj - 1) / cj) return HAC_EFORMAT;
        max_nnz = std::max(max_nnz, cnt);
        const uint64_t bits = v.colbit[j + 1] - v.colbit[j];
        max_bits = std::max<uint64_t>(max_bits, bits);
        // every chunk entry points inside its column, in ascending order
        uint64_t prev_rel = 0, prev_row = 0;
        for (uint64_t g = v.colchunk[j]; g < v.colchunk[j + 1]; ++g) {
            uint64_t rel, row;
            v.entry(g, rel, row);
            if (rel >= bits || row >= d.n) return HAC_EFORMAT;
            if (g == v.colchunk[j] ? (rel != 0 || row != 0) : (rel <= prev_rel || ((d.format == HAC_FORMAT_HAC || d.ri_coding == HAC_RI_RICE) && row <= prev_row)))
                return HAC_EFORMAT;
            prev_rel = rel; prev_row = row;
        }
    }
    if (max_nnz != d.max_col_nnz || max_bits != d.max_col_bits) return HAC_EFORMAT;
    if (d.chunk_rows) {
        // row index: every column starts at (0, 0), ends at (its bits, its non-zeros), never steps back,
        // and no entry claims more non-zeros than rows passed
        const uint64_t nq = (d.n + d.chunk_rows - 1) / d.chunk_rows;
        for (uint64_t j = 0; j < d.m; ++j) {
            const uint64_t bits = v.colbit[j + 1] - v.colbit[j], cnt = v.colpos[j + 1] - v.colpos[j];
            uint64_t pb = 0, pp = 0;
            for (uint64_t q = 0; q <= nq; ++q) {
                uint64_t rb, rp;
                v.row_entry(j * (nq + 1) + q, rb, rp);
                if (q == 0 && (rb || rp)) return HAC_EFORMAT;
                if (rb < pb || rp < pp || rb > bits || rp > cnt) return HAC_EFORMAT;
                if (rp - pp > d.chunk_rows) return HAC_EFORMAT;
                if (q == nq && (rb != bits || rp != cnt)) return HAC_EFORMAT;
                pb = rb; pp = rp;
            }
        }
    }
    return HAC_OK;
}

int check_deep(const View& v)
{
    const hac_desc_t& d = v.d;
    SeqDecoder dec(v);
    // row index: every entry against the sequential decode, and the fullest tile of 16 columns x 4 entries
    const uint64_t cr = d.chunk_rows, nq = cr ? (d.n + cr - 1) / cr : 0;
    std::vector<uint64_t> tile(cr ? (size_t)((d.n + 4 * cr - 1) / (4 * cr)) : 0, 0);
    uint64_t worst_tile = 0;
    auto row_entry_is = [&](uint64_t j, uint64_t q, uint64_t bit, uint64_t pos) {
        uint64_t rb, rp;
        v.row_entry(j * (nq + 1) + q, rb, rp);
        return rb == bit - v.colbit[j] && rp == pos - v.colpos[j];
    };
    auto tile_add = [&](uint64_t row) { if (cr) tile[(size_t)(row / (4 * cr))]++; };
    auto tile_column_done = [&](uint64_t j) {
        if (cr && ((j & 15) == 15 || j + 1 == d.m)) {
            for (uint64_t& t : tile) { worst_tile = std::max(worst_tile, t); t = 0; }
        }
    };
    if (d.format == HAC_FORMAT_HAC) {
        uint64_t pos = 0;
        for (uint64_t j = 0; j < d.m; ++j) {
            if (v.colbit[j] != dec.bitpos || v.colpos[j] != pos) return HAC_EFORMAT;
            uint64_t g = v.colchunk[j];
            uint64_t last_bit = dec.bitpos, last_row = 0;     // where the next chunk would start
            for (uint64_t i = 0; i < d.n; ++i) {
                if (cr && i % cr == 0 && !row_entry_is(j, i / cr, dec.bitpos, pos)) return HAC_EFORMAT;
                const int64_t s = dec.next();
                if (s < 0) return HAC_EFORMAT;
                if (d.has_zero && s == 0) continue;
                tile_add(i);
                if ((pos - v.colpos[j]) % chunk_of_column(d.chunk, v.colpos[j + 1] - v.colpos[j]) == 0) {     // first non-zero of a chunk
                    uint64_t rel, row;
                    if (g >= v.colchunk[j + 1]) return HAC_EFORMAT;
                    v.entry(g, rel, row);
                    if (rel != last_bit - v.colbit[j] || row != last_row) return HAC_EFORMAT;
                    ++g;
                }
                ++pos;
                last_bit = dec.bitpos; last_row = i + 1;
            }
            if (g != v.colchunk[j + 1]) return HAC_EFORMAT;
            tile_column_done(j);
        }
        if (pos != d.nnz || dec.bitpos != d.total_bits) return HAC_EFORMAT;
    } else if (d.ri_coding == HAC_RI_RICE) {
        uint64_t gap_bits = 0;
        for (uint64_t j = 0; j < d.m; ++j) {
            if (v.colbit[j] != dec.bitpos) return HAC_EFORMAT;
            uint64_t g = v.colchunk[j];
            int64_t prev = -1;
            for (uint64_t p = v.colpos[j]; p < v.colpos[j + 1]; ++p) {
                if ((p - v.colpos[j]) % chunk_of_column(d.chunk, v.colpos[j + 1] - v.colpos[j]) == 0) {
                    uint64_t rel, row;
                    v.entry(g, rel, row);
                    if (rel != dec.bitpos - v.colbit[j] || row != (uint64_t)(prev + 1)) return HAC_EFORMAT;
                    ++g;
                }
                const uint64_t before = dec.bitpos;
                const int64_t gap = dec.next_gap(d.rice_k);
                if (gap < 0) return HAC_EFORMAT;
                if (((uint64_t)gap >> d.rice_k) >= kRiceEscape && dec.bitpos - before != kRiceEscape + 1 + 32) return HAC_EFORMAT;
                if (((uint64_t)gap >> d.rice_k) < kRiceEscape && dec.bitpos - before == kRiceEscape + 1 + 32) return HAC_EFORMAT;
                gap_bits += dec.bitpos - before;
                const int64_t r = prev + 1 + gap;
                if (r >= (int64_t)d.n) return HAC_EFORMAT;
                prev = r;
                if (dec.next() < 0) return HAC_EFORMAT;
            }
        }
        if (dec.bitpos != d.total_bits || gap_bits != d.gap_bits) return HAC_EFORMAT;
    } else {
        for (uint64_t j = 0; j < d.m; ++j) {
            if (v.colbit[j] != dec.bitpos) return HAC_EFORMAT;
            uint64_t g = v.colchunk[j];
            int64_t prev = -1;
            uint64_t q = 0;                                   // next entry of the row index to check
            for (uint64_t p = v.colpos[j]; p < v.colpos[j + 1]; ++p) {
                if ((p - v.colpos[j]) % chunk_of_column(d.chunk, v.colpos[j + 1] - v.colpos[j]) == 0) {
                    uint64_t rel, row;
                    v.entry(g, rel, row);
                    if (rel != dec.bitpos - v.colbit[j]) return HAC_EFORMAT;
                    ++g;
                }
                const uint32_t r = ri_field(v.ri, p, d.ri_bits);
                if (r >= d.n || (int64_t)r <= prev) return HAC_EFORMAT;
                for (; cr && q < nq && q * cr <= r; ++q)
                    if (!row_entry_is(j, q, dec.bitpos, p)) return HAC_EFORMAT;
                if (dec.next() < 0) return HAC_EFORMAT;
                tile_add(r);
                prev = r;
            }
            for (; cr && q < nq; ++q)
                if (!row_entry_is(j, q, dec.bitpos, v.colpos[j + 1])) return HAC_EFORMAT;
            tile_column_done(j);
        }
        if (dec.bitpos != d.total_bits) return HAC_EFORMAT;
    }
    if (cr && d.max_tile_nnz != std::min<uint64_t>(worst_tile, 65535)) return HAC_EFORMAT;
    return HAC_OK;
}

} // namespace

namespace {

inline uint32_t im_pointer(const hac_desc_t& d, const uint8_t* base, uint64_t i, uint64_t j)
{
    const uint64_t at = i * d.idx_pitch + j;
    return d.ent_bits == 8 ? base[d.off_stream + at]
                           : reinterpret_cast<const uint16_t*>(base + d.off_stream)[at];
}

// representatives finite and ascending after the optional 0.0; every pointer below k; padding 0;
// nnz = number of pointers to a value other than 0.0
// A layer of a network blob (dict_shared): the value list is checked once for the network, and
// a non-zero is a pointer to a value other than 0.0, wherever 0.0 sits in the list.
int check_index_map(const void* blob, const hac_desc_t& d, bool deep)
{
    const uint8_t* base = static_cast<const uint8_t*>(blob);
    const float* cb = reinterpret_cast<const float*>(base + d.off_codebook);
    if (!d.dict_shared) {
        for (uint32_t s = 0; s < d.k_sym; ++s) {
            if (!std::isfinite(cb[s])) return HAC_EFORMAT;
            if (s > d.has_zero && !(cb[s - 1] < cb[s])) return HAC_EFORMAT;
            if ((cb[s] == 0.0f) != (d.has_zero && s == 0)) return HAC_EFORMAT;
        }
        if (d.has_zero && float_bits(cb[0]) != 0) return HAC_EFORMAT;
    }
    if (!deep) return HAC_OK;
    uint64_t nnz = 0;
    for (uint64_t i = 0; i < d.n; ++i)
        for (uint64_t j = 0; j < d.idx_pitch; ++j) {
            const uint32_t p = im_pointer(d, base, i, j);
            if (j >= d.m) { if (p) return HAC_EFORMAT; continue; }
            if (p >= d.k_sym) return HAC_EFORMAT;
            if (d.dict_shared ? cb[p] != 0.0f : !(d.has_zero && p == 0)) ++nnz;
        }
    return nnz == d.nnz ? HAC_OK : HAC_EFORMAT;
}

} // namespace

extern "C" int hac_validate(const void* blob, size_t bytes, int deep)
{
    hac_desc_t d;
    int rc = check_header(blob, bytes, d);
    if (rc) return rc;
    if (d.format == HAC_FORMAT_IM) return check_index_map(blob, d, deep != 0);
    try {
        View v; make_view(blob, d, v);
        if ((rc = check_tables(v))) return rc;
        if ((rc = check_index_shallow(v))) return rc;
        if (deep && (rc = check_deep(v))) return rc;
    } catch (const std::bad_alloc&) {
        return HAC_ENOMEM;
    }
    return HAC_OK;
}

extern "C" int hac_describe(const void* blob, size_t bytes, hac_desc_t* desc)
{
    if (!desc) return HAC_EINVAL;
    return check_header(blob, bytes, *desc);
}

namespace {

// how often each symbol occurs in a layer's stream (sequential decode)
int count_symbols(const View& v, std::vector<uint64_t>& cnt)
{
    const hac_desc_t& d = v.d;
    SeqDecoder dec(v);
    const uint64_t symbols = d.format == HAC_FORMAT_HAC ? d.n * d.m : d.nnz;
    for (uint64_t i = 0; i < symbols; ++i) {
        if (d.ri_coding == HAC_RI_RICE && dec.next_gap(d.rice_k) < 0) return HAC_EFORMAT;
        const int64_t s = dec.next();
        if (s < 0) return HAC_EFORMAT;
        cnt[(size_t)s]++;
    }
    return HAC_OK;
}

// the paper's size of one layer without its dictionaries: words (+ ri and cb for sHAC)
uint64_t layer_paper_bits(const hac_desc_t& d)
{
    if (d.format == HAC_FORMAT_HAC) return 32 * d.n_words;
    const bool rice = d.ri_coding == HAC_RI_RICE;
    return 32 * d.n_words + 32 * ((rice ? 0 : d.nnz) + d.m + 1);
}

// a validated index map: W_out row-major, sym_out the pointers in column order
int decode_index_map(const void* blob, const hac_desc_t& d, float* W_out, int32_t* sym_out)
{
    const uint8_t* base = static_cast<const uint8_t*>(blob);
    const float* cb = reinterpret_cast<const float*>(base + d.off_codebook);
    for (uint64_t i = 0; i < d.n; ++i)
        for (uint64_t j = 0; j < d.m; ++j) {
            const uint32_t p = im_pointer(d, base, i, j);
            if (sym_out) sym_out[j * d.n + i] = (int32_t)p;
            if (W_out) W_out[i * d.m + j] = cb[p];
        }
    return HAC_OK;
}

// the library's sequential decoder over one validated layer
int decode_layer(const View& v, float* W_out, int32_t* sym_out, int32_t* row_out, int32_t* col_out)
{
    const hac_desc_t& d = v.d;
    SeqDecoder dec(v);
    if (d.format == HAC_FORMAT_HAC) {
        if (row_out || col_out) return HAC_EINVAL;
        for (uint64_t j = 0; j < d.m; ++j)
            for (uint64_t i = 0; i < d.n; ++i) {
                const int64_t s = dec.next();
                if (s < 0) return HAC_EFORMAT;
                if (sym_out) sym_out[j * d.n + i] = (int32_t)s;
                if (W_out) W_out[i * d.m + j] = v.codebook[s];
            }
    } else {
        if (W_out) std::memset(W_out, 0, sizeof(float) * (size_t)(d.n * d.m));
        const bool rice = d.ri_coding == HAC_RI_RICE;
        for (uint64_t j = 0; j < d.m; ++j) {
            int64_t prev = -1;
            for (uint64_t p = v.colpos[j]; p < v.colpos[j + 1]; ++p) {
                uint64_t r;
                if (rice) {
                    const int64_t gap = dec.next_gap(d.rice_k);
                    if (gap < 0) return HAC_EFORMAT;
                    r = (uint64_t)(prev + 1 + gap);
                    prev = (int64_t)r;
                }
                const int64_t s = dec.next();
                if (s < 0) return HAC_EFORMAT;
                if (!rice) r = ri_field(v.ri, p, d.ri_bits);
                if (r >= d.n) return HAC_EFORMAT;
                if (sym_out) sym_out[p] = (int32_t)s;
                if (row_out) row_out[p] = (int32_t)r;
                if (col_out) col_out[p] = (int32_t)j;
                if (W_out) W_out[(uint64_t)r * d.m + j] = v.codebook[s];
            }
        }
    }
    return HAC_OK;
}

} // namespace

extern "C" int hac_stats(const void* blob, size_t bytes, hac_stats_t* out)
{
    if (!out) return HAC_EINVAL;
    hac_desc_t d;
    int rc = check_header(blob, bytes, d);
    if (rc) return rc;
    if (d.format == HAC_FORMAT_IM) {
        if ((rc = check_index_map(blob, d, true))) return rc;
        std::memset(out, 0, sizeof *out);
        const uint8_t* base = static_cast<const uint8_t*>(blob);
        out->stream_bits = d.total_bits;
        out->stream_bytes = d.n * d.idx_pitch * (d.ent_bits / 8);
        out->table_bytes = 4ull * d.k_sym;
        out->blob_bytes = d.blob_bytes;
        out->paper_bits = d.total_bits + 32ull * d.k_sym;          // bbar*n*m + k*b
        out->bound_bits = (double)out->paper_bits;                 // the paper gives this size exactly, not a bound
        std::vector<uint64_t> cnt(d.k_sym, 0);
        for (uint64_t i = 0; i < d.n; ++i)
            for (uint64_t j = 0; j < d.m; ++j) cnt[im_pointer(d, base, i, j)]++;
        const double nm = (double)d.n * (double)d.m;
        double H = 0.0;
        for (uint32_t s = 0; s < d.k_sym; ++s)
            if (cnt[s]) { const double p = (double)cnt[s] / nm; H -= p * std::log2(p); }
        out->entropy_bits = H;
        out->avg_code_bits = (double)d.ent_bits;
        out->psi = (double)d.blob_bytes / (4.0 * nm);
        return HAC_OK;
    }
    View v; make_view(blob, d, v);
    if ((rc = check_tables(v))) return rc;
    if ((rc = check_index_shallow(v))) return rc;
    std::memset(out, 0, sizeof *out);
    out->stream_bits = d.total_bits;
    out->stream_bytes = 4 * d.n_words;
    out->table_bytes = 4ull * d.k_sym + d.k_sym + 3 * 33 * 4 + 4ull * d.k_sym + (4ull << d.lut_bits);
    out->blob_bytes = d.blob_bytes;
    const double nm = (double)d.n * (double)d.m;
    const double k = (double)std::max<uint32_t>(d.k_sym, 1);
    const uint64_t ent_bytes = d.n_chunks * (d.ent_bits / 8);
    out->row_index_bytes = row_index_entries(d) * (d.rent_bits / 8);
    if (d.format == HAC_FORMAT_HAC) {
        out->index_bytes = 3 * 4 * (d.m + 1) + ent_bytes;
        out->paper_bits = layer_paper_bits(d) + 6ull * 32 * d.k_sym;
        out->bound_bits = nm * (1.0 + std::log2(k)) + 6.0 * k * 32.0;
    } else {
        const bool rice = d.ri_coding == HAC_RI_RICE;
        out->index_bytes = 2 * 4 * (d.m + 1) + ent_bytes;
        out->ri_bytes = rice ? 0 : 4 * ((d.nnz * d.ri_bits + 31) / 32);
        out->cb_bytes = 4 * (d.m + 1);
        out->paper_bits = layer_paper_bits(d) + 6ull * 32 * d.k_sym;
        out->bound_bits = (double)d.nnz * (1.0 + std::log2(k)) + 32.0 * (6.0 * k + (double)d.nnz + (double)d.m + 1.0);
    }
    // entropy from the code lengths is not available; recompute symbol counts by a sequential decode
    std::vector<uint64_t> cnt(d.k_sym, 0);
    if ((rc = count_symbols(v, cnt))) return rc;
    const uint64_t symbols = d.format == HAC_FORMAT_HAC ? d.n * d.m : d.nnz;
    double H = 0.0;
    for (uint32_t s = 0; s < d.k_sym; ++s)
        if (cnt[s]) { const double p = (double)cnt[s] / (double)symbols; H -= p * std::log2(p); }
    out->entropy_bits = H;
    out->avg_code_bits = symbols ? (double)(d.total_bits - d.gap_bits) / (double)symbols : 0.0;
    out->psi = (double)d.blob_bytes / (4.0 * nm);
    return HAC_OK;
}

extern "C" int hac_decode_host(const void* blob, size_t bytes, float* W_out, int32_t* sym_out,
                               int32_t* row_out, int32_t* col_out)
{
    hac_desc_t d;
    int rc = check_header(blob, bytes, d);
    if (rc) return rc;
    if (d.format == HAC_FORMAT_IM) {
        if (row_out || col_out) return HAC_EINVAL;
        if ((rc = check_index_map(blob, d, true))) return rc;
        return decode_index_map(blob, d, W_out, sym_out);
    }
    View v; make_view(blob, d, v);
    if ((rc = check_tables(v))) return rc;
    if ((rc = check_index_shallow(v))) return rc;
    return decode_layer(v, W_out, sym_out, row_out, col_out);
}

// =================================================================================
// network blob: description, validation, accounting, decode
// =================================================================================
namespace {

int check_net_header(const void* blob, size_t bytes, hac_net_t& net)
{
    if (!blob) return HAC_EINVAL;
    if (bytes < sizeof(hac_net_t)) return HAC_EFORMAT;
    std::memcpy(&net, blob, sizeof net);
    if (net.magic != kNetMagic || net.version != kNetVersion || net.header_bytes != 256) return HAC_EFORMAT;
    if (net.n_layers < 1 || net.n_layers > 65536) return HAC_EFORMAT;
    if (net.blob_bytes > bytes || net.blob_bytes < sizeof(hac_net_t)) return HAC_EFORMAT;
    for (size_t i = 0; i < sizeof net.reserved / sizeof net.reserved[0]; ++i) if (net.reserved[i]) return HAC_EFORMAT;
    if (net.off_layers != sizeof(hac_net_t)) return HAC_EFORMAT;
    if (net.off_layers + (uint64_t)net.n_layers * sizeof(hac_desc_t) > net.blob_bytes) return HAC_EFORMAT;
    if (net.has_zero > 1 || net.lmax > 32 || net.lut_bits < 1 || net.lut_bits > 12) return HAC_EFORMAT;
    if (net.reserved32 || net.k_values < net.k_sym || net.k_values > net.k_sym + 65536u) return HAC_EFORMAT;
    if (net.has_zero > net.k_sym) return HAC_EFORMAT;
    return HAC_OK;
}

// The network's tables, checked once: the shared code (as for a layer blob) and the value list
// behind it (the values only index-map layers hold: finite, 0.0 first if present, then ascending,
// none of them a shared symbol's value).
int check_net_tables(const void* blob, const hac_net_t& net)
{
    hac_desc_t d;
    std::memset(&d, 0, sizeof d);
    d.format = HAC_FORMAT_SHAC;                               // zero_len is a HAC layer's own field
    d.k_sym = net.k_sym; d.lmax = net.lmax; d.lut_bits = net.lut_bits; d.has_zero = net.has_zero;
    d.off_codebook = net.off_codebook; d.off_codelen = net.off_codelen; d.off_canon = net.off_canon;
    d.off_symsort = net.off_symsort; d.off_lut = net.off_lut; d.blob_bytes = net.blob_bytes;
    const size_t tot = (size_t)net.blob_bytes;
    const uint64_t first = net.off_layers + (uint64_t)net.n_layers * sizeof(hac_desc_t);
    if (net.off_codebook < first || net.off_codelen < first || net.off_canon < first || net.off_symsort < first ||
        net.off_lut < first) return HAC_EFORMAT;
    if (!section_ok(d, d.off_codebook, 4ull * net.k_values, tot) || !section_ok(d, d.off_codelen, d.k_sym, tot) ||
        !section_ok(d, d.off_canon, 3 * 33 * 4, tot) || !section_ok(d, d.off_symsort, 4ull * d.k_sym, tot) ||
        !section_ok(d, d.off_lut, 4ull << d.lut_bits, tot)) return HAC_EFORMAT;
    View v; make_view(blob, d, v);
    int rc = check_tables(v);
    if (rc) return rc;
    const float* cb = v.codebook;
    const uint32_t k = net.k_sym, kv = net.k_values;
    for (uint32_t s = k; s < kv; ++s) {
        if (!std::isfinite(cb[s])) return HAC_EFORMAT;
        if (cb[s] == 0.0f && (s != k || net.has_zero || float_bits(cb[s]) != 0)) return HAC_EFORMAT;
        if (s > k && cb[s - 1] != 0.0f && !(cb[s - 1] < cb[s])) return HAC_EFORMAT;
        if (cb[s] != 0.0f && std::binary_search(cb + net.has_zero, cb + k, cb[s])) return HAC_EFORMAT;
    }
    return HAC_OK;
}

// header of layer l, checked against the network header
int net_layer_desc(const void* blob, const hac_net_t& net, uint32_t l, hac_desc_t& d)
{
    if (l >= net.n_layers) return HAC_EINVAL;
    std::memcpy(&d, static_cast<const uint8_t*>(blob) + net.off_layers + (uint64_t)l * sizeof(hac_desc_t), sizeof d);
    if (d.blob_bytes != net.blob_bytes) return HAC_EFORMAT;
    int rc = check_desc(d, (size_t)net.blob_bytes, true);
    if (rc) return rc;
    const uint64_t behind = net.off_layers + (uint64_t)net.n_layers * sizeof(hac_desc_t);
    if (d.format == HAC_FORMAT_IM)
        return (d.off_codebook == net.off_codebook && d.k_sym == net.k_values && d.off_stream >= behind) ? HAC_OK : HAC_EFORMAT;
    if (d.off_codebook != net.off_codebook || d.off_codelen != net.off_codelen || d.off_canon != net.off_canon ||
        d.off_symsort != net.off_symsort || d.off_lut != net.off_lut || d.k_sym != net.k_sym || d.lmax != net.lmax ||
        d.lut_bits != net.lut_bits || d.has_zero != net.has_zero) return HAC_EFORMAT;
    // a layer's own sections lie behind the headers
    const uint64_t first = net.off_layers + (uint64_t)net.n_layers * sizeof(hac_desc_t);
    if (d.off_codebook < first || d.off_stream < first || d.off_col_chunk < first || d.off_col_pos < first ||
        d.off_col_bit < first || d.off_chunk_ent < first || (d.off_ri && d.off_ri < first)) return HAC_EFORMAT;
    return HAC_OK;
}

} // namespace

extern "C" int hac_net_describe(const void* blob, size_t bytes, hac_net_t* net)
{
    if (!net) return HAC_EINVAL;
    return check_net_header(blob, bytes, *net);
}

extern "C" int hac_net_layer(const void* blob, size_t bytes, uint32_t layer, hac_desc_t* desc)
{
    if (!desc) return HAC_EINVAL;
    hac_net_t net;
    int rc = check_net_header(blob, bytes, net);
    if (rc) return rc;
    return net_layer_desc(blob, net, layer, *desc);
}

extern "C" int hac_net_validate(const void* blob, size_t bytes, int deep)
{
    hac_net_t net;
    int rc = check_net_header(blob, bytes, net);
    if (rc) return rc;
    try {
        if ((rc = check_net_tables(blob, net))) return rc;
        for (uint32_t l = 0; l < net.n_layers; ++l) {
            hac_desc_t d;
            if ((rc = net_layer_desc(blob, net, l, d))) return rc;
            if (d.format == HAC_FORMAT_IM) {
                if ((rc = check_index_map(blob, d, deep != 0))) return rc;
                continue;
            }
            View v; make_view(blob, d, v);
            if (d.format == HAC_FORMAT_HAC && (rc = check_tables(v))) return rc;   // zero_len against the code
            if ((rc = check_index_shallow(v))) return rc;
            if (deep && (rc = check_deep(v))) return rc;
        }
    } catch (const std::bad_alloc&) {
        return HAC_ENOMEM;
    }
    return HAC_OK;
}

extern "C" int hac_net_stats(const void* blob, size_t bytes, hac_net_stats_t* out)
{
    if (!out) return HAC_EINVAL;
    hac_net_t net;
    int rc = check_net_header(blob, bytes, net);
    if (rc) return rc;
    try {
        std::memset(out, 0, sizeof *out);
        std::vector<uint64_t> cnt(net.k_sym, 0);
        uint64_t gap_bits = 0, map_bits = 0;
        if ((rc = check_net_tables(blob, net))) return rc;
        for (uint32_t l = 0; l < net.n_layers; ++l) {
            hac_desc_t d;
            if ((rc = net_layer_desc(blob, net, l, d))) return rc;
            if (d.format == HAC_FORMAT_IM) {
                if ((rc = check_index_map(blob, d, true))) return rc;
                out->entries += d.n * d.m;
                out->nnz += d.nnz;
                out->stream_bits += d.total_bits;
                out->paper_bits += d.total_bits;              // bbar * n * m
                map_bits += d.total_bits;
                continue;
            }
            View v; make_view(blob, d, v);
            if (d.format == HAC_FORMAT_HAC && (rc = check_tables(v))) return rc;
            if ((rc = check_index_shallow(v))) return rc;
            if ((rc = count_symbols(v, cnt))) return rc;
            out->entries += d.n * d.m;
            out->nnz += d.nnz;
            out->symbols += d.format == HAC_FORMAT_HAC ? d.n * d.m : d.nnz;
            out->stream_bits += d.total_bits;
            out->paper_bits += layer_paper_bits(d);
            gap_bits += d.gap_bits;
        }
        out->n_layers = net.n_layers;
        out->paper_bits += 6ull * 32 * net.k_sym + 32ull * (net.k_values - net.k_sym);
        out->table_bytes = 4ull * net.k_values + net.k_sym + 3 * 33 * 4 + 4ull * net.k_sym + (4ull << net.lut_bits);
        out->blob_bytes = net.blob_bytes;
        double H = 0.0;
        for (uint32_t s = 0; s < net.k_sym; ++s)
            if (cnt[s]) { const double p = (double)cnt[s] / (double)out->symbols; H -= p * std::log2(p); }
        out->entropy_bits = H;
        out->avg_code_bits = out->symbols ? (double)(out->stream_bits - gap_bits - map_bits) / (double)out->symbols : 0.0;
        out->psi = (double)net.blob_bytes / (4.0 * (double)out->entries);
    } catch (const std::bad_alloc&) {
        return HAC_ENOMEM;
    }
    return HAC_OK;
}

extern "C" int hac_net_decode_host(const void* blob, size_t bytes, uint32_t layer, float* W_out,
                                   int32_t* sym_out, int32_t* row_out, int32_t* col_out)
{
    hac_net_t net;
    int rc = check_net_header(blob, bytes, net);
    if (rc) return rc;
    hac_desc_t d;
    if ((rc = net_layer_desc(blob, net, layer, d))) return rc;
    if ((rc = check_net_tables(blob, net))) return rc;
    if (d.format == HAC_FORMAT_IM) {
        if (row_out || col_out) return HAC_EINVAL;
        if ((rc = check_index_map(blob, d, true))) return rc;
        return decode_index_map(blob, d, W_out, sym_out);
    }
    View v; make_view(blob, d, v);
    if (d.format == HAC_FORMAT_HAC && (rc = check_tables(v))) return rc;
    if ((rc = check_index_shallow(v))) return rc;
    return decode_layer(v, W_out, sym_out, row_out, col_out);
}

extern "C" int hac_choose_format(int64_t n, int64_t m, uint64_t nnz, uint32_t k)
{
    if (n < 1 || m < 1 || k < 1 || (double)nnz > (double)n * (double)m) return HAC_EINVAL;
    const double nm = (double)n * (double)m;
    const double a = (1.0 + std::log2((double)k)) / 32.0;
    const double s_star = (a - ((double)m + 1.0) / nm) / (1.0 + a);
    return (double)nnz / nm < s_star ? HAC_FORMAT_SHAC : HAC_FORMAT_HAC;
}

extern "C" const char* hac_strerror(int status)
{
    switch (status) {
    case HAC_OK: return "ok";
    case HAC_EINVAL: return "invalid argument";
    case HAC_ENOMEM: return "out of host memory";
    case HAC_EFORMAT: return "blob fails validation";
    case HAC_ERANGE: return "value outside the limits of the format (codeword > 32 bits or count too large)";
    case HAC_EHIP: return "HIP call failed";
    case HAC_EWORKSPACE: return "workspace missing or too small";
    default: return "unknown status";
    }
}
