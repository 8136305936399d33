/* hac.h -- C ABI of libhac: HAC / sHAC compressed layer matrices and the
 * product Y = X.W computed straight from the compressed form on an MI355X.
 *
 * Source of the definitions: "Compact representations of convolutional neural
 * networks via weight pruning and quantization" (arXiv 2108.12704), Sect. IV.
 *   HAC  (Sect. IV-B): all n*m entries of W, zeros included, in column order,
 *        each replaced by its Huffman codeword; the bit stream is cut into
 *        32-bit words, the last one zero-padded.
 *   sHAC (Sect. IV-C): CSC form (nz, ri, cb of Sect. IV-A); nz Huffman-coded
 *        without the symbol 0; ri and cb stored beside it.
 *   dot  (Algorithms 1-3): Y = X.W where W is the decoded matrix; X holds one
 *        input vector per row.
 *
 *   IM   (Sect. III-C1, "index map"): the k representatives in a vector and one
 *        pointer per entry of W (8 bits for k <= 256, else 16); the form the
 *        paper uses for quantized, unpruned (convolutional) layers.  Pointers
 *        number the values like the HAC alphabet: 0.0 first when it occurs,
 *        then ascending.
 *
 *   Network blobs (Sect. V-H, V-K): all layers of a network written with one
 *        shared dictionary, index-map layers sharing its value list; see
 *        hac_net_encode below.
 *   Chain of layers (an extension): hac_forward evaluates
 *        A <- act(A.W_l + b_l) layer after layer; see below.
 *
 * An extension beyond the paper, selected with hac_opts_t.ri_coding =
 * HAC_RI_RICE: sHAC whose row-index vector ri is replaced by Golomb-Rice coded
 * row gaps written into the stream itself.  For the non-zero at CSC position p
 * of column j let d = ri[p] - prev - 1, prev being the row of the non-zero
 * before it in the same column, or -1 for the column's first.  With q = d >> k:
 *        q <  31: q bits 0, one bit 1, the k low bits of d (MSB first);
 *        q >= 31: 31 bits 0, one bit 1, d as 32 bits.
 * The stream is the concatenation over p of  Rice_k(d_p) | H(nz_p); nz, its
 * Huffman code and cb are those of sHAC; k (0..15) minimises the gap bits, the
 * smaller k on ties.  Corollary 2 still bounds the size (there is no ri).
 *
 * Conventions
 *   - W is n x m (n input features, m outputs).  X is B x n, Y is B x m, both
 *     row-major fp32 with leading dimensions ldx >= n, ldy >= m (in elements).
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device
 *     memory of the current device.  The library never allocates or frees
 *     device memory; only hac_encode_dev synchronises a stream (it says so).
 *   - Every function returns HAC_OK (0) or a negative hac_status; nothing
 *     throws across this boundary.  No global mutable state; calls on distinct
 *     arguments may run concurrently from several threads.
 *   - A blob is one flat, relocatable byte buffer: a 256-byte header
 *     (hac_desc_t) followed by 256-byte-aligned sections.  Copy it to the
 *     device verbatim (any 256-byte-aligned address); keep the header on the
 *     host and pass it to the device calls as `desc`.
 *
 * Stream bit order: the first bit of the stream is bit 31 of word 0 (Sect.
 * IV-B leaves the order inside a word open).  The code is a canonical Huffman
 * code: optimal lengths, codewords assigned in order of (length, symbol) --
 * any optimal prefix code is a valid H_W.  Symbols number the distinct fp32
 * values that occur in W: 0.0 first when it occurs, then ascending.
 */
#ifndef HAC_H
#define HAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HAC_OK         =  0,
    HAC_EINVAL     = -1,   /* null pointer, bad size, wrong format for this call        */
    HAC_ENOMEM     = -2,   /* host allocation failed                                     */
    HAC_EFORMAT    = -3,   /* blob fails validation (magic, bounds, index, code tables)  */
    HAC_ERANGE     = -4,   /* codeword > 32 bits, or a count exceeds the format's limits */
    HAC_EHIP       = -5,   /* a HIP call failed; see hac_last_hip_error()                */
    HAC_EWORKSPACE = -6    /* workspace missing or smaller than hac_workspace_bytes()    */
} hac_status;

enum { HAC_FORMAT_HAC = 1, HAC_FORMAT_SHAC = 2, HAC_FORMAT_IM = 3 };

/* A hipStream_t, spelled without pulling in the HIP headers. */
typedef void *hac_stream_t;

/* Encoder options; pass NULL for the defaults given in brackets. */
typedef struct {
    uint32_t chunk_nnz;   /* non-zeros per index entry, restarting at every column; 0 = default
                             [max(4, ceil(most non-zeros in a column / 64))]: one wavefront
                             then decodes a whole column side by side.
                             HAC_CHUNK_PER_COLUMN: every column its own chunk size,
                             max(4, ceil(its non-zeros / 64)), so that every long column
                             fills the 64 lanes, not only the longest                       */
    uint32_t ri_bits;     /* sHAC row-index field width: 0 = ceil(log2 n) (footnote of
                             Sect. IV-A), 32 = one word per index as in Corollary 2        */
    uint32_t lut_bits;    /* width of the first-level decode table, 1..12 [min(Lmax,10)]  */
    uint32_t ri_coding;   /* sHAC: HAC_RI_FIELDS [default] or HAC_RI_RICE (ri_bits must
                             then be 0); hac_encode requires 0                             */
    uint32_t chunk_rows;  /* rows of W per entry of the row index (see hac_desc_t), a multiple
                             of 4 when below n; 0 = no row index [default];
                             HAC_CHUNK_ROWS_AUTO = about 8 non-zeros per entry.  Not with
                             HAC_RI_RICE                                                   */
} hac_opts_t;

enum { HAC_RI_FIELDS = 0, HAC_RI_RICE = 1 };
#define HAC_CHUNK_ROWS_AUTO 0xffffffffu
#define HAC_CHUNK_PER_COLUMN 0xffffffffu
#define HAC_CHUNK_FLAG_PER_COLUMN 0x80000000u   /* in hac_desc_t.chunk */

/* Blob header == descriptor.  All offsets are bytes from the start of the blob.
 *
 * The index added for the GPU (not part of the paper's formats; its conclusions
 * propose per-column bit offsets so that columns can be decoded in parallel):
 * per column its first stream bit, its first CSC position and
 * its first chunk; per chunk of `chunk` consecutive non-zeros of a column the
 * bit at which its decoding starts, relative to the column's first bit, and
 * for HAC the row of the first symbol decoded there.  Chunk k of column j
 * holds the non-zeros col_pos[j] + k*chunk ... and, for HAC, starts right
 * after the codeword of the non-zero before them (at the column's first bit
 * for k = 0), so the zeros in front of its first non-zero belong to it.
 *
 * Row index (optional, hac_opts_t.chunk_rows): a second index that cuts every
 * column at the same rows, so that a block of the large-batch kernel can own a
 * range of rows of W for a group of columns and keep the matching rows of X in
 * LDS.  With nq = ceil(n / chunk_rows), column j has nq + 1 entries, stored
 * column after column; entry q < nq says where the column's rows >= q*chunk_rows
 * begin: rel_bit, the stream bit relative to col_bit[j] of the first codeword
 * decoded for them (HAC: the codeword of entry (q*chunk_rows, j) itself; sHAC:
 * the codeword of the first non-zero in those rows), and rel_pos, the number of
 * the column's non-zeros in rows < q*chunk_rows.  Entry nq holds the column's
 * length in bits and its number of non-zeros. */
typedef struct {
    uint32_t magic;        /* 'HAC1' = 0x31434148                                          */
    uint32_t version;      /* 2                                                            */
    uint32_t format;       /* HAC_FORMAT_HAC / HAC_FORMAT_SHAC                             */
    uint32_t header_bytes; /* 256                                                          */
    uint64_t n, m;         /* shape of W                                                   */
    uint64_t nnz;          /* q: entries different from 0.0                                */
    uint64_t total_bits;   /* |HAC(W)| resp. |HAC(nz)|: exact stream length                */
    uint64_t n_words;      /* N resp. N1 = ceil(total_bits / 32)                           */
    uint32_t k_sym;        /* alphabet size (HAC counts the value 0 when it occurs)        */
    uint32_t lmax;         /* longest codeword, <= 32                                      */
    uint32_t lut_bits;     /* first-level table has 2^lut_bits entries                     */
    uint32_t has_zero;     /* HAC: 1 when 0.0 occurs in W; it is then symbol 0             */
    uint32_t zero_len;     /* HAC: codeword length of symbol 0 when that codeword is all
                              zero bits (it is one of the shortest), else 0                */
    uint32_t chunk;        /* non-zeros per chunk; with HAC_CHUNK_FLAG_PER_COLUMN set the low
                              bits are the smallest chunk size and column j is cut into chunks of
                              max(that, ceil(non-zeros of j / 64)) non-zeros                  */
    uint32_t ri_bits;      /* sHAC: width of one row-index field                           */
    uint32_t ent_bits;     /* width of one chunk entry: HAC and Rice-coded sHAC 32 or 64,
                              sHAC with ri fields 16 or 32                                 */
    uint64_t n_chunks;     /* sum over columns of ceil(non-zeros in the column / its chunk size) */
    uint64_t off_codebook; /* float[k_sym]: symbol -> shared value (H^-1's values)         */
    uint64_t off_codelen;  /* uint8[k_sym]: codeword length per symbol                     */
    uint64_t off_canon;    /* uint32[3][33]: first_code[l], count[l], first_index[l]       */
    uint64_t off_symsort;  /* uint32[k_sym]: symbols in (length, symbol) order             */
    uint64_t off_lut;      /* uint32[2^lut_bits]: (symbol << 6) | length, 0 = longer code  */
    uint64_t off_stream;   /* uint32[n_words], followed by >= 64 bytes of zeros            */
    uint64_t off_col_chunk;/* uint32[m + 1]: first chunk of each column                    */
    uint64_t off_col_pos;  /* uint32[m + 1]: CSC position of each column's first non-zero;
                              for sHAC this is the paper's cb (0-based, cb[m] = nnz)       */
    uint64_t off_col_bit;  /* uint32[m + 1]: first stream bit of each column               */
    uint64_t off_chunk_ent;/* n_chunks entries of ent_bits bits (+ >= 8 bytes of zeros):
                              sHAC: bit offset relative to col_bit[j];
                              HAC : (relative bit offset << row_bits) | first row, as one
                              uint32, or as uint32 pair {first row, relative bit offset};
                              Rice-coded sHAC: as HAC, "first row" being the row from
                              which the chunk's first gap counts (prev + 1)                */
    uint64_t off_ri;       /* sHAC: row indices, ri_bits-wide fields packed MSB-first into
                              uint32 words, followed by >= 64 bytes of zeros               */
    uint64_t blob_bytes;   /* total size                                                   */
    uint64_t max_col_bits; /* longest stretch of stream bits that one column occupies      */
    uint64_t max_col_nnz;  /* most non-zeros in one column                                 */
    uint32_t row_bits;     /* ent_bits = 32 with a row: low bits of an entry that hold it  */
    uint32_t ri_coding;    /* sHAC: HAC_RI_FIELDS or HAC_RI_RICE                           */
    uint32_t rice_k;       /* HAC_RI_RICE: the parameter k                                 */
    uint32_t dict_shared;  /* 1 in the headers of a network blob (hac_net_encode): offsets count
                              from the start of the network blob, the table offsets are those
                              of the one shared dictionary, k_sym / has_zero describe that
                              dictionary (a layer need not use every symbol); else 0       */
    uint64_t gap_bits;     /* HAC_RI_RICE: part of total_bits spent on the gap codewords   */
    uint64_t idx_pitch;    /* IM: elements from one row of the index map to the next, a
                              multiple of 16; the columns past m hold 0                    */
    uint64_t off_row_ent;  /* row index: m * (nq + 1) entries of rent_bits bits (+ >= 8 bytes
                              of zeros): (rel_bit << rpos_bits) | rel_pos as one uint32, or
                              the uint32 pair {rel_pos, rel_bit}; 0 without a row index      */
    uint32_t chunk_rows;   /* rows per entry of the row index; 0 = the blob has none        */
    uint8_t  rent_bits;    /* 32 or 64                                                      */
    uint8_t  rpos_bits;    /* rent_bits = 32: low bits of an entry that hold rel_pos        */
    uint16_t max_tile_nnz; /* most non-zeros in a tile of 16 columns x 4 entries of the row
                              index (columns 16a .. 16a+15, rows 4b*chunk_rows ...), or
                              65535 when that is more                                       */
} hac_desc_t;

/* An IM blob uses the header like this: format = HAC_FORMAT_IM; k_sym
 * representatives at off_codebook; ent_bits = 8 or 16, the width of a pointer;
 * the index map at off_stream, n rows of idx_pitch pointers, row-major (followed
 * by >= 64 bytes of zeros); total_bits = ent_bits * n * m, the paper's bbar*n*m;
 * has_zero as for HAC.  Every other offset and count is 0. */

/* Sizes as the paper accounts for them (Sect. IV-B/IV-C) next to the real ones. */
typedef struct {
    uint64_t stream_bits;      /* exact |HAC(.)|                                           */
    uint64_t stream_bytes;     /* 4 * n_words                                              */
    uint64_t table_bytes;      /* codebook + lengths + canonical tables + first-level table*/
    uint64_t index_bytes;      /* index added for the GPU (not part of the paper's format):
                                  col_chunk, col_bit, chunk entries, and for HAC col_pos   */
    uint64_t ri_bytes, cb_bytes; /* sHAC: packed ri (0 when Rice-coded: the gaps are part of
                                  the stream), and cb (= col_pos)                          */
    uint64_t blob_bytes;
    uint64_t paper_bits;       /* 32*N + 6*32*k (+ 32*(q + m + 1) for sHAC, 32*(m + 1) when
                                  Rice-coded): the quantity bounded by Corollary 1 / 2     */
    double   bound_bits;       /* Corollary 1 / Corollary 2 with b = 32                    */
    double   entropy_bits;     /* source entropy H per symbol                              */
    double   avg_code_bits;    /* total_bits / symbols, H <= avg <= H + 1                  */
    double   psi;              /* blob_bytes / (4 n m): occupancy ratio of what is stored  */
    uint64_t row_index_bytes;  /* the optional row index (0 without one); a dot call reads
                                  either it or the chunk entries counted in index_bytes   */
} hac_stats_t;

/* Optional launch overrides for the dot calls (NULL = library defaults).  Any
 * field left 0 keeps its default.  Values outside the documented range give
 * HAC_EINVAL.  They change how the work is split, never what is computed; where
 * a split changes the order of the fp32 additions, the flag says so. */
typedef struct {
    uint32_t cols_per_wave;   /* columns of W one wavefront handles, 1..32                 */
    uint32_t waves_per_block; /* 1..16                                                     */
    uint32_t variant;         /* 0, or an OR of the HAC_LAUNCH_* flags below                */
    uint32_t list_entries;    /* entries of the per-wavefront list of decoded non-zeros,
                                 64..4096 [sized from the blob header]                     */
    uint32_t staging_words;   /* words of the per-wavefront LDS buffer for stream (and ri)
                                 words, 16..16384, a multiple of 4 [from the header]       */
    uint32_t pass_width;      /* batch columns one pass over the list covers:
                                 32 / 64 / 128 / 256 [32]                                  */
    uint32_t free_running;    /* 1 = do not hold a block's wavefronts on the same pass
                                 (measurement aid) [0]                                     */
    uint32_t tile_width;      /* batch columns one block covers: 32 / 64 / 128 / 256, not
                                 below pass_width; every column of W is decoded once per
                                 such tile of the batch [256]                              */
    uint32_t sessions_per_block; /* row-blocked kernel: groups of 4 row-index entries one block
                                 works off before it writes its sums [so that there is
                                 about one block per compute unit]; changes the order of
                                 the additions                                             */
} hac_launch_t;

/* The workspace already holds the feature-major copy of this very X (same B,
 * same n) left there by an earlier call: skip the re-layout pass.  Meant for
 * one X multiplied with several compressed matrices of the same height. */
#define HAC_LAUNCH_REUSE_XT 0x100u

/* Batches of at most 4 rows normally run a kernel in which every lane
 * multiplies the non-zeros it decodes itself; this flag sends them through the
 * kernel of the larger batches (decoded non-zeros listed in LDS, then shared by
 * lanes that each own batch columns).  Same result up to summation order. */
#define HAC_LAUNCH_LIST_KERNEL 0x200u

/* Batches of 2 to 8 rows with a short X (n * B' <= 8192, B' = B rounded up to
 * a power of two) normally run without a re-layout pass and without workspace:
 * every block copies X into LDS.  This flag sends them the other way (re-layout
 * in the workspace first).  Same result up to summation order. */
#define HAC_LAUNCH_NO_X_LDS 0x1000u

/* Blobs with a row index (hac_opts_t.chunk_rows) and batches of more than 128 rows run the
 * row-blocked kernel: a block owns 256 columns of W, up to 256 batch rows and a range of rows,
 * keeps the matching rows of X in LDS and the sums of all its columns in registers; ranges are
 * added by a second kernel in a fixed order, through the workspace.  The first flag sends any
 * batch that way (given a row index), the second none.  Same result up to summation order. */
#define HAC_LAUNCH_ROWS_KERNEL    0x2000u
#define HAC_LAUNCH_NO_ROWS_KERNEL 0x4000u

/* Force one of the two routes of hac_dot / shac_dot (not both). */
#define HAC_LAUNCH_SPARSE_ROUTE 0x400u
#define HAC_LAUNCH_DENSE_ROUTE  0x800u

/* ---- host side ------------------------------------------------------------ */

/* Encode W as an index map (Sect. III-C1).  opts must be NULL.  Same ownership and
 * errors as hac_encode; more than 65536 distinct values give HAC_ERANGE. */
int im_encode(const float *W, int64_t n, int64_t m, int64_t ldw,
              const hac_opts_t *opts, void **blob, size_t *blob_bytes);

/* Encode W (host, row-major, leading dimension ldw >= m) into a HAC blob
 * (Sect. IV-B).  -0.0 is stored as +0.0; NaN/Inf give HAC_EINVAL.  n, m >= 1.
 * On success *blob is malloc'ed by the library (release with hac_free) and
 * *blob_bytes is its size. */
int hac_encode(const float *W, int64_t n, int64_t m, int64_t ldw,
               const hac_opts_t *opts, void **blob, size_t *blob_bytes);

/* Same for sHAC (Sect. IV-C): CSC with Huffman-coded nz, packed ri, cb. */
int shac_encode(const float *W, int64_t n, int64_t m, int64_t ldw,
                const hac_opts_t *opts, void **blob, size_t *blob_bytes);

/* Release a blob returned by an encode call (NULL is allowed). */
void hac_free(void *blob);

/* Check a host blob: header, section bounds, code tables (Kraft equality,
 * canonical order, first-level table), monotone column arrays with
 * col_pos[m] = nnz.  With deep != 0 the stream is also decoded from bit 0 and
 * every index entry, symbol count and row index (< n, ascending in a column)
 * is checked against it.  Never reads outside [blob, blob + bytes). */
int hac_validate(const void *blob, size_t bytes, int deep);

/* Copy the header of a validated host blob into *desc (header checks only). */
int hac_describe(const void *blob, size_t bytes, hac_desc_t *desc);

/* Size accounting for a host blob. */
int hac_stats(const void *blob, size_t bytes, hac_stats_t *out);

/* The library's own sequential CPU decoder (it ignores the chunk index).
 * HAC : W_out (n*m, row-major, may be NULL), sym_out (n*m symbols in column
 *       order, may be NULL); row_out, col_out must be NULL.
 * sHAC: W_out as above; sym_out, row_out, col_out (each nnz entries, CSC
 *       order, each may be NULL). */
int hac_decode_host(const void *blob, size_t bytes, float *W_out, int32_t *sym_out,
                    int32_t *row_out, int32_t *col_out);

/* ---- one dictionary for all layers of a network (Sect. V-H) ----------------- */

/* When the layers of a network are quantized together ("unified" quantization,
 * Sect. V-H; used for whole networks in Sect. V-K) they draw their weights from
 * one set of representatives, and one dictionary serves all of them.  A network
 * blob holds L layers, each HAC or sHAC, written with ONE Huffman code: every
 * layer contributes the symbols it writes into its own stream (all n*m entries
 * for HAC, the non-zeros for sHAC) to one pooled source; the alphabet numbers
 * the pooled values as usual (0.0 first when a HAC layer holds a zero, then
 * ascending) and the code is built from the pooled counts.  (The paper does not
 * say what is pooled when HAC and sHAC layers are mixed; this makes the code
 * optimal for all streams together.)
 *
 * A layer may also be an index map (the hybrid of Sect. V-K: index map for the
 * convolutional part, HAC / sHAC for the fully connected part, all sharing the
 * same representatives).  It writes no codewords and so adds nothing to the
 * pooled source; its pointers index the network's one value list: the k_sym
 * shared symbols followed by the values that occur in index-map layers only
 * (0.0 first if it is one of them, then ascending), k_values entries in all.
 * Pointers take 8 bits when k_values <= 256, else 16.  In such a layer's header
 * k_sym = k_values and has_zero = 0; the layer is multiplied with im_dot.
 *
 * Layout: this 256-byte header, L layer headers (hac_desc_t with dict_shared =
 * 1), the shared tables, then every layer's own sections (stream, per-column
 * arrays, chunk entries, ri).  All offsets count from the start of the network
 * blob, so a layer is multiplied with
 *        hac_dot(&layer_desc, d_network_blob, ...)   (or shac_dot)
 * exactly like a blob of its own, d_network_blob being the device copy of the
 * whole network blob. */
typedef struct {
    uint32_t magic;         /* 'HACN' = 0x4e434148                                         */
    uint32_t version;       /* 1                                                           */
    uint32_t header_bytes;  /* 256                                                         */
    uint32_t n_layers;      /* L >= 1                                                      */
    uint64_t blob_bytes;    /* total size                                                  */
    uint64_t off_layers;    /* hac_desc_t[L]                                               */
    uint64_t off_codebook, off_codelen, off_canon, off_symsort, off_lut;   /* as in hac_desc_t */
    uint32_t k_sym, lmax, lut_bits, has_zero;                              /* as in hac_desc_t */
    uint32_t k_values;      /* entries of the value list at off_codebook: the k_sym shared
                               symbols, then the values only index-map layers hold         */
    uint32_t reserved32;
    uint64_t reserved[20];
} hac_net_t;

typedef struct {
    uint64_t n_layers;
    uint64_t entries;          /* sum of n*m                                               */
    uint64_t nnz;              /* sum of the layers' non-zeros                             */
    uint64_t symbols;          /* codewords in all streams (the pooled source's length)    */
    uint64_t stream_bits;      /* sum of the layers' total_bits                            */
    uint64_t table_bytes;      /* the one dictionary                                       */
    uint64_t blob_bytes;
    uint64_t paper_bits;       /* the layers' words (+ ri, cb for sHAC) as in hac_stats_t,
                                  8 or 16 bits per entry of an index-map layer, plus
                                  6*32*k_sym ONCE for the two dictionaries and 32 bits per
                                  value only index-map layers hold                         */
    double   entropy_bits;     /* entropy of the pooled source per symbol                  */
    double   avg_code_bits;    /* bits spent on value codewords / symbols: H <= avg <= H+1 */
    double   psi;              /* blob_bytes / (4 * entries)                               */
} hac_net_stats_t;

/* Encode L layers with one shared dictionary.  formats[l] is HAC_FORMAT_HAC or
 * HAC_FORMAT_SHAC or HAC_FORMAT_IM; W[l] is n[l] x m[l], row-major, leading
 * dimension ldw[l] (all host).  opts (may be NULL) applies to every layer: chunk_nnz and ri_bits = 0
 * are chosen per layer, ri_coding affects the sHAC layers only.  Ownership and
 * errors as for hac_encode; L > 65536 gives HAC_EINVAL. */
int hac_net_encode(uint32_t n_layers, const uint32_t *formats, const float *const *W,
                   const int64_t *n, const int64_t *m, const int64_t *ldw,
                   const hac_opts_t *opts, void **blob, size_t *blob_bytes);

/* Copy the network header / the header of one layer of a host network blob
 * (header checks only). */
int hac_net_describe(const void *blob, size_t bytes, hac_net_t *net);
int hac_net_layer(const void *blob, size_t bytes, uint32_t layer, hac_desc_t *desc);

/* hac_validate for a network blob: the shared tables once, then every layer;
 * also that all layers point at the shared tables. */
int hac_net_validate(const void *blob, size_t bytes, int deep);

/* Size accounting with the dictionary counted once. */
int hac_net_stats(const void *blob, size_t bytes, hac_net_stats_t *out);

/* hac_decode_host for one layer of a network blob. */
int hac_net_decode_host(const void *blob, size_t bytes, uint32_t layer, float *W_out,
                        int32_t *sym_out, int32_t *row_out, int32_t *col_out);

/* ---- device side (asynchronous on `stream`) -------------------------------- */

/* Which of the two compressed formats the paper's size bounds favour for an
 * n x m matrix with nnz non-zeros and k distinct values: sHAC when the non-zero
 * ratio s = nnz / (n m) is below (a - (m+1)/(n m)) / (1 + a), a = (1 + log2 k) / 32
 * (the inequality psi_sHAC < psi_HAC at the end of Sect. IV-C, from Eqs. (2) and
 * (3)), else HAC.  Returns HAC_FORMAT_HAC or HAC_FORMAT_SHAC, or HAC_EINVAL.  The
 * bounds are loose for HAC (real streams are 2-6 times smaller, Sect. V), so this
 * is the paper's rule of thumb, not a size guarantee. */
int hac_choose_format(int64_t n, int64_t m, uint64_t nnz, uint32_t k);

/* Encode on the device: W (n x m, row-major, leading dimension ldw >= m) is in
 * device memory and so is the blob that comes out, byte for byte the blob
 * hac_encode / shac_encode (format = HAC_FORMAT_HAC / HAC_FORMAT_SHAC) build on
 * the host with the same options (Rice-coded row gaps included).  The value
 * histogram, the code bits, the gap bits for every Rice parameter and the bit
 * packing run on the GPU; the Huffman code, the choice of the parameter and the
 * prefix sums over columns are made on the host in between, so the call
 * synchronises `stream` (two or three times) and returns with the blob complete.
 * d_ws: hac_encode_dev_workspace_bytes(n, m) bytes, 256-byte aligned.  *desc
 * receives the header.  If d_blob is NULL or blob_capacity < desc->blob_bytes the
 * call returns HAC_EWORKSPACE with desc filled in: allocate desc->blob_bytes
 * (256-byte aligned) and call again.  n is limited to 65535 * 1024 rows. */
size_t hac_encode_dev_workspace_bytes(int64_t n, int64_t m);
int hac_encode_dev(uint32_t format, const float *d_W, int64_t n, int64_t m, int64_t ldw,
                   const hac_opts_t *opts, void *d_blob, size_t blob_capacity, hac_desc_t *desc,
                   void *d_ws, size_t ws_bytes, hac_stream_t stream);

/* Bytes of device workspace hac_dot / shac_dot need for a batch of B rows with
 * default launch settings (0 when none is needed: a single row, or a few rows
 * over a short X, see HAC_LAUNCH_NO_X_LDS).  The workspace holds X re-laid out
 * feature-major, or, on the dense route (see hac_dot), the decoded index map
 * of W.  A launch that forces another way may need more: size the workspace
 * with hac_workspace_bytes_for().  Both return 0 for B <= 0 and for a header
 * that no encoder could have written (zero sizes, unknown format). */
size_t hac_workspace_bytes(const hac_desc_t *desc, int64_t B);
size_t hac_workspace_bytes_for(const hac_desc_t *desc, int64_t B, const hac_launch_t *launch);

/* Which route hac_dot / shac_dot take for this blob, batch and launch (see
 * hac_dot): HAC_ROUTE_SPARSE or HAC_ROUTE_DENSE, or HAC_EINVAL. */
enum { HAC_ROUTE_SPARSE = 0, HAC_ROUTE_DENSE = 1 };
int hac_dot_route(const hac_desc_t *desc, int64_t B, const hac_launch_t *launch);

/* Y[B x m] = X[B x n] . W with W given as a HAC blob on the device
 * (Algorithm 1 for every row of X as in Algorithm 3; the stream is decoded
 * once per launch, not once per row).  Y is overwritten.  d_blob must be
 * 256-byte aligned, d_ws 256-byte aligned and >= hac_workspace_bytes().
 * B = 0 is a no-op.  fp32 accumulation; the order of the additions is fixed,
 * so results are bitwise reproducible run to run.
 *
 * The device calls check desc and their arguments, not the bytes of the blob:
 * d_blob must hold a blob that hac_validate (deep) accepts, as every encoder
 * returns.  On other bytes a walk still ends (rows are bounded by n), but the
 * result and the addresses it reads from X are undefined.
 *
 * Two routes.  Sparse: every non-zero is decoded and applied to the batch by
 * vector FMAs.  Dense: the stream is decoded once into an index map
 * (Sect. III-C1) in the workspace and multiplied tile by tile on the matrix
 * cores (fp32 MFMA); with few output tiles the K loop is split and the parts
 * are added in a fixed order.  The library estimates both times from desc and
 * B (the dense route wins for layers that are a fifth or more non-zero at
 * batches of several hundred rows) and takes the shorter; hac_dot_route() tells
 * which.  HAC_LAUNCH_SPARSE_ROUTE / HAC_LAUNCH_DENSE_ROUTE in launch->variant
 * force one (the dense route needs at most 65536 symbols). */
int hac_dot(const hac_desc_t *desc, const void *d_blob,
            const float *d_X, int64_t B, int64_t ldx,
            float *d_Y, int64_t ldy,
            void *d_ws, size_t ws_bytes,
            const hac_launch_t *launch, hac_stream_t stream);

/* Same for an sHAC blob (Algorithm 2): also unpacks the row-index fields and
 * writes 0 to the columns that hold no non-zero. */
int shac_dot(const hac_desc_t *desc, const void *d_blob,
             const float *d_X, int64_t B, int64_t ldx,
             float *d_Y, int64_t ldy,
             void *d_ws, size_t ws_bytes,
             const hac_launch_t *launch, hac_stream_t stream);

/* For callers that cannot allocate device memory or must not call an allocator (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): hac_dot / shac_dot
 * (picked by desc->format) with the workspace taken from a fixed array of
 * HAC_NOALLOC_WORKSPACE_BYTES inside the library's device image instead of from the caller.
 * The call allocates and frees nothing, on the host or on the device.  A product whose
 * workspace (hac_workspace_bytes_for(desc, B, launch)) exceeds the array returns
 * HAC_EWORKSPACE and launches nothing.  Each GPU holds one such array until the process ends;
 * every call on that GPU uses it, so calls that may overlap on one GPU (different streams or
 * threads) race on it: order them.  Nothing is kept in the array between calls (each call
 * writes what it reads).  Otherwise as hac_dot. */
#define HAC_NOALLOC_WORKSPACE_BYTES (16u << 20)
int hac_dot_noalloc(const hac_desc_t *desc, const void *d_blob,
                    const float *d_X, int64_t B, int64_t ldx,
                    float *d_Y, int64_t ldy,
                    const hac_launch_t *launch, hac_stream_t stream);

/* A chain of layers (not in the paper, which gives the product of one layer):
 *     A_0 = X,   A_{l+1} = act_l(A_l . W_l + bias_l),   Y = A_L
 * with W_l given compressed (HAC, sHAC or IM; layer blobs of their own or the
 * layers of a network blob), bias_l an optional vector of m_l floats added to
 * every row, act_l the identity or max(., 0).  Bias and activation are applied
 * where a sum is finished, and between two layers that both take the sparse
 * route the activations are written in the feature-major layout the next layer
 * gathers from, so only X itself is re-laid out.  n of layer l must equal m of
 * layer l - 1; at most 256 layers.  The result is that of calling the dot of
 * every layer in turn (same kernels, same order of additions). */
enum { HAC_ACT_NONE = 0, HAC_ACT_RELU = 1 };
typedef struct {
    const hac_desc_t *desc;  /* host: the layer's header                                    */
    const void *d_blob;      /* device: the blob that header's offsets count from            */
    const float *d_bias;     /* device: m floats, or NULL                                    */
    uint32_t activation;     /* HAC_ACT_NONE / HAC_ACT_RELU                                  */
    uint32_t reserved;       /* 0                                                            */
} hac_layer_t;

/* Device workspace for hac_forward on a batch of B rows: two activation buffers
 * and the largest workspace any layer needs (0 on bad arguments or B = 0). */
size_t hac_forward_workspace_bytes(const hac_layer_t *layers, uint32_t n_layers, int64_t B);

/* Y[B x m_L] = the chain applied to X[B x n_0] (row-major, ldx >= n_0, ldy >= m_L).
 * d_ws: 256-byte aligned, >= hac_forward_workspace_bytes().  Asynchronous on
 * `stream`; errors as for hac_dot (HAC_EINVAL also when the shapes do not chain). */
int hac_forward(const hac_layer_t *layers, uint32_t n_layers,
                const float *d_X, int64_t B, int64_t ldx, float *d_Y, int64_t ldy,
                void *d_ws, size_t ws_bytes, hac_stream_t stream);

/* Y = X . W for an index-map blob (Sect. III-C1).  Up to 32 rows of X the map is
 * streamed once per group of 8 rows and multiplied by vector FMAs; beyond that,
 * pointers are expanded through the representatives tile by tile and multiplied
 * on the matrix cores (fp32 in, fp32 accumulate).  The workspace
 * (hac_workspace_bytes(), 0 for large batches) holds partial sums when the rows
 * of W are split over blocks; launch must be NULL.  Otherwise as hac_dot. */
int im_dot(const hac_desc_t *desc, const void *d_blob,
           const float *d_X, int64_t B, int64_t ldx,
           float *d_Y, int64_t ldy,
           void *d_ws, size_t ws_bytes,
           const hac_launch_t *launch, hac_stream_t stream);

/* TEST ONLY: materialise what the device decoder sees.
 * d_W  : n*m floats, row-major (every entry written);
 * d_sym: n*m int32 symbols in column order (every entry written). */
int hac_decode_dev(const hac_desc_t *desc, const void *d_blob,
                   float *d_W, int32_t *d_sym, hac_stream_t stream);

/* TEST ONLY: d_nz, d_sym, d_row, d_col each hold nnz entries in CSC order. */
int shac_decode_dev(const hac_desc_t *desc, const void *d_blob,
                    float *d_nz, int32_t *d_sym, int32_t *d_row, int32_t *d_col,
                    hac_stream_t stream);

/* The kernels launched by the calling thread's most recent successful hac_dot / shac_dot /
 * im_dot / hac_dot_noalloc call, in launch order, separated by "; ", spelled as a profiler prints
 * them without their namespace (e.g. "transpose_panel32_kernel; dot_batch_kernel<false, 4, true,
 * false>").  For attributing profiler rows to calls; never NULL. */
const char *hac_last_kernels(void);

/* Text for a status code; never NULL. */
const char *hac_strerror(int status);

/* hipError_t value of the most recent HIP failure on the calling thread
 * (0 if none); cleared by the next successful device call of that thread. */
int hac_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HAC_H */
