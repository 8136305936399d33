/* CPU oracle in plain C for the HAC / sHAC formats and their dot procedures.
 *
 * TEST INFRASTRUCTURE.  Written from the paper (arXiv 2108.12704, Sect. IV);
 * shares nothing with the HIP library.  Same readings as the Python oracle:
 * b = 32-bit words, first stream bit = most significant bit of word 0,
 * decoders stop on the symbol count, fp64 accumulation.  The sequential dot
 * routines are written as what they compute -- the columns of W summed as
 * their codewords are read off the stream by a bit-serial tree walk -- not as
 * a transcription of the paper's listings.
 *
 * The Huffman code itself is built by the Python oracle and handed in as
 *   - values[k], code[k], len[k]      for encoding (H_W), and
 *   - left[k-1 or 1], right[..], root for decoding (H_W^-1 as a binary tree:
 *     node ids < k are leaves, internal node id i has children left[i-k],
 *     right[i-k]).
 *
 * Build: gcc -O2 -shared -fPIC -pthread oracle.c -o liboracle.so
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- bit writer: append `len` bits of `code`, most significant first ---- */
typedef struct {
    uint32_t *words;
    int64_t cap;      /* capacity in words */
    int64_t nbits;    /* bits written so far */
    int overflow;
} bitwriter;

static void put_bits(bitwriter *bw, uint32_t code, int len)
{
    for (int t = len - 1; t >= 0; --t) {
        int64_t w = bw->nbits / 32;
        int pos = (int)(bw->nbits % 32);          /* 0 = most significant bit */
        if (w >= bw->cap) { bw->overflow = 1; return; }
        if ((code >> t) & 1u) bw->words[w] |= (uint32_t)1 << (31 - pos);
        bw->nbits++;
    }
}

static int find_symbol(const float *values, int k, float v)
{
    for (int i = 0; i < k; ++i)
        if (values[i] == v) return i;
    return -1;
}

/* HAC(W) (Sect. IV-B): all n*m entries in column order, zeros included.
 * W is row-major with leading dimension m.  words[] must be zero-filled by
 * the caller (that is the zero padding).  Returns 0, or -1 on a value outside
 * the alphabet, -2 on overflow of words[]. */
int oracle_hac_encode(const float *W, int64_t n, int64_t m,
                      const float *values, const uint32_t *code, const int32_t *len, int32_t k,
                      uint32_t *words, int64_t cap_words, int64_t *nbits_out)
{
    bitwriter bw = { words, cap_words, 0, 0 };
    for (int64_t j = 0; j < m; ++j)
        for (int64_t i = 0; i < n; ++i) {
            int z = find_symbol(values, k, W[i * m + j]);
            if (z < 0) return -1;
            put_bits(&bw, code[z], len[z]);
            if (bw.overflow) return -2;
        }
    *nbits_out = bw.nbits;
    return 0;
}

/* sHAC(W) (Sect. IV-C): CSC arrays, nz Huffman-coded without the symbol 0.
 * ri has room for cap_nz entries, cb for m+1. */
int oracle_shac_encode(const float *W, int64_t n, int64_t m,
                       const float *values, const uint32_t *code, const int32_t *len, int32_t k,
                       uint32_t *words, int64_t cap_words, int64_t *nbits_out,
                       int64_t *ri, int64_t cap_nz, int64_t *cb)
{
    bitwriter bw = { words, cap_words, 0, 0 };
    int64_t q = 0;
    cb[0] = 0;
    for (int64_t j = 0; j < m; ++j) {
        for (int64_t i = 0; i < n; ++i) {
            float v = W[i * m + j];
            if (v == 0.0f) continue;
            int z = find_symbol(values, k, v);
            if (z < 0) return -1;
            if (q >= cap_nz) return -2;
            put_bits(&bw, code[z], len[z]);
            if (bw.overflow) return -2;
            ri[q++] = i;
        }
        cb[j + 1] = q;
    }
    *nbits_out = bw.nbits;
    return 0;
}

/* ---- the code tree and a bit-serial reader ----
 * The stream is one long run of bits, bit p being bit (31 - p % 32) of word
 * p / 32; a codeword may straddle two words.  A symbol is read by walking the
 * tree from the root, one edge per bit (0 left, 1 right), down to a leaf. */
typedef struct { const int32_t *left, *right; int32_t k, root; } tree_t;

static int bit_at(const uint32_t *C, int64_t pos)
{
    return (int)((C[pos / 32] >> (31 - (int)(pos % 32))) & 1u);
}

/* symbol whose codeword starts at bit *pos; advances *pos past it.  Never reads
 * past bit `end`: returns -1 when the codeword does not end before it. */
static int next_symbol(const uint32_t *C, int64_t *pos, int64_t end, const tree_t *t)
{
    int32_t node = t->root;
    while (node >= t->k) {
        if (*pos >= end) return -1;
        node = bit_at(C, *pos) ? t->right[node - t->k] : t->left[node - t->k];
        (*pos)++;
    }
    return node;
}

int oracle_unpack(const uint32_t *words, int64_t N, int64_t count,
                  const int32_t *left, const int32_t *right, int32_t k, int32_t root,
                  int32_t *sym_out)
{
    tree_t t = { left, right, k, root };
    int64_t pos = 0;
    for (int64_t got = 0; got < count; ++got) {
        int z = next_symbol(words, &pos, N * 32, &t);
        if (z < 0) return -1;
        sym_out[got] = z;
    }
    return 0;
}

/* x^T W from a HAC stream (what Algorithm 1 returns): the stream is W column
 * after column, every entry a codeword, so column j is the next n symbols;
 * each is multiplied with its row's x as it is read.  out[m], x has n entries. */
int oracle_dot_hac(const uint32_t *C, int64_t N,
                   const int32_t *left, const int32_t *right, int32_t k, int32_t root,
                   const float *value, const float *x, int64_t n, int64_t m, double *out)
{
    tree_t t = { left, right, k, root };
    int64_t pos = 0;
    for (int64_t j = 0; j < m; ++j) {
        double sum = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            int z = next_symbol(C, &pos, N * 32, &t);
            if (z < 0) return -1;
            sum += (double)x[i] * (double)value[z];
        }
        out[j] = sum;
    }
    return 0;
}

/* x^T W from the sHAC triple (what Algorithm 2 returns): the stream holds the
 * non-zeros only, in CSC order; column j owns positions cb[j] .. cb[j+1] - 1
 * (none for an empty column, whose sum stays 0) and position p is in row ri[p]. */
int oracle_dot_shac(const uint32_t *C, int64_t N1, const int64_t *ri, const int64_t *cb,
                    const int32_t *left, const int32_t *right, int32_t k, int32_t root,
                    const float *value, const float *x, int64_t n, int64_t m, double *out)
{
    tree_t t = { left, right, k, root };
    int64_t pos = 0;
    (void)n;
    for (int64_t j = 0; j < m; ++j) {
        double sum = 0.0;
        for (int64_t p = cb[j]; p < cb[j + 1]; ++p) {
            int z = next_symbol(C, &pos, N1 * 32, &t);
            if (z < 0) return -1;
            sum += (double)x[ri[p]] * (double)value[z];
        }
        out[j] = sum;
    }
    return 0;
}

/* Algorithm 3 (ParDot): rows of X in q chunks of ceil(rows/q), one thread per
 * chunk, each row through Dot on the whole compressed matrix. */
typedef struct {
    int shac;
    const uint32_t *C; int64_t N;
    const int64_t *ri, *cb;
    const int32_t *left, *right; int32_t k, root;
    const float *values;
    const float *X; int64_t ldx;
    int64_t n, m;
    double *out;
    int64_t start, end;
    int status;
} par_job;

static void *par_worker(void *arg)
{
    par_job *j = (par_job *)arg;
    for (int64_t i = j->start; i < j->end; ++i) {
        const float *x = j->X + i * j->ldx;
        double *y = j->out + i * j->m;
        int rc = j->shac
            ? oracle_dot_shac(j->C, j->N, j->ri, j->cb, j->left, j->right, j->k, j->root,
                              j->values, x, j->n, j->m, y)
            : oracle_dot_hac(j->C, j->N, j->left, j->right, j->k, j->root,
                             j->values, x, j->n, j->m, y);
        if (rc) j->status = rc;
    }
    return NULL;
}

static int pardot(par_job proto, int64_t rows, int32_t q)
{
    if (rows <= 0) return 0;
    if (q < 1) q = 1;
    int64_t chunk = (rows + q - 1) / q;
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)q);
    par_job *jobs = (par_job *)malloc(sizeof(par_job) * (size_t)q);
    if (!th || !jobs) { free(th); free(jobs); return -3; }
    int started = 0, rc = 0;
    for (int32_t t = 0; t < q; ++t) {
        int64_t s = (int64_t)t * chunk, e = s + chunk < rows ? s + chunk : rows;
        if (s >= rows) break;
        jobs[started] = proto;
        jobs[started].start = s;
        jobs[started].end = e;
        jobs[started].status = 0;
        if (pthread_create(&th[started], NULL, par_worker, &jobs[started])) { rc = -3; break; }
        started++;
    }
    for (int t = 0; t < started; ++t) {
        pthread_join(th[t], NULL);
        if (jobs[t].status) rc = jobs[t].status;
    }
    free(th);
    free(jobs);
    return rc;
}

int oracle_pardot_hac(const uint32_t *C, int64_t N,
                      const int32_t *left, const int32_t *right, int32_t k, int32_t root,
                      const float *values, const float *X, int64_t rows, int64_t ldx,
                      int64_t n, int64_t m, int32_t q, double *out)
{
    par_job p;
    memset(&p, 0, sizeof p);
    p.shac = 0; p.C = C; p.N = N; p.left = left; p.right = right; p.k = k; p.root = root;
    p.values = values; p.X = X; p.ldx = ldx; p.n = n; p.m = m; p.out = out;
    return pardot(p, rows, q);
}

int oracle_pardot_shac(const uint32_t *C, int64_t N1, const int64_t *ri, const int64_t *cb,
                       const int32_t *left, const int32_t *right, int32_t k, int32_t root,
                       const float *values, const float *X, int64_t rows, int64_t ldx,
                       int64_t n, int64_t m, int32_t q, double *out)
{
    par_job p;
    memset(&p, 0, sizeof p);
    p.shac = 1; p.C = C; p.N = N1; p.ri = ri; p.cb = cb;
    p.left = left; p.right = right; p.k = k; p.root = root;
    p.values = values; p.X = X; p.ldx = ldx; p.n = n; p.m = m; p.out = out;
    return pardot(p, rows, q);
}

/* ---- decode once, all rows of X at a time, threads over ranges of columns ----
 *
 * The paper's conclusions propose to store the bit offset at which every
 * column begins, so that columns can be handed to different threads.  This is
 * that variant, written plainly: one sequential pass finds the offsets; then
 * thread t takes a contiguous range of columns, walks each column's codewords
 * from its offset (one tree step per bit, as above) and adds x[b][row] * value
 * to the column's B sums for every non-zero it meets.  X is transposed first
 * (xt[row][b]) so that the B products of one non-zero touch consecutive
 * memory.  fp64 accumulation, rows in ascending order: the result is the
 * dense product up to rounding, and does not depend on the thread count. */

/* HAC: colbit[j] = first bit of column j (m + 1 entries, colbit[m] = stream length). */
int oracle_hac_column_offsets(const uint32_t *C, int64_t nbits,
                              const int32_t *left, const int32_t *right, int32_t k, int32_t root,
                              int64_t n, int64_t m, int64_t *colbit)
{
    tree_t t = { left, right, k, root };
    int64_t pos = 0;
    for (int64_t j = 0; j < m; ++j) {
        colbit[j] = pos;
        for (int64_t i = 0; i < n; ++i)
            if (next_symbol(C, &pos, nbits, &t) < 0) return -1;
    }
    colbit[m] = pos;
    return pos == nbits ? 0 : -1;
}

/* sHAC: colbit[j] = first bit of the codeword of nz[cb[j]]. */
int oracle_shac_column_offsets(const uint32_t *C, int64_t nbits, const int64_t *cb,
                               const int32_t *left, const int32_t *right, int32_t k, int32_t root,
                               int64_t m, int64_t *colbit)
{
    tree_t t = { left, right, k, root };
    int64_t pos = 0;
    for (int64_t j = 0; j < m; ++j) {
        colbit[j] = pos;
        for (int64_t p = cb[j]; p < cb[j + 1]; ++p)
            if (next_symbol(C, &pos, nbits, &t) < 0) return -1;
    }
    colbit[m] = pos;
    return pos == nbits ? 0 : -1;
}

typedef struct {
    int shac;
    const uint32_t *C; const int64_t *colbit;
    const int64_t *ri, *cb;
    tree_t tree;
    const float *values;
    const float *xt;          /* n x B */
    int64_t B, n, m;
    double *out;              /* B x m */
    double *sums;             /* this thread's B sums */
    int64_t c0, c1;
    int status;
} col_job;

static void *col_worker(void *arg)
{
    col_job *j = (col_job *)arg;
    const int64_t end = j->colbit[j->m];          /* the stream's length in bits */
    for (int64_t col = j->c0; col < j->c1; ++col) {
        int64_t pos = j->colbit[col];
        for (int64_t b = 0; b < j->B; ++b) j->sums[b] = 0.0;
        if (j->shac) {
            for (int64_t p = j->cb[col]; p < j->cb[col + 1]; ++p) {
                const int z = next_symbol(j->C, &pos, end, &j->tree);
                if (z < 0) { j->status = -1; return NULL; }
                const double v = (double)j->values[z];
                const float *x = j->xt + j->ri[p] * j->B;
                for (int64_t b = 0; b < j->B; ++b) j->sums[b] += (double)x[b] * v;
            }
        } else {
            for (int64_t i = 0; i < j->n; ++i) {
                const int z = next_symbol(j->C, &pos, end, &j->tree);
                if (z < 0) { j->status = -1; return NULL; }
                const float w = j->values[z];
                if (w == 0.0f) continue;
                const float *x = j->xt + i * j->B;
                for (int64_t b = 0; b < j->B; ++b) j->sums[b] += (double)x[b] * (double)w;
            }
        }
        for (int64_t b = 0; b < j->B; ++b) j->out[b * j->m + col] = j->sums[b];
    }
    return NULL;
}

/* out[B x m] = X[B x n] . W, W given as a HAC (ri = cb = NULL) or sHAC stream with its column offsets. */
int oracle_coldot(const uint32_t *C, const int64_t *colbit, const int64_t *ri, const int64_t *cb,
                  const int32_t *left, const int32_t *right, int32_t k, int32_t root,
                  const float *values, const float *X, int64_t B, int64_t ldx,
                  int64_t n, int64_t m, int32_t q, double *out)
{
    if (B <= 0 || m <= 0) return 0;
    if (q < 1) q = 1;
    if (q > m) q = (int32_t)m;
    float *xt = (float *)malloc(sizeof(float) * (size_t)n * (size_t)B);
    double *sums = (double *)malloc(sizeof(double) * (size_t)B * (size_t)q);
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)q);
    col_job *jobs = (col_job *)malloc(sizeof(col_job) * (size_t)q);
    int rc = 0, started = 0;
    if (!xt || !sums || !th || !jobs) { rc = -3; goto done; }
    for (int64_t b = 0; b < B; ++b)
        for (int64_t i = 0; i < n; ++i) xt[i * B + b] = X[b * ldx + i];
    {
        const int64_t chunk = (m + q - 1) / q;
        for (int32_t t = 0; t < q; ++t) {
            const int64_t c0 = (int64_t)t * chunk, c1 = c0 + chunk < m ? c0 + chunk : m;
            if (c0 >= m) break;
            col_job *j = &jobs[started];
            j->shac = cb != NULL; j->C = C; j->colbit = colbit; j->ri = ri; j->cb = cb;
            j->tree.left = left; j->tree.right = right; j->tree.k = k; j->tree.root = root;
            j->values = values; j->xt = xt; j->B = B; j->n = n; j->m = m; j->out = out;
            j->sums = sums + (size_t)started * (size_t)B; j->c0 = c0; j->c1 = c1; j->status = 0;
            if (pthread_create(&th[started], NULL, col_worker, j)) { rc = -3; break; }
            started++;
        }
    }
    for (int t = 0; t < started; ++t) {
        pthread_join(th[t], NULL);
        if (jobs[t].status) rc = jobs[t].status;
    }
done:
    free(xt); free(sums); free(th); free(jobs);
    return rc;
}
