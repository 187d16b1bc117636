/*
 * CPU oracle for compressed-layer inference (pruned, codebook-quantised,
 * relative-indexed, Huffman-coded weight matrices).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, single-purpose restatement
 * of what the paper computes, used only by the tests, by the smoke check and by
 * the CPU-baseline leg of the benchmark.  The product library never calls it and
 * shares no source, table or helper with it.
 *
 * Every function cites the passage of the paper it restates.  Arithmetic that
 * decides an integer (the nearest-centre choice) and all sums are in fp64; the
 * stored weights and activations are fp32 as the paper states (Sec. III-A).
 *
 * Readings taken where the text is silent or ambiguous are marked READING.
 *
 * Build: gcc -O2 -std=c99 -ffp-contract=off -fopenmp -shared -fPIC oracle.c -o liboracle.so
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ECORRUPT (-2)
#define ORC_ENOMEM (-3)

/* ------------------------------------------------------------------------- */
/* Sec. III-B, quantisation paragraph: r bits give at most 2^r - 1 distinct   */
/* non-zero shared values plus 0; each val entry is an r-bit index of its     */
/* cluster centre; the centres are kept in the codebook.                      */
/*                                                                            */
/* READING: index 0 is the reserved value 0 (used by padding entries only).   */
/* READING: "clustered" is realised as linear quantisation: the 2^r - 1       */
/* centres are equally spaced from the smallest to the largest surviving      */
/* weight, evaluated in fp64 and rounded to fp32.  A single centre (r = 1)    */
/* sits at the midpoint.                                                      */
/* ------------------------------------------------------------------------- */
int orc_linear_codebook(const float *W, int64_t n, int r, float *codebook)
{
    if (!W || !codebook || n < 0 || r < 1 || r > 8) return ORC_EINVAL;
    int nc = (1 << r) - 1;
    int have = 0;
    double lo = 0.0, hi = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        float w = W[i];
        if (!isfinite(w)) return ORC_EINVAL;
        if (w == 0.0f) continue;
        if (!have) { lo = hi = (double)w; have = 1; }
        else { if ((double)w < lo) lo = (double)w; if ((double)w > hi) hi = (double)w; }
    }
    codebook[0] = 0.0f;
    for (int t = 1; t <= nc; ++t) {
        double c;
        if (!have) c = 0.0;
        else if (nc == 1) c = 0.5 * (lo + hi);
        else c = lo + (double)(t - 1) * (hi - lo) / (double)(nc - 1);
        codebook[t] = (float)c;
    }
    return ORC_OK;
}

/* Same passage.  A pruned weight (exactly 0) gets index 0.  A surviving weight
 * gets the index in [1, 2^r - 1] of the centre nearest to it in fp64 distance;
 * READING: ties go to the lower index.  A surviving weight never gets index 0,
 * even when its centre's value happens to be 0. */
int orc_quantize(const float *W, int64_t n, int r, const float *codebook, uint8_t *q)
{
    if (!W || !codebook || !q || n < 0 || r < 1 || r > 8) return ORC_EINVAL;
    int nc = (1 << r) - 1;
    for (int64_t i = 0; i < n; ++i) {
        float w = W[i];
        if (!isfinite(w)) return ORC_EINVAL;
        if (w == 0.0f) { q[i] = 0; continue; }
        int best = 1;
        double bestd = fabs((double)w - (double)codebook[1]);
        for (int t = 2; t <= nc; ++t) {
            double d = fabs((double)w - (double)codebook[t]);
            if (d < bestd) { bestd = d; best = t; }
        }
        q[i] = (uint8_t)best;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Block geometry: Sec. IV-A (blocks stored contiguously, one block per row   */
/* of the re-laid-out matrix) and Algorithm 2 (block i covers rows starting   */
/* at row_id = (i / nbw) * bh and columns starting at col_id = (i % nbw) * bw */
/* where nbw is the number of blocks across).                                 */
/* READING: when bh or bw does not divide the matrix the count of blocks is   */
/* rounded up and edge blocks keep their true, smaller shape.                 */
/* ------------------------------------------------------------------------- */
static void block_geom(int M, int K, int bh, int bw, int64_t bi,
                       int *row_id, int *col_id, int *bhp, int *bwp)
{
    int64_t nbw = (K + bw - 1) / bw;
    *row_id = (int)((bi / nbw) * bh);
    *col_id = (int)((bi % nbw) * bw);
    *bhp = (M - *row_id < bh) ? (M - *row_id) : bh;
    *bwp = (K - *col_id < bw) ? (K - *col_id) : bw;
}

int64_t orc_num_blocks(int M, int K, int bh, int bw)
{
    if (M < 1 || K < 1 || bh < 1 || bw < 1) return ORC_EINVAL;
    return (int64_t)((M + bh - 1) / bh) * (int64_t)((K + bw - 1) / bw);
}

/* ------------------------------------------------------------------------- */
/* Sec. III-B, relative index paragraph: each non-zero stores, in k bits, how  */
/* many zeros lie between it and the previous non-zero of its row (for the    */
/* first non-zero: how many lie before it, i.e. its position); when that      */
/* count does not fit the k-bit field a zero is added to both val and col_ind.*/
/* Here "row" is a row of the block-contiguous matrix of Sec. IV-A, i.e. one  */
/* flattened block.                                                            */
/*                                                                            */
/* READING: the field holds z in [0, 2^k - 1]; a padding entry carries value  */
/* index 0 and z = 2^k - 1 and itself occupies a position, so it advances the */
/* running position by 2^k.  (With k = 2 a first non-zero at 0-based position */
/* >= 4 yields a padding entry standing at position 3, the "fourth location"  */
/* of the paper's example.)                                                   */
/* READING: nothing is stored for the zeros that follow a block's last        */
/* non-zero.                                                                   */
/* READING: colmajor == 0 flattens a block row by row (p = r*bw' + c), as the  */
/* paper's 8x8 -> 4x16 illustration does (a block's elements stored           */
/* contiguously, the re-laid matrix then kept as relative-indexed CSR); a     */
/* block of a single column then is a CSC column with a relative row index.   */
/* colmajor != 0 flattens a block column by column (p = c*bh' + r) instead.   */
/*                                                                            */
/* q: M x K row-major quantised indices (0 = pruned).  With val == NULL only  */
/* the number of entries is returned.  block_ptr (nblocks + 1, 0-based entry  */
/* offsets) may be NULL.                                                       */
/* ------------------------------------------------------------------------- */
int64_t orc_build_entries(const uint8_t *q, int M, int K, int bh, int bw, int kbits,
                          int colmajor, uint8_t *val, uint8_t *idx, int64_t *block_ptr)
{
    if (!q || M < 1 || K < 1 || bh < 1 || bw < 1 || kbits < 1 || kbits > 8) return ORC_EINVAL;
    int64_t nblocks = orc_num_blocks(M, K, bh, bw);
    int64_t R = (int64_t)1 << kbits;
    int64_t n = 0;
    for (int64_t bi = 0; bi < nblocks; ++bi) {
        int row_id, col_id, bhp, bwp;
        block_geom(M, K, bh, bw, bi, &row_id, &col_id, &bhp, &bwp);
        if (block_ptr) block_ptr[bi] = n;
        int64_t prev = -1;
        int64_t np = (int64_t)bhp * bwp;
        for (int64_t p = 0; p < np; ++p) {
            int r = colmajor ? (int)(p % bhp) : (int)(p / bwp);
            int c = colmajor ? (int)(p / bhp) : (int)(p % bwp);
            uint8_t s = q[(int64_t)(row_id + r) * K + (col_id + c)];
            if (!s) continue;
            int64_t g = p - prev - 1;
            while (g > R - 1) {
                if (val) { val[n] = 0; idx[n] = (uint8_t)(R - 1); }
                ++n;
                prev += R;
                g -= R;
            }
            if (val) { val[n] = s; idx[n] = (uint8_t)g; }
            ++n;
            prev = p;
        }
    }
    if (block_ptr) block_ptr[nblocks] = n;
    return n;
}

/* ------------------------------------------------------------------------- */
/* Sec. III-B, last paragraph / Han et al. pipeline: the val and col_ind       */
/* arrays are each Huffman coded.  Textbook construction: repeatedly merge    */
/* the two least-weight trees.  Symbols that never occur get no codeword      */
/* (length 0).  READING: an alphabet with a single occurring symbol gets a    */
/* 1-bit codeword.  Tie-breaking is unspecified (any optimal prefix code is   */
/* a correct Huffman code).                                                    */
/*                                                                            */
/* code[s] holds the codeword with bit i (LSB = bit 0) being the i-th bit      */
/* written to the stream, i.e. bit 0 is the decision taken at the tree root.  */
/* ------------------------------------------------------------------------- */
int orc_huffman_code(const int64_t *counts, int nsym, uint8_t *len, uint64_t *code)
{
    if (!counts || !len || !code || nsym < 1 || nsym > 256) return ORC_EINVAL;
    int maxn = 2 * nsym;
    int64_t *w = (int64_t *)malloc(sizeof(int64_t) * maxn);
    int *left = (int *)malloc(sizeof(int) * maxn);
    int *right = (int *)malloc(sizeof(int) * maxn);
    int *alive = (int *)malloc(sizeof(int) * maxn);
    if (!w || !left || !right || !alive) { free(w); free(left); free(right); free(alive); return ORC_ENOMEM; }
    int nn = 0, nalive = 0;
    for (int s = 0; s < nsym; ++s) { len[s] = 0; code[s] = 0; }
    /* leaves: node id = order of insertion; remember which symbol */
    int *symof = (int *)malloc(sizeof(int) * maxn);
    if (!symof) { free(w); free(left); free(right); free(alive); return ORC_ENOMEM; }
    for (int s = 0; s < nsym; ++s) {
        if (counts[s] < 0) { free(w); free(left); free(right); free(alive); free(symof); return ORC_EINVAL; }
        if (counts[s] > 0) { w[nn] = counts[s]; left[nn] = right[nn] = -1; alive[nn] = 1; symof[nn] = s; ++nn; ++nalive; }
    }
    int rc = ORC_OK;
    if (nalive == 0) { /* empty stream: no codewords */
    } else if (nalive == 1) {
        len[symof[0]] = 1; code[symof[0]] = 0;
    } else {
        while (nalive > 1) {
            int a = -1, b = -1; /* a = smallest, b = second smallest */
            for (int i = 0; i < nn; ++i) {
                if (!alive[i]) continue;
                if (a < 0 || w[i] < w[a]) { b = a; a = i; }
                else if (b < 0 || w[i] < w[b]) { b = i; }
            }
            alive[a] = alive[b] = 0;
            w[nn] = w[a] + w[b]; left[nn] = a; right[nn] = b; alive[nn] = 1; symof[nn] = -1;
            ++nn; --nalive;
        }
        /* walk down from the root (last node) assigning bits: left = 0, right = 1 */
        int root = nn - 1;
        int *stack = (int *)malloc(sizeof(int) * maxn);
        uint8_t *d = (uint8_t *)calloc(maxn, 1);
        uint64_t *cw = (uint64_t *)calloc(maxn, sizeof(uint64_t));
        if (!stack || !d || !cw) { rc = ORC_ENOMEM; }
        else {
            int sp = 0; stack[sp++] = root;
            while (sp) {
                int u = stack[--sp];
                if (left[u] < 0) {
                    if (d[u] > 64) { rc = ORC_EINVAL; break; }
                    len[symof[u]] = d[u]; code[symof[u]] = cw[u];
                } else {
                    int l = left[u], r = right[u];
                    d[l] = d[r] = (uint8_t)(d[u] + 1);
                    cw[l] = cw[u];
                    cw[r] = cw[u] | ((uint64_t)1 << d[u]);
                    stack[sp++] = l; stack[sp++] = r;
                }
            }
        }
        free(stack); free(d); free(cw);
    }
    free(w); free(left); free(right); free(alive); free(symof);
    return rc;
}

/* Stream convention: bit b of a stream is bit (b mod 8) of byte b / 8, and a
 * codeword's bits are written in the order the tree is walked. */
static inline int get_bit(const uint8_t *bytes, int64_t b) { return (bytes[b >> 3] >> (b & 7)) & 1; }
static inline void put_bit(uint8_t *bytes, int64_t b, int v)
{
    if (v) bytes[b >> 3] |= (uint8_t)(1u << (b & 7));
    else bytes[b >> 3] &= (uint8_t)~(1u << (b & 7));
}

/* Append the codewords of sym[0..n) starting at bit start_bit.  bytes == NULL
 * only measures.  Returns the bit position after the last codeword. */
int64_t orc_huffman_encode(const uint8_t *sym, int64_t n, int nsym, const uint8_t *len,
                           const uint64_t *code, uint8_t *bytes, int64_t start_bit)
{
    if ((!sym && n > 0) || !len || !code || n < 0 || start_bit < 0) return ORC_EINVAL;
    int64_t b = start_bit;
    for (int64_t i = 0; i < n; ++i) {
        int s = sym[i];
        if (s >= nsym || len[s] == 0) return ORC_EINVAL;
        if (bytes) for (int j = 0; j < len[s]; ++j) put_bit(bytes, b + j, (int)((code[s] >> j) & 1));
        b += len[s];
    }
    return b;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1 steps 5-6 / Algorithm 2 steps 5-6: Huffman decoding of a span  */
/* of a bit stream.  Bit-serial: one tree edge per bit.  The tree is rebuilt  */
/* from the (len, code) table, which also verifies that the table is a prefix */
/* code.  Decodes exactly n symbols from start_bit; a walk that leaves the    */
/* tree or runs past total_bits is an error.  bitpos (optional, n entries)    */
/* receives the bit address at which each codeword starts.  Returns the bit   */
/* position after the last decoded codeword, or a negative error.             */
/* ------------------------------------------------------------------------- */
typedef struct { int (*child)[2]; int *leaf; int nn; } orc_trie;

/* Rebuild the code tree from a (len, code) table; fails unless the table is a
 * prefix code. */
static int64_t trie_build(orc_trie *t, int nsym, const uint8_t *len, const uint64_t *code)
{
    int cap = 2;
    for (int s = 0; s < nsym; ++s) { if (len[s] > 64) return ORC_EINVAL; cap += len[s]; }
    t->child = (int (*)[2])malloc(sizeof(int[2]) * cap);
    t->leaf = (int *)malloc(sizeof(int) * cap);
    if (!t->child || !t->leaf) { free(t->child); free(t->leaf); return ORC_ENOMEM; }
    int nn = 1; t->child[0][0] = t->child[0][1] = -1; t->leaf[0] = -1;
    int64_t rc = 0;
    for (int s = 0; s < nsym && rc == 0; ++s) {
        if (!len[s]) continue;
        int u = 0;
        for (int j = 0; j < len[s]; ++j) {
            if (t->leaf[u] >= 0) { rc = ORC_ECORRUPT; break; }      /* a codeword is a prefix of this one */
            int bit = (int)((code[s] >> j) & 1);
            if (t->child[u][bit] < 0) {
                t->child[nn][0] = t->child[nn][1] = -1; t->leaf[nn] = -1; t->child[u][bit] = nn++;
            }
            u = t->child[u][bit];
        }
        if (rc) break;
        if (t->leaf[u] >= 0 || t->child[u][0] >= 0 || t->child[u][1] >= 0) { rc = ORC_ECORRUPT; break; }
        t->leaf[u] = s;
    }
    t->nn = nn;
    if (rc) { free(t->child); free(t->leaf); }
    return rc;
}

/* Walk one codeword starting at bit *b.  Returns the symbol or a negative error. */
static int trie_walk(const orc_trie *t, const uint8_t *bytes, int64_t total_bits, int64_t *b)
{
    int u = 0;
    while (t->leaf[u] < 0) {
        if (*b >= total_bits) return ORC_ECORRUPT;
        int nx = t->child[u][get_bit(bytes, *b)];
        ++*b;
        if (nx < 0) return ORC_ECORRUPT;
        u = nx;
    }
    if (u == 0) return ORC_ECORRUPT; /* empty code table */
    return t->leaf[u];
}

int64_t orc_huffman_decode_serial(const uint8_t *bytes, int64_t total_bits, int64_t start_bit,
                                  int64_t n, int nsym, const uint8_t *len, const uint64_t *code,
                                  uint8_t *out, int64_t *bitpos)
{
    if ((!bytes && total_bits > 0) || !len || !code || n < 0 || start_bit < 0 || nsym < 1 || nsym > 256) return ORC_EINVAL;
    orc_trie t;
    int64_t rc = trie_build(&t, nsym, len, code);
    if (rc) return rc;
    int64_t b = start_bit;
    for (int64_t i = 0; i < n; ++i) {
        if (bitpos) bitpos[i] = b;
        int s = trie_walk(&t, bytes, total_bits, &b);
        if (s < 0) { rc = s; break; }
        out[i] = (uint8_t)s;
    }
    free(t.child); free(t.leaf);
    return rc ? rc : b;
}

/* The same walk in the form the algorithms state it: decode the span of the
 * stream between two bit addresses (val_begin .. val_end of a row_ptr pair).
 * A codeword that straddles end_bit is an error.  Returns the number of symbols
 * decoded (at most max_out), or a negative error. */
int64_t orc_huffman_decode_span(const uint8_t *bytes, int64_t start_bit, int64_t end_bit,
                                int nsym, const uint8_t *len, const uint64_t *code,
                                uint8_t *out, int64_t max_out)
{
    if ((!bytes && end_bit > 0) || !len || !code || start_bit < 0 || end_bit < start_bit || nsym < 1 || nsym > 256) return ORC_EINVAL;
    orc_trie t;
    int64_t rc = trie_build(&t, nsym, len, code);
    if (rc) return rc;
    int64_t b = start_bit, n = 0;
    while (b < end_bit) {
        int s = trie_walk(&t, bytes, end_bit, &b);
        if (s < 0) { rc = s; break; }
        if (n >= max_out) { rc = ORC_EINVAL; break; }
        out[n++] = (uint8_t)s;
    }
    free(t.child); free(t.leaf);
    return rc ? rc : n;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1 steps 7-8 / Algorithm 2 steps 7-9: prefix sum of the relative   */
/* indices gives absolute positions; each value index is replaced by its      */
/* codebook entry; the block's entries are arranged as a bh x bw block placed */
/* at (row_id, col_id).  The position of entry j of a block is                */
/* sum_{j' <= j}(z_j' + 1) - 1.  Padding entries (value index 0) only advance */
/* the position.  Wd: M x K row-major fp32, overwritten (zero-filled first).  */
/* ------------------------------------------------------------------------- */
int orc_reconstruct(const uint8_t *val, const uint8_t *idx, const int64_t *block_ptr,
                    const float *codebook, int M, int K, int bh, int bw, int kbits,
                    int colmajor, float *Wd, uint8_t *qd /* optional M*K index matrix */)
{
    if (!block_ptr || !codebook || !Wd || M < 1 || K < 1 || bh < 1 || bw < 1 || kbits < 1 || kbits > 8) return ORC_EINVAL;
    int64_t nblocks = orc_num_blocks(M, K, bh, bw);
    memset(Wd, 0, sizeof(float) * (size_t)M * K);
    if (qd) memset(qd, 0, (size_t)M * K);
    int64_t R = (int64_t)1 << kbits;
    for (int64_t bi = 0; bi < nblocks; ++bi) {
        int row_id, col_id, bhp, bwp;
        block_geom(M, K, bh, bw, bi, &row_id, &col_id, &bhp, &bwp);
        int64_t np = (int64_t)bhp * bwp;
        int64_t pos = -1;
        if (block_ptr[bi + 1] < block_ptr[bi]) return ORC_ECORRUPT;
        for (int64_t e = block_ptr[bi]; e < block_ptr[bi + 1]; ++e) {
            if (idx[e] >= R) return ORC_ECORRUPT;
            pos += (int64_t)idx[e] + 1;
            if (pos >= np) return ORC_ECORRUPT;
            if (val[e] == 0) continue;
            int r = colmajor ? (int)(pos % bhp) : (int)(pos / bwp);
            int c = colmajor ? (int)(pos / bhp) : (int)(pos % bwp);
            int64_t at = (int64_t)(row_id + r) * K + (col_id + c);
            Wd[at] = codebook[val[e]];
            if (qd) qd[at] = val[e];
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Eq. (1)-(2): b_i = sum_j W_ij a_j + v_i, for every image of the batch.     */
/* W: M x K row-major fp32, X: B x K row-major fp32, bias: M or NULL,         */
/* Y: B x M row-major fp64.  Products and sums in fp64, j ascending.          */
/* relu != 0 applies max(0, .) (the activation between stacked layers).       */
/* Rows are independent, so nthreads > 1 only splits the (image, row) loop.   */
/* ------------------------------------------------------------------------- */
int orc_fc_forward(const float *W, const float *X, const float *bias, int M, int K, int B,
                   int relu, int nthreads, double *Y)
{
    if (!W || !X || !Y || M < 1 || K < 1 || B < 0) return ORC_EINVAL;
    if (nthreads < 1) nthreads = 1;
    int64_t total = (int64_t)B * M;
#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (int64_t t = 0; t < total; ++t) {
        int b = (int)(t / M), i = (int)(t % M);
        const float *w = W + (int64_t)i * K;
        const float *x = X + (int64_t)b * K;
        double acc = 0.0;
        for (int j = 0; j < K; ++j) acc += (double)w[j] * (double)x[j];
        if (bias) acc += (double)bias[i];
        if (relu && acc < 0.0) acc = 0.0;
        Y[t] = acc;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Sec. III-A, convolution paragraph: every filter is slid over the width and */
/* height of the input volume and a dot product with the receptive field is   */
/* taken at each location; stacking the maps gives the output volume.  This   */
/* is that definition written out (no im2col).  Filters are the rows of W:    */
/* row oc holds the (C/groups) x R x S filter flattened as ((c*R + r)*S + s). */
/* READING (standard grouped convolution, as in AlexNet): output channel oc   */
/* of group g = oc / (OC/groups) sees input channels g*(C/groups) ... only.   */
/* X: B x C x H x Wd (NCHW) fp32; Y: B x OC x P x Q fp64;                      */
/* P = (H + 2 pad - R) / stride + 1, Q likewise.  Zero padding.               */
/* ------------------------------------------------------------------------- */
int orc_conv_forward(const float *W, const float *X, const float *bias,
                     int B, int C, int H, int Wd, int OC, int R, int S, int stride, int pad, int groups,
                     int relu, int nthreads, double *Y)
{
    if (!W || !X || !Y || B < 0 || C < 1 || H < 1 || Wd < 1 || OC < 1 || R < 1 || S < 1 || stride < 1 || pad < 0 || groups < 1) return ORC_EINVAL;
    if (C % groups || OC % groups) return ORC_EINVAL;
    int P = (H + 2 * pad - R) / stride + 1, Q = (Wd + 2 * pad - S) / stride + 1;
    if (P < 1 || Q < 1) return ORC_EINVAL;
    int Cg = C / groups, OCg = OC / groups;
    int K = Cg * R * S;
    if (nthreads < 1) nthreads = 1;
    int64_t total = (int64_t)B * OC;
#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (int64_t t = 0; t < total; ++t) {
        int b = (int)(t / OC), oc = (int)(t % OC);
        int g = oc / OCg;
        const float *w = W + (int64_t)oc * K;
        for (int p = 0; p < P; ++p)
            for (int qq = 0; qq < Q; ++qq) {
                double acc = 0.0;
                for (int c = 0; c < Cg; ++c)
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < S; ++s) {
                            int h = p * stride - pad + r, x = qq * stride - pad + s;
                            if (h < 0 || h >= H || x < 0 || x >= Wd) continue;
                            acc += (double)w[(c * R + r) * S + s] *
                                   (double)X[(((int64_t)b * C + (g * Cg + c)) * H + h) * Wd + x];
                        }
                if (bias) acc += (double)bias[oc];
                if (relu && acc < 0.0) acc = 0.0;
                Y[(((int64_t)b * OC + oc) * P + p) * Q + qq] = acc;
            }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* The fixed-function layers between the convolutions of the paper's AlexNet  */
/* runs (Table IV lists norm1/2 and pool1/2/5; Sec. II: "the RELU/POOL layers */
/* implement fixed functions").  The paper does not define them; READING: the */
/* layers of the AlexNet it evaluates - max pooling over size x size windows  */
/* with a stride, no padding, windows fully inside the image; and local        */
/* response normalisation across channels,                                     */
/*   y[c] = x[c] / (k + alpha / n * sum_{c' in window(c)} x[c']^2)^beta,       */
/* the window being the n channels centred on c and clipped to [0, C).         */
/* X: B x C x H x W fp32 (NCHW); Y fp64.                                       */
/* ------------------------------------------------------------------------- */
int orc_maxpool_forward(const float *X, int B, int C, int H, int Wd, int size, int stride, double *Y)
{
    if (!X || !Y || B < 0 || C < 1 || H < size || Wd < size || size < 1 || stride < 1) return ORC_EINVAL;
    int P = (H - size) / stride + 1, Q = (Wd - size) / stride + 1;
    for (int64_t bc = 0; bc < (int64_t)B * C; ++bc)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                double m = -INFINITY;
                for (int r = 0; r < size; ++r)
                    for (int s = 0; s < size; ++s) {
                        double v = (double)X[(bc * H + (p * stride + r)) * Wd + (q * stride + s)];
                        if (v > m) m = v;
                    }
                Y[(bc * P + p) * Q + q] = m;
            }
    return ORC_OK;
}

int orc_lrn_forward(const float *X, int B, int C, int H, int Wd, int n, double alpha, double beta, double k, double *Y)
{
    if (!X || !Y || B < 0 || C < 1 || H < 1 || Wd < 1 || n < 1 || !(n & 1)) return ORC_EINVAL;
    int64_t hw = (int64_t)H * Wd;
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < C; ++c)
            for (int64_t i = 0; i < hw; ++i) {
                double ss = 0.0;
                for (int d = -(n / 2); d <= n / 2; ++d) {
                    int cc = c + d;
                    if (cc < 0 || cc >= C) continue;
                    double v = (double)X[((int64_t)b * C + cc) * hw + i];
                    ss += v * v;
                }
                Y[((int64_t)b * C + c) * hw + i] = (double)X[((int64_t)b * C + c) * hw + i] / pow(k + alpha / n * ss, beta);
            }
    return ORC_OK;
}
