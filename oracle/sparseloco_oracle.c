/*
 * SparseLoCo compress + aggregate path: plain CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of what the hot path computes.  It is used by the tests, by the smoke check
 * and by the benchmark's reported CPU baseline; the product (the HIP library)
 * never calls it and shares no code, header, table or helper with it.
 *
 * Every function cites the passage of the SparseLoCo paper (arXiv 2508.15706)
 * it follows.  Where the paper is silent the reading taken is stated next to
 * the code.  Floating point: the path itself is fp32 (the error buffer, the
 * pseudo-gradient and the parameters are fp32 tensors); all quantizer
 * statistics are fp64 with a fixed summation tree so that the bytes of a
 * payload are a function of the inputs alone.
 *
 * Parity pins (tests marked "not gpu"): brute-force Top-k on tiny chunks,
 * exactly-rounded rational arithmetic for the accumulate, hand-computed tree
 * sums, the closed form of the quantizer on +-c inputs, exact rational
 * quantizer statistics on dyadic inputs, a big-integer bit-stream model of the
 * wire format, a dense numpy model of the aggregation, and the invariants of
 * Eq. (2).  No function here is "parity unpinned"; what is pinned for the
 * quantizer is the reading of Section 4's description stated below, since the
 * paper prints no worked example of it.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC
 *        (no -ffast-math, no -march: fmaf must stay a single correctly
 *        rounded operation and nothing else may be contracted).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define SLO_OK 0
#define SLO_ERR_ARG (-1)
#define SLO_ERR_PAYLOAD (-2)
#define SLO_ERR_NOMEM (-3)

#define SLO_LAYOUT_FLAT 0 /* contiguous runs of tile*tile elements (1-D rule)   */
#define SLO_LAYOUT_TILE 1 /* tile x tile blocks of a row-major matrix (2-D rule) */

/* One tensor of the list.  All tensors live in flat fp32 arenas (e, delta,
 * theta) at element offset `offset`, row-major rows x cols.  A 1-D tensor is
 * rows = 1. */
typedef struct {
    int64_t rows, cols, offset;
    int32_t layout;
    int32_t reserved;
} slo_tensor;

/* ------------------------------------------------------------------------- */
/* Chunk geometry (Section 3.3, last paragraph; Section 4 "chunk size 4096,   */
/* non-overlapping square 64x64 grids for 2D parameters").                    */
/*                                                                           */
/* 2-D rule: the matrix is cut into tile x tile blocks, blocks numbered       */
/* row-major over the block grid; inside a block the local index is           */
/* j = tile*lr + lc.  1-D rule: runs of C = tile*tile consecutive elements,   */
/* j = position in the run.  Reading for shapes that are not multiples of     */
/* the tile: edge chunks are partial, only in-range positions are candidates, */
/* j keeps the full-tile stride, k is not scaled down.                        */
/* ------------------------------------------------------------------------- */

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

int64_t slo_tensor_chunks(const slo_tensor *t, int tile)
{
    int64_t C = (int64_t)tile * tile;
    if (t->layout == SLO_LAYOUT_TILE)
        return ceil_div(t->rows, tile) * ceil_div(t->cols, tile);
    return ceil_div(t->rows * t->cols, C);
}

int64_t slo_num_chunks(const slo_tensor *t, int nt, int tile)
{
    int64_t n = 0;
    for (int i = 0; i < nt; ++i) n += slo_tensor_chunks(&t[i], tile);
    return n;
}

/* Arena element index of local position j of chunk c of tensor t, or -1 when
 * that position lies outside the tensor. */
int64_t slo_element_of(const slo_tensor *t, int tile, int64_t c, int j)
{
    if (t->layout == SLO_LAYOUT_TILE) {
        int64_t tiles_c = ceil_div(t->cols, tile);
        int64_t tr = c / tiles_c, tc = c % tiles_c;
        int64_t row = tr * tile + j / tile;
        int64_t col = tc * tile + j % tile;
        if (row >= t->rows || col >= t->cols) return -1;
        return t->offset + row * t->cols + col;
    } else {
        int64_t C = (int64_t)tile * tile;
        int64_t pos = c * C + j;
        if (pos >= t->rows * t->cols) return -1;
        return t->offset + pos;
    }
}

/* ------------------------------------------------------------------------- */
/* Wire format.  Appendix "Compression of indices in Top-k" fixes only the    */
/* bit counts: an index inside a chunk of 4096 needs 12 bits, a quantized     */
/* value 2 bits.  Reading for the byte layout:                                */
/*   per tensor, at a 16-byte aligned offset: float LUT[4] (little endian),   */
/*   then one record per chunk in chunk order; a record is the k indices in   */
/*   ascending order as a little-endian stream of 12-bit fields, followed by  */
/*   the k codes, four per byte, entry m in bits 2*(m mod 4).                 */
/* Record size 7k/4 bytes (k a multiple of 4), tensor block padded to 16.     */
/* ------------------------------------------------------------------------- */

int64_t slo_record_bytes(int k) { return (int64_t)7 * k / 4; }

int64_t slo_tensor_block_bytes(const slo_tensor *t, int tile, int k)
{
    int64_t b = 16 + slo_tensor_chunks(t, tile) * slo_record_bytes(k);
    return (b + 15) / 16 * 16;
}

int64_t slo_payload_bytes(const slo_tensor *t, int nt, int tile, int k)
{
    int64_t n = 0;
    for (int i = 0; i < nt; ++i) n += slo_tensor_block_bytes(&t[i], tile, k);
    return n;
}

/* Encode one record: idx[0..k) ascending 12-bit values, code[0..k) in 0..3. */
void slo_pack_record(const uint16_t *idx, const uint8_t *code, int k, uint8_t *out)
{
    int nidx = 3 * k / 2;
    memset(out, 0, (size_t)slo_record_bytes(k));
    for (int m = 0; m < k; ++m) {
        int bit = 12 * m; /* first bit of field m in the stream */
        unsigned v = idx[m] & 0xFFFu;
        for (int b = 0; b < 12; ++b)
            if (v >> b & 1u) out[(bit + b) / 8] |= (uint8_t)(1u << ((bit + b) % 8));
    }
    for (int m = 0; m < k; ++m)
        out[nidx + m / 4] |= (uint8_t)((code[m] & 3u) << (2 * (m % 4)));
}

void slo_unpack_record(const uint8_t *in, int k, uint16_t *idx, uint8_t *code)
{
    int nidx = 3 * k / 2;
    for (int m = 0; m < k; ++m) {
        int bit = 12 * m;
        unsigned v = 0;
        for (int b = 0; b < 12; ++b)
            v |= (unsigned)(in[(bit + b) / 8] >> ((bit + b) % 8) & 1u) << b;
        idx[m] = (uint16_t)v;
    }
    for (int m = 0; m < k; ++m) code[m] = (uint8_t)(in[nidx + m / 4] >> (2 * (m % 4)) & 3u);
}

/* The record encoder alone over n_chunks records (what sl_pack_indices does). */
int slo_pack_indices(const uint16_t *idx, const uint8_t *code, int64_t n_chunks, int k,
                     uint8_t *out)
{
    if (k < 4 || k % 4 || k > 4096 || n_chunks < 0) return SLO_ERR_ARG;
    for (int64_t c = 0; c < n_chunks; ++c)
        slo_pack_record(idx + c * k, code + c * k, k, out + c * slo_record_bytes(k));
    return SLO_OK;
}

/* ------------------------------------------------------------------------- */
/* Fixed-shape fp64 summation.  The paper does not say in which order the     */
/* quantizer's sums are taken; since a payload has to be reproducible bit for */
/* bit, the reading is: pad the sequence on the right with +0.0 to the next   */
/* power of two, then replace it by the sums of adjacent pairs until one      */
/* value is left.                                                             */
/* ------------------------------------------------------------------------- */

double slo_tree_sum(const double *s, int64_t n)
{
    int64_t P = 1;
    while (P < n) P *= 2;
    double *w = (double *)malloc((size_t)P * sizeof(double));
    if (!w) return NAN;
    for (int64_t i = 0; i < P; ++i) w[i] = i < n ? s[i] : 0.0;
    for (int64_t m = P; m > 1; m /= 2)
        for (int64_t i = 0; i < m / 2; ++i) w[i] = w[2 * i] + w[2 * i + 1];
    double r = w[0];
    free(w);
    return r;
}

/* Sum over a tensor's selected entries of a per-entry quantity y, laid out
 * y[c*k + m]: first the tree sum of each chunk's k entries, then the tree sum
 * of those per-chunk leaves in chunk order. */
static double two_level_sum(const double *y, int64_t n_chunks, int k)
{
    double *leaf = (double *)malloc((size_t)(n_chunks > 0 ? n_chunks : 1) * sizeof(double));
    for (int64_t c = 0; c < n_chunks; ++c) leaf[c] = slo_tree_sum(y + c * k, k);
    double r = slo_tree_sum(leaf, n_chunks);
    free(leaf);
    return r;
}

/* ------------------------------------------------------------------------- */
/* Step 1: error-feedback accumulate, first line of Eq. (2) / the argument of */
/* Top-k in Algorithm 1:  a = beta * e + delta.  Reading for the rounding:    */
/* one fused multiply-add in fp32 (a single rounding).                        */
/* ------------------------------------------------------------------------- */

void slo_accumulate(float *e, const float *delta, float beta, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) e[i] = fmaf(beta, e[i], delta[i]);
}

/* ------------------------------------------------------------------------- */
/* Step 2: chunk-wise Top-k by magnitude (Section 3.3 last paragraph;         */
/* "Top-k largest magnitude entries", Section 4.2).  Plain definition: sort   */
/* the chunk's valid positions by |a| descending and keep the first k.        */
/* |a| is compared through its bit pattern with the sign cleared, which is    */
/* the same order as the real magnitude for finite values.  Ties (paper       */
/* silent): the lower local index wins.  Output is in ascending local index.  */
/* ------------------------------------------------------------------------- */

typedef struct {
    uint32_t key;
    int32_t j;
} slo_cand;

static int cmp_mag_desc_then_index(const void *pa, const void *pb)
{
    const slo_cand *a = (const slo_cand *)pa, *b = (const slo_cand *)pb;
    if (a->key != b->key) return a->key > b->key ? -1 : 1;
    return a->j < b->j ? -1 : (a->j > b->j ? 1 : 0);
}

static int cmp_index_asc(const void *pa, const void *pb)
{
    const slo_cand *a = (const slo_cand *)pa, *b = (const slo_cand *)pb;
    return a->j < b->j ? -1 : (a->j > b->j ? 1 : 0);
}

static uint32_t f32_bits(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    return u;
}

/* Select within one chunk of tensor t.  a = arena holding the accumulated
 * values.  Returns the number of valid positions in the chunk, or -1 when it
 * has fewer than k. */
int slo_topk_chunk(const slo_tensor *t, int tile, int64_t c, const float *a, int k,
                   uint16_t *sel_idx, float *sel_val)
{
    int C = tile * tile, n = 0;
    slo_cand *cand = (slo_cand *)malloc((size_t)C * sizeof(slo_cand));
    for (int j = 0; j < C; ++j) {
        int64_t i = slo_element_of(t, tile, c, j);
        if (i < 0) continue;
        cand[n].key = f32_bits(a[i]) & 0x7FFFFFFFu;
        cand[n].j = j;
        ++n;
    }
    if (n < k) {
        free(cand);
        return -1;
    }
    qsort(cand, (size_t)n, sizeof(slo_cand), cmp_mag_desc_then_index);
    qsort(cand, (size_t)k, sizeof(slo_cand), cmp_index_asc);
    for (int m = 0; m < k; ++m) {
        sel_idx[m] = (uint16_t)cand[m].j;
        sel_val[m] = a[slo_element_of(t, tile, c, cand[m].j)];
    }
    free(cand);
    return n;
}

/* ------------------------------------------------------------------------- */
/* Step 3: 2-bit statistical quantizer (Section 4, experimental set-up: all   */
/* selected values of one tensor are quantized together; they are centred by  */
/* their mean, [-6 sigma, 6 sigma] is cut into uniform bins - four for 2 bits */
/* - and each bin keeps the centroid of the values assigned to it as a        */
/* look-up table).  Readings where the paper gives no formula:                */
/*   - statistics in fp64 over x in canonical order (chunk, then index) with  */
/*     the two-level tree above; S1 = sum x, S2 = sum x*x;                    */
/*   - mu = S1/M; var = S2/M - mu*mu (population), clamped at 0;              */
/*   - bin width 3 sigma, edges -3 sigma, 0, +3 sigma on d = x - mu, bins     */
/*     half-open [lo, hi), values beyond +-6 sigma fall in the end bins;      */
/*     decided on squares so that no square root is involved:                 */
/*        T = 9*var, dd = d*d,                                                */
/*        code = d < 0 ? (dd > T ? 0 : 1) : (dd >= T ? 3 : 2);                */
/*   - LUT[b] = centroid of the raw values with code b, fp64 sum / count,     */
/*     rounded to fp32; an empty bin, or a centroid equal to zero, is +0.0f.  */
/* Dequantisation is then the single look-up LUT[code].                       */
/* stats (optional, 8 doubles out): S1, S2, mu, var, n0..n3.                  */
/* ------------------------------------------------------------------------- */

int slo_quantize_tensor(const float *x, int64_t n_chunks, int k, uint8_t *code, float lut[4],
                        double *stats)
{
    int64_t M = n_chunks * k;
    for (int b = 0; b < 4; ++b) lut[b] = 0.0f;
    if (M == 0) return SLO_OK;
    double *y = (double *)calloc((size_t)M, sizeof(double));
    if (!y) return SLO_ERR_NOMEM;

    for (int64_t i = 0; i < M; ++i) y[i] = (double)x[i];
    double S1 = two_level_sum(y, n_chunks, k);
    for (int64_t i = 0; i < M; ++i) y[i] = (double)x[i] * (double)x[i];
    double S2 = two_level_sum(y, n_chunks, k);

    double mu = S1 / (double)M;
    double q = S2 / (double)M;
    double p = mu * mu;
    double var = q - p;
    if (var < 0.0) var = 0.0;
    double T = 9.0 * var;

    int64_t cnt[4] = {0, 0, 0, 0};
    for (int64_t i = 0; i < M; ++i) {
        double d = (double)x[i] - mu;
        double dd = d * d;
        int cde = d < 0.0 ? (dd > T ? 0 : 1) : (dd >= T ? 3 : 2);
        code[i] = (uint8_t)cde;
        cnt[cde]++;
    }
    for (int b = 0; b < 4; ++b) {
        for (int64_t i = 0; i < M; ++i) y[i] = code[i] == b ? (double)x[i] : 0.0;
        double Sb = two_level_sum(y, n_chunks, k);
        float cen = cnt[b] ? (float)(Sb / (double)cnt[b]) : 0.0f;
        if (cen == 0.0f) cen = 0.0f; /* -0.0f -> +0.0f */
        lut[b] = cen;
    }
    if (stats) {
        stats[0] = S1, stats[1] = S2, stats[2] = mu, stats[3] = var;
        for (int b = 0; b < 4; ++b) stats[4 + b] = (double)cnt[b];
    }
    free(y);
    return SLO_OK;
}

/* ------------------------------------------------------------------------- */
/* The compression half of Algorithm 1 ("Compression + Error Feedback"; first */
/* two lines of Eq. (2)) over a tensor list:                                  */
/*     a      = beta*e + delta                                                */
/*     payload= Q(Top-k(a))                                                   */
/*     e      = a - dequantised payload   (a itself where nothing was sent)   */
/* e is updated in place.  Optional outputs (may be NULL), all laid out in    */
/* list chunk order: sel_idx/sel_val/sel_code [n_chunks*k], lut [nt*4].       */
/* ef_frozen != 0 is the error-feedback freeze of Appendix "Freezing Error    */
/* Feedback": the buffer is neither used nor accumulated, i.e. a = delta and  */
/* e is left untouched.                                                       */
/* ------------------------------------------------------------------------- */

int slo_compress(const slo_tensor *t, int nt, int tile, int k, float *e, const float *delta,
                 float beta, int ef_frozen, uint8_t *payload, uint16_t *sel_idx, float *sel_val,
                 uint8_t *sel_code, float *lut_out)
{
    if (nt < 0 || tile < 1 || tile > 64 || k < 4 || k % 4 || k > tile * tile) return SLO_ERR_ARG;
    int64_t rec = slo_record_bytes(k);
    int64_t chunk0 = 0, pay_off = 0;
    int status = SLO_OK;

    for (int ti = 0; ti < nt; ++ti) {
        const slo_tensor *T = &t[ti];
        int64_t n = T->rows * T->cols;
        int64_t nc = slo_tensor_chunks(T, tile);
        int64_t M = nc * k;

        /* a = beta*e + delta; while frozen a = delta and e is not touched.
         * `a` points at the tensor's first element; L is the same tensor
         * addressed from there. */
        slo_tensor L = *T;
        L.offset = 0;
        const float *a;
        if (ef_frozen) {
            a = delta + T->offset;
        } else {
            slo_accumulate(e + T->offset, delta + T->offset, beta, n);
            a = e + T->offset;
        }

        uint16_t *idx = (uint16_t *)malloc((size_t)(M > 0 ? M : 1) * sizeof(uint16_t));
        float *val = (float *)malloc((size_t)(M > 0 ? M : 1) * sizeof(float));
        uint8_t *code = (uint8_t *)malloc((size_t)(M > 0 ? M : 1));
        int bad = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(| : bad)
        for (int64_t c = 0; c < nc; ++c)
            if (slo_topk_chunk(&L, tile, c, a, k, idx + c * k, val + c * k) < 0) bad |= 1;
        if (bad) status = SLO_ERR_ARG;

        float lut[4];
        if (!bad) {
            slo_quantize_tensor(val, nc, k, code, lut, NULL);

            /* residual: last part of Eq. (2) line 2 / Algorithm 1 error update */
            if (!ef_frozen)
                for (int64_t c = 0; c < nc; ++c)
                    for (int m = 0; m < k; ++m) {
                        int64_t i = slo_element_of(&L, tile, c, idx[c * k + m]);
                        e[T->offset + i] = a[i] - lut[code[c * k + m]];
                    }

            if (payload) {
                uint8_t *blk = payload + pay_off;
                memset(blk, 0, (size_t)slo_tensor_block_bytes(T, tile, k));
                memcpy(blk, lut, 16);
                for (int64_t c = 0; c < nc; ++c)
                    slo_pack_record(idx + c * k, code + c * k, k, blk + 16 + c * rec);
            }
            if (sel_idx) memcpy(sel_idx + chunk0 * k, idx, (size_t)M * sizeof(uint16_t));
            if (sel_val) memcpy(sel_val + chunk0 * k, val, (size_t)M * sizeof(float));
            if (sel_code) memcpy(sel_code + chunk0 * k, code, (size_t)M);
            if (lut_out) memcpy(lut_out + 4 * ti, lut, 16);
        }
        free(idx), free(val), free(code);
        if (bad) return status;
        chunk0 += nc;
        pay_off += slo_tensor_block_bytes(T, tile, k);
    }
    return status;
}

/* ------------------------------------------------------------------------- */
/* The aggregation half of Algorithm 1 ("Aggregate + Outer Update"; last two  */
/* lines of Eq. (2)): dequantise every worker's payload, average over the R   */
/* workers (a coordinate a worker did not send counts as zero), and take the  */
/* outer SGD step theta <- theta - lr * average.  Order (paper silent): per   */
/* chunk a zero fp32 accumulator, workers added in order r = 0..R-1, then     */
/* theta = fma(-lr, acc * (1/R), theta) with 1/R rounded once to fp32.        */
/* ------------------------------------------------------------------------- */

int slo_decompress_avg_apply(const slo_tensor *t, int nt, int tile, int k, float *theta,
                             const uint8_t *const *payloads, int R, float lr)
{
    if (nt < 0 || tile < 1 || tile > 64 || k < 4 || k % 4 || k > tile * tile || R < 1)
        return SLO_ERR_ARG;
    int C = tile * tile;
    int64_t rec = slo_record_bytes(k);
    float invR = 1.0f / (float)R;
    int64_t pay_off = 0;
    int bad = 0;

    for (int ti = 0; ti < nt; ++ti) {
        const slo_tensor *T = &t[ti];
        int64_t nc = slo_tensor_chunks(T, tile);
#pragma omp parallel for schedule(dynamic, 16) reduction(| : bad)
        for (int64_t c = 0; c < nc; ++c) {
            float *acc = (float *)calloc((size_t)C, sizeof(float));
            uint16_t *idx = (uint16_t *)malloc((size_t)k * sizeof(uint16_t));
            uint8_t *code = (uint8_t *)malloc((size_t)k);
            for (int r = 0; r < R; ++r) {
                const uint8_t *blk = payloads[r] + pay_off;
                float lut[4];
                memcpy(lut, blk, 16);
                slo_unpack_record(blk + 16 + c * rec, k, idx, code);
                for (int m = 0; m < k; ++m) {
                    if (idx[m] >= C) {
                        bad |= 1;
                        continue;
                    }
                    acc[idx[m]] = acc[idx[m]] + lut[code[m]];
                }
            }
            for (int j = 0; j < C; ++j) {
                int64_t i = slo_element_of(T, tile, c, j);
                if (i < 0) continue;
                theta[i] = fmaf(-lr, acc[j] * invR, theta[i]);
            }
            free(acc), free(idx), free(code);
        }
        pay_off += slo_tensor_block_bytes(T, tile, k);
    }
    return bad ? SLO_ERR_PAYLOAD : SLO_OK;
}

/* Dense view of one worker's payload: out[i] = dequantised value at every
 * transmitted coordinate, untouched elsewhere (callers pass zeros).  A helper
 * for tests of the identities of Eq. (2); not a step of the path. */
int slo_decompress_dense(const slo_tensor *t, int nt, int tile, int k, const uint8_t *payload,
                         float *out)
{
    int64_t rec = slo_record_bytes(k), pay_off = 0;
    uint16_t *idx = (uint16_t *)malloc((size_t)k * sizeof(uint16_t));
    uint8_t *code = (uint8_t *)malloc((size_t)k);
    for (int ti = 0; ti < nt; ++ti) {
        const slo_tensor *T = &t[ti];
        int64_t nc = slo_tensor_chunks(T, tile);
        float lut[4];
        memcpy(lut, payload + pay_off, 16);
        for (int64_t c = 0; c < nc; ++c) {
            slo_unpack_record(payload + pay_off + 16 + c * rec, k, idx, code);
            for (int m = 0; m < k; ++m) {
                int64_t i = slo_element_of(T, tile, c, idx[m]);
                if (i < 0) {
                    free(idx), free(code);
                    return SLO_ERR_PAYLOAD;
                }
                out[i] = lut[code[m]];
            }
        }
        pay_off += slo_tensor_block_bytes(T, tile, k);
    }
    free(idx), free(code);
    return SLO_OK;
}

/* ------------------------------------------------------------------------- */
/* Other value widths (ablation "Effect of quantization on loss": 1-, 2-, 3-,  */
/* 4-bit and full-precision values; the quantizer of Section 4 cuts            */
/* [-6 sigma, 6 sigma] into uniform bins, 2^b of them for b bits).  The *_b     */
/* functions repeat the path above with the number of value bits as a          */
/* parameter: bits in {1, 2, 3, 4}, or 32 for unquantized fp32 values.  With    */
/* bits = 2 they produce the same bytes as the functions above.  Readings:     */
/*   - bin q of 2^b is [mu + sigma*c_q, mu + sigma*c_(q+1)) with               */
/*     c_j = 12 j / 2^b - 6, the end bins open-ended; a value's code is the    */
/*     number of inner edges j = 1 .. 2^b - 1 it has reached, each edge        */
/*     decided on squares against T_j = (c_j*c_j) * var;                       */
/*   - wire format: per tensor a header of 2^b floats padded to 16 bytes (none */
/*     for 32 bits), then per chunk the k 12-bit indices followed by the k     */
/*     codes as a little-endian stream of b-bit fields, or by the k fp32       */
/*     values; k must be a multiple of 8 unless bits = 2;                      */
/*   - 32 bits: nothing is quantized, the residual at a sent position is       */
/*     a - a.                                                                  */
/* ------------------------------------------------------------------------- */

static int bits_ok(int k, int bits, int tile)
{
    if (!(bits == 1 || bits == 2 || bits == 3 || bits == 4 || bits == 32)) return 0;
    if (k < 4 || k % 4 || k > tile * tile) return 0;
    if (bits != 2 && k % 8) return 0;
    return 1;
}

int64_t slo_header_bytes_b(int bits)
{
    if (bits == 32) return 0;
    int64_t h = (int64_t)4 << bits;
    return h < 16 ? 16 : h;
}

int64_t slo_record_bytes_b(int k, int bits)
{
    return (int64_t)3 * k / 2 + (bits == 32 ? (int64_t)4 * k : (int64_t)k * bits / 8);
}

int64_t slo_tensor_block_bytes_b(const slo_tensor *t, int tile, int k, int bits)
{
    int64_t b = slo_header_bytes_b(bits) + slo_tensor_chunks(t, tile) * slo_record_bytes_b(k, bits);
    return (b + 15) / 16 * 16;
}

int64_t slo_payload_bytes_b(const slo_tensor *t, int nt, int tile, int k, int bits)
{
    int64_t n = 0;
    for (int i = 0; i < nt; ++i) n += slo_tensor_block_bytes_b(&t[i], tile, k, bits);
    return n;
}

/* code is used for bits <= 4, val for bits = 32 (the other may be NULL). */
void slo_pack_record_b(const uint16_t *idx, const uint8_t *code, const float *val, int k, int bits,
                       uint8_t *out)
{
    int nidx = 3 * k / 2;
    memset(out, 0, (size_t)slo_record_bytes_b(k, bits));
    for (int m = 0; m < k; ++m) {
        int bit = 12 * m;
        unsigned v = idx[m] & 0xFFFu;
        for (int b = 0; b < 12; ++b)
            if (v >> b & 1u) out[(bit + b) / 8] |= (uint8_t)(1u << ((bit + b) % 8));
    }
    if (bits == 32) {
        memcpy(out + nidx, val, (size_t)4 * k);
        return;
    }
    for (int m = 0; m < k; ++m) {
        int bit = bits * m;
        for (int b = 0; b < bits; ++b)
            if (code[m] >> b & 1u) out[nidx + (bit + b) / 8] |= (uint8_t)(1u << ((bit + b) % 8));
    }
}

void slo_unpack_record_b(const uint8_t *in, int k, int bits, uint16_t *idx, uint8_t *code, float *val)
{
    int nidx = 3 * k / 2;
    for (int m = 0; m < k; ++m) {
        int bit = 12 * m;
        unsigned v = 0;
        for (int b = 0; b < 12; ++b)
            v |= (unsigned)(in[(bit + b) / 8] >> ((bit + b) % 8) & 1u) << b;
        idx[m] = (uint16_t)v;
    }
    if (bits == 32) {
        memcpy(val, in + nidx, (size_t)4 * k);
        return;
    }
    for (int m = 0; m < k; ++m) {
        int bit = bits * m;
        unsigned v = 0;
        for (int b = 0; b < bits; ++b)
            v |= (unsigned)(in[nidx + (bit + b) / 8] >> ((bit + b) % 8) & 1u) << b;
        code[m] = (uint8_t)v;
    }
}

/* lut has 2^bits entries; stats (optional): S1, S2, mu, var, then 2^bits counts. */
int slo_quantize_tensor_b(const float *x, int64_t n_chunks, int k, int bits, uint8_t *code,
                          float *lut, double *stats)
{
    if (bits < 1 || bits > 4) return SLO_ERR_ARG;
    int nb = 1 << bits;
    int64_t M = n_chunks * k;
    for (int b = 0; b < nb; ++b) lut[b] = 0.0f;
    if (M == 0) return SLO_OK;
    double *y = (double *)calloc((size_t)M, sizeof(double));
    if (!y) return SLO_ERR_NOMEM;

    for (int64_t i = 0; i < M; ++i) y[i] = (double)x[i];
    double S1 = two_level_sum(y, n_chunks, k);
    for (int64_t i = 0; i < M; ++i) y[i] = (double)x[i] * (double)x[i];
    double S2 = two_level_sum(y, n_chunks, k);

    double mu = S1 / (double)M;
    double q = S2 / (double)M;
    double p = mu * mu;
    double var = q - p;
    if (var < 0.0) var = 0.0;

    int64_t cnt[16] = {0};
    for (int64_t i = 0; i < M; ++i) {
        double d = (double)x[i] - mu;
        double dd = d * d;
        int reached = 0;
        for (int j = 1; j < nb; ++j) {
            double cj = 12.0 * (double)j / (double)nb - 6.0; /* edge in units of sigma, exact */
            double Tj = (cj * cj) * var;
            int at_or_above;
            if (cj < 0.0)
                at_or_above = d >= 0.0 || dd <= Tj;
            else if (cj == 0.0)
                at_or_above = d >= 0.0;
            else
                at_or_above = d >= 0.0 && dd >= Tj;
            reached += at_or_above;
        }
        code[i] = (uint8_t)reached;
        cnt[reached]++;
    }
    for (int b = 0; b < nb; ++b) {
        for (int64_t i = 0; i < M; ++i) y[i] = code[i] == b ? (double)x[i] : 0.0;
        double Sb = two_level_sum(y, n_chunks, k);
        float cen = cnt[b] ? (float)(Sb / (double)cnt[b]) : 0.0f;
        if (cen == 0.0f) cen = 0.0f;
        lut[b] = cen;
    }
    if (stats) {
        stats[0] = S1, stats[1] = S2, stats[2] = mu, stats[3] = var;
        for (int b = 0; b < nb; ++b) stats[4 + b] = (double)cnt[b];
    }
    free(y);
    return SLO_OK;
}

/* slo_compress with a value width.  Optional outputs as there; lut_out holds
 * 2^bits floats per tensor (unused for bits = 32, where sel_code is unused too
 * and the sent values are sel_val). */
int slo_compress_b(const slo_tensor *t, int nt, int tile, int k, int bits, float *e,
                   const float *delta, float beta, int ef_frozen, uint8_t *payload,
                   uint16_t *sel_idx, float *sel_val, uint8_t *sel_code, float *lut_out)
{
    if (nt < 0 || tile < 1 || tile > 64 || !bits_ok(k, bits, tile)) return SLO_ERR_ARG;
    int nb = bits == 32 ? 0 : 1 << bits;
    int64_t rec = slo_record_bytes_b(k, bits), hdr = slo_header_bytes_b(bits);
    int64_t chunk0 = 0, pay_off = 0;

    for (int ti = 0; ti < nt; ++ti) {
        const slo_tensor *T = &t[ti];
        int64_t n = T->rows * T->cols;
        int64_t nc = slo_tensor_chunks(T, tile);
        int64_t M = nc * k;
        slo_tensor L = *T;
        L.offset = 0;
        const float *a;
        if (ef_frozen) {
            a = delta + T->offset;
        } else {
            slo_accumulate(e + T->offset, delta + T->offset, beta, n);
            a = e + T->offset;
        }

        uint16_t *idx = (uint16_t *)malloc((size_t)(M > 0 ? M : 1) * sizeof(uint16_t));
        float *val = (float *)malloc((size_t)(M > 0 ? M : 1) * sizeof(float));
        uint8_t *code = (uint8_t *)calloc((size_t)(M > 0 ? M : 1), 1);
        int bad = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(| : bad)
        for (int64_t c = 0; c < nc; ++c)
            if (slo_topk_chunk(&L, tile, c, a, k, idx + c * k, val + c * k) < 0) bad |= 1;
        if (bad) {
            free(idx), free(val), free(code);
            return SLO_ERR_ARG;
        }

        float lut[16] = {0};
        if (bits != 32) slo_quantize_tensor_b(val, nc, k, bits, code, lut, NULL);

        if (!ef_frozen)
            for (int64_t c = 0; c < nc; ++c)
                for (int m = 0; m < k; ++m) {
                    int64_t i = slo_element_of(&L, tile, c, idx[c * k + m]);
                    float sent = bits == 32 ? val[c * k + m] : lut[code[c * k + m]];
                    e[T->offset + i] = a[i] - sent;
                }

        if (payload) {
            uint8_t *blk = payload + pay_off;
            memset(blk, 0, (size_t)slo_tensor_block_bytes_b(T, tile, k, bits));
            memcpy(blk, lut, (size_t)4 * nb);
            for (int64_t c = 0; c < nc; ++c)
                slo_pack_record_b(idx + c * k, code + c * k, val + c * k, k, bits, blk + hdr + c * rec);
        }
        if (sel_idx) memcpy(sel_idx + chunk0 * k, idx, (size_t)M * sizeof(uint16_t));
        if (sel_val) memcpy(sel_val + chunk0 * k, val, (size_t)M * sizeof(float));
        if (sel_code) memcpy(sel_code + chunk0 * k, code, (size_t)M);
        if (lut_out && nb) memcpy(lut_out + (size_t)nb * ti, lut, (size_t)4 * nb);
        free(idx), free(val), free(code);
        chunk0 += nc;
        pay_off += slo_tensor_block_bytes_b(T, tile, k, bits);
    }
    return SLO_OK;
}

/* slo_decompress_avg_apply with a value width (same order of operations). */
int slo_decompress_avg_apply_b(const slo_tensor *t, int nt, int tile, int k, int bits, float *theta,
                               const uint8_t *const *payloads, int R, float lr)
{
    if (nt < 0 || tile < 1 || tile > 64 || !bits_ok(k, bits, tile) || R < 1) return SLO_ERR_ARG;
    int C = tile * tile;
    int nb = bits == 32 ? 0 : 1 << bits;
    int64_t rec = slo_record_bytes_b(k, bits), hdr = slo_header_bytes_b(bits);
    float invR = 1.0f / (float)R;
    int64_t pay_off = 0;
    int bad = 0;

    for (int ti = 0; ti < nt; ++ti) {
        const slo_tensor *T = &t[ti];
        int64_t nc = slo_tensor_chunks(T, tile);
#pragma omp parallel for schedule(dynamic, 16) reduction(| : bad)
        for (int64_t c = 0; c < nc; ++c) {
            float *acc = (float *)calloc((size_t)C, sizeof(float));
            uint16_t *idx = (uint16_t *)malloc((size_t)k * sizeof(uint16_t));
            uint8_t *code = (uint8_t *)calloc((size_t)k, 1);
            float *val = (float *)calloc((size_t)k, sizeof(float));
            for (int r = 0; r < R; ++r) {
                const uint8_t *blk = payloads[r] + pay_off;
                float lut[16] = {0};
                memcpy(lut, blk, (size_t)4 * nb);
                slo_unpack_record_b(blk + hdr + c * rec, k, bits, idx, code, val);
                for (int m = 0; m < k; ++m) {
                    if (idx[m] >= C) {
                        bad |= 1;
                        continue;
                    }
                    float sent = bits == 32 ? val[m] : lut[code[m]];
                    acc[idx[m]] = acc[idx[m]] + sent;
                }
            }
            for (int j = 0; j < C; ++j) {
                int64_t i = slo_element_of(T, tile, c, j);
                if (i < 0) continue;
                theta[i] = fmaf(-lr, acc[j] * invR, theta[i]);
            }
            free(acc), free(idx), free(code), free(val);
        }
        pay_off += slo_tensor_block_bytes_b(T, tile, k, bits);
    }
    return bad ? SLO_ERR_PAYLOAD : SLO_OK;
}

int slo_decompress_dense_b(const slo_tensor *t, int nt, int tile, int k, int bits,
                           const uint8_t *payload, float *out)
{
    if (!bits_ok(k, bits, tile)) return SLO_ERR_ARG;
    int nb = bits == 32 ? 0 : 1 << bits;
    int64_t rec = slo_record_bytes_b(k, bits), hdr = slo_header_bytes_b(bits), pay_off = 0;
    uint16_t *idx = (uint16_t *)malloc((size_t)k * sizeof(uint16_t));
    uint8_t *code = (uint8_t *)calloc((size_t)k, 1);
    float *val = (float *)calloc((size_t)k, sizeof(float));
    int status = SLO_OK;
    for (int ti = 0; ti < nt && status == SLO_OK; ++ti) {
        const slo_tensor *T = &t[ti];
        int64_t nc = slo_tensor_chunks(T, tile);
        float lut[16] = {0};
        memcpy(lut, payload + pay_off, (size_t)4 * nb);
        for (int64_t c = 0; c < nc && status == SLO_OK; ++c) {
            slo_unpack_record_b(payload + pay_off + hdr + c * rec, k, bits, idx, code, val);
            for (int m = 0; m < k; ++m) {
                int64_t i = slo_element_of(T, tile, c, idx[m]);
                if (i < 0) {
                    status = SLO_ERR_PAYLOAD;
                    break;
                }
                out[i] = bits == 32 ? val[m] : lut[code[m]];
            }
        }
        pay_off += slo_tensor_block_bytes_b(T, tile, k, bits);
    }
    free(idx), free(code), free(val);
    return status;
}

/* ------------------------------------------------------------------------- */
/* Random-k (ablation "SparseLoCo with Random-k vs. Top-k sparsification":    */
/* the same pipeline with k randomly chosen positions per chunk instead of    */
/* the k largest, "for the same number of indices selected").  Reading: every */
/* valid position of a chunk gets a pseudo-random 31-bit key from a           */
/* counter-based generator -                                                  */
/*     key = fmix32(fmix32(fmix32(seed) ^ chunk) ^ j) >> 1                    */
/* with the 32-bit finalizer of MurmurHash3 (Appleby, public domain), chunk = */
/* the chunk's index in the whole list, j = local index (the seed is hashed   */
/* on its own first, so that small seeds and small chunk numbers do not       */
/* cancel each other) - and the k positions                                   */
/* with the largest keys are taken, ties to the lower index: a uniformly      */
/* random k-subset that both sides can reproduce from (seed, chunk, j).       */
/* Everything after the selection (quantizer, residual, wire format) is as in */
/* slo_compress_b.                                                            */
/* ------------------------------------------------------------------------- */

uint32_t slo_fmix32(uint32_t h)
{
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}

uint32_t slo_random_key(uint32_t seed, uint32_t chunk, uint32_t j)
{
    return slo_fmix32(slo_fmix32(slo_fmix32(seed) ^ chunk) ^ j) >> 1;
}

/* Random selection within chunk c of tensor t (chunk_list = its index in the
 * whole list).  Same outputs as slo_topk_chunk. */
int slo_randk_chunk(const slo_tensor *t, int tile, int64_t c, int64_t chunk_list, const float *a, int k,
                    uint32_t seed, uint16_t *sel_idx, float *sel_val)
{
    int C = tile * tile, n = 0;
    slo_cand *cand = (slo_cand *)malloc((size_t)C * sizeof(slo_cand));
    for (int j = 0; j < C; ++j) {
        if (slo_element_of(t, tile, c, j) < 0) continue;
        cand[n].key = slo_random_key(seed, (uint32_t)chunk_list, (uint32_t)j);
        cand[n].j = j;
        ++n;
    }
    if (n < k) {
        free(cand);
        return -1;
    }
    qsort(cand, (size_t)n, sizeof(slo_cand), cmp_mag_desc_then_index);
    qsort(cand, (size_t)k, sizeof(slo_cand), cmp_index_asc);
    for (int m = 0; m < k; ++m) {
        sel_idx[m] = (uint16_t)cand[m].j;
        sel_val[m] = a[slo_element_of(t, tile, c, cand[m].j)];
    }
    free(cand);
    return n;
}

/* slo_compress_b with Random-k in place of Top-k. */
int slo_compress_random_b(const slo_tensor *t, int nt, int tile, int k, int bits, float *e,
                          const float *delta, float beta, uint32_t seed, uint8_t *payload,
                          uint16_t *sel_idx_out)
{
    if (nt < 0 || tile < 1 || tile > 64 || !bits_ok(k, bits, tile)) return SLO_ERR_ARG;
    int nb = bits == 32 ? 0 : 1 << bits;
    int64_t rec = slo_record_bytes_b(k, bits), hdr = slo_header_bytes_b(bits);
    int64_t chunk0 = 0, pay_off = 0;
    for (int ti = 0; ti < nt; ++ti) {
        const slo_tensor *T = &t[ti];
        int64_t n = T->rows * T->cols;
        int64_t nc = slo_tensor_chunks(T, tile);
        int64_t M = nc * k;
        slo_tensor L = *T;
        L.offset = 0;
        slo_accumulate(e + T->offset, delta + T->offset, beta, n);
        const float *a = e + T->offset;
        uint16_t *idx = (uint16_t *)malloc((size_t)(M > 0 ? M : 1) * sizeof(uint16_t));
        float *val = (float *)malloc((size_t)(M > 0 ? M : 1) * sizeof(float));
        uint8_t *code = (uint8_t *)calloc((size_t)(M > 0 ? M : 1), 1);
        int bad = 0;
        for (int64_t c = 0; c < nc; ++c)
            if (slo_randk_chunk(&L, tile, c, chunk0 + c, a, k, seed, idx + c * k, val + c * k) < 0) bad = 1;
        if (bad) {
            free(idx), free(val), free(code);
            return SLO_ERR_ARG;
        }
        float lut[16] = {0};
        if (bits != 32) slo_quantize_tensor_b(val, nc, k, bits, code, lut, NULL);
        for (int64_t c = 0; c < nc; ++c)
            for (int m = 0; m < k; ++m) {
                int64_t i = slo_element_of(&L, tile, c, idx[c * k + m]);
                float sent = bits == 32 ? val[c * k + m] : lut[code[c * k + m]];
                e[T->offset + i] = a[i] - sent;
            }
        if (payload) {
            uint8_t *blk = payload + pay_off;
            memset(blk, 0, (size_t)slo_tensor_block_bytes_b(T, tile, k, bits));
            memcpy(blk, lut, (size_t)4 * nb);
            for (int64_t c = 0; c < nc; ++c)
                slo_pack_record_b(idx + c * k, code + c * k, val + c * k, k, bits, blk + hdr + c * rec);
        }
        if (sel_idx_out) memcpy(sel_idx_out + chunk0 * k, idx, (size_t)M * sizeof(uint16_t));
        free(idx), free(val), free(code);
        chunk0 += nc;
        pay_off += slo_tensor_block_bytes_b(T, tile, k, bits);
    }
    return SLO_OK;
}

/* Well-formedness of a received payload (a receiver-side check, not a step of
 * the method): every record lists k strictly ascending positions, each of them
 * inside the tensor.  Returns SLO_OK or SLO_ERR_PAYLOAD. */
int slo_validate_payload(const slo_tensor *t, int nt, int tile, int k, const uint8_t *payload)
{
    int64_t rec = slo_record_bytes(k), pay_off = 0;
    uint16_t *idx = (uint16_t *)malloc((size_t)k * sizeof(uint16_t));
    uint8_t *code = (uint8_t *)malloc((size_t)k);
    int status = SLO_OK;
    for (int ti = 0; ti < nt && status == SLO_OK; ++ti) {
        const slo_tensor *T = &t[ti];
        int64_t nc = slo_tensor_chunks(T, tile);
        for (int64_t c = 0; c < nc && status == SLO_OK; ++c) {
            slo_unpack_record(payload + pay_off + 16 + c * rec, k, idx, code);
            for (int m = 0; m < k; ++m) {
                if (m > 0 && idx[m] <= idx[m - 1]) status = SLO_ERR_PAYLOAD;
                if (slo_element_of(T, tile, c, idx[m]) < 0) status = SLO_ERR_PAYLOAD;
            }
        }
        pay_off += slo_tensor_block_bytes(T, tile, k);
    }
    free(idx), free(code);
    return status;
}

/* ------------------------------------------------------------------------- */
/* Outer steps of the DiLoCo family that SparseLoCo is built up from and       */
/* compared with (Eq. (1): DiLoCo's Nesterov outer momentum; Section 3.2:      */
/* DiLoCo-LOM and DiLoCo-LOM-Sub-k; appendix "Exact algorithmic description of */
/* DiLoCo variants": DiLoCo+Top-k[+EF], DiLoCo-LOM+Top-k[+EF]).  They reuse    */
/* the chunk-wise Top-k and the sparse aggregate above (with unquantized       */
/* values: these variants have no Q) and add dense elementwise steps.          */
/* Readings for the rounding, as for Eq. (2): every "x <- c*y + z" is one fp32 */
/* fused multiply-add; a dense average is an fp32 accumulator that starts at   */
/* +0.0f, adds the R buffers in the order r = 0..R-1 and is multiplied by 1/R  */
/* rounded once.  Only elements that belong to a tensor are touched.           */
/* ------------------------------------------------------------------------- */

/* Local outer momentum and local Nesterov direction of one worker (Section
 * 3.2; first two lines of the LOM outer step):
 *     m <- mu*m + delta ;  dir <- delta + mu*m.
 * dir may be the same buffer as delta. */
void slo_lom_direction(const slo_tensor *t, int nt, float *m, const float *delta, float mu, float *dir)
{
    for (int ti = 0; ti < nt; ++ti) {
        int64_t o = t[ti].offset, n = t[ti].rows * t[ti].cols;
        for (int64_t i = o; i < o + n; ++i) {
            float mn = fmaf(mu, m[i], delta[i]);
            m[i] = mn;
            dir[i] = fmaf(mu, mn, delta[i]);
        }
    }
}

/* Dense aggregate and outer step.  avg = (1/R) sum_r dirs[r].
 *   m == NULL : theta <- theta - lr*avg          (last two lines of the LOM outer
 *               step; with dirs = the raw pseudo-gradients: plain averaging,
 *               what Eq. (1) reduces to without its second line)
 *   m != NULL : Eq. (1), DiLoCo:  m <- mu*m + avg ; d <- avg + mu*m ;
 *               theta <- theta - lr*d. */
int slo_dense_avg_apply(const slo_tensor *t, int nt, float *theta, float *m, const float *const *dirs,
                        int R, float lr, float mu)
{
    if (R < 1) return SLO_ERR_ARG;
    float invR = 1.0f / (float)R;
    for (int ti = 0; ti < nt; ++ti) {
        int64_t o = t[ti].offset, n = t[ti].rows * t[ti].cols;
        for (int64_t i = o; i < o + n; ++i) {
            float acc = 0.0f;
            for (int r = 0; r < R; ++r) acc = acc + dirs[r][i];
            float d = acc * invR;
            if (m) {
                float mn = fmaf(mu, m[i], d);
                m[i] = mn;
                d = fmaf(mu, mn, d);
            }
            theta[i] = fmaf(-lr, d, theta[i]);
        }
    }
    return SLO_OK;
}

/* Sparse aggregate followed by DiLoCo's global Nesterov momentum (appendix
 * algorithm "Outer step for DiLoCo+Top-k[+EF]", last four lines): the average
 * of the R sparse payloads as in slo_decompress_avg_apply_b, then
 *     m <- mu*m + avg ;  d <- avg + mu*m ;  theta <- theta - lr*d
 * at EVERY element (m is dense: it keeps moving where nothing was sent). */
int slo_decompress_avg_apply_nesterov_b(const slo_tensor *t, int nt, int tile, int k, int bits,
                                        float *theta, float *m, const uint8_t *const *payloads, int R,
                                        float lr, float mu)
{
    if (nt < 0 || tile < 1 || tile > 64 || !bits_ok(k, bits, tile) || R < 1) return SLO_ERR_ARG;
    int C = tile * tile;
    int nb = bits == 32 ? 0 : 1 << bits;
    int64_t rec = slo_record_bytes_b(k, bits), hdr = slo_header_bytes_b(bits);
    float invR = 1.0f / (float)R;
    int64_t pay_off = 0;
    int bad = 0;
    for (int ti = 0; ti < nt; ++ti) {
        const slo_tensor *T = &t[ti];
        int64_t nc = slo_tensor_chunks(T, tile);
        for (int64_t c = 0; c < nc; ++c) {
            float *acc = (float *)calloc((size_t)C, sizeof(float));
            uint16_t *idx = (uint16_t *)malloc((size_t)k * sizeof(uint16_t));
            uint8_t *code = (uint8_t *)calloc((size_t)k, 1);
            float *val = (float *)calloc((size_t)k, sizeof(float));
            for (int r = 0; r < R; ++r) {
                const uint8_t *blk = payloads[r] + pay_off;
                float lut[16] = {0};
                memcpy(lut, blk, (size_t)4 * nb);
                slo_unpack_record_b(blk + hdr + c * rec, k, bits, idx, code, val);
                for (int q = 0; q < k; ++q) {
                    if (idx[q] >= C) {
                        bad |= 1;
                        continue;
                    }
                    float sent = bits == 32 ? val[q] : lut[code[q]];
                    acc[idx[q]] = acc[idx[q]] + sent;
                }
            }
            for (int j = 0; j < C; ++j) {
                int64_t i = slo_element_of(T, tile, c, j);
                if (i < 0) continue;
                float d = acc[j] * invR;
                float mn = fmaf(mu, m[i], d);
                m[i] = mn;
                d = fmaf(mu, mn, d);
                theta[i] = fmaf(-lr, d, theta[i]);
            }
            free(acc), free(idx), free(code), free(val);
        }
        pay_off += slo_tensor_block_bytes_b(T, tile, k, bits);
    }
    return bad ? SLO_ERR_PAYLOAD : SLO_OK;
}

/* DiLoCo-LOM-Sub-k (Section 3.2; boxed line of the LOM outer step):
 *     m <- m - Top-k(m)
 * with the chunk-wise Top-k of SparseLoCo (same magnitude order and tie
 * rule).  At a selected position the result is m - m = +0.0f; every other
 * element is untouched.  sel_idx (optional): the selected local indices,
 * [n_chunks * k] in list chunk order. */
int slo_sub_topk(const slo_tensor *t, int nt, int tile, int k, float *m, uint16_t *sel_idx)
{
    if (nt < 0 || tile < 1 || tile > 64 || k < 1 || k > tile * tile) return SLO_ERR_ARG;
    int64_t chunk0 = 0;
    uint16_t *idx = (uint16_t *)malloc((size_t)k * sizeof(uint16_t));
    float *val = (float *)malloc((size_t)k * sizeof(float));
    int status = SLO_OK;
    for (int ti = 0; ti < nt && status == SLO_OK; ++ti) {
        const slo_tensor *T = &t[ti];
        int64_t nc = slo_tensor_chunks(T, tile);
        for (int64_t c = 0; c < nc; ++c) {
            if (slo_topk_chunk(T, tile, c, m, k, idx, val) < 0) {
                status = SLO_ERR_ARG;
                break;
            }
            for (int q = 0; q < k; ++q) {
                int64_t i = slo_element_of(T, tile, c, idx[q]);
                m[i] = val[q] - val[q];
            }
            if (sel_idx) memcpy(sel_idx + (chunk0 + c) * k, idx, (size_t)k * sizeof(uint16_t));
        }
        chunk0 += nc;
    }
    free(idx), free(val);
    return status;
}

int slo_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------- */
/* Index coder (appendix "Compression of indices in Top-k").  The paper names */
/* its coder ("sub-chunking and Rice coding") and the rates it reaches (8.9,  */
/* 6.6, 5.6 bits per index for k = 32, 128, 256 against the bounds 8.3, 6.3,  */
/* 5.3) but does not describe it.  PARITY UNPINNED beyond: lossless round     */
/* trip, size between the information bound and the paper's reached rates on  */
/* uniformly random index sets, and the hand-computed bytes of tiny records.  */
/*                                                                           */
/* Reading (this build's own format, "SLRICE02"; it is the wire format of a   */
/* round: the compressor emits it and the aggregation consumes it):           */
/*   - an ascending index list is coded as gaps g_0 = idx_0,                  */
/*     g_i = idx_i - idx_(i-1) - 1, each as a Rice code with parameter b:     */
/*     quotient q_i = g_i >> b in unary (q_i one-bits, then a zero bit) and   */
/*     the b low bits of g_i as the remainder;                                */
/*     b = floor(log2(floor(4096 ln 2) / k)) = floor(log2(2839 / k)), 0 when  */
/*     2839 / k < 1 (the optimum for uniformly random positions);             */
/*   - the two halves of the codes are stored apart, so that a decoder can    */
/*     take a chunk's entries side by side instead of one after the other:    */
/*     the remainders as k fields of b bits at fixed places, the quotients    */
/*     as one bit vector per chunk (the unary codes back to back: k zero      */
/*     bits, Q = sum of the q_i one-bits; entry i ends at the i-th zero,      */
/*     which sits at bit i + q_0 + ... + q_i).  The bits are the Rice codes'  */
/*     bits, regrouped: k (1 + b) + Q per chunk;                              */
/*   - bits fill bytes LSB first (as the 12-bit fields of the plain format);  */
/*   - fixed record of a chunk: the k remainders (b bits each, LSB first)     */
/*     padded with zero bits to a multiple of 4 bytes, then the k value       */
/*     fields exactly as they stand in the plain record (k * bits / 8 bytes), */
/*     zero padding to a multiple of 4 bytes (both parts start on a 4-byte    */
/*     boundary; neither padding is ever present when k is a multiple of 32); */
/*   - directory: one entry per group of 16 consecutive chunks of a tensor:   */
/*     uint32 = offset of the group's run of quotient bit vectors, in 4-byte  */
/*     words from the start of the quotient section, then 16 fields with the  */
/*     Q of each chunk of the group - one byte each when the largest possible */
/*     Q, (4096 - k) >> b, is below 256, else two (little endian); fields of  */
/*     chunks beyond the tensor's last are zero.  A chunk's bit vector starts */
/*     at bit  sum over the earlier chunks of its group of (k + Q)  of the    */
/*     group's run;                                                           */
/*   - tensor block, 16-byte aligned, at an offset that follows from the list */
/*     alone: look-up table header as in the plain format; the directory; the */
/*     fixed records in chunk order; zero padding to 16 bytes;                */
/*   - quotient section, after the last block: the groups' runs in list       */
/*     order, the chunks of a group back to back without padding, every run   */
/*     zero-padded to a 4-byte boundary; zero padding to 16 bytes at the end; */
/*   - buffer: "SLRICE02", uint64 total bytes, the blocks, the section.       */
/* ("Group" is this format's own unit and no reading of the paper's           */
/* "sub-chunking"; the format does not split a chunk.)                        */
/* ------------------------------------------------------------------------- */

#define SLO_RICE_GROUP 16
static const char SLO_RICE_MAGIC[8] = {'S', 'L', 'R', 'I', 'C', 'E', '0', '2'};

int slo_rice_param(int k)
{
    int q = 2839 / k, b = 0;
    while ((2 << b) <= q) ++b;
    return q < 1 ? 0 : b;
}

/* bytes of a quotient-sum field, of a directory entry and of a fixed record */
int slo_rice_qfield_bytes(int k) { return ((4096 - k) >> slo_rice_param(k)) < 256 ? 1 : 2; }
int64_t slo_rice_dir_entry_bytes(int k) { return 4 + SLO_RICE_GROUP * (int64_t)slo_rice_qfield_bytes(k); }
int64_t slo_rice_rem_bytes(int k) { return ((int64_t)k * slo_rice_param(k) + 31) / 32 * 4; }
int64_t slo_rice_fixed_bytes(int k, int bits)
{
    return (slo_rice_rem_bytes(k) + (int64_t)k * bits / 8 + 3) / 4 * 4;
}

static void put_bit(uint8_t *p, int64_t bit, unsigned v)
{
    if (v & 1u) p[bit / 8] |= (uint8_t)(1u << (bit % 8));
}

static unsigned get_bit(const uint8_t *p, int64_t bit) { return p[bit / 8] >> (bit % 8) & 1u; }

/* Bytes of the part whose layout follows from the list alone (header + blocks). */
static int64_t rice_fixed_part(const slo_tensor *t, int nt, int tile, int k, int bits)
{
    int64_t pos = 16;
    for (int i = 0; i < nt; ++i) {
        int64_t nc = slo_tensor_chunks(&t[i], tile), ng = ceil_div(nc, SLO_RICE_GROUP);
        pos += ceil_div(slo_header_bytes_b(bits) + ng * slo_rice_dir_entry_bytes(k) +
                        nc * slo_rice_fixed_bytes(k, bits), 16) * 16;
    }
    return pos;
}

/* Upper bound of the coded size of payloads of this list (every Q at its maximum). */
int64_t slo_rice_max_bytes_b(const slo_tensor *t, int nt, int tile, int k, int bits)
{
    if (!bits_ok(k, bits, tile)) return SLO_ERR_ARG;
    int64_t qmax = (4096 - k) >> slo_rice_param(k);
    int64_t total = rice_fixed_part(t, nt, tile, k, bits);
    for (int i = 0; i < nt; ++i) {
        int64_t nc = slo_tensor_chunks(&t[i], tile);
        for (int64_t c0 = 0; c0 < nc; c0 += SLO_RICE_GROUP) {
            int64_t in_group = nc - c0 < SLO_RICE_GROUP ? nc - c0 : SLO_RICE_GROUP;
            total += ceil_div(in_group * (k + qmax), 32) * 4;
        }
    }
    return ceil_div(total, 16) * 16;
}

/* payload (plain wire format) -> coded buffer; returns the coded size or <0. */
int64_t slo_rice_encode_b(const slo_tensor *t, int nt, int tile, int k, int bits,
                          const uint8_t *payload, uint8_t *out, int64_t cap)
{
    if (!bits_ok(k, bits, tile)) return SLO_ERR_ARG;
    const int b = slo_rice_param(k), qf = slo_rice_qfield_bytes(k);
    const int64_t rec = slo_record_bytes_b(k, bits), hdr = slo_header_bytes_b(bits);
    const int64_t fix = slo_rice_fixed_bytes(k, bits), dent = slo_rice_dir_entry_bytes(k);
    const int64_t section = rice_fixed_part(t, nt, tile, k, bits);   /* start of the quotient section */
    if (section > cap) return SLO_ERR_ARG;
    uint16_t *idx = (uint16_t *)malloc((size_t)k * sizeof(uint16_t));
    uint8_t *code = (uint8_t *)calloc((size_t)k, 1);
    float *val = (float *)calloc((size_t)k, sizeof(float));
    memset(out, 0, (size_t)cap);
    int64_t pos = 16, pay_off = 0, word = 0;      /* next block; tensor's plain block; next run, in words */
    int status = SLO_OK;
    for (int ti = 0; ti < nt && status == SLO_OK; ++ti) {
        int64_t nc = slo_tensor_chunks(&t[ti], tile), ng = ceil_div(nc, SLO_RICE_GROUP);
        uint8_t *blk = out + pos, *dir = blk + hdr, *fixed = dir + ng * dent;
        memcpy(blk, payload + pay_off, (size_t)hdr);             /* look-up table */
        for (int64_t g = 0; g < ng && status == SLO_OK; ++g) {
            uint32_t w32 = (uint32_t)word;
            memcpy(dir + g * dent, &w32, 4);
            int64_t bit = 0;                                      /* bit inside the group's run */
            for (int64_t c = g * SLO_RICE_GROUP; c < nc && c < (g + 1) * SLO_RICE_GROUP; ++c) {
                const uint8_t *r = payload + pay_off + hdr + c * rec;
                slo_unpack_record_b(r, k, bits, idx, code, val);
                int prev = -1;
                int64_t Q = 0;
                /* worst case of this chunk's vector, checked before it is written */
                if (section + 4 * word + (bit + k + ((4096 - k) >> b) + 7) / 8 > cap) {
                    status = SLO_ERR_ARG;
                    break;
                }
                for (int m = 0; m < k; ++m) {
                    uint32_t gap = (uint32_t)(idx[m] - prev - 1);
                    prev = idx[m];
                    for (uint32_t q = gap >> b; q > 0; --q, ++bit, ++Q) put_bit(out + section + 4 * word, bit, 1u);
                    ++bit;                                        /* the zero bit */
                    for (int i = 0; i < b; ++i) put_bit(fixed + c * fix, (int64_t)m * b + i, gap >> i);
                }
                /* the value fields: the tail of the plain record, byte for byte */
                memcpy(fixed + c * fix + slo_rice_rem_bytes(k), r + 3 * k / 2, (size_t)((int64_t)k * bits / 8));
                uint8_t *field = dir + g * dent + 4 + (c - g * SLO_RICE_GROUP) * qf;
                field[0] = (uint8_t)(Q & 0xFF);
                if (qf == 2) field[1] = (uint8_t)(Q >> 8);
            }
            word += ceil_div(bit, 32);
        }
        pos += ceil_div(hdr + ng * dent + nc * fix, 16) * 16;
        pay_off += slo_tensor_block_bytes_b(&t[ti], tile, k, bits);
    }
    free(idx), free(code), free(val);
    if (status != SLO_OK) return status;
    int64_t total = ceil_div(section + 4 * word, 16) * 16;
    if (total > cap) return SLO_ERR_ARG;
    memcpy(out, SLO_RICE_MAGIC, 8);
    uint64_t t64 = (uint64_t)total;
    memcpy(out + 8, &t64, 8);
    return total;
}

/* coded buffer of in_bytes bytes -> payload in the plain wire format (every byte written).
 * SLO_ERR_PAYLOAD: wrong magic or size, a run or a bit vector that leaves the buffer, a
 * vector that does not hold k zero bits within its k + Q bits, an index beyond 4095. */
int slo_rice_decode_b(const slo_tensor *t, int nt, int tile, int k, int bits, const uint8_t *in,
                      int64_t in_bytes, uint8_t *payload)
{
    if (!bits_ok(k, bits, tile)) return SLO_ERR_ARG;
    const int b = slo_rice_param(k), qf = slo_rice_qfield_bytes(k);
    const int64_t rec = slo_record_bytes_b(k, bits), hdr = slo_header_bytes_b(bits);
    const int64_t fix = slo_rice_fixed_bytes(k, bits), dent = slo_rice_dir_entry_bytes(k);
    const int64_t section = rice_fixed_part(t, nt, tile, k, bits);
    uint64_t total;
    if (in_bytes < 16 || memcmp(in, SLO_RICE_MAGIC, 8)) return SLO_ERR_PAYLOAD;
    memcpy(&total, in + 8, 8);
    if ((int64_t)total != in_bytes || in_bytes < section) return SLO_ERR_PAYLOAD;
    uint16_t *idx = (uint16_t *)malloc((size_t)k * sizeof(uint16_t));
    uint8_t *code = (uint8_t *)calloc((size_t)k, 1);
    float *val = (float *)calloc((size_t)k, sizeof(float));
    int64_t pos = 16, pay_off = 0;
    int status = SLO_OK;
    for (int ti = 0; ti < nt && status == SLO_OK; ++ti) {
        int64_t nc = slo_tensor_chunks(&t[ti], tile), ng = ceil_div(nc, SLO_RICE_GROUP);
        const uint8_t *blk = in + pos, *dir = blk + hdr, *fixed = dir + ng * dent;
        memset(payload + pay_off, 0, (size_t)slo_tensor_block_bytes_b(&t[ti], tile, k, bits));
        memcpy(payload + pay_off, blk, (size_t)hdr);
        for (int64_t c = 0; c < nc && status == SLO_OK; ++c) {
            const int64_t g = c / SLO_RICE_GROUP;
            uint32_t word;
            memcpy(&word, dir + g * dent, 4);
            int64_t bit = 0, Q = 0;                               /* start of the chunk's vector in the run */
            for (int64_t c2 = g * SLO_RICE_GROUP; c2 <= c; ++c2) {
                const uint8_t *field = dir + g * dent + 4 + (c2 - g * SLO_RICE_GROUP) * qf;
                Q = field[0] | (qf == 2 ? field[1] << 8 : 0);
                if (c2 < c) bit += k + Q;
            }
            const uint8_t *run = in + section + 4 * (int64_t)word;
            if (section + 4 * (int64_t)word + (bit + k + Q + 7) / 8 > in_bytes) {
                status = SLO_ERR_PAYLOAD;
                break;
            }
            const int64_t end = bit + k + Q;
            int prev = -1;
            for (int m = 0; m < k; ++m) {
                uint32_t q = 0, rem = 0;
                while (bit < end && get_bit(run, bit)) ++q, ++bit;
                if (bit >= end) {
                    status = SLO_ERR_PAYLOAD;                     /* fewer than k zero bits */
                    break;
                }
                ++bit;
                for (int i = 0; i < b; ++i) rem |= get_bit(fixed + c * fix, (int64_t)m * b + i) << i;
                int v = prev + 1 + (int)(q << b | rem);
                if (v > 4095) status = SLO_ERR_PAYLOAD, v = 4095;
                idx[m] = (uint16_t)v;
                prev = v;
            }
            if (status != SLO_OK) break;
            if (bit != end) status = SLO_ERR_PAYLOAD;             /* Q does not match the vector */
            uint8_t *r = payload + pay_off + hdr + c * rec;
            /* indices through the record encoder (with all-zero value fields), then the value
             * fields byte for byte */
            slo_pack_record_b(idx, code, val, k, bits, r);
            memcpy(r + 3 * k / 2, fixed + c * fix + slo_rice_rem_bytes(k), (size_t)((int64_t)k * bits / 8));
        }
        pos += ceil_div(hdr + ng * dent + nc * fix, 16) * 16;
        pay_off += slo_tensor_block_bytes_b(&t[ti], tile, k, bits);
    }
    free(idx), free(code), free(val);
    return status;
}

/* The paper's setting, 2-bit values. */
int64_t slo_rice_max_bytes(const slo_tensor *t, int nt, int tile, int k)
{
    return slo_rice_max_bytes_b(t, nt, tile, k, 2);
}

int64_t slo_rice_encode(const slo_tensor *t, int nt, int tile, int k, const uint8_t *payload,
                        uint8_t *out, int64_t cap)
{
    return slo_rice_encode_b(t, nt, tile, k, 2, payload, out, cap);
}

int slo_rice_decode(const slo_tensor *t, int nt, int tile, int k, const uint8_t *in, int64_t in_bytes,
                    uint8_t *payload)
{
    return slo_rice_decode_b(t, nt, tile, k, 2, in, in_bytes, payload);
}
