/*
 * CPU oracle for FlashOmni attention (Algorithm 1, Definitions 1-2, Section 3.3
 * "Sparse Symbols Compression", Section 3.1 for the dense definition).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
 * library is checked against.  Nothing in the product path may call it, and it shares
 * no code with the HIP sources.
 *
 * What is computed, for every batch b, head h and query block i (b_q rows):
 *   - cache flag set (the paper's F(S_c, i) == 0, "cache-then-reuse" branch of
 *     Algorithm 1 with OP_reuse = identity): the block of O is the block of the cached
 *     output, copied as raw 16-bit patterns.  With no cached tensor the block is left
 *     untouched (the early-continue of that branch).
 *   - otherwise ("compute-on-demand" branch): with J_i the set of key blocks whose
 *     symbol bit J(S_s, i, j) is 1, every row r of the block gets
 *         s_k = <Q_r, K_k> / sqrt(d)          for all keys k in the kept blocks
 *         p_k = exp(s_k - max_k s_k)
 *         O_r = sum_k p_k V_k / sum_k p_k
 *     i.e. Section 3.1's softmax attention restricted to the kept keys.  Algorithm 1
 *     updates the running max and sum only inside the J == 1 branch, so the softmax
 *     normalises over kept keys only.  The online (running max) form of Algorithm 1
 *     reaches this two-pass result exactly up to rounding, so the two-pass definition
 *     is what is written here.  A computed row with no kept key block is defined as 0.
 *
 * Symbol layout (Section 3.3): logical bit t of a row of symbols is stored in byte t/8
 * at bit position 7 - t%8 (most significant bit first, zero padding at the end), which
 * is what the worked example [1,1,1,0] -> 0b11100000 = 224 fixes.  Each (b,h,i) row of
 * S_s is padded to a whole number of bytes.
 *
 * All arithmetic is IEEE double.  Inputs are bf16 bit patterns widened exactly.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double widen_bf16(uint16_t bits)
{
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* round-to-nearest-even narrowing double -> float -> bf16, used only for the bf16
 * statistics copy of computed blocks (never for cached blocks, which are raw copies) */
static uint16_t narrow_bf16(double x)
{
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* J(S_s, i, j) for one row of packed symbols: 1 = compute the pair */
static int symbol_bit(const uint8_t *row, int t)
{
    return (row[t >> 3] >> (7 - (t & 7))) & 1;
}

int oracle_mask_row_bytes(int Tkv)
{
    return (Tkv + 7) / 8;
}

/*
 * One query block of one head.  Kd, Vd: that head's keys/values widened to double,
 * [L][D].  Qh: that head's bf16 queries [L][D].  mask_row: packed symbols of this
 * (b,h,i) or NULL for "all kept".  out: [bq][D] doubles.  scores: scratch of L doubles.
 * Definition 1 counts ceil(L / b) blocks: the last query block and the last key block may be
 * short; rows of `out` past the end of the sequence are left untouched.
 */
static void compute_block(const uint16_t *Qh, const double *Kd, const double *Vd,
                          const uint8_t *mask_row, int i, int L, int D, int bq, int bk,
                          double *out, double *scores)
{
    const int Tkv = (L + bk - 1) / bk;
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    double *q = (double *)malloc((size_t)D * sizeof(double));

    for (int r = 0; r < bq && i * bq + r < L; ++r) {
        const uint16_t *qrow = Qh + ((size_t)i * bq + r) * D;
        double *orow = out + (size_t)r * D;
        for (int c = 0; c < D; ++c) {
            q[c] = widen_bf16(qrow[c]);
            orow[c] = 0.0;
        }

        /* pass 1: scores of kept keys and their maximum */
        double m = -INFINITY;
        int any = 0;
        for (int j = 0; j < Tkv; ++j) {
            if (mask_row && !symbol_bit(mask_row, j))
                continue;
            any = 1;
            for (int k = j * bk; k < (j + 1) * bk && k < L; ++k) {
                const double *krow = Kd + (size_t)k * D;
                double dot = 0.0;
                for (int c = 0; c < D; ++c)
                    dot += q[c] * krow[c];
                double s = dot * inv_sqrt_d;
                scores[k] = s;
                if (s > m)
                    m = s;
            }
        }
        if (!any)
            continue; /* no kept key block: row defined as zero */

        /* pass 2: weights, their sum, weighted sum of values */
        double l = 0.0;
        for (int j = 0; j < Tkv; ++j) {
            if (mask_row && !symbol_bit(mask_row, j))
                continue;
            for (int k = j * bk; k < (j + 1) * bk && k < L; ++k) {
                double p = exp(scores[k] - m);
                const double *vrow = Vd + (size_t)k * D;
                l += p;
                for (int c = 0; c < D; ++c)
                    orow[c] += p * vrow[c];
            }
        }
        for (int c = 0; c < D; ++c)
            orow[c] /= l;
    }
    free(q);
}

static void widen_head(const uint16_t *src, double *dst, size_t n)
{
#pragma omp parallel for schedule(static)
    for (long long t = 0; t < (long long)n; ++t)
        dst[t] = widen_bf16(src[t]);
}

/*
 * Selected query blocks.  items[n] = flattened (b*H + h)*Tq + i, in any order.
 * O_f64: [n_items][bq][D] doubles; O_bits: [n_items][bq][D] bf16 patterns (may be NULL).
 * A cached item gets the raw cached bits (and their widened value); with O_cache NULL
 * its slots are left untouched.
 * Returns 0, or -1 on bad arguments.
 */
int oracle_sparse_attn_blocks(const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                              const uint8_t *cache_flags, const uint8_t *kv_mask,
                              const uint16_t *O_cache, int B, int H, int L, int D,
                              int bq, int bk, const int64_t *items, int64_t n_items,
                              double *O_f64, uint16_t *O_bits)
{
    if (!Q || !K || !V || !O_f64 || B <= 0 || H <= 0 || L <= 0 || D <= 0 || bq <= 0 || bk <= 0)
        return -1;
    const int Tq = (L + bq - 1) / bq, Tkv = (L + bk - 1) / bk;
    const int row_bytes = oracle_mask_row_bytes(Tkv);
    const size_t head_elems = (size_t)L * D;
    const size_t blk_elems = (size_t)bq * D;

    double *Kd = (double *)malloc(head_elems * sizeof(double));
    double *Vd = (double *)malloc(head_elems * sizeof(double));
    if (!Kd || !Vd) {
        free(Kd);
        free(Vd);
        return -1;
    }

    for (int64_t bh = 0; bh < (int64_t)B * H; ++bh) {
        int needed = 0;
        for (int64_t n = 0; n < n_items && !needed; ++n) {
            if (items[n] / Tq == bh && !(cache_flags && cache_flags[items[n]]))
                needed = 1;
        }
        if (needed) {
            widen_head(K + bh * head_elems, Kd, head_elems);
            widen_head(V + bh * head_elems, Vd, head_elems);
        }
#pragma omp parallel
        {
            double *scores = (double *)malloc((size_t)L * sizeof(double));
#pragma omp for schedule(dynamic, 1)
            for (int64_t n = 0; n < n_items; ++n) {
                if (items[n] / Tq != bh)
                    continue;
                const int i = (int)(items[n] % Tq);
                double *out = O_f64 + (size_t)n * blk_elems;
                uint16_t *outb = O_bits ? O_bits + (size_t)n * blk_elems : NULL;
                if (cache_flags && cache_flags[items[n]]) {
                    if (O_cache) {
                        const uint16_t *src = O_cache + bh * head_elems + (size_t)i * blk_elems;
                        const int rows = L - i * bq < bq ? L - i * bq : bq;
                        for (size_t t = 0; t < (size_t)rows * D; ++t) {
                            out[t] = widen_bf16(src[t]);
                            if (outb)
                                outb[t] = src[t];
                        }
                    }
                    continue;
                }
                const uint8_t *mrow = kv_mask ? kv_mask + (size_t)items[n] * row_bytes : NULL;
                compute_block(Q + bh * head_elems, Kd, Vd, mrow, i, L, D, bq, bk, out, scores);
                if (outb) {
                    const int rows = L - i * bq < bq ? L - i * bq : bq;
                    for (size_t t = 0; t < (size_t)rows * D; ++t)
                        outb[t] = narrow_bf16(out[t]);
                }
            }
            free(scores);
        }
    }
    free(Kd);
    free(Vd);
    return 0;
}

/* Every query block: O_f64 and O_bits have the tensor shape [B][H][L][D]. */
int oracle_sparse_attn(const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                       const uint8_t *cache_flags, const uint8_t *kv_mask,
                       const uint16_t *O_cache, int B, int H, int L, int D, int bq, int bk,
                       double *O_f64, uint16_t *O_bits)
{
    if (B <= 0 || H <= 0 || L <= 0 || bq <= 0)
        return -1;
    const int Tq = (L + bq - 1) / bq;
    const int64_t n = (int64_t)B * H * Tq;
    int64_t *items = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    if (!items)
        return -1;
    for (int64_t t = 0; t < n; ++t)
        items[t] = t;
    int rc = 0;
    if (L % bq == 0) {
        /* the blocks of [n][bq][D] are the rows of [B][H][L][D] in order */
        rc = oracle_sparse_attn_blocks(Q, K, V, cache_flags, kv_mask, O_cache, B, H, L, D, bq, bk,
                                       items, n, O_f64, O_bits);
    } else {
        /* short last block: go through [n][bq][D] staging arrays, seeded with what O holds so that
         * "left untouched" keeps its meaning, and copy the rows that exist back */
        const size_t blk = (size_t)bq * D;
        double *tf = (double *)calloc((size_t)n * blk, sizeof(double));
        uint16_t *tb = (uint16_t *)calloc((size_t)n * blk, sizeof(uint16_t));
        if (!tf || !tb) {
            free(tf);
            free(tb);
            free(items);
            return -1;
        }
        for (int pass = 0; pass < 2; ++pass) {
            if (pass == 1)
                rc = oracle_sparse_attn_blocks(Q, K, V, cache_flags, kv_mask, O_cache, B, H, L, D, bq,
                                               bk, items, n, tf, O_bits ? tb : NULL);
            for (int64_t t = 0; t < n; ++t) {
                const int64_t bh = t / Tq;
                const int i = (int)(t % Tq);
                const int rows = L - i * bq < bq ? L - i * bq : bq;
                const size_t at = ((size_t)bh * L + (size_t)i * bq) * D;
                for (size_t e = 0; e < (size_t)rows * D; ++e) {
                    if (pass == 0) {
                        tf[(size_t)t * blk + e] = O_f64[at + e];
                        if (O_bits)
                            tb[(size_t)t * blk + e] = O_bits[at + e];
                    } else {
                        O_f64[at + e] = tf[(size_t)t * blk + e];
                        if (O_bits)
                            O_bits[at + e] = tb[(size_t)t * blk + e];
                    }
                }
            }
        }
        free(tf);
        free(tb);
    }
    free(items);
    return rc;
}

/*
 * Pair accounting of Section 4.1 ("Sparsity = skip / total" over the
 * (Q_i K_j^T, P_ij V_j) pairs): kept = pairs actually computed, i.e. set symbol bits of
 * non-cached rows; total = B*H*Tq*Tkv.
 */
int oracle_count_pairs(const uint8_t *cache_flags, const uint8_t *kv_mask, int B, int H,
                       int L, int bq, int bk, int64_t *kept, int64_t *total)
{
    if (B <= 0 || H <= 0 || L <= 0 || bq <= 0 || bk <= 0)
        return -1;
    const int Tq = (L + bq - 1) / bq, Tkv = (L + bk - 1) / bk;
    const int row_bytes = oracle_mask_row_bytes(Tkv);
    int64_t k = 0;
    for (int64_t row = 0; row < (int64_t)B * H * Tq; ++row) {
        if (cache_flags && cache_flags[row])
            continue;
        for (int j = 0; j < Tkv; ++j)
            k += kv_mask ? symbol_bit(kv_mask + (size_t)row * row_bytes, j) : 1;
    }
    *kept = k;
    *total = (int64_t)B * H * Tq * Tkv;
    return 0;
}

/* number of OpenMP threads the parallel loops above will use */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
