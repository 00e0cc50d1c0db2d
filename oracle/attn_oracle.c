/*
 * fp64 CPU oracle for MM-DiT joint attention, dense or under a block mask.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, definition-level checker
 * the GPU library is compared against.  Nothing in the product path may call,
 * link or import it; it shares no code with the HIP kernels.
 *
 * What it computes (RAPID^3, Sec. 3.1 Eq. 1: the self-attention block F_SA of
 * a DiT layer over the joint image+text token sequence; Sec. 3.2 "Level-3:
 * Sparse-Attention", Eq. 4: the same block with a pruned attention map,
 * controlled per layer and per head; Sec. 3.3 (c): action 0 = full attention,
 * actions 1..N_sparse = progressively sparser maps).  The paper cites the
 * standard scaled-dot-product attention and never prints the formula, so the
 * oracle is that definition written out:
 *
 *   for every sample b, head h and query row r:
 *     r >= kv_len                      -> O[r,:] = 0            (padded query)
 *     A(r) = { c < kv_len : M[b,h,r/block,c/block] != 0 }   (dense: M == 1)
 *     A(r) empty                       -> O[r,:] = 0
 *     s_c = scale * sum_d Q[r,d] K[c,d]            c in A(r)
 *     p_c = exp(s_c - max_c s_c);  Z = sum_c p_c
 *     O[r,:] = sum_c (p_c / Z) V[c,:]
 *
 * Pruned entries are removed BEFORE the softmax (the kept entries renormalise);
 * that is the only reading under which a pruned tile needs no computation.
 *
 * Inputs are bf16 bit patterns (uint16), widened exactly to fp64; every
 * operation is fp64; the output stays fp64 (never rounded to bf16).
 * No blocking, no fusion, no online softmax: two plain passes per row.
 *
 * Pins (tests/test_oracle_pins.py, tests/test_oracle_mutants.py): library
 * softmax+matmul brute force with an explicit 0/-inf bias, closed forms
 * (single key, identical keys, V == 1, block indicator V), invariances (shift,
 * permutation, masked-block perturbation, sample/head independence), convexity.
 * No value printed in the paper pins attention numerically.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* bf16 is the upper half of an IEEE binary32. */
static double bf16_to_f64(uint16_t bits)
{
    uint32_t w = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* One output row.  q_row: D values of this query.  k, v: [N, D] of this
 * (sample, head).  mask_row: nb bytes = row r/block of this (sample, head)'s
 * block mask, or NULL for dense.  score: caller scratch of N doubles. */
static void attn_row(const uint16_t *q_row, const uint16_t *k, const uint16_t *v,
                     const uint8_t *mask_row, int block, int kv_len, int D,
                     double scale, double *score, double *out)
{
    int c, d;
    int any = 0;
    double m = -INFINITY, Z = 0.0;

    for (d = 0; d < D; ++d) out[d] = 0.0;

    /* scores of allowed keys, and their maximum */
    for (c = 0; c < kv_len; ++c) {
        int allowed = (mask_row == NULL) || (mask_row[c / block] != 0);
        if (!allowed) { score[c] = -INFINITY; continue; }
        double dot = 0.0;
        for (d = 0; d < D; ++d)
            dot += bf16_to_f64(q_row[d]) * bf16_to_f64(k[(size_t)c * D + d]);
        score[c] = scale * dot;
        if (!any || score[c] > m) m = score[c];
        any = 1;
    }
    if (!any) return;                     /* no allowed key: row stays 0 */

    /* softmax over the allowed set */
    for (c = 0; c < kv_len; ++c) {
        if (score[c] == -INFINITY) { score[c] = 0.0; continue; }
        score[c] = exp(score[c] - m);
        Z += score[c];
    }
    /* weighted sum of value rows */
    for (c = 0; c < kv_len; ++c) {
        if (score[c] == 0.0) continue;
        double p = score[c] / Z;
        for (d = 0; d < D; ++d)
            out[d] += p * bf16_to_f64(v[(size_t)c * D + d]);
    }
}

static int check_args(const void *q, const void *k, const void *v, const void *o,
                      int B, int H, int N, int D, int block, const uint8_t *mask,
                      int kv_len)
{
    if (!q || !k || !v || !o) return -1;
    if (B <= 0 || H <= 0 || N <= 0 || D <= 0) return -2;
    if (kv_len < 1 || kv_len > N) return -2;
    if (mask) { if (block <= 0 || N % block != 0) return -2; }
    return 0;
}

/*
 * Whole tensor.  q,k,v: bf16 bits [B,H,N,D] (D fastest).  o: fp64 [B,H,N,D].
 * mask: uint8 [B,H,N/block,N/block] (query-block, key-block), nonzero = keep;
 * NULL = dense (block ignored).  kv_len = number of valid tokens (a prefix).
 * scale <= 0 selects 1/sqrt(D).  Returns 0, or a negative code on bad args.
 */
int rapid_oracle_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                      double *o, int B, int H, int N, int D, int block,
                      const uint8_t *mask, int kv_len, double scale)
{
    int rc = check_args(q, k, v, o, B, H, N, D, block, mask, kv_len);
    if (rc) return rc;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)D);
    const int nb = mask ? N / block : 0;
    const long long rows = (long long)B * H * N;
    int failed = 0;

#pragma omp parallel
    {
        double *score = (double *)malloc(sizeof(double) * (size_t)N);
        if (!score) {
#pragma omp atomic write
            failed = 1;
        }
        long long t;
#pragma omp for schedule(dynamic, 16)
        for (t = 0; t < rows; ++t) {
            if (!score) continue;
            const long long bh = t / N;
            const int r = (int)(t % N);
            double *out = o + (size_t)t * D;
            if (r >= kv_len) { for (int d = 0; d < D; ++d) out[d] = 0.0; continue; }
            const size_t base = (size_t)bh * N * D;
            const uint8_t *mrow = mask
                ? mask + ((size_t)bh * nb + (size_t)(r / block)) * nb : NULL;
            attn_row(q + base + (size_t)r * D, k + base, v + base, mrow, block,
                     kv_len, D, scale, score, out);
        }
        free(score);
    }
    return failed ? -7 : 0;
}

/*
 * Selected rows only (for full-size parity on sampled outputs and for the
 * bounded timing sample).  rows: n_rows triples (b, h, r).  o: fp64 [n_rows, D].
 */
int rapid_oracle_attn_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                           double *o, int B, int H, int N, int D, int block,
                           const uint8_t *mask, int kv_len, double scale,
                           int n_rows, const int *rows)
{
    int rc = check_args(q, k, v, o, B, H, N, D, block, mask, kv_len);
    if (rc) return rc;
    if (n_rows < 0 || (n_rows > 0 && !rows)) return -2;
    for (int i = 0; i < n_rows; ++i) {
        const int b = rows[3 * i], h = rows[3 * i + 1], r = rows[3 * i + 2];
        if (b < 0 || b >= B || h < 0 || h >= H || r < 0 || r >= N) return -2;
    }
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)D);
    const int nb = mask ? N / block : 0;
    int failed = 0;

#pragma omp parallel
    {
        double *score = (double *)malloc(sizeof(double) * (size_t)N);
        if (!score) {
#pragma omp atomic write
            failed = 1;
        }
        int i;
#pragma omp for schedule(dynamic, 4)
        for (i = 0; i < n_rows; ++i) {
            if (!score) continue;
            const int b = rows[3 * i], h = rows[3 * i + 1], r = rows[3 * i + 2];
            double *out = o + (size_t)i * D;
            if (r >= kv_len) { for (int d = 0; d < D; ++d) out[d] = 0.0; continue; }
            const size_t bh = (size_t)b * H + h;
            const size_t base = bh * N * D;
            const uint8_t *mrow = mask
                ? mask + (bh * nb + (size_t)(r / block)) * nb : NULL;
            attn_row(q + base + (size_t)r * D, k + base, v + base, mrow, block,
                     kv_len, D, scale, score, out);
        }
        free(score);
    }
    return failed ? -7 : 0;
}

/*
 * Kept-tile lists (the "which tiles are visited" part of the sparse action):
 * for each (b, h, query-block i) the ascending key-blocks j with M[b,h,i,j] != 0
 * whose first token lies below kv_len.  counts: int32 [B,H,nb];
 * indices: int32 [B,H,nb,nb], first counts[...] entries valid, the rest -1.
 */
int rapid_oracle_kept_tiles(const uint8_t *mask, int B, int H, int N, int block,
                            int kv_len, int32_t *counts, int32_t *indices)
{
    if (!mask || !counts || !indices) return -1;
    if (B <= 0 || H <= 0 || N <= 0 || block <= 0 || N % block != 0) return -2;
    if (kv_len < 1 || kv_len > N) return -2;
    const int nb = N / block;
    for (size_t bhi = 0; bhi < (size_t)B * H * nb; ++bhi) {
        int n = 0;
        for (int j = 0; j < nb; ++j) {
            indices[bhi * nb + j] = -1;
            if (mask[bhi * nb + j] != 0 && (long long)j * block < kv_len)
                indices[bhi * nb + n++] = j;
        }
        counts[bhi] = n;
    }
    return 0;
}

int rapid_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
