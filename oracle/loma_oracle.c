/*
 * CPU fp64 oracle for LoMA attention, scalable variant -- TEST INFRASTRUCTURE.
 *
 * Same definition as oracle/loma_oracle.py, written so the large configurations
 * finish in seconds to minutes: the 0/1 mask row of a query is still built
 * explicitly (one byte per column, from the zone rules of Sec. 4.3 / Eq. 1-3),
 * but one row at a time instead of as an S x S array, and every masked pair is
 * left out of the softmax (Eq. 5-7).  No tiling, no skipping derived from the
 * block structure, no fusion: for each row, for each column with mask 1, one
 * dot product, then a max, exps, a sum and a weighted sum of V rows.
 *
 * Inputs are float32 or bf16 bit patterns (uint16); both widen exactly to fp64.
 * All arithmetic is fp64 with libm exp/log.  OpenMP splits independent rows
 * (mask pass) or independent (b, h) pairs (generation form) over host threads.
 *
 * This file shares nothing with the HIP library.  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may load it.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F32 0
#define ORACLE_BF16 1

enum { Z_READ = 0, Z_MEM = 1, Z_REP = 2 };

static inline double elem(const void* base, size_t idx, int dtype) {
    if (dtype == ORACLE_F32) return (double)((const float*)base)[idx];
    uint32_t bits = ((uint32_t)((const uint16_t*)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static void widen_row(const void* base, size_t row, int d, int dtype, double* dst) {
    for (int e = 0; e < d; ++e) dst[e] = elem(base, row * (size_t)d + e, dtype);
}

/* zone of an in-chunk offset, chunk = [read tc | mem t | rep tc] (Sec. 4.1) */
static inline int zone_of(int o, int R, int t) { return o < R ? Z_READ : (o < R + t ? Z_MEM : Z_REP); }

/* Fill mask[0..S) for query row p: Eq. 1 inside the chunk, Eq. 3 against earlier chunks. */
static void build_mask_row(int p, int t, int c, int n, const int* col_chunk, const int* col_zone,
                           const int* col_off, uint8_t* mask) {
    const int R = t * c, s = 2 * R + t, S = n * s;
    const int y = p / s, o = p % s, z = zone_of(o, R, t);
    for (int q = 0; q < S; ++q) {
        int vis;
        if (z == Z_READ) {
            if (col_chunk[q] < y) vis = (col_zone[q] == Z_MEM);              /* S block */
            else vis = (col_chunk[q] == y && col_zone[q] == Z_READ && col_off[q] <= o); /* L block */
        } else if (z == Z_MEM) {
            vis = (col_chunk[q] == y && col_zone[q] != Z_REP);               /* [1 1 0] */
        } else {
            vis = (col_chunk[q] == y && (col_zone[q] == Z_MEM || q == p));   /* [0 1 I] */
        }
        mask[q] = (uint8_t)vis;
    }
}

/* softmax(scale * q.K^T over listed keys) V for one query; keys given by row indices. */
static void attend_one(const double* qrow, const void* k, const void* v, int dtype, size_t base_row,
                       const int* key_rows, int nkeys, int d, double scale,
                       double* scores, double* krow, double* out, double* lse) {
    double mx = -INFINITY;
    for (int j = 0; j < nkeys; ++j) {
        widen_row(k, base_row + (size_t)key_rows[j], d, dtype, krow);
        double acc = 0.0;
        for (int e = 0; e < d; ++e) acc += qrow[e] * krow[e];
        scores[j] = acc * scale;
        if (scores[j] > mx) mx = scores[j];
    }
    double den = 0.0;
    for (int j = 0; j < nkeys; ++j) { scores[j] = exp(scores[j] - mx); den += scores[j]; }
    for (int e = 0; e < d; ++e) out[e] = 0.0;
    for (int j = 0; j < nkeys; ++j) {
        widen_row(v, base_row + (size_t)key_rows[j], d, dtype, krow);
        const double w = scores[j] / den;
        for (int e = 0; e < d; ++e) out[e] += w * krow[e];
    }
    if (lse) *lse = mx + log(den);
}

/*
 * Mask pass.  q, k, v: [B, H, S, d], S = n * t(2c+1).  rows: nrows query indices in [0, S)
 * (NULL = all S rows, nrows ignored).  out: [B, H, nrows, d] fp64; lse: [B, H, nrows] or NULL.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int loma_oracle_mask_attn(const void* q, const void* k, const void* v, double* out, double* lse,
                          int B, int H, int d, int t, int c, int n, double scale, int dtype,
                          const int* rows, int nrows, int nthreads) {
    if (!q || !k || !v || !out || B < 1 || H < 1 || d < 1 || t < 1 || c < 1 || n < 1) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
    const int R = t * c, s = 2 * R + t, S = n * s;
    if (!rows) nrows = S;
    for (int i = 0; rows && i < nrows; ++i) if (rows[i] < 0 || rows[i] >= S) return -1;
    int* col_chunk = malloc(sizeof(int) * S);
    int* col_zone = malloc(sizeof(int) * S);
    int* col_off = malloc(sizeof(int) * S);
    if (!col_chunk || !col_zone || !col_off) { free(col_chunk); free(col_zone); free(col_off); return -1; }
    for (int x = 0; x < S; ++x) { col_chunk[x] = x / s; col_off[x] = x % s; col_zone[x] = zone_of(x % s, R, t); }
    int failed = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
#pragma omp parallel
    {
        uint8_t* mask = malloc((size_t)S);
        int* key_rows = malloc(sizeof(int) * S);
        double* scores = malloc(sizeof(double) * S);
        double* qrow = malloc(sizeof(double) * d);
        double* krow = malloc(sizeof(double) * d);
        if (!mask || !key_rows || !scores || !qrow || !krow) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(dynamic, 4)
            for (int i = 0; i < nrows; ++i) {
                const int p = rows ? rows[i] : i;
                build_mask_row(p, t, c, n, col_chunk, col_zone, col_off, mask);
                int nk = 0;
                for (int x = 0; x < S; ++x) if (mask[x]) key_rows[nk++] = x;
                for (int bh = 0; bh < B * H; ++bh) {
                    const size_t base = (size_t)bh * S;
                    widen_row(q, base + p, d, dtype, qrow);
                    attend_one(qrow, k, v, dtype, base, key_rows, nk, d, scale, scores, krow,
                               out + ((size_t)bh * nrows + i) * d, lse ? lse + (size_t)bh * nrows + i : NULL);
                }
            }
        }
        free(mask); free(key_rows); free(scores); free(qrow); free(krow);
    }
    free(col_chunk); free(col_zone); free(col_off);
    return failed ? -1 : 0;
}

/*
 * Gradients of the mask pass for an upstream gradient dout of the output (Sec. 4.4, Eq. 5-7
 * differentiated; masked pairs have weight 0 and carry nothing).  Row by row, with the row's mask
 * written out explicitly as in the forward routine: weights w_j = softmax over the visible keys,
 * o = sum_j w_j v_j, delta = dout . o, and for every visible key j
 *     da_j = w_j (dout . v_j - delta);  dq += scale da_j k_j;  dk_j += scale da_j q;  dv_j += w_j dout.
 * One thread owns a (b, h) pair, so the sums into dk/dv need no atomics.
 * q, k, v, dout: [B, H, S, d] (float32 or bf16 bits); dq, dk, dv: [B, H, S, d] fp64.
 */
int loma_oracle_mask_attn_bwd(const void* q, const void* k, const void* v, const void* dout,
                              double* dq, double* dk, double* dv,
                              int B, int H, int d, int t, int c, int n, double scale, int dtype, int nthreads) {
    if (!q || !k || !v || !dout || !dq || !dk || !dv || B < 1 || H < 1 || d < 1 || t < 1 || c < 1 || n < 1) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
    const int R = t * c, s = 2 * R + t, S = n * s;
    int* col_chunk = malloc(sizeof(int) * S);
    int* col_zone = malloc(sizeof(int) * S);
    int* col_off = malloc(sizeof(int) * S);
    if (!col_chunk || !col_zone || !col_off) { free(col_chunk); free(col_zone); free(col_off); return -1; }
    for (int x = 0; x < S; ++x) { col_chunk[x] = x / s; col_off[x] = x % s; col_zone[x] = zone_of(x % s, R, t); }
    memset(dk, 0, sizeof(double) * (size_t)B * H * S * d);
    memset(dv, 0, sizeof(double) * (size_t)B * H * S * d);
    int failed = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
#pragma omp parallel
    {
        uint8_t* mask = malloc((size_t)S);
        int* key_rows = malloc(sizeof(int) * S);
        double* w = malloc(sizeof(double) * S);
        double* qrow = malloc(sizeof(double) * d);
        double* krow = malloc(sizeof(double) * d);
        double* grow = malloc(sizeof(double) * d);
        double* orow = malloc(sizeof(double) * d);
        if (!mask || !key_rows || !w || !qrow || !krow || !grow || !orow) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int bh = 0; bh < B * H; ++bh) {
                const size_t base = (size_t)bh * S;
                for (int p = 0; p < S; ++p) {
                    build_mask_row(p, t, c, n, col_chunk, col_zone, col_off, mask);
                    int nk = 0;
                    for (int x = 0; x < S; ++x) if (mask[x]) key_rows[nk++] = x;
                    widen_row(q, base + p, d, dtype, qrow);
                    widen_row(dout, base + p, d, dtype, grow);
                    attend_one(qrow, k, v, dtype, base, key_rows, nk, d, scale, w, krow, orow, NULL);
                    /* attend_one leaves exp(score - max) in w; normalise to the weights */
                    double den = 0.0;
                    for (int j = 0; j < nk; ++j) den += w[j];
                    double delta = 0.0;
                    for (int e = 0; e < d; ++e) delta += grow[e] * orow[e];
                    double* dqp = dq + (base + p) * (size_t)d;
                    for (int e = 0; e < d; ++e) dqp[e] = 0.0;
                    for (int j = 0; j < nk; ++j) {
                        const size_t kr = base + (size_t)key_rows[j];
                        const double wj = w[j] / den;
                        widen_row(v, kr, d, dtype, krow);
                        double dw = 0.0;
                        for (int e = 0; e < d; ++e) dw += grow[e] * krow[e];
                        double* dvp = dv + kr * (size_t)d;
                        for (int e = 0; e < d; ++e) dvp[e] += wj * grow[e];
                        const double da = wj * (dw - delta) * scale;
                        widen_row(k, kr, d, dtype, krow);
                        double* dkp = dk + kr * (size_t)d;
                        for (int e = 0; e < d; ++e) { dqp[e] += da * krow[e]; dkp[e] += da * qrow[e]; }
                    }
                }
            }
        }
        free(mask); free(key_rows); free(w); free(qrow); free(krow); free(grow); free(orow);
    }
    free(col_chunk); free(col_zone); free(col_off);
    return failed ? -1 : 0;
}

/*
 * Generation form, attention of Lq queries over an explicit key list made of two
 * segments (all pairs visible: the appendix masks for one new token, and for the
 * <m> pass, are all ones).  Per (b, h):
 *   queries  q   [B, H, Lq, d]
 *   segment1 k1/v1 rows [0, n1) of a buffer with stride1 rows per (b, h)
 *   segment2 k2/v2 rows [0, n2) of a buffer with stride2 rows per (b, h)
 * decode:   Lq = 1, segment1 = memory cache (n1 = n_mem_chunks*t), segment2 = reading zone
 *           INCLUDING the new token (n2 = fill).
 * compress: Lq = t, segment1 = reading zone (n1 = t*c), segment2 = the <m> tokens' own K/V (n2 = t).
 * bh_list: optional subset of (b*H + h) indices (NULL = all); out: [nbh, Lq, d] fp64;
 * lse (optional, may be NULL): [nbh, Lq] fp64, log of the softmax denominator of Eq. 7 taken over the
 * scaled scores: max + log(sum exp(score - max)).
 */
int loma_oracle_attend_segments(const void* q, int Lq,
                                const void* k1, const void* v1, long stride1, int n1,
                                const void* k2, const void* v2, long stride2, int n2,
                                double* out, double* lse, int B, int H, int d, double scale, int dtype,
                                const int* bh_list, int nbh, int nthreads) {
    if (!q || !out || B < 1 || H < 1 || d < 1 || Lq < 1 || n1 < 0 || n2 < 0 || n1 + n2 < 1) return -1;
    if ((n1 > 0 && (!k1 || !v1 || stride1 < n1)) || (n2 > 0 && (!k2 || !v2 || stride2 < n2))) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
    if (!bh_list) nbh = B * H;
    for (int i = 0; bh_list && i < nbh; ++i) if (bh_list[i] < 0 || bh_list[i] >= B * H) return -1;
    const int L = n1 + n2;
    int failed = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
#pragma omp parallel
    {
        double* scores = malloc(sizeof(double) * L);
        double* qrow = malloc(sizeof(double) * d);
        double* krow = malloc(sizeof(double) * d);
        if (!scores || !qrow || !krow) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int i = 0; i < nbh; ++i) {
                const int bh = bh_list ? bh_list[i] : i;
                for (int r = 0; r < Lq; ++r) {
                    widen_row(q, (size_t)bh * Lq + r, d, dtype, qrow);
                    double mx = -INFINITY;
                    for (int j = 0; j < L; ++j) {
                        if (j < n1) widen_row(k1, (size_t)bh * stride1 + j, d, dtype, krow);
                        else widen_row(k2, (size_t)bh * stride2 + (j - n1), d, dtype, krow);
                        double acc = 0.0;
                        for (int e = 0; e < d; ++e) acc += qrow[e] * krow[e];
                        scores[j] = acc * scale;
                        if (scores[j] > mx) mx = scores[j];
                    }
                    double den = 0.0;
                    for (int j = 0; j < L; ++j) { scores[j] = exp(scores[j] - mx); den += scores[j]; }
                    double* o = out + ((size_t)i * Lq + r) * d;
                    for (int e = 0; e < d; ++e) o[e] = 0.0;
                    for (int j = 0; j < L; ++j) {
                        if (j < n1) widen_row(v1, (size_t)bh * stride1 + j, d, dtype, krow);
                        else widen_row(v2, (size_t)bh * stride2 + (j - n1), d, dtype, krow);
                        const double w = scores[j] / den;
                        for (int e = 0; e < d; ++e) o[e] += w * krow[e];
                    }
                    if (lse) lse[(size_t)i * Lq + r] = mx + log(den);
                }
            }
        }
        free(scores); free(qrow); free(krow);
    }
    return failed ? -1 : 0;
}

int loma_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
