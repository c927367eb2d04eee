/* Driver for a sanitizer build of the C oracle: runs every routine on small seeded inputs, over all the
 * argument forms the tests use (row subsets, (b,h) subsets, optional outputs, both input types), and prints
 * the results in full precision; the Python test compares them with the ordinary build's. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int loma_oracle_mask_attn(const void*, const void*, const void*, double*, double*, int, int, int, int, int, int, double,
                          int, const int*, int, int);
int loma_oracle_mask_attn_bwd(const void*, const void*, const void*, const void*, double*, double*, double*, int, int, int,
                              int, int, int, double, int, int);
int loma_oracle_attend_segments(const void*, int, const void*, const void*, long, int, const void*, const void*, long, int,
                                double*, double*, int, int, int, double, int, const int*, int, int);

static uint32_t state = 9486u;
static float next_float(void) {                 /* small LCG: values in [-1, 1) */
    state = state * 1664525u + 1013904223u;
    return (float)((int32_t)state) / 2147483648.0f;
}
static void dump(const char* name, const double* x, size_t n) {
    printf("%s", name);
    for (size_t i = 0; i < n; ++i) printf(" %.17g", x[i]);
    printf("\n");
}

int main(void) {
    const int B = 2, H = 2, d = 8, t = 2, c = 3, n = 3;
    const int R = t * c, s = 2 * R + t, S = n * s;
    const size_t N = (size_t)B * H * S * d;
    float* f = malloc(sizeof(float) * N * 4);
    uint16_t* h = malloc(sizeof(uint16_t) * N * 4);
    if (!f || !h) return 2;
    for (size_t i = 0; i < 4 * N; ++i) {
        f[i] = next_float();
        union { float x; uint32_t u; } cv = {f[i]};
        h[i] = (uint16_t)(cv.u >> 16);             /* truncation is fine here: any bf16 pattern will do */
    }
    double* out = malloc(sizeof(double) * N);
    double* lse = malloc(sizeof(double) * (size_t)B * H * S);
    double* g[3] = {malloc(sizeof(double) * N), malloc(sizeof(double) * N), malloc(sizeof(double) * N)};
    if (!out || !lse || !g[0] || !g[1] || !g[2]) return 2;
    for (int dtype = 0; dtype < 2; ++dtype) {
        const void* q = dtype ? (const void*)h : (const void*)f;
        const void* k = dtype ? (const void*)(h + N) : (const void*)(f + N);
        const void* v = dtype ? (const void*)(h + 2 * N) : (const void*)(f + 2 * N);
        const void* go = dtype ? (const void*)(h + 3 * N) : (const void*)(f + 3 * N);
        if (loma_oracle_mask_attn(q, k, v, out, lse, B, H, d, t, c, n, 0.35, dtype, NULL, 0, 3)) return 3;
        dump("mask_out", out, N);
        dump("mask_lse", lse, (size_t)B * H * S);
        const int rows[5] = {0, R - 1, R, R + t, S - 1};
        if (loma_oracle_mask_attn(q, k, v, out, NULL, B, H, d, t, c, n, 0.35, dtype, rows, 5, 1)) return 3;
        dump("mask_rows", out, (size_t)B * H * 5 * d);
        if (loma_oracle_mask_attn_bwd(q, k, v, go, g[0], g[1], g[2], B, H, d, t, c, n, 0.35, dtype, 2)) return 3;
        dump("dq", g[0], N); dump("dk", g[1], N); dump("dv", g[2], N);
        /* generation form: [B, H, S, d] buffers read as caches of S rows, n1 + n2 keys, Lq queries */
        const int bh[2] = {3, 0};
        if (loma_oracle_attend_segments(q, 1, k, v, S, 7, v, k, S, 4, out, lse, B, H, d, 0.35, dtype, NULL, 0, 2)) return 3;
        dump("decode_out", out, (size_t)B * H * d); dump("decode_lse", lse, (size_t)B * H);
        if (loma_oracle_attend_segments(q, t, k, v, S, R, v, k, S, t, out, NULL, B, H, d, 0.35, dtype, bh, 2, 1)) return 3;
        dump("compress_out", out, (size_t)2 * t * d);
        if (loma_oracle_attend_segments(q, 1, NULL, NULL, 0, 0, v, k, S, 1, out, lse, B, H, d, 0.35, dtype, NULL, 0, 0)) return 3;
        dump("single_key", out, (size_t)B * H * d);
    }
    /* rejected argument sets: no access may happen */
    if (loma_oracle_mask_attn(NULL, f, f, out, NULL, B, H, d, t, c, n, 1.0, 0, NULL, 0, 0) != -1) return 4;
    const int bad_row[1] = {S};
    if (loma_oracle_mask_attn(f, f, f, out, NULL, B, H, d, t, c, n, 1.0, 0, bad_row, 1, 0) != -1) return 4;
    const int bad_bh[1] = {B * H};
    if (loma_oracle_attend_segments(f, 1, f, f, S, 2, NULL, NULL, 0, 0, out, NULL, B, H, d, 1.0, 0, bad_bh, 1, 0) != -1) return 4;
    if (loma_oracle_attend_segments(f, 1, f, f, 1, 2, NULL, NULL, 0, 0, out, NULL, B, H, d, 1.0, 0, NULL, 0, 0) != -1) return 4;
    free(f); free(h); free(out); free(lse); free(g[0]); free(g[1]); free(g[2]);
    printf("oracle driver ok\n");
    return 0;
}
