/* Runs every entry point of the CPU oracle on small, ragged and extreme shapes.  Built with
 * -fsanitize=address,undefined by tests/test_sanitizers.py: any out-of-bounds access, use of
 * uninitialised heap, signed overflow or misaligned access inside the oracle ends the run with a
 * report and a non-zero exit status.  The inputs are filled by a small LCG; no values are checked
 * here (the oracle's pins do that), only that it runs clean. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_d_pad(int d);
int oracle_n_proj(int d, int k, int tau);
void oracle_set_threads(int n);
int oracle_hash(const void *x, int x_dtype, const int8_t *signs, uint16_t *codes, int64_t n, int d, int k, int tau,
                int n_rounds);
int oracle_forward(const void *x, int x_dtype, const int8_t *signs, const void *tables, int table_dtype, float *y,
                   uint16_t *codes_out, int64_t n, int d, int k, int tau, int d_out, int n_rounds, int acc64);
int oracle_forward_weighted(const void *x, int x_dtype, const int8_t *signs, const void *tables, int table_dtype,
                            float *y, uint16_t *codes_out, double *w_out, int64_t n, int d, int k, int tau,
                            int d_out, int n_rounds);
int oracle_forward_probes(const void *x, int x_dtype, const int8_t *signs, const void *tables, int table_dtype,
                          float *y, uint16_t *codes_out, double *p_out, int64_t n, int d, int k, int tau, int d_out,
                          int n_rounds);
int oracle_bh_forward(const void *x, int x_dtype, const float *bmats, const void *tables, int table_dtype, float *y,
                      uint16_t *codes_out, int64_t n, int d, int k, int tau, int d_out, int block, int n_factors,
                      int acc64);

static uint32_t lcg = 12345u;
static uint32_t next(void) { return lcg = lcg * 1664525u + 1013904223u; }
static float unit(void) { return (float)(next() >> 8) / 8388608.0f - 1.0f; }

static int run(int64_t n, int d, int k, int tau, int d_out, int rounds, int x16, int t16, int block)
{
    const int d_pad = oracle_d_pad(d), P = oracle_n_proj(d, k, tau);
    const size_t rows = (size_t)1 << tau;
    /* exact-size heap buffers: one element past any of them is a sanitizer report */
    void *x = malloc((size_t)(n ? n : 1) * d * (x16 ? 2 : 4));
    int8_t *signs = malloc((size_t)P * rounds * d_pad);
    void *tables = malloc((size_t)k * rows * d_out * (t16 ? 2 : 4));
    float *y = malloc(sizeof(float) * (size_t)(n ? n : 1) * d_out);
    uint16_t *codes = malloc(sizeof(uint16_t) * (size_t)(n ? n : 1) * k);
    float *bm = malloc(sizeof(float) * (size_t)P * 4 * d_pad * block);
    if (!x || !signs || !tables || !y || !codes || !bm) return 99;
    for (size_t i = 0; i < (size_t)n * d; ++i) {
        const float v = unit() * 2.0f;
        if (x16) {
            uint32_t u;
            memcpy(&u, &v, 4);
            ((uint16_t *)x)[i] = (uint16_t)(u >> 16);
        } else
            ((float *)x)[i] = v;
    }
    for (size_t i = 0; i < (size_t)P * rounds * d_pad; ++i) signs[i] = (next() & 0x10000) ? 1 : -1;
    for (size_t i = 0; i < (size_t)k * rows * d_out; ++i) {
        const float v = unit() * 0.02f;
        if (t16) {
            uint32_t u;
            memcpy(&u, &v, 4);
            ((uint16_t *)tables)[i] = (uint16_t)(u >> 16);
        } else
            ((float *)tables)[i] = v;
    }
    for (size_t i = 0; i < (size_t)P * 4 * d_pad * block; ++i) bm[i] = unit() * 0.25f;
    int rc = oracle_hash(x, x16, signs, codes, n, d, k, tau, rounds);
    for (int acc64 = 0; acc64 < 2 && !rc; ++acc64)
        rc = oracle_forward(x, x16, signs, tables, t16, y, codes, n, d, k, tau, d_out, rounds, acc64);
    if (!rc) rc = oracle_forward_weighted(x, x16, signs, tables, t16, y, codes, NULL, n, d, k, tau, d_out, rounds);
    if (!rc) rc = oracle_forward_probes(x, x16, signs, tables, t16, y, codes, NULL, n, d, k, tau, d_out, rounds);
    if (!rc && block <= d_pad) rc = oracle_bh_forward(x, x16, bm, tables, t16, y, codes, n, d, k, tau, d_out, block, 4, 1);
    free(x);
    free(signs);
    free(tables);
    free(y);
    free(codes);
    free(bm);
    if (rc) printf("oracle returned %d for n=%lld d=%d k=%d tau=%d d_out=%d\n", rc, (long long)n, d, k, tau, d_out);
    return rc;
}

int main(void)
{
    int rc = 0;
    for (int threads = 1; threads <= 3 && !rc; threads += 2) {
        oracle_set_threads(threads);
        rc = run(64, 64, 8, 8, 64, 2, 0, 0, 16);                 /* the tiny configuration */
        if (!rc) rc = run(5, 48, 6, 8, 12, 3, 0, 1, 16);         /* padded width, bf16 rows */
        if (!rc) rc = run(7, 100, 20, 5, 8, 3, 1, 0, 32);        /* d_pad = 128, bf16 input */
        if (!rc) rc = run(3, 200, 30, 13, 4, 1, 0, 0, 64);       /* two projections, a code straddles them */
        if (!rc) rc = run(2, 64, 4, 16, 4, 2, 0, 0, 16);         /* widest code */
        if (!rc) rc = run(1, 1, 1, 1, 4, 1, 0, 0, 1);            /* the smallest of everything */
        if (!rc) rc = run(0, 64, 8, 8, 64, 2, 0, 0, 16);         /* an empty batch */
        if (!rc) rc = run(33, 768, 96, 8, 8, 3, 0, 0, 64);       /* the benchmark's hash shape, narrow rows */
    }
    printf(rc ? "FAILED\n" : "oracle ran clean\n");
    return rc;
}
