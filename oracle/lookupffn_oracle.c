/*
 * CPU oracle for the LookupFFN inference forward pass.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the method computes, used to check the GPU library and to report a host
 * baseline.  It shares no code with the GPU path and nothing in the product
 * path may call it.
 *
 * What is computed (paper notation; h = number of tables, here `k`):
 *
 *   Sec. 3.1, eq. "lookup":        y = sum_{j<k} T_j[ f_j(x) ]          (no 1/k factor)
 *   Sec. 3.1, hyperplane hash:     f_j(x) = decimal(sign(z_j)),  z_j = x R_j
 *   Sec. 3.2, "The problem":       all z_j are slices of one wide projection x R,
 *                                  cut into k consecutive tau-vectors
 *   Sec. 3.2, eq. "hadamard":      R = D_1 H D_2 H D_3 H   (D_i = +-1 diagonals,
 *                                  H = Hadamard transform), x a row vector, so
 *                                  each round flips signs first and transforms second
 *   Sec. 3.1, eq. "optimal_index": one row per table (the arg-max row = the
 *                                  sign pattern itself)
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - H is the Sylvester (natural-order) Walsh-Hadamard matrix scaled by
 *     d_pad^(-1/2); it is applied as the textbook in-place butterfly with
 *     ascending stride 1, 2, 4, ... in fp32, round-to-nearest, no fused ops.
 *   - d that is not a power of two is zero-padded at the tail to
 *     d_pad = next power of two; when k*tau > d_pad, P = ceil(k*tau/d_pad)
 *     independent projections (each with its own sign diagonals) are
 *     concatenated (this is the rule the paper's FLOP tables imply).
 *   - bit b of code j is [ z[j*tau + b] >= 0 ]  (+1 <-> 1, little-endian);
 *     +0 and -0 both give 1.
 *   - codes are 0-based, in [0, 2^tau).
 *
 * Weighted variant (Sec. 4, the form every experiment of the paper uses; the "linearly scaled"
 * version of eq. "partial_softmax" with N(z_k) = {g(z_k)}):
 *
 *   y = sum_k  <z_k,S_g> exp(<z_k,S_g>) / prod_j (exp(z_kj) + exp(-z_kj))  *  T_k[g(z_k)]
 *
 * with S_g the +-1 row selected by the code (Sec. 3.1, eq. "optimal_index").  The soft codes
 * z stay in fp32 (they are the hash's values); the weights and the weighted sum are fp64.
 *
 * BH4 hash (Sec. 3.2, eq. "block_acdc"): R = prod_{i=1..m} B_i H with block-diagonal B_i
 * (block size 16/32/64 in the paper, m = 4), applied to the row vector x left to right:
 * v <- (v B_i) H / sqrt(d_pad).  (v B)_j = sum_c v_c B[c][j] over the block of j, accumulated in
 * fp32 with one fused multiply-add per term, c ascending, starting from +0 (the order is part of
 * the definition here: fp32 addition is not associative and the sign bits are compared exactly).
 *
 * Parity pins (tests/test_oracle_*.py): dense Sylvester matrix from
 * scipy.linalg.hadamard, orthonormality, involution, closed-form inputs,
 * the arg-max form of the hash by brute force over all 2^tau sign rows,
 * fp64 dense recount of every bit, torch embedding_bag for the gather.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };
enum { ORACLE_OK = 0, ORACLE_E_ARG = -1, ORACLE_E_NOMEM = -2 };

/* host threads the token loops may use (tokens are independent, Sec. 2.1 "point-wise") */
int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* smallest power of two >= d (the padded width of one projection) */
int oracle_d_pad(int d)
{
    int p = 1;
    while (p < d) p <<= 1;
    return p;
}

/* number of independent d_pad-wide projections needed for k*tau sign bits */
int oracle_n_proj(int d, int k, int tau)
{
    int d_pad = oracle_d_pad(d);
    return (int)(((int64_t)k * tau + d_pad - 1) / d_pad);
}

/*
 * Value of an IEEE 754 binary16 bit pattern (1 sign, 5 exponent, 10 fraction bits), exact in fp32:
 *   exponent 0:      (-1)^s * fraction * 2^-24          (zero and subnormals)
 *   exponent 1..30:  (-1)^s * (1024 + fraction) * 2^(exponent - 25)
 *   exponent 31:     infinity (fraction 0) or NaN
 */
static float half_value(uint16_t h)
{
    const int s = h >> 15, e = (h >> 10) & 31, m = h & 1023;
    float v;
    if (e == 0)
        v = ldexpf((float)m, -24);
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexpf((float)(1024 + m), e - 25);
    return s ? -v : v;
}

void oracle_half_to_float(const uint16_t *h, float *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = half_value(h[i]);
}

/*
 * fp32 -> 16-bit storage, round to nearest, ties to even (for outputs kept in 16 bits).
 * bf16 keeps the top 16 bits of the fp32 pattern: add half an ulp of the kept part, plus the
 * kept part's last bit on a tie, and cut; NaN stays NaN (quiet bit set).
 */
void oracle_float_to_bf16(const float *f, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        uint32_t u;
        memcpy(&u, &f[i], 4);
        if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu))
            out[i] = (uint16_t)((u >> 16) | 0x0040u);
        else
            out[i] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
    }
}

/*
 * fp32 -> binary16, round to nearest even, by search: among the 2 * 0x7C01 finite-or-infinite
 * patterns of the value's sign, the one whose value is nearest (ties: even fraction bit).  Written as
 * the definition, not as bit tricks: the candidates are found by bisection on the magnitude
 * (half_value is monotone in the pattern for a fixed sign).
 */
void oracle_float_to_half(const float *f, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        const float v = f[i];
        if (v != v) {
            out[i] = 0x7E00;
            continue;
        }
        const uint16_t sign = signbit(v) ? 0x8000 : 0;
        const double a = fabs((double)v);
        /* largest pattern lo in [0, 0x7C00] with value <= a (0x7C00 = infinity) */
        int lo = 0, hi = 0x7C00;
        while (lo < hi) {
            const int mid = (lo + hi + 1) / 2;
            if ((double)half_value((uint16_t)mid) <= a)
                lo = mid;
            else
                hi = mid - 1;
        }
        int pick = lo;
        if (lo < 0x7C00) {
            /* beyond the largest finite value the upper neighbour counts as 2^16 (the next power of
             * two), as IEEE rounding to an unbounded exponent range prescribes */
            const double below = (double)half_value((uint16_t)lo);
            const double above = lo + 1 == 0x7C00 ? 65536.0 : (double)half_value((uint16_t)(lo + 1));
            const double dl = a - below, du = above - a;
            if (du < dl || (du == dl && (lo & 1))) pick = lo + 1;
        }
        out[i] = (uint16_t)(sign | pick);
    }
}

/* element `i` of a row stored as fp32, bf16 or binary16, widened exactly to fp32 */
static float load_elt(const void *base, int dtype, int64_t i)
{
    if (dtype == ORACLE_F32) return ((const float *)base)[i];
    if (dtype == ORACLE_F16) return half_value(((const uint16_t *)base)[i]);
    uint32_t w = (uint32_t)((const uint16_t *)base)[i] << 16; /* bf16 = top half of fp32 */
    float f;
    memcpy(&f, &w, sizeof f);
    return f;
}

/*
 * In-place unnormalised Walsh-Hadamard transform of v[0..n), n a power of two,
 * Sylvester order: out[i] = sum_j (-1)^popcount(i & j) v[j].
 * Sec. 3.2, eq. "hadamard" ("H is Hadamard transform").
 */
void oracle_fwht(float *v, int n)
{
    for (int h = 1; h < n; h <<= 1) {
        for (int b = 0; b < n; b += 2 * h) {
            for (int j = b; j < b + h; ++j) {
                float a = v[j];
                float c = v[j + h];
                v[j] = a + c;
                v[j + h] = a - c;
            }
        }
    }
}

/*
 * One structured projection of one token, Sec. 3.2 eq. "hadamard":
 *   v <- pad(x);  for r = 1..R:  v <- (v D_r) H / sqrt(d_pad)
 * signs_p points at this projection's R diagonals, [R][d_pad] int8 (+1/-1).
 * z receives the d_pad soft-hash coordinates.
 */
static void project_token(const void *x_row, int x_dtype, int d, int d_pad,
                          const int8_t *signs_p, int n_rounds, float *z)
{
    const float scale = (float)(1.0 / sqrt((double)d_pad));
    for (int i = 0; i < d; ++i) z[i] = load_elt(x_row, x_dtype, i);
    for (int i = d; i < d_pad; ++i) z[i] = 0.0f;
    for (int r = 0; r < n_rounds; ++r) {
        const int8_t *D = signs_p + (int64_t)r * d_pad;
        for (int i = 0; i < d_pad; ++i)
            if (D[i] < 0) z[i] = -z[i];
        oracle_fwht(z, d_pad);
        for (int i = 0; i < d_pad; ++i) z[i] = z[i] * scale;
    }
}

static int check_shape(int64_t n, int d, int k, int tau, int n_rounds)
{
    if (n < 0 || d < 1 || k < 1 || tau < 1 || tau > 16 || n_rounds < 1) return ORACLE_E_ARG;
    return ORACLE_OK;
}

/*
 * Soft hash codes z = x R for every token (Sec. 3.1 "soft hash code";
 * Sec. 3.2 "The problem": one wide projection for all tables).
 *   x     [n][d]              fp32 or bf16
 *   signs [P][n_rounds][d_pad] int8
 *   z     [n][P*d_pad]        fp32 out (projection 0's coordinates first)
 */
int oracle_soft_codes(const void *x, int x_dtype, const int8_t *signs, float *z,
                      int64_t n, int d, int k, int tau, int n_rounds)
{
    if (check_shape(n, d, k, tau, n_rounds) || !x || !signs || !z) return ORACLE_E_ARG;
    const int d_pad = oracle_d_pad(d);
    const int P = oracle_n_proj(d, k, tau);
    const size_t esz = x_dtype == ORACLE_F32 ? 4 : 2;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        const char *row = (const char *)x + (size_t)t * d * esz;
        for (int p = 0; p < P; ++p)
            project_token(row, x_dtype, d, d_pad,
                          signs + (int64_t)p * n_rounds * d_pad, n_rounds,
                          z + ((int64_t)t * P + p) * d_pad);
    }
    return ORACLE_OK;
}

/*
 * decimal(sign(z_j)) for one token (Sec. 3.1): table j owns coordinates
 * [j*tau, (j+1)*tau) of the concatenated projections; coordinate b of z_j is
 * bit b of the code; bit = 1 when the coordinate is >= 0.
 */
static void pack_codes(const float *z_cat, int k, int tau, uint16_t *codes)
{
    for (int j = 0; j < k; ++j) {
        unsigned c = 0;
        for (int b = 0; b < tau; ++b)
            if (z_cat[(int64_t)j * tau + b] >= 0.0f) c |= 1u << b;
        codes[j] = (uint16_t)c;
    }
}

/*
 * Hash step: codes[n][k] (uint16), code = f_j(x) of Sec. 3.1.
 */
int oracle_hash(const void *x, int x_dtype, const int8_t *signs, uint16_t *codes,
                int64_t n, int d, int k, int tau, int n_rounds)
{
    if (check_shape(n, d, k, tau, n_rounds) || !x || !signs || !codes) return ORACLE_E_ARG;
    const int d_pad = oracle_d_pad(d);
    const int P = oracle_n_proj(d, k, tau);
    const size_t esz = x_dtype == ORACLE_F32 ? 4 : 2;
    int err = 0;
#pragma omp parallel
    {
        float *z = (float *)malloc(sizeof(float) * (size_t)P * d_pad);
        if (!z) {
#pragma omp atomic write
            err = 1;
        }
#pragma omp barrier
        if (!err) {
#pragma omp for schedule(static)
            for (int64_t t = 0; t < n; ++t) {
                const char *row = (const char *)x + (size_t)t * d * esz;
                for (int p = 0; p < P; ++p)
                    project_token(row, x_dtype, d, d_pad,
                                  signs + (int64_t)p * n_rounds * d_pad, n_rounds,
                                  z + (int64_t)p * d_pad);
                pack_codes(z, k, tau, codes + t * k);
            }
        }
        free(z);
    }
    return err ? ORACLE_E_NOMEM : ORACLE_OK;
}

/*
 * Gather step, Sec. 3.1 eq. "lookup": y[t] = sum_{j<k} T_j[codes[t][j]].
 *   tables [k][2^tau][d_out] fp32 or bf16;  y [n][d_out] fp32.
 *   acc64 != 0: sum in fp64 in table order, round once to fp32 (the reference
 *               any summation order is judged against);
 *   acc64 == 0: sum in fp32 sequentially j = 0, 1, ..., k-1.
 */
int oracle_gather(const uint16_t *codes, const void *tables, int table_dtype, float *y,
                  int64_t n, int k, int tau, int d_out, int acc64)
{
    if (n < 0 || k < 1 || tau < 1 || tau > 16 || d_out < 1 || !codes || !tables || !y)
        return ORACLE_E_ARG;
    const int64_t rows = (int64_t)1 << tau;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        for (int c = 0; c < d_out; ++c) {
            double s64 = 0.0;
            float s32 = 0.0f;
            for (int j = 0; j < k; ++j) {
                int64_t code = codes[t * k + j];
                if (code >= rows) {
#pragma omp atomic write
                    bad = 1;
                    code = 0;
                }
                float e = load_elt(tables, table_dtype, ((int64_t)j * rows + code) * d_out + c);
                s64 += (double)e;
                s32 = s32 + e;
            }
            y[t * d_out + c] = acc64 ? (float)s64 : s32;
        }
    }
    return bad ? ORACLE_E_ARG : ORACLE_OK;
}

/*
 * One BH{m} projection of one token (Sec. 3.2, eq. "block_acdc"):
 *   v <- pad(x);  for i = 1..m:  u_j = sum_{c in block(j)} v_c B_i[c][j];  v <- H u / sqrt(d_pad)
 * bm_p points at this projection's m block-diagonal factors, [m][d_pad/b][b][b] fp32 with
 * element [i][blk][c][j] = B_i[blk*b + c][blk*b + j].
 */
static void project_token_bh(const void *x_row, int x_dtype, int d, int d_pad, const float *bm_p,
                             int block, int n_factors, float *z, float *tmp)
{
    const float scale = (float)(1.0 / sqrt((double)d_pad));
    for (int i = 0; i < d; ++i) z[i] = load_elt(x_row, x_dtype, i);
    for (int i = d; i < d_pad; ++i) z[i] = 0.0f;
    for (int f = 0; f < n_factors; ++f) {
        const float *Bf = bm_p + (int64_t)f * d_pad * block;
        for (int blk = 0; blk < d_pad / block; ++blk) {
            const float *Bb = Bf + (int64_t)blk * block * block;
            for (int j = 0; j < block; ++j) {
                float acc = 0.0f;
                for (int c = 0; c < block; ++c) acc = fmaf(z[blk * block + c], Bb[c * block + j], acc);
                tmp[blk * block + j] = acc;
            }
        }
        oracle_fwht(tmp, d_pad);
        for (int i = 0; i < d_pad; ++i) z[i] = tmp[i] * scale;
    }
}

static int check_bh(int64_t n, int d, int k, int tau, int block, int n_factors)
{
    if (check_shape(n, d, k, tau, n_factors)) return ORACLE_E_ARG;
    if (block < 1 || (block & (block - 1)) || block > oracle_d_pad(d)) return ORACLE_E_ARG;
    return ORACLE_OK;
}

/*
 * BH{m} soft codes and hash codes for every token; same conventions as oracle_soft_codes /
 * oracle_hash with the sign diagonals replaced by
 *   bmats [P][n_factors][d_pad/block][block][block] fp32.
 * z (may be NULL) receives [n][P*d_pad]; codes (may be NULL) receives [n][k].
 */
int oracle_bh_hash(const void *x, int x_dtype, const float *bmats, float *z, uint16_t *codes, int64_t n, int d,
                   int k, int tau, int block, int n_factors)
{
    if (check_bh(n, d, k, tau, block, n_factors) || !x || !bmats || (!z && !codes)) return ORACLE_E_ARG;
    const int d_pad = oracle_d_pad(d);
    const int P = oracle_n_proj(d, k, tau);
    const size_t esz = x_dtype == ORACLE_F32 ? 4 : 2;
    int err = 0;
#pragma omp parallel
    {
        float *zt = (float *)malloc(sizeof(float) * (size_t)(P + 1) * d_pad);
        if (!zt) {
#pragma omp atomic write
            err = 1;
        }
#pragma omp barrier
        if (!err) {
#pragma omp for schedule(static)
            for (int64_t t = 0; t < n; ++t) {
                const char *row = (const char *)x + (size_t)t * d * esz;
                for (int p = 0; p < P; ++p)
                    project_token_bh(row, x_dtype, d, d_pad, bmats + (int64_t)p * n_factors * d_pad * block, block,
                                     n_factors, zt + (int64_t)p * d_pad, zt + (int64_t)P * d_pad);
                if (z) memcpy(z + t * P * d_pad, zt, sizeof(float) * (size_t)P * d_pad);
                if (codes) pack_codes(zt, k, tau, codes + t * k);
            }
        }
        free(zt);
    }
    return err ? ORACLE_E_NOMEM : ORACLE_OK;
}

/* Whole forward pass with the BH{m} hash: codes, then the plain gather of eq. "lookup". */
int oracle_bh_forward(const void *x, int x_dtype, const float *bmats, const void *tables, int table_dtype,
                      float *y, uint16_t *codes_out, int64_t n, int d, int k, int tau, int d_out, int block,
                      int n_factors, int acc64)
{
    if (!y || !tables || !codes_out) return ORACLE_E_ARG;
    int rc = oracle_bh_hash(x, x_dtype, bmats, NULL, codes_out, n, d, k, tau, block, n_factors);
    if (rc == ORACLE_OK) rc = oracle_gather(codes_out, tables, table_dtype, y, n, k, tau, d_out, acc64);
    return rc;
}

/*
 * Gather weights from given soft codes (Sec. 4, weighted variant above), literally:
 *   s_k = <z_k, S_g>,  S_g[b] = +1 where z_k[b] >= 0 else -1   (the row the code selects)
 *   w_k = s_k * exp(s_k) / prod_b (exp(z_k[b]) + exp(-z_k[b]))
 *   z [n][zstride] fp32 (table k owns coordinates [k*tau, (k+1)*tau));  w [n][k] fp64.
 * The product in the denominator is the closed form of sum_i exp(<z_k, S_i>) over all
 * 2^tau sign rows (Sec. 3.1, the identity after eq. "full_softmax").
 */
int oracle_weights_from_z(const float *z, int64_t zstride, double *w, int64_t n, int k, int tau)
{
    if (n < 0 || k < 1 || tau < 1 || tau > 16 || zstride < (int64_t)k * tau || !z || !w) return ORACLE_E_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        for (int j = 0; j < k; ++j) {
            const float *zk = z + t * zstride + (int64_t)j * tau;
            double s = 0.0, denom = 1.0;
            for (int b = 0; b < tau; ++b) {
                const double zb = (double)zk[b];
                s += (zk[b] >= 0.0f) ? zb : -zb;
                denom *= exp(zb) + exp(-zb);
            }
            w[t * k + j] = s * exp(s) / denom;
        }
    }
    return ORACLE_OK;
}

/* Weights for every token: Hash (fp32) then oracle_weights_from_z. */
int oracle_weights(const void *x, int x_dtype, const int8_t *signs, double *w, int64_t n, int d, int k,
                   int tau, int n_rounds)
{
    if (check_shape(n, d, k, tau, n_rounds) || !x || !signs || !w) return ORACLE_E_ARG;
    const int64_t zs = (int64_t)oracle_n_proj(d, k, tau) * oracle_d_pad(d);
    float *z = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1) * zs);
    if (!z) return ORACLE_E_NOMEM;
    int rc = oracle_soft_codes(x, x_dtype, signs, z, n, d, k, tau, n_rounds);
    if (rc == ORACLE_OK) rc = oracle_weights_from_z(z, zs, w, n, k, tau);
    free(z);
    return rc;
}

/*
 * Weighted gather (Sec. 4): y[t] = sum_j w[t][j] * T_j[codes[t][j]], accumulated in fp64 in
 * table order and rounded once to fp32.
 */
int oracle_gather_weighted(const uint16_t *codes, const double *w, const void *tables, int table_dtype,
                           float *y, int64_t n, int k, int tau, int d_out)
{
    if (n < 0 || k < 1 || tau < 1 || tau > 16 || d_out < 1 || !codes || !w || !tables || !y)
        return ORACLE_E_ARG;
    const int64_t rows = (int64_t)1 << tau;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        for (int c = 0; c < d_out; ++c) {
            double s = 0.0;
            for (int j = 0; j < k; ++j) {
                int64_t code = codes[t * k + j];
                if (code >= rows) {
#pragma omp atomic write
                    bad = 1;
                    code = 0;
                }
                s += w[t * k + j] * (double)load_elt(tables, table_dtype, ((int64_t)j * rows + code) * d_out + c);
            }
            y[t * d_out + c] = (float)s;
        }
    }
    return bad ? ORACLE_E_ARG : ORACLE_OK;
}

/* Whole weighted forward pass (Sec. 4): codes, weights, weighted gather.  w_out may be NULL. */
int oracle_forward_weighted(const void *x, int x_dtype, const int8_t *signs, const void *tables,
                            int table_dtype, float *y, uint16_t *codes_out, double *w_out, int64_t n,
                            int d, int k, int tau, int d_out, int n_rounds)
{
    if (check_shape(n, d, k, tau, n_rounds) || !y || !tables || !codes_out) return ORACLE_E_ARG;
    double *w = w_out;
    if (!w) {
        w = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * k);
        if (!w) return ORACLE_E_NOMEM;
    }
    int rc = oracle_hash(x, x_dtype, signs, codes_out, n, d, k, tau, n_rounds);
    if (rc == ORACLE_OK) rc = oracle_weights(x, x_dtype, signs, w, n, d, k, tau, n_rounds);
    if (rc == ORACLE_OK) rc = oracle_gather_weighted(codes_out, w, tables, table_dtype, y, n, k, tau, d_out);
    if (!w_out) free(w);
    return rc;
}

/*
 * Multi-probe lookup (Sec. 3.1, eq. "partial_softmax") with the neighbourhood
 *   N(z_k) = { i : || S_i - sign(z_k) ||_0 <= 1 }
 * i.e. the row g(z_k) and the tau rows one sign flip away from it ("sampled according to the l0
 * difference"), each weighted by its soft-max share:
 *   y = sum_k sum_{i in N(z_k)} exp(<z_k,S_i>) T_k[i] / prod_j (exp(z_kj) + exp(-z_kj)).
 * Probe order per table: g, then g with bit 0 flipped, bit 1 flipped, ...  The soft codes z are the
 * hash's fp32 values; weights and sums are fp64.
 *   z [n][zstride] fp32;  codes (out, may be NULL) [n][k];  p (out, may be NULL) [n][k][1+tau] fp64
 */
int oracle_probe_weights_from_z(const float *z, int64_t zstride, uint16_t *codes, double *p, int64_t n, int k, int tau)
{
    if (n < 0 || k < 1 || tau < 1 || tau > 16 || zstride < (int64_t)k * tau || !z) return ORACLE_E_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        for (int j = 0; j < k; ++j) {
            const float *zk = z + t * zstride + (int64_t)j * tau;
            unsigned g = 0;
            double denom = 1.0;
            for (int b = 0; b < tau; ++b) {
                if (zk[b] >= 0.0f) g |= 1u << b;
                denom *= exp((double)zk[b]) + exp(-(double)zk[b]);
            }
            if (codes) codes[t * k + j] = (uint16_t)g;
            if (!p) continue;
            for (int probe = 0; probe <= tau; ++probe) {
                const unsigned i = probe == 0 ? g : g ^ (1u << (probe - 1));
                double score = 0.0;  /* <z_k, S_i>, S_i[b] = +1 where bit b of i is set, else -1 */
                for (int b = 0; b < tau; ++b) score += ((i >> b) & 1u) ? (double)zk[b] : -(double)zk[b];
                p[(t * k + j) * (tau + 1) + probe] = exp(score) / denom;
            }
        }
    }
    return ORACLE_OK;
}

/* y[t] = sum_j sum_probe p[t][j][probe] * T_j[row(probe)], fp64 accumulation, one rounding. */
int oracle_gather_probes(const uint16_t *codes, const double *p, const void *tables, int table_dtype, float *y,
                         int64_t n, int k, int tau, int d_out)
{
    if (n < 0 || k < 1 || tau < 1 || tau > 16 || d_out < 1 || !codes || !p || !tables || !y) return ORACLE_E_ARG;
    const int64_t rows = (int64_t)1 << tau;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        for (int c = 0; c < d_out; ++c) {
            double s = 0.0;
            for (int j = 0; j < k; ++j) {
                int64_t g = codes[t * k + j];
                if (g >= rows) {
#pragma omp atomic write
                    bad = 1;
                    g = 0;
                }
                for (int probe = 0; probe <= tau; ++probe) {
                    const int64_t i = probe == 0 ? g : g ^ ((int64_t)1 << (probe - 1));
                    s += p[(t * k + j) * (tau + 1) + probe] *
                         (double)load_elt(tables, table_dtype, ((int64_t)j * rows + i) * d_out + c);
                }
            }
            y[t * d_out + c] = (float)s;
        }
    }
    return bad ? ORACLE_E_ARG : ORACLE_OK;
}

/* Whole multi-probe forward pass: sign-diagonal hash (fp32 z), probe weights, weighted sum. */
int oracle_forward_probes(const void *x, int x_dtype, const int8_t *signs, const void *tables, int table_dtype,
                          float *y, uint16_t *codes_out, double *p_out, int64_t n, int d, int k, int tau, int d_out,
                          int n_rounds)
{
    if (check_shape(n, d, k, tau, n_rounds) || !y || !tables || !codes_out) return ORACLE_E_ARG;
    const int64_t zs = (int64_t)oracle_n_proj(d, k, tau) * oracle_d_pad(d);
    const size_t cnt = (size_t)(n > 0 ? n : 1);
    float *z = (float *)malloc(sizeof(float) * cnt * zs);
    double *p = p_out ? p_out : (double *)malloc(sizeof(double) * cnt * k * (tau + 1));
    int rc = (z && p) ? ORACLE_OK : ORACLE_E_NOMEM;
    if (rc == ORACLE_OK) rc = oracle_soft_codes(x, x_dtype, signs, z, n, d, k, tau, n_rounds);
    if (rc == ORACLE_OK) rc = oracle_probe_weights_from_z(z, zs, codes_out, p, n, k, tau);
    if (rc == ORACLE_OK) rc = oracle_gather_probes(codes_out, p, tables, table_dtype, y, n, k, tau, d_out);
    free(z);
    if (!p_out) free(p);
    return rc;
}

/*
 * Whole forward pass: Hash then Gather (Sec. 3.1 "Two main operations").
 * codes_out may be NULL.
 */
int oracle_forward(const void *x, int x_dtype, const int8_t *signs, const void *tables,
                   int table_dtype, float *y, uint16_t *codes_out, int64_t n, int d, int k,
                   int tau, int d_out, int n_rounds, int acc64)
{
    if (check_shape(n, d, k, tau, n_rounds) || !y || !tables) return ORACLE_E_ARG;
    uint16_t *codes = codes_out;
    if (!codes) {
        codes = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)(n > 0 ? n : 1) * k);
        if (!codes) return ORACLE_E_NOMEM;
    }
    int rc = oracle_hash(x, x_dtype, signs, codes, n, d, k, tau, n_rounds);
    if (rc == ORACLE_OK)
        rc = oracle_gather(codes, tables, table_dtype, y, n, k, tau, d_out, acc64);
    if (!codes_out) free(codes);
    return rc;
}
