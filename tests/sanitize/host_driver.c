/* Drives the host side of liblookupffn.so -- argument validation, size queries, planning arithmetic,
 * options -- through the C ABI on a machine without a GPU.  Built, like the library's host code, with
 * -fsanitize=address,undefined by tests/test_sanitizers.py.  Every call here returns before its first HIP
 * call (bad arguments, empty batches, pure size queries), so no device is needed; the pointers are
 * stand-ins that are never dereferenced. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "lookupffn.h"

#define FAKE ((void *)(uintptr_t)(1u << 20))
static int failures = 0;
#define EXPECT(expr, want)                                                              \
    do {                                                                                \
        long long got_ = (long long)(expr), want_ = (long long)(want);                  \
        if (got_ != want_) {                                                            \
            printf("%s:%d: %s = %lld, expected %lld\n", __FILE__, __LINE__, #expr, got_, want_); \
            ++failures;                                                                 \
        }                                                                               \
    } while (0)

int main(void)
{
    /* size queries over a sweep of shapes, including the extremes the validation admits */
    const int ks[] = {1, 2, 7, 96, 128, 170, 1 << 20};
    const int taus[] = {1, 7, 8, 9, 10, 13, 16};
    const int64_t ns[] = {0, 1, 8, 1000, 16384, 65536, (int64_t)1 << 31, (int64_t)1 << 40};
    for (unsigned a = 0; a < sizeof ks / sizeof *ks; ++a)
        for (unsigned b = 0; b < sizeof taus / sizeof *taus; ++b)
            for (unsigned c = 0; c < sizeof ns / sizeof *ns; ++c) {
                const int k = ks[a], tau = taus[b];
                const int64_t n = ns[c];
                const int64_t w0 = lookupffn_workspace_bytes(n, k), w1 = lookupffn_workspace_bytes_weighted(n, k),
                              w2 = lookupffn_workspace_bytes_probes(n, k, tau), g0 = lookupffn_workspace_bytes_gather(n, k),
                              g1 = lookupffn_workspace_bytes_gather_weighted(n, k),
                              g2 = lookupffn_workspace_bytes_gather_probes(n, k, tau);
                if (w0 < 0 || w1 < w0 || w2 < w0 || g0 < 0 || g1 < g0 || g2 < g0 || (n == 0 && (w0 | w1 | w2 | g0 | g1 | g2))) {
                    printf("size query out of order: n=%lld k=%d tau=%d\n", (long long)n, k, tau);
                    ++failures;
                }
                for (int d_out = 4; d_out <= 4096; d_out *= 4)
                    if (lookupffn_prepared_tables_bytes(k, tau, d_out, LFFN_F32) < 0) ++failures;
                for (int block = 16; block <= 64; block *= 2) {
                    (void)lookupffn_workspace_bytes_bh(n, 768, k, tau, block, 4);
                    (void)lookupffn_workspace_bytes_bh_weighted(n, 768, k, tau, block | LFFN_PREPARED, 4);
                    (void)lookupffn_prepared_bh_bytes(768, k, tau, block, 4);
                }
            }
    /* argument validation of every entry point: errors and empty batches return before any HIP call */
    EXPECT(lookupffn_hash(FAKE, FAKE, FAKE, 0, 768, 96, 8, 3, LFFN_F32, NULL), LFFN_OK);
    EXPECT(lookupffn_hash(NULL, FAKE, FAKE, 5, 768, 96, 8, 3, LFFN_F32, NULL), LFFN_E_NULL);
    EXPECT(lookupffn_hash(FAKE, FAKE, FAKE, 5, 768, 96, 17, 3, LFFN_F32, NULL), LFFN_E_TAU);
    EXPECT(lookupffn_hash(FAKE, FAKE, FAKE, 5, 5000, 96, 8, 3, LFFN_F32, NULL), LFFN_E_UNSUPPORTED);
    EXPECT(lookupffn_hash(FAKE, FAKE, FAKE, -1, 768, 96, 8, 3, LFFN_F32, NULL), LFFN_E_SIZE);
    EXPECT(lookupffn_gather(FAKE, FAKE, FAKE, 0, 96, 8, 768, LFFN_F32, NULL, 0, NULL), LFFN_OK);
    EXPECT(lookupffn_gather(FAKE, FAKE, FAKE, 5, 96, 8, 770, LFFN_F32, NULL, 0, NULL), LFFN_E_ALIGN);
    EXPECT(lookupffn_gather(FAKE, FAKE, FAKE, 1000, 96, 8, 768, LFFN_F32, FAKE, 16, NULL), LFFN_E_WORKSPACE);
    EXPECT(lookupffn_gather_weighted(FAKE, NULL, FAKE, FAKE, 5, 96, 8, 768, LFFN_F32, NULL, 0, NULL), LFFN_E_NULL);
    EXPECT(lookupffn_gather_probes(FAKE, FAKE, FAKE, FAKE, 0, 96, 8, 768, LFFN_BF16, NULL, 0, NULL), LFFN_OK);
    EXPECT(lookupffn_forward(FAKE, FAKE, FAKE, FAKE, 0, 768, 96, 8, 768, 3, LFFN_F32, LFFN_F32 | LFFN_PREPARED, NULL, 0, NULL), LFFN_OK);
    EXPECT(lookupffn_forward(FAKE, FAKE, FAKE, FAKE, 1000, 768, 96, 8, 768, 3, LFFN_F32, LFFN_F32, FAKE, 16, NULL), LFFN_E_WORKSPACE);
    EXPECT(lookupffn_forward_weighted(FAKE, FAKE, FAKE, FAKE, 5, 768, 96, 0, 768, 3, LFFN_F32, LFFN_F32, NULL, 0, NULL), LFFN_E_TAU);
    EXPECT(lookupffn_forward_probes(FAKE, FAKE, FAKE, FAKE, 5, 768, 96, 8, 768, 3, 9, LFFN_F32, NULL, 0, NULL), LFFN_E_DTYPE);
    EXPECT(lookupffn_forward_static(FAKE, FAKE, FAKE, FAKE, 45000, 768, 96, 8, 768, 3, LFFN_F32, LFFN_F32, NULL), LFFN_E_WORKSPACE);
    EXPECT(lookupffn_forward_static(FAKE, FAKE, FAKE, FAKE, 0, 768, 96, 8, 768, 3, LFFN_F32, LFFN_F32, NULL), LFFN_OK);
    {
        const int8_t *signs[33];
        const void *tables[33];
        for (int i = 0; i < 33; ++i) signs[i] = FAKE, tables[i] = FAKE;
        EXPECT(lookupffn_forward_stack(FAKE, signs, tables, FAKE, 0, 768, 96, 8, 768, 3, 12, LFFN_F32, LFFN_F32, NULL), LFFN_OK);
        EXPECT(lookupffn_forward_stack(FAKE, signs, tables, FAKE, 0, 768, 96, 8, 768, 3, 33, LFFN_F32, LFFN_F32, NULL), LFFN_E_SIZE);
        EXPECT(lookupffn_forward_stack(FAKE, signs, tables, FAKE, 0, 64, 8, 8, 64, 2, 1, LFFN_F32, LFFN_F32, NULL), LFFN_E_UNSUPPORTED);
        signs[5] = NULL;
        EXPECT(lookupffn_forward_stack(FAKE, signs, tables, FAKE, 4, 768, 96, 8, 768, 3, 12, LFFN_F32, LFFN_F32, NULL), LFFN_E_NULL);
    }
    EXPECT(lookupffn_hash_bh(FAKE, FAKE, FAKE, 0, 768, 96, 8, 64, 4, LFFN_F32, NULL, 0, NULL), LFFN_OK);
    EXPECT(lookupffn_hash_bh(FAKE, FAKE, FAKE, 5, 768, 96, 8, 48, 4, LFFN_F32, NULL, 0, NULL), LFFN_E_UNSUPPORTED);
    EXPECT(lookupffn_forward_bh(FAKE, FAKE, FAKE, FAKE, 0, 768, 96, 8, 768, 64, 4, LFFN_F32, LFFN_F32, NULL, 0, NULL), LFFN_OK);
    EXPECT(lookupffn_prepare_tables(FAKE, 96, 8, 768, LFFN_F32, FAKE, 16, NULL), LFFN_E_WORKSPACE);
    EXPECT(lookupffn_prepare_bh(FAKE, 768, 96, 8, 64, 4, FAKE, 16, NULL), LFFN_E_WORKSPACE);
    /* options and the small text interfaces */
    EXPECT(lookupffn_set_option("token_slots", 8), LFFN_OK);
    EXPECT(lookupffn_set_option("token_slots", 0), LFFN_OK);
    EXPECT(lookupffn_set_option("small_tokens", -2), LFFN_E_SIZE);
    EXPECT(lookupffn_set_option("nothing", 1), LFFN_E_SIZE);
    EXPECT(lookupffn_set_option(NULL, 1), LFFN_E_NULL);
    for (int st = 1; st >= -9; --st) EXPECT(strlen(lookupffn_strerror(st)) > 0, 1);
    EXPECT(strlen(lookupffn_last_hip_error()), 0);
    EXPECT(strlen(lookupffn_last_gather_kernel()), 0);
    EXPECT(lookupffn_version() > 0, 1);
    {
        double ms[4];
        int64_t cnt = -1;
        EXPECT(lookupffn_timing_read_each(0, ms, 4, &cnt), LFFN_OK);
        EXPECT(cnt, 0);
        EXPECT(lookupffn_timing_read_each(2, ms, 4, &cnt), LFFN_E_SIZE);
    }
    printf(failures ? "FAILED: %d checks\n" : "host code ran clean\n", failures);
    return failures != 0;
}
