/*
 * Runs every function of the oracle on small inputs, edge cases included, so that a build with
 * -fsanitize=address,undefined can flag out-of-bounds accesses, invalid shifts or conversions and leaks.
 * Test infrastructure like the oracle itself (tests/test_oracle_sanitize.py compiles and runs it); it
 * checks no values -- the pins under tests/ do that.
 */
#include <stdio.h>

#include "condensa_oracle.c"

static float frand(uint32_t* s) {
    *s = *s * 1664525u + 1013904223u;
    return ((float)(*s >> 8) / 8388608.0f - 1.0f) * 0.05f;
}

int main(void) {
    uint32_t seed = 1911;
    enum { N = 1260 };                                       /* 6*5*6*7 = 3*4*5*7*3 */
    float *w = malloc(N * sizeof(float)), *lam = malloc(N * sizeof(float)), *v = malloc(N * sizeof(float)),
          *theta = malloc(N * sizeof(float)), *lam2 = malloc(N * sizeof(float)), *grad = malloc(N * sizeof(float)),
          *dq = malloc(N * sizeof(float)), *buf = malloc(N * sizeof(float));
    uint64_t *keys = malloc(N * sizeof(uint64_t)), *sorted = malloc(N * sizeof(uint64_t));
    uint8_t *keep = malloc(N), *q8 = malloc(N), *mask = malloc(N);
    uint16_t* q16 = malloc(N * sizeof(uint16_t));
    double* s = malloc(N * sizeof(double));
    float* norms = malloc(N * sizeof(float));
    for (int i = 0; i < N; ++i) { w[i] = frand(&seed); lam[i] = frand(&seed); buf[i] = frand(&seed); }
    w[3] = 0.0f; w[4] = -0.0f; w[5] = w[6]; w[7] = 1e-30f; w[8] = 7e4f; w[9] = -1e9f;   /* zeros, a tie, tiny, beyond binary16 */
    const int sizes[] = {0, 1, 2, 3, 5, 337, N};
    for (unsigned si = 0; si < sizeof sizes / sizeof sizes[0]; ++si) {
        const uint64_t n = (uint64_t)sizes[si];
        oracle_magnitude_keys(w, n, keys);
        memcpy(sorted, keys, n * sizeof(uint64_t));
        oracle_sort_desc(sorted, n);
        for (uint64_t kk = 0; kk <= n; kk += (n > 8 ? n / 3 + 1 : 1)) {
            oracle_select sel;
            oracle_select_keep(keys, sorted, n, kk, &sel, keep);
            oracle_apply_keep(w, keep, n, theta);
        }
        oracle_quantize_f16(w, n, q16, dq);
        oracle_quantize_f16(w, n, q16, NULL);
        oracle_dequantize_f16(q16, n, dq);
        (void)oracle_count_nonzero_f16(q16, n);
        oracle_quantize_bf16(w, n, q16, dq);
        oracle_dequantize_bf16(q16, n, dq);
        for (int fmt = 0; fmt < 2; ++fmt) {
            (void)oracle_quantize_fp8(w, n, fmt, q8, dq);
            (void)oracle_dequantize_fp8(q8, n, fmt, dq);
        }
        (void)oracle_quantize_fp8(w, n, 7, q8, dq);           /* unknown format: refused */
        oracle_lc_shifted(w, lam, n, 1e-3f, v);
        memset(keep, 0, N);
        for (uint64_t i = 0; i < n; i += 3) keep[i] = 1;
        oracle_lc_update(w, lam, v, keep, n, 1e-3f, theta, lam2, grad);
        oracle_lc_update_pq(w, lam, v, keep, n, 1e-3f, q16, theta, lam2, grad);
        oracle_lc_sgd_step(w, grad, theta, lam, buf, n, 1e-3f, 0.1f, 0.9f, lam2, dq);
        (void)oracle_count_nonzero_f32(theta, n);
        (void)oracle_count_nonzero_u8(q8, n);
    }
    (void)oracle_kept_count(0.02, 1048576);
    (void)oracle_kept_count(1.0, 0);
    (void)oracle_kept_count(0.5, 3);
    /* aggregates and structure applies: filters of [6, 210], 5x7 blocks of [30, 42], ragged 4-D blocks of [3,4,5,21] */
    memset(keep, 0, N);
    for (int i = 0; i < N; i += 2) keep[i] = 1;
    oracle_filter_sumsq(w, 6, 210, s);
    oracle_aggregate_keys(s, 6, keys);
    oracle_norms(s, 6, norms);
    oracle_filter_apply(w, 6, 210, keep, theta, mask);
    oracle_block_sumsq(w, 30, 42, 5, 7, s);
    oracle_block_apply(w, 30, 42, 5, 7, keep, theta, mask);
    {
        const uint64_t d[4] = {3, 4, 5, 21}, b[4] = {2, 3, 2, 4};
        oracle_block_sumsq_nd(w, d, b, s);
        oracle_block_apply_nd(w, d, b, keep, theta, mask);
    }
    {   /* thinning of [6, 5, 42]; the function takes ids inside the tensor only (its callers filter the others) */
        const int32_t ko[4] = {0, 5, 2, 5}, ki[3] = {4, 0, 3};
        oracle_thin(w, 6, 5, 42, ko, 4, ki, 3, theta);
        oracle_thin(w, 6, 5, 42, NULL, 6, NULL, 5, theta);
    }
    free(w); free(lam); free(v); free(theta); free(lam2); free(grad); free(dq); free(buf); free(keys); free(sorted);
    free(keep); free(q8); free(mask); free(q16); free(s); free(norms);
    printf("sanitize_check ok\n");
    return 0;
}
