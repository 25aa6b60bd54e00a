/* Driver for a host-sanitizer build of the CPU oracle: exact-size heap buffers (so that any
 * out-of-bounds index trips AddressSanitizer) over every input type, row subsets, masks, the
 * probability hook and the rejection paths.  Built and run by tests/test_oracle_sanitized.py. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_self_attn(const void *q, const void *k, const void *v, int32_t dtype, int32_t B, int32_t H,
                     int32_t D, const int32_t grid[3], const int32_t origin[3], const int32_t split[3],
                     double base, double scale, const int64_t *rows, int64_t n_rows, double *out,
                     double *lse, double *probs, int32_t pb, int32_t ph);
int oracle_cross_attn(const void *q, const void *k, const void *v, const uint8_t *kv_valid, int32_t dtype,
                      int32_t B, int32_t H, int32_t D, int64_t Lq, int64_t Lk, double scale,
                      const int64_t *rows, int64_t n_rows, double *out, double *lse, double *probs,
                      int32_t pb, int32_t ph);
int oracle_rope3d(const double *x, double *y, int64_t L, int32_t D, const int64_t *pos, const int32_t split[3],
                  double base);
int oracle_token_positions(const int32_t grid[3], const int32_t origin[3], int64_t n_tokens, int64_t *pos_out);

static uint32_t state = 12345u;
static double rnd(void)
{
    state = state * 1664525u + 1013904223u;
    return ((double)(state >> 8) / 16777216.0) * 2.0 - 1.0;
}

/* dtype 0: bf16 bit patterns, 1: float, 2: double */
static void *make(int dtype, size_t n)
{
    size_t es = dtype == 0 ? 2 : dtype == 1 ? 4 : 8;
    void *p = malloc(n * es);
    for (size_t i = 0; i < n; ++i) {
        float f = (float)rnd();
        if (dtype == 0) {
            uint32_t u;
            __builtin_memcpy(&u, &f, 4);
            ((uint16_t *)p)[i] = (uint16_t)(u >> 16);
        } else if (dtype == 1) {
            ((float *)p)[i] = f;
        } else {
            ((double *)p)[i] = f;
        }
    }
    return p;
}

static int finite_all(const double *x, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        if (!isfinite(x[i])) return 0;
    return 1;
}

int main(void)
{
    int fails = 0;
    for (int dtype = 0; dtype < 3; ++dtype) {
        const int32_t B = 2, H = 3, D = 8, grid[3] = {2, 3, 5}, origin[3] = {4, -2, 9}, split[3] = {4, 2, 2};
        const int64_t L = 30, rows[4] = {0, 7, 29, 13};
        size_t n = (size_t)B * L * H * D;
        void *q = make(dtype, n), *k = make(dtype, n), *v = make(dtype, n);
        double *out = malloc(sizeof(double) * B * 4 * H * D), *lse = malloc(sizeof(double) * B * H * 4);
        double *probs = malloc(sizeof(double) * 4 * L);
        int rc = oracle_self_attn(q, k, v, dtype, B, H, D, grid, origin, split, 10000.0, 0.0, rows, 4, out, lse,
                                  probs, 1, 2);
        if (rc != 0 || !finite_all(out, (size_t)B * 4 * H * D) || !finite_all(lse, B * H * 4)) ++fails;
        for (int r = 0; r < 4; ++r) {
            double s = 0;
            for (int m = 0; m < L; ++m) s += probs[r * L + m];
            if (fabs(s - 1.0) > 1e-12) ++fails;
        }
        /* rejected arguments must not touch the outputs */
        const int64_t bad_rows[1] = {30};
        if (oracle_self_attn(q, k, v, dtype, B, H, D, grid, origin, split, 10000.0, 0.0, bad_rows, 1, NULL, NULL, NULL,
                             0, 0) == 0)
            ++fails;
        const int32_t bad_split[3] = {4, 2, 4};
        if (oracle_self_attn(q, k, v, dtype, B, H, D, grid, origin, bad_split, 10000.0, 0.0, rows, 4, NULL, NULL, NULL,
                             0, 0) == 0)
            ++fails;
        free(q); free(k); free(v); free(out); free(lse); free(probs);

        const int64_t Lq = 5, Lk = 11, crows[3] = {4, 0, 2};
        void *cq = make(dtype, (size_t)B * Lq * H * D), *ck = make(dtype, (size_t)B * Lk * H * D),
             *cv = make(dtype, (size_t)B * Lk * H * D);
        uint8_t *valid = malloc((size_t)B * Lk);
        for (int i = 0; i < B * Lk; ++i) valid[i] = (uint8_t)(i % 3 != 1);
        for (int i = 0; i < Lk; ++i) valid[Lk + i] = 0; /* second request: nothing to attend to */
        double *cout = malloc(sizeof(double) * B * 3 * H * D), *clse = malloc(sizeof(double) * B * H * 3);
        double *cprobs = malloc(sizeof(double) * 3 * Lk);
        rc = oracle_cross_attn(cq, ck, cv, valid, dtype, B, H, D, Lq, Lk, 0.3, crows, 3, cout, clse, cprobs, 0, 1);
        if (rc != 0 || !finite_all(cout, (size_t)B * 3 * H * D)) ++fails;
        for (int i = 0; i < 3 * H * D; ++i)
            if (cout[3 * H * D + i] != 0.0) ++fails; /* fully masked request: zeros */
        rc = oracle_cross_attn(cq, ck, cv, NULL, dtype, B, H, D, Lq, Lk, 0.0, crows, 3, cout, NULL, NULL, 0, 0);
        if (rc != 0) ++fails;
        free(cq); free(ck); free(cv); free(valid); free(cout); free(clse); free(cprobs);
    }
    {
        const int32_t grid[3] = {3, 2, 4}, origin[3] = {0, 0, 0}, split[3] = {2, 2, 2};
        int64_t *pos = malloc(sizeof(int64_t) * 3 * 24);
        double *x = malloc(sizeof(double) * 24 * 6), *y = malloc(sizeof(double) * 24 * 6);
        for (int i = 0; i < 24 * 6; ++i) x[i] = rnd();
        if (oracle_token_positions(grid, origin, 24, pos) != 0) ++fails;
        if (oracle_rope3d(x, y, 24, 6, pos, split, 100.0) != 0 || !finite_all(y, 24 * 6)) ++fails;
        free(pos); free(x); free(y);
    }
    printf("oracle sanitizer driver: %d failure(s)\n", fails);
    return fails != 0;
}
