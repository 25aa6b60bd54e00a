/*
 * dit_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, fp64 CPU statement of what the DiT attention hot path computes:
 * dense softmax attention over every token of a (T,Hg,Wg) latent grid with a 3-axis
 * rotary position embedding on q and k (self-attention), and dense softmax attention
 * over a short conditioning sequence with a key-padding mask (cross-attention).
 *
 * The OnePiece paper (Sec. 2.4 "The AIGC Workflow", Diffusion stage; Sec. 4.4
 * "TaskWorker", user function on device-resident tensors) names the workload but gives
 * no mathematics for it, so every convention below is this repository's own reading and
 * is stated where it is used.  The code is the textbook definition written out: rotate,
 * dot, two-pass softmax, weighted sum.  No tiling, no online softmax, no tables, nothing
 * shared with the GPU implementation.  Only tests, the smoke check and the CPU-baseline
 * leg of the benchmark may call it.
 *
 * Pins (tests/test_oracle_pins.py): brute force with complex arithmetic on tiny grids,
 * rows of the softmax summing to 1, constant V, shift invariance of RoPE scores, single
 * key, q = 0 closed form, dominant key, isometry/identity of the rotation, reduction to
 * 1-D RoPE in closed form, axis separability, permutation invariance, mask = compaction,
 * log-sum-exp merge.  The RoPE pair/frequency convention itself cannot be checked
 * against an external model (none is available): "parity unpinned" for that choice only.
 *
 * Layout: every tensor is dense [B, L, H, D] (token-major), element type given by
 * `dtype`: 0 = bf16 bit patterns (uint16), 1 = float, 2 = double.  Inputs are widened
 * exactly to double; nothing is rounded on the way in.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double load_elem(const void *p, int dtype, int64_t i)
{
    if (dtype == 0) {
        uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
        float f;
        memcpy(&f, &u, 4);
        return (double)f;
    }
    if (dtype == 1)
        return (double)((const float *)p)[i];
    return ((const double *)p)[i];
}

/* Token n of the row-major (T,Hg,Wg) lattice, w fastest, plus an integer origin. */
static void token_pos(int64_t n, const int32_t grid[3], const int32_t origin[3], int64_t pos[3])
{
    int64_t hw = (int64_t)grid[1] * grid[2];
    pos[0] = origin[0] + n / hw;
    pos[1] = origin[1] + (n / grid[2]) % grid[1];
    pos[2] = origin[2] + n % grid[2];
}

/*
 * 3-axis rotary embedding of one head vector.  The D channels are three contiguous
 * sections (t, h, w) of sizes split[0..2]; inside section a, pair i is channels
 * (o_a+2i, o_a+2i+1), rotated by the angle pos_a * base^(-2i/d_a): the pair, read as
 * the complex number x0 + j x1, is multiplied by e^{j phi}.
 */
static void rope3d_vec(const double *x, double *y, const int64_t pos[3], const int32_t split[3],
                       double base)
{
    int o = 0;
    for (int a = 0; a < 3; ++a) {
        int da = split[a];
        for (int i = 0; i < da / 2; ++i) {
            double omega = pow(base, -2.0 * (double)i / (double)da);
            double phi = (double)pos[a] * omega;
            double c = cos(phi), s = sin(phi);
            double x0 = x[o + 2 * i], x1 = x[o + 2 * i + 1];
            y[o + 2 * i] = x0 * c - x1 * s;
            y[o + 2 * i + 1] = x0 * s + x1 * c;
        }
        o += da;
    }
}

/*
 * Softmax attention of one query vector over n_keys keys (kk, vv dense [n_keys, D]).
 * valid == NULL means every key attends.  Two passes: maximum, then normalised
 * exponentials.  A row with no valid key gives zeros and lse = -inf.
 * probs (optional) receives the n_keys probabilities.
 */
static void attend_row(const double *q, const double *kk, const double *vv, const uint8_t *valid,
                       int64_t n_keys, int D, double scale, double *s, double *out, double *lse,
                       double *probs)
{
    double mx = -INFINITY;
    for (int64_t m = 0; m < n_keys; ++m) {
        if (valid && !valid[m]) {
            s[m] = -INFINITY;
            continue;
        }
        double acc = 0.0;
        for (int c = 0; c < D; ++c)
            acc += q[c] * kk[m * D + c];
        s[m] = scale * acc;
        if (s[m] > mx)
            mx = s[m];
    }
    for (int c = 0; c < D; ++c)
        out[c] = 0.0;
    if (mx == -INFINITY) {
        if (lse)
            *lse = -INFINITY;
        if (probs)
            for (int64_t m = 0; m < n_keys; ++m)
                probs[m] = 0.0;
        return;
    }
    double sum = 0.0;
    for (int64_t m = 0; m < n_keys; ++m) {
        s[m] = (s[m] == -INFINITY) ? 0.0 : exp(s[m] - mx);
        sum += s[m];
    }
    for (int64_t m = 0; m < n_keys; ++m) {
        double p = s[m] / sum;
        if (probs)
            probs[m] = p;
        if (p != 0.0)
            for (int c = 0; c < D; ++c)
                out[c] += p * vv[m * D + c];
    }
    if (lse)
        *lse = mx + log(sum);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* (t,h,w) of each of n tokens: pos_out[n][3]. */
int oracle_token_positions(const int32_t grid[3], const int32_t origin[3], int64_t n_tokens,
                           int64_t *pos_out)
{
    for (int64_t n = 0; n < n_tokens; ++n)
        token_pos(n, grid, origin, pos_out + 3 * n);
    return 0;
}

/* Rotate x[L, D] (double) at explicit positions pos[L][3] into y[L, D]. */
int oracle_rope3d(const double *x, double *y, int64_t L, int32_t D, const int64_t *pos,
                  const int32_t split[3], double base)
{
    if (split[0] + split[1] + split[2] != D || (split[0] | split[1] | split[2]) & 1)
        return -1;
    for (int64_t n = 0; n < L; ++n)
        rope3d_vec(x + n * D, y + n * D, pos + 3 * n, split, base);
    return 0;
}

/*
 * Self-attention for the listed query rows of every (batch, head).
 *   q, k, v : [B, L, H, D] of `dtype`, L = grid[0]*grid[1]*grid[2]
 *   rows    : n_rows token indices in [0, L); the same list is used for every (b, h)
 *   out     : [B, n_rows, H, D] double;  lse (nullable): [B, H, n_rows] double
 *   probs   : nullable; when given, [n_rows, L] probabilities of (b, h) = (pb, ph)
 *   scale <= 0 selects 1/sqrt(D).
 * All L keys attend (no mask).  Returns 0, or -1 on bad arguments, -2 out of memory.
 */
int oracle_self_attn(const void *q, const void *k, const void *v, int32_t dtype, int32_t B,
                     int32_t H, int32_t D, const int32_t grid[3], const int32_t origin[3],
                     const int32_t split[3], double base, double scale, const int64_t *rows,
                     int64_t n_rows, double *out, double *lse, double *probs, int32_t pb,
                     int32_t ph)
{
    int64_t L = (int64_t)grid[0] * grid[1] * grid[2];
    if (B < 1 || H < 1 || D < 2 || L < 1 || split[0] + split[1] + split[2] != D ||
        ((split[0] | split[1] | split[2]) & 1) || split[0] < 0 || split[1] < 0 || split[2] < 0)
        return -1;
    for (int64_t r = 0; r < n_rows; ++r)
        if (rows[r] < 0 || rows[r] >= L)
            return -1;
    if (scale <= 0.0)
        scale = 1.0 / sqrt((double)D);

    double *kr = malloc(sizeof(double) * L * D);
    double *vv = malloc(sizeof(double) * L * D);
    if (!kr || !vv) {
        free(kr);
        free(vv);
        return -2;
    }
    int fail = 0;
    for (int32_t b = 0; b < B; ++b)
        for (int32_t h = 0; h < H; ++h) {
#pragma omp parallel
            {
                double *tmp = malloc(sizeof(double) * D);
                if (!tmp) {
#pragma omp atomic write
                    fail = 1;
                }
#pragma omp for schedule(static)
                for (int64_t m = 0; m < L; ++m) {
                    if (!tmp)
                        continue;
                    int64_t base_idx = (((int64_t)b * L + m) * H + h) * D;
                    int64_t pos[3];
                    token_pos(m, grid, origin, pos);
                    for (int c = 0; c < D; ++c) {
                        tmp[c] = load_elem(k, dtype, base_idx + c);
                        vv[m * D + c] = load_elem(v, dtype, base_idx + c);
                    }
                    rope3d_vec(tmp, kr + m * D, pos, split, base);
                }
                free(tmp);
            }
            if (fail)
                break;
#pragma omp parallel
            {
                double *s = malloc(sizeof(double) * L);
                double *qv = malloc(sizeof(double) * 2 * D);
                if (!s || !qv) {
#pragma omp atomic write
                    fail = 1;
                }
#pragma omp for schedule(dynamic, 1)
                for (int64_t r = 0; r < n_rows; ++r) {
                    if (!s || !qv)
                        continue;
                    int64_t n = rows[r];
                    int64_t base_idx = (((int64_t)b * L + n) * H + h) * D;
                    int64_t pos[3];
                    token_pos(n, grid, origin, pos);
                    for (int c = 0; c < D; ++c)
                        qv[c] = load_elem(q, dtype, base_idx + c);
                    rope3d_vec(qv, qv + D, pos, split, base);
                    double *o = out + (((int64_t)b * n_rows + r) * H + h) * D;
                    double *l = lse ? lse + ((int64_t)b * H + h) * n_rows + r : NULL;
                    double *pr = (probs && b == pb && h == ph) ? probs + r * L : NULL;
                    attend_row(qv + D, kr, vv, NULL, L, D, scale, s, o, l, pr);
                }
                free(s);
                free(qv);
            }
            if (fail)
                break;
        }
    free(kr);
    free(vv);
    return fail ? -2 : 0;
}

/*
 * Cross-attention (no positional rotation) for the listed query rows.
 *   q : [B, Lq, H, D];  k, v : [B, Lk, H, D];  kv_valid (nullable): [B, Lk], 1 = attend
 *   out : [B, n_rows, H, D] double;  lse (nullable): [B, H, n_rows]
 *   probs (nullable): [n_rows, Lk] for (b, h) = (pb, ph)
 * One joint softmax over all Lk keys of the request; masked keys take no part in the
 * maximum or the sum.
 */
int oracle_cross_attn(const void *q, const void *k, const void *v, const uint8_t *kv_valid,
                      int32_t dtype, int32_t B, int32_t H, int32_t D, int64_t Lq, int64_t Lk,
                      double scale, const int64_t *rows, int64_t n_rows, double *out, double *lse,
                      double *probs, int32_t pb, int32_t ph)
{
    if (B < 1 || H < 1 || D < 1 || Lq < 1 || Lk < 1)
        return -1;
    for (int64_t r = 0; r < n_rows; ++r)
        if (rows[r] < 0 || rows[r] >= Lq)
            return -1;
    if (scale <= 0.0)
        scale = 1.0 / sqrt((double)D);
    double *kk = malloc(sizeof(double) * Lk * D);
    double *vv = malloc(sizeof(double) * Lk * D);
    if (!kk || !vv) {
        free(kk);
        free(vv);
        return -2;
    }
    int fail = 0;
    for (int32_t b = 0; b < B; ++b)
        for (int32_t h = 0; h < H; ++h) {
            for (int64_t m = 0; m < Lk; ++m) {
                int64_t base_idx = (((int64_t)b * Lk + m) * H + h) * D;
                for (int c = 0; c < D; ++c) {
                    kk[m * D + c] = load_elem(k, dtype, base_idx + c);
                    vv[m * D + c] = load_elem(v, dtype, base_idx + c);
                }
            }
            const uint8_t *valid = kv_valid ? kv_valid + (int64_t)b * Lk : NULL;
#pragma omp parallel
            {
                double *s = malloc(sizeof(double) * Lk);
                double *qv = malloc(sizeof(double) * D);
                if (!s || !qv) {
#pragma omp atomic write
                    fail = 1;
                }
#pragma omp for schedule(static)
                for (int64_t r = 0; r < n_rows; ++r) {
                    if (!s || !qv)
                        continue;
                    int64_t base_idx = (((int64_t)b * Lq + rows[r]) * H + h) * D;
                    for (int c = 0; c < D; ++c)
                        qv[c] = load_elem(q, dtype, base_idx + c);
                    double *o = out + (((int64_t)b * n_rows + r) * H + h) * D;
                    double *l = lse ? lse + ((int64_t)b * H + h) * n_rows + r : NULL;
                    double *pr = (probs && b == pb && h == ph) ? probs + r * Lk : NULL;
                    attend_row(qv, kk, vv, valid, Lk, D, scale, s, o, l, pr);
                }
                free(s);
                free(qv);
            }
            if (fail)
                break;
        }
    free(kk);
    free(vv);
    return fail ? -2 : 0;
}
