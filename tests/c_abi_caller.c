/* A C99 caller of the library's C ABI, with no Python and no C++ in between: device buffers from the
 * HIP runtime's C API, one self-attention, one masked cross-attention, one projection and the fused q/k/v projection
 * route through include/dit_attn.h,
 * results compared with the CPU oracle (oracle/dit_oracle.c, linked in) to the parity bar.
 * Built by paper_2601_20655_amd/build.py (build_c_caller), run by tests/test_gpu_c_caller.py. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "dit_attn.h"

int oracle_self_attn(const void *q, const void *k, const void *v, int32_t dtype, int32_t B, int32_t H,
                     int32_t D, const int32_t grid[3], const int32_t origin[3], const int32_t split[3],
                     double base, double scale, const int64_t *rows, int64_t n_rows, double *out,
                     double *lse, double *probs, int32_t pb, int32_t ph);
int oracle_cross_attn(const void *q, const void *k, const void *v, const uint8_t *kv_valid, int32_t dtype,
                      int32_t B, int32_t H, int32_t D, int64_t Lq, int64_t Lk, double scale,
                      const int64_t *rows, int64_t n_rows, double *out, double *lse, double *probs,
                      int32_t pb, int32_t ph);

#define CHECK_HIP(x)                                                                  \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));            \
            return 2;                                                                 \
        }                                                                             \
    } while (0)

static uint64_t rng_state = 0x2601206550ull;
static float gauss(void)
{ /* sum of 12 uniforms - 6: close enough to N(0,1) for a stand-in activation */
    float s = 0.f;
    for (int i = 0; i < 12; ++i) {
        rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
        s += (float)(rng_state >> 40) / 16777216.0f;
    }
    return s - 6.0f;
}

static uint16_t *make_bf16(size_t n)
{
    uint16_t *p = (uint16_t *)malloc(n * 2);
    for (size_t i = 0; i < n; ++i) {
        float f = gauss();
        uint32_t u;
        memcpy(&u, &f, 4);
        u += 0x7fffu + ((u >> 16) & 1u); /* nearest even */
        p[i] = (uint16_t)(u >> 16);
    }
    return p;
}

static void *to_device(const void *h, size_t bytes)
{
    void *d = NULL;
    if (hipMalloc(&d, bytes) != hipSuccess) return NULL;
    if (h && hipMemcpy(d, h, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL;
    return d;
}

/* max |gpu - ref| / RMS(ref) */
static double rel_err(const float *gpu, const double *ref, size_t n)
{
    double ss = 0, mx = 0;
    for (size_t i = 0; i < n; ++i) {
        ss += ref[i] * ref[i];
        double e = fabs((double)gpu[i] - ref[i]);
        if (e > mx) mx = e;
    }
    return mx / sqrt(ss / (double)n);
}

int main(void)
{
    int n_dev = 0;
    CHECK_HIP(hipGetDeviceCount(&n_dev));
    if (n_dev < 1) {
        fprintf(stderr, "no GPU\n");
        return 2;
    }
    printf("libdit_attn version %d\n", dit_attn_version());

    /* ---- self-attention: grid 3 x 7 x 19 = 399 tokens, 2 heads, d128 ---- */
    {
        const int32_t B = 1, H = 2, D = 128, grid[3] = {3, 7, 19}, origin[3] = {0, 0, 0}, split[3] = {44, 42, 42};
        const int64_t L = 399;
        const size_t n = (size_t)B * L * H * D;
        uint16_t *q = make_bf16(n), *k = make_bf16(n), *v = make_bf16(n);
        void *dq = to_device(q, n * 2), *dk = to_device(k, n * 2), *dv = to_device(v, n * 2);
        void *dout = to_device(NULL, n * 4);
        if (!dq || !dk || !dv || !dout) return 2;

        dit_self_attn_params p;
        memset(&p, 0, sizeof(p));
        p.B = B; p.H = H; p.D = D;
        p.T = grid[0]; p.Hg = grid[1]; p.Wg = grid[2];
        p.d_t = split[0]; p.d_h = split[1]; p.d_w = split[2];
        p.rope_base = 10000.0f;
        p.in_dtype = DIT_BF16; p.out_dtype = DIT_F32;
        dit_strides s = {(int64_t)L * H * D, (int64_t)H * D, D};
        p.sq = p.sk = p.sv = p.so = s;
        size_t ws_bytes = dit_attn_workspace_bytes(&p);
        void *ws = to_device(NULL, ws_bytes);
        if (!ws_bytes || !ws) return 2;
        dit_status st = dit_attn_forward(dq, dk, dv, dout, NULL, &p, ws, ws_bytes, NULL);
        if (st != DIT_OK) {
            fprintf(stderr, "dit_attn_forward: %s %s\n", dit_strerror(st), dit_last_hip_error());
            return 1;
        }
        CHECK_HIP(hipDeviceSynchronize());
        float *out = (float *)malloc(n * 4);
        CHECK_HIP(hipMemcpy(out, dout, n * 4, hipMemcpyDeviceToHost));

        int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * L);
        for (int64_t i = 0; i < L; ++i) rows[i] = i;
        double *ref = (double *)malloc(n * 8);
        if (oracle_self_attn(q, k, v, 0, B, H, D, grid, origin, split, 10000.0, 0.0, rows, L, ref, NULL, NULL, 0, 0))
            return 1;
        double e = rel_err(out, ref, n);
        printf("self-attention  max|err|/RMS = %.3e\n", e);
        if (!(e < 2e-2)) return 1;
        /* a bad call is refused before anything is launched */
        p.d_w = 40;
        if (dit_attn_forward(dq, dk, dv, dout, NULL, &p, ws, ws_bytes, NULL) != DIT_ERR_INVALID_ARG) return 1;
        hipFree(dq); hipFree(dk); hipFree(dv); hipFree(dout); hipFree(ws);
        free(q); free(k); free(v); free(out); free(rows); free(ref);
    }

    /* ---- cross-attention: 2 requests x 200 queries x 129 keys (96 text, padded, + 33 image) ---- */
    {
        const int32_t B = 2, H = 2, D = 128;
        const int64_t Lq = 200, Lk = 129;
        const size_t nq = (size_t)B * Lq * H * D, nk = (size_t)B * Lk * H * D;
        uint16_t *q = make_bf16(nq), *k = make_bf16(nk), *v = make_bf16(nk);
        uint8_t *valid = (uint8_t *)malloc((size_t)B * Lk);
        const int text_len[2] = {37, 96};
        for (int b = 0; b < B; ++b)
            for (int m = 0; m < Lk; ++m) valid[b * Lk + m] = (uint8_t)(m < text_len[b] || m >= 96);
        void *dq = to_device(q, nq * 2), *dk = to_device(k, nk * 2), *dv = to_device(v, nk * 2);
        void *dvalid = to_device(valid, (size_t)B * Lk), *dout = to_device(NULL, nq * 4);
        if (!dq || !dk || !dv || !dvalid || !dout) return 2;

        dit_cross_attn_params p;
        memset(&p, 0, sizeof(p));
        p.B = B; p.H = H; p.D = D; p.Lq = (int32_t)Lq; p.Lk = (int32_t)Lk;
        p.in_dtype = DIT_BF16; p.out_dtype = DIT_F32;
        dit_strides sq = {Lq * H * D, (int64_t)H * D, D}, sk = {Lk * H * D, (int64_t)H * D, D};
        p.sq = p.so = sq;
        p.sk = p.sv = sk;
        size_t ws_bytes = dit_cross_attn_workspace_bytes(&p);
        void *ws = to_device(NULL, ws_bytes);
        if (!ws_bytes || !ws) return 2;
        dit_status st = dit_cross_attn_forward(dq, dk, dv, (const uint8_t *)dvalid, dout, NULL, &p, ws, ws_bytes, NULL);
        if (st != DIT_OK) {
            fprintf(stderr, "dit_cross_attn_forward: %s %s\n", dit_strerror(st), dit_last_hip_error());
            return 1;
        }
        CHECK_HIP(hipDeviceSynchronize());
        float *out = (float *)malloc(nq * 4);
        CHECK_HIP(hipMemcpy(out, dout, nq * 4, hipMemcpyDeviceToHost));
        int64_t *rows = (int64_t *)malloc(sizeof(int64_t) * Lq);
        for (int64_t i = 0; i < Lq; ++i) rows[i] = i;
        double *ref = (double *)malloc(nq * 8);
        if (oracle_cross_attn(q, k, v, valid, 0, B, H, D, Lq, Lk, 0.0, rows, Lq, ref, NULL, NULL, 0, 0)) return 1;
        double e = rel_err(out, ref, nq);
        printf("cross-attention max|err|/RMS = %.3e\n", e);
        if (!(e < 2e-2)) return 1;
        hipFree(dq); hipFree(dk); hipFree(dv); hipFree(dvalid); hipFree(dout); hipFree(ws);
        free(q); free(k); free(v); free(valid); free(out); free(rows); free(ref);
    }
    /* ---- projection: y = x w^T + bias, 300 tokens, 192 -> 264 features (ragged tiles on both axes),
     * checked against a triple loop in double written out here ---- */
    {
        const int32_t M = 300, N = 264, K = 192;
        uint16_t *x = make_bf16((size_t)M * K), *w = make_bf16((size_t)N * K), *b = make_bf16((size_t)N);
        void *dx = to_device(x, (size_t)M * K * 2), *dw = to_device(w, (size_t)N * K * 2);
        void *db = to_device(b, (size_t)N * 2), *dy = to_device(NULL, (size_t)M * N * 4);
        if (!dx || !dw || !db || !dy) return 2;
        dit_linear_params p;
        memset(&p, 0, sizeof(p));
        p.M = M; p.N = N; p.K = K; p.ldx = K; p.ldw = K; p.ldy = N; p.out_dtype = DIT_F32;
        dit_status st = dit_linear_forward(dx, dw, db, dy, &p, NULL);
        if (st != DIT_OK) {
            fprintf(stderr, "dit_linear_forward: %s %s\n", dit_strerror(st), dit_last_hip_error());
            return 1;
        }
        CHECK_HIP(hipDeviceSynchronize());
        float *y = (float *)malloc((size_t)M * N * 4);
        CHECK_HIP(hipMemcpy(y, dy, (size_t)M * N * 4, hipMemcpyDeviceToHost));
        double *ref = (double *)malloc((size_t)M * N * 8);
        for (int m = 0; m < M; ++m)
            for (int n = 0; n < N; ++n) {
                double acc = 0.0;
                for (int k = 0; k < K; ++k) {
                    uint32_t ux = (uint32_t)x[(size_t)m * K + k] << 16, uw = (uint32_t)w[(size_t)n * K + k] << 16;
                    float fx, fw;
                    memcpy(&fx, &ux, 4);
                    memcpy(&fw, &uw, 4);
                    acc += (double)fx * (double)fw;
                }
                uint32_t ub = (uint32_t)b[n] << 16;
                float fb;
                memcpy(&fb, &ub, 4);
                ref[(size_t)m * N + n] = acc + (double)fb;
            }
        double e = rel_err(y, ref, (size_t)M * N);
        printf("projection      max|err|/RMS = %.3e\n", e);
        if (!(e < 1e-5)) return 1;
        p.K = 100; /* not a multiple of 64: refused before anything is launched */
        if (dit_linear_forward(dx, dw, db, dy, &p, NULL) != DIT_ERR_UNSUPPORTED) return 1;
        hipFree(dx); hipFree(dw); hipFree(db); hipFree(dy);
        free(x); free(w); free(b); free(y); free(ref);
    }
    /* ---- q/k/v projection that writes the attention's tile images, then attention on them: bit for bit the
     * result of the separate calls (projection with bf16 output, attention on the q, k, v columns of that output) ---- */
    {
        const int32_t H = 2, D = 128, K = 128, grid[3] = {3, 7, 11}, split[3] = {44, 42, 42};
        const int64_t L = 3 * 7 * 11, HD = (int64_t)H * D, N = 3 * HD;
        uint16_t *x = make_bf16((size_t)L * K), *w = make_bf16((size_t)N * K), *b = make_bf16((size_t)N);
        /* weights of the size a projection has, so that q and k stay of order one */
        for (size_t i = 0; i < (size_t)N * K; ++i) {
            uint32_t u = (uint32_t)w[i] << 16;
            float f;
            memcpy(&f, &u, 4);
            f *= 0.09f;
            memcpy(&u, &f, 4);
            w[i] = (uint16_t)(u >> 16);
        }
        void *dx = to_device(x, (size_t)L * K * 2), *dw = to_device(w, (size_t)N * K * 2), *db = to_device(b, (size_t)N * 2);
        void *dy = to_device(NULL, (size_t)L * N * 2), *dqo = to_device(NULL, (size_t)L * HD * 2);
        void *o1 = to_device(NULL, (size_t)L * HD * 4), *o2 = to_device(NULL, (size_t)L * HD * 4);
        if (!dx || !dw || !db || !dy || !dqo || !o1 || !o2) return 2;
        dit_self_attn_params ap;
        memset(&ap, 0, sizeof(ap));
        ap.B = 1; ap.H = H; ap.D = D;
        ap.T = grid[0]; ap.Hg = grid[1]; ap.Wg = grid[2];
        ap.d_t = split[0]; ap.d_h = split[1]; ap.d_w = split[2];
        ap.rope_base = 10000.0f;
        ap.in_dtype = DIT_BF16; ap.out_dtype = DIT_F32;
        dit_strides dense = {L * HD, HD, D};
        ap.sq = ap.sk = ap.sv = ap.so = dense;
        size_t ws_bytes = dit_attn_workspace_bytes(&ap);
        void *ws = to_device(NULL, ws_bytes), *ws2 = to_device(NULL, ws_bytes);
        if (!ws || !ws2) return 2;
        dit_linear_params lp;
        memset(&lp, 0, sizeof(lp));
        lp.M = (int32_t)L; lp.N = (int32_t)N; lp.K = K; lp.ldx = K; lp.ldw = K; lp.ldy = N; lp.out_dtype = DIT_BF16;
        dit_status st = dit_qkv_proj_forward(dx, dw, db, dqo, &lp, &ap, ws, ws_bytes, NULL);
        if (st != DIT_OK) {
            fprintf(stderr, "dit_qkv_proj_forward: %s %s\n", dit_strerror(st), dit_last_hip_error());
            return 1;
        }
        dit_self_attn_params ar = ap;
        ar.flags |= DIT_FLAG_KV_RESIDENT;
        st = dit_attn_forward(dqo, NULL, NULL, o1, NULL, &ar, ws, ws_bytes, NULL);
        if (st != DIT_OK) {
            fprintf(stderr, "dit_attn_forward on resident tiles: %s %s\n", dit_strerror(st), dit_last_hip_error());
            return 1;
        }
        /* the separate route: rows of [q | k | v] with a token stride of 3 H D */
        st = dit_linear_forward(dx, dw, db, dy, &lp, NULL);
        if (st != DIT_OK) return 1;
        dit_self_attn_params as = ap;
        dit_strides cols = {L * N, N, D};
        as.sq = as.sk = as.sv = cols;
        st = dit_attn_forward(dy, (uint16_t *)dy + HD, (uint16_t *)dy + 2 * HD, o2, NULL, &as, ws2, ws_bytes, NULL);
        if (st != DIT_OK) {
            fprintf(stderr, "dit_attn_forward on projected rows: %s %s\n", dit_strerror(st), dit_last_hip_error());
            return 1;
        }
        CHECK_HIP(hipDeviceSynchronize());
        float *h1 = (float *)malloc((size_t)L * HD * 4), *h2 = (float *)malloc((size_t)L * HD * 4);
        CHECK_HIP(hipMemcpy(h1, o1, (size_t)L * HD * 4, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(h2, o2, (size_t)L * HD * 4, hipMemcpyDeviceToHost));
        double sq = 0.0;
        for (size_t i = 0; i < (size_t)L * HD; ++i) sq += (double)h1[i] * h1[i];
        const int same = memcmp(h1, h2, (size_t)L * HD * 4) == 0;
        printf("fused q/k/v projection + attention: %s the separate calls (output RMS %.3e)\n",
               same ? "bit for bit" : "DIFFERS from", sqrt(sq / (double)(L * HD)));
        if (!same || !(sq > 0.0)) return 1;
        hipFree(dx); hipFree(dw); hipFree(db); hipFree(dy); hipFree(dqo); hipFree(o1); hipFree(o2); hipFree(ws); hipFree(ws2);
        free(x); free(w); free(b); free(h1); free(h2);
    }
    printf("c caller ok\n");
    return 0;
}
