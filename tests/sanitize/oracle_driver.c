/* Sanitizer driver for the CPU oracle (test infrastructure): calls every exported function of
 * thi_oracle.c on small seeded inputs, including the smallest legal extents, and prints a checksum.
 * Built by tests/test_sanitizers_cpu.py with -fsanitize=address,undefined; a clean run prints "ok". */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int thi_oracle_threads(void);
double thi_oracle_half_to_double(uint16_t h);
double thi_oracle_silu(double t);
int thi_oracle_linear(const uint16_t *x, const uint16_t *w, double *y, double *s, long M, long N, long K);
int thi_oracle_rmsnorm_qkv(const uint16_t *x, const uint16_t *gamma, float eps, const uint16_t *w, double *y, double *s,
                           long M, long N, long K);
int thi_oracle_swiglu_mlp(const uint16_t *x, const uint16_t *wg, const uint16_t *wu, const uint16_t *wd, double *y,
                          double *s, double *h_out, long M, long H, long I);
int thi_oracle_linear_residual(const uint16_t *x, const uint16_t *w, const uint16_t *res, double *y, double *s, long M,
                               long N, long K);
int thi_oracle_rmsnorm_swiglu_mlp(const uint16_t *x, const uint16_t *gamma, float eps, const uint16_t *wg,
                                  const uint16_t *wu, const uint16_t *wd, const uint16_t *res, double *y, double *s,
                                  double *h_out, long M, long H, long I);
int thi_oracle_rope_inplace(double *y, double *s, const int32_t *pos, const float *theta, long M, long N, long n_rot,
                            long head_dim);
int thi_oracle_rmsnorm_qkv_rope(const uint16_t *x, const uint16_t *gamma, float eps, const uint16_t *w, const int32_t *pos,
                                const float *theta, double *y, double *s, long M, long N, long K, long n_rot, long head_dim);
int thi_oracle_decode_attention(const uint16_t *q, const uint16_t *k, const uint16_t *v, const int32_t *len, float scale,
                                double *y, double *s, long B, long Hq, long Hkv, long D, long S_max);

static uint32_t rng_state = 12345u;
static uint16_t small_half(void)
{   /* finite fp16 patterns with exponent <= 15 (|v| < 2), both signs, subnormals included */
    rng_state = rng_state * 1664525u + 1013904223u;
    uint32_t r = rng_state >> 8;
    return (uint16_t)(((r & 1u) << 15) | ((r >> 1) % 0x4000u));
}
static uint16_t *halves(long n)
{
    uint16_t *p = (uint16_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(uint16_t));
    if (!p) exit(3);
    for (long i = 0; i < n; ++i) p[i] = small_half();
    return p;
}
static double *doubles(long n)
{
    double *p = (double *)calloc((size_t)(n > 0 ? n : 1), sizeof(double));
    if (!p) exit(3);
    return p;
}
static double sum(const double *p, long n)
{
    double t = 0;
    for (long i = 0; i < n; ++i) t += p[i];
    return t;
}

int main(void)
{
    double check = 0;
    const long shapes[][3] = {{1, 1, 8}, {1, 3, 8}, {2, 5, 16}, {7, 33, 40}, {33, 17, 264}};
    for (unsigned c = 0; c < sizeof(shapes) / sizeof(shapes[0]); ++c) {
        const long M = shapes[c][0], N = shapes[c][1], K = shapes[c][2], I = N + 3;
        uint16_t *x = halves(M * K), *w = halves(N * K), *g = halves(K), *res = halves(M * N);
        uint16_t *wg = halves(I * K), *wu = halves(I * K), *wd = halves(K * I), *resm = halves(M * K);
        double *y = doubles(M * N), *s = doubles(M * N), *ym = doubles(M * K), *sm = doubles(M * K), *h = doubles(M * I);
        if (thi_oracle_linear(x, w, y, s, M, N, K)) return 4;
        check += sum(y, M * N) + sum(s, M * N);
        if (thi_oracle_rmsnorm_qkv(x, g, 1e-6f, w, y, s, M, N, K)) return 4;
        check += sum(y, M * N);
        if (thi_oracle_linear_residual(x, w, res, y, s, M, N, K)) return 4;
        check += sum(y, M * N);
        if (thi_oracle_swiglu_mlp(x, wg, wu, wd, ym, sm, h, M, K, I)) return 4;
        check += sum(ym, M * K) + sum(h, M * I);
        if (thi_oracle_swiglu_mlp(x, wg, wu, wd, ym, sm, NULL, M, K, I)) return 4;
        if (thi_oracle_rmsnorm_swiglu_mlp(x, g, 1e-6f, wg, wu, wd, resm, ym, sm, h, M, K, I)) return 4;
        if (thi_oracle_rmsnorm_swiglu_mlp(x, g, 1e-6f, wg, wu, wd, NULL, ym, sm, NULL, M, K, I)) return 4;
        check += sum(ym, M * K);
        free(x); free(w); free(g); free(res); free(wg); free(wu); free(wd); free(resm);
        free(y); free(s); free(ym); free(sm); free(h);
    }
    {   /* rotary embedding: two heads of eight columns rotated, four columns left alone */
        const long M = 3, N = 20, K = 16, hd = 8, n_rot = 16;
        uint16_t *x = halves(M * K), *w = halves(N * K), *g = halves(K);
        double *y = doubles(M * N), *s = doubles(M * N);
        int32_t pos[3] = {0, 5, 4095};
        float theta[4] = {1.0f, 0.1f, 0.01f, 0.001f};
        if (thi_oracle_rmsnorm_qkv_rope(x, g, 1e-6f, w, pos, theta, y, s, M, N, K, n_rot, hd)) return 5;
        check += sum(y, M * N) + sum(s, M * N);
        if (thi_oracle_rope_inplace(y, NULL, pos, theta, M, N, n_rot, hd)) return 5;
        if (thi_oracle_rope_inplace(y, s, pos, theta, M, N, 12, hd) != -2) return 5;      /* not whole heads: refused */
        free(x); free(w); free(g); free(y); free(s);
    }
    {   /* decode attention: ragged lengths with an empty request, grouped heads */
        const long B = 3, Hq = 6, Hkv = 2, D = 8, S = 11;
        uint16_t *q = halves(B * Hq * D), *k = halves(B * Hkv * S * D), *v = halves(B * Hkv * S * D);
        double *y = doubles(B * Hq * D), *s = doubles(B * Hq * D);
        int32_t len[3] = {11, 0, 1};
        if (thi_oracle_decode_attention(q, k, v, len, 0.35f, y, s, B, Hq, Hkv, D, S)) return 6;
        check += sum(y, B * Hq * D) + sum(s, B * Hq * D);
        free(q); free(k); free(v); free(y); free(s);
    }
    check += thi_oracle_silu(-3.0) + thi_oracle_half_to_double(0x3c00) + thi_oracle_half_to_double(0x0001) +
             (double)thi_oracle_threads();
    if (!isfinite(check)) return 7;
    printf("ok %.6f\n", check);
    return 0;
}
