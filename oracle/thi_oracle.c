/*
 * thi_oracle -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * A plain, slow, fp64 CPU statement of what the Llama decoder-layer linear
 * operators compute.  Only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg may call it.  It shares no code, header, table or helper
 * with the HIP library and is never a fallback for it.
 *
 * What is computed, and where the paper fixes it:
 *   - the linear operator Y = X * W                (Sec. III-B.1, the GEMM
 *     statement before Eq. 1); weights are held [N,K] row-major here, i.e. the
 *     paper's W transposed (the layout this library's boundary uses);
 *   - "FP16 storage, FP32 accumulation", with normalisation statistics kept in
 *     higher precision (Sec. III-B.4).  The oracle reads the same fp16 bit
 *     patterns as the GPU, widens them exactly to fp64 and rounds nothing
 *     afterwards, so it is the mathematical result up to ~K*2^-53 relative;
 *   - low-density operators wrapped around the high-density one
 *     (Sec. III-C.1, the "[low]-high-[low]" fusion unit): RMSNorm before the QKV
 *     projection, SiLU(gate)*up after the gate/up projections.  The paper does
 *     not print the RMSNorm and SwiGLU formulas; the standard Llama definitions
 *     are used: rmsnorm(x)[k] = x[k] * gamma[k] / sqrt(mean_k x[k]^2 + eps),
 *     silu(t) = t / (1 + exp(-t)), h = silu(gate) * up.
 *
 * Every function also returns S[m,n] = sum_k |a[m,k] * w[n,k]|, the magnitude
 * against which the acceptance tolerance is scaled.
 *
 * Loop order is the index order of the definitions.  The only parallelism is
 * an OpenMP "for" over output rows n (each output element is still one serial
 * sum in index order, so results do not depend on the thread count).
 *
 * Parity pins (tests/test_oracle_*.py): identity / one-hot / all-ones / +-1
 * weights, RMSNorm of constant vectors, RMSNorm scale invariance and
 * factorisation, SiLU reference values and identities, SwiGLU with selector
 * matrices, exact rational brute force on tiny shapes, a numpy fp64 witness on
 * mid-size shapes, linearity, residuals that cancel the product exactly, the
 * normalised MLP against its pinned parts, and the paper's Eq. 1-3 / Eq. 7
 * arithmetic for the roofline helpers used by the benchmark.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE binary16 bit pattern -> double, exact (subnormals, inf, nan kept). */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);            /* subnormal or zero: frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

static void widen_row(const uint16_t *src, double *dst, long count)
{
    for (long i = 0; i < count; ++i) dst[i] = half_bits_to_double(src[i]);
}

int thi_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

double thi_oracle_half_to_double(uint16_t h) { return half_bits_to_double(h); }

double thi_oracle_silu(double t) { return t / (1.0 + exp(-t)); }

/*
 * Core of every operator: a[M,K] (fp64, already widened or already an fp64
 * intermediate) against fp16 weights w[N,K]:
 *     y[m,n] = sum_k a[m,k] * w[n,k],   s[m,n] = sum_k |a[m,k] * w[n,k]|.
 * s may be NULL.
 */
static int dense_rows(const double *a, const uint16_t *w, double *y, double *s,
                      long M, long N, long K)
{
    int failed = 0;
#pragma omp parallel
    {
        double *wrow = (double *)malloc((size_t)K * sizeof(double));
        if (!wrow) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(static)
            for (long n = 0; n < N; ++n) {
                widen_row(w + n * K, wrow, K);
                for (long m = 0; m < M; ++m) {
                    const double *arow = a + m * K;
                    double acc = 0.0, mag = 0.0;
                    for (long k = 0; k < K; ++k) {
                        double p = arow[k] * wrow[k];
                        acc += p;
                        mag += fabs(p);
                    }
                    y[m * N + n] = acc;
                    if (s) s[m * N + n] = mag;
                }
            }
        }
        free(wrow);
    }
    return failed ? -1 : 0;
}

/* Sec. III-B.1: y = x * w^T with x[M,K], w[N,K] fp16 bit patterns. */
int thi_oracle_linear(const uint16_t *x, const uint16_t *w, double *y, double *s,
                      long M, long N, long K)
{
    double *a = (double *)malloc((size_t)M * K * sizeof(double));
    if (!a) return -1;
    widen_row(x, a, M * K);
    int rc = dense_rows(a, w, y, s, M, N, K);
    free(a);
    return rc;
}

/*
 * Sec. III-B.4 (RMSNorm statistics in higher precision) + Sec. III-C.1 (low-
 * density operator placed in front of the linear operator):
 *   ms_m = (1/K) sum_k x[m,k]^2,  r_m = 1/sqrt(ms_m + eps),
 *   xhat[m,k] = x[m,k] * r_m * gamma[k]   (never rounded),
 *   y = xhat * w^T.
 * eps is the fp32 value the GPU entry point receives, widened exactly.
 */
int thi_oracle_rmsnorm_qkv(const uint16_t *x, const uint16_t *gamma, float eps,
                           const uint16_t *w, double *y, double *s,
                           long M, long N, long K)
{
    double *a = (double *)malloc((size_t)M * K * sizeof(double));
    double *g = (double *)malloc((size_t)K * sizeof(double));
    if (!a || !g) { free(a); free(g); return -1; }
    widen_row(x, a, M * K);
    widen_row(gamma, g, K);
    for (long m = 0; m < M; ++m) {
        double *row = a + m * K;
        double sumsq = 0.0;
        for (long k = 0; k < K; ++k) sumsq += row[k] * row[k];
        double r = 1.0 / sqrt(sumsq / (double)K + (double)eps);
        for (long k = 0; k < K; ++k) row[k] = row[k] * r * g[k];
    }
    int rc = dense_rows(a, w, y, s, M, N, K);
    free(a);
    free(g);
    return rc;
}

/*
 * Sec. III-C.1 (low-density operator placed behind the linear operators):
 *   gate = x * wg^T, up = x * wu^T          x[M,H], wg/wu[I,H]
 *   h    = silu(gate) * up                  (fp64, never rounded)
 *   y    = h * wd^T                         wd[H,I]
 *   s[m,n] = sum_j |h[m,j] * wd[n,j]|
 * h_out (may be NULL) receives h[M,I] so tests can check the composition.
 */
int thi_oracle_swiglu_mlp(const uint16_t *x, const uint16_t *wg, const uint16_t *wu,
                          const uint16_t *wd, double *y, double *s, double *h_out,
                          long M, long H, long I)
{
    double *a = (double *)malloc((size_t)M * H * sizeof(double));
    double *gate = (double *)malloc((size_t)M * I * sizeof(double));
    double *up = (double *)malloc((size_t)M * I * sizeof(double));
    int rc = -1;
    if (a && gate && up) {
        widen_row(x, a, M * H);
        rc = dense_rows(a, wg, gate, NULL, M, I, H);
        if (rc == 0) rc = dense_rows(a, wu, up, NULL, M, I, H);
        if (rc == 0) {
            for (long i = 0; i < M * I; ++i) gate[i] = thi_oracle_silu(gate[i]) * up[i];
            if (h_out) memcpy(h_out, gate, (size_t)M * I * sizeof(double));
            rc = dense_rows(gate, wd, y, s, M, H, I);
        }
    }
    free(a);
    free(gate);
    free(up);
    return rc;
}

/*
 * The decoder layer of Sec. III-D.3 (norm -> attention -> norm -> FFN, each block wrapped in a
 * residual connection as in the Llama layer the paper takes as given) closes two fusion units with
 * an addition and opens the second one with a normalisation:
 *   linear_residual     : y = res + x * w^T                      (O projection, down projection)
 *   rmsnorm_swiglu_mlp  : n = rmsnorm(x; gamma, eps) (never rounded), h = silu(n wg^T) * (n wu^T),
 *                         y = res + h * wd^T                     (res may be NULL: no addition)
 * The residual is fp16 like every activation and is widened exactly; S gains |res[m,n]|.
 */
int thi_oracle_linear_residual(const uint16_t *x, const uint16_t *w, const uint16_t *res, double *y, double *s,
                               long M, long N, long K)
{
    int rc = thi_oracle_linear(x, w, y, s, M, N, K);
    if (rc) return rc;
    for (long i = 0; i < M * N; ++i) {
        const double r = half_bits_to_double(res[i]);
        y[i] += r;
        if (s) s[i] += fabs(r);
    }
    return 0;
}

int thi_oracle_rmsnorm_swiglu_mlp(const uint16_t *x, const uint16_t *gamma, float eps, const uint16_t *wg,
                                  const uint16_t *wu, const uint16_t *wd, const uint16_t *res, double *y,
                                  double *s, double *h_out, long M, long H, long I)
{
    double *a = (double *)malloc((size_t)M * H * sizeof(double));
    double *g = (double *)malloc((size_t)H * sizeof(double));
    double *gate = (double *)malloc((size_t)M * I * sizeof(double));
    double *up = (double *)malloc((size_t)M * I * sizeof(double));
    int rc = -1;
    if (a && g && gate && up) {
        widen_row(x, a, M * H);
        widen_row(gamma, g, H);
        for (long m = 0; m < M; ++m) {
            double *row = a + m * H;
            double sumsq = 0.0;
            for (long k = 0; k < H; ++k) sumsq += row[k] * row[k];
            double r = 1.0 / sqrt(sumsq / (double)H + (double)eps);
            for (long k = 0; k < H; ++k) row[k] = row[k] * r * g[k];
        }
        rc = dense_rows(a, wg, gate, NULL, M, I, H);
        if (rc == 0) rc = dense_rows(a, wu, up, NULL, M, I, H);
        if (rc == 0) {
            for (long i = 0; i < M * I; ++i) gate[i] = thi_oracle_silu(gate[i]) * up[i];
            if (h_out) memcpy(h_out, gate, (size_t)M * I * sizeof(double));
            rc = dense_rows(gate, wd, y, s, M, H, I);
        }
        if (rc == 0 && res) {
            for (long i = 0; i < M * H; ++i) {
                const double r = half_bits_to_double(res[i]);
                y[i] += r;
                if (s) s[i] += fabs(r);
            }
        }
    }
    free(a);
    free(g);
    free(gate);
    free(up);
    return rc;
}

/*
 * Rotary position embedding fused behind the QKV projection (Algorithm 1, "Linear-RoPE fusion":
 * the rotation is applied to the accumulator tile before it is stored).  Reading taken: the
 * listing builds its "mix" vector by swapping neighbouring elements with a sign, i.e. the pairs
 * are the interleaved neighbours (2i, 2i+1) of each head; the angle of pair i at token m is
 * pos[m] * theta[i], with theta a caller-supplied fp32 table of head_dim/2 entries (the listing
 * loads theta from memory and multiplies it by the row's position).
 *
 *   (a, b) = (y[m, c], y[m, c+1]),  c even, c < n_rot,  i = (c mod head_dim) / 2
 *   out[m, c]   = a cos(ang) - b sin(ang)
 *   out[m, c+1] = b cos(ang) + a sin(ang)
 * Columns >= n_rot (the V projection) are left as they are.  S follows the same linear map with
 * absolute values: S'[c] = S[c]|cos| + S[c+1]|sin|, S'[c+1] = S[c+1]|cos| + S[c]|sin|.
 * The angle is formed in fp64 from the exact values of the int32 position and the fp32 theta.
 */
int thi_oracle_rope_inplace(double *y, double *s, const int32_t *pos, const float *theta,
                            long M, long N, long n_rot, long head_dim)
{
    if (head_dim <= 0 || (head_dim & 1) || n_rot < 0 || n_rot > N || (n_rot % head_dim)) return -2;
    for (long m = 0; m < M; ++m) {
        for (long c = 0; c < n_rot; c += 2) {
            long i = (c % head_dim) / 2;
            double ang = (double)pos[m] * (double)theta[i];
            double cs = cos(ang), sn = sin(ang);
            double a = y[m * N + c], b = y[m * N + c + 1];
            y[m * N + c] = a * cs - b * sn;
            y[m * N + c + 1] = b * cs + a * sn;
            if (s) {
                double sa = s[m * N + c], sb = s[m * N + c + 1];
                s[m * N + c] = sa * fabs(cs) + sb * fabs(sn);
                s[m * N + c + 1] = sb * fabs(cs) + sa * fabs(sn);
            }
        }
    }
    return 0;
}

int thi_oracle_rmsnorm_qkv_rope(const uint16_t *x, const uint16_t *gamma, float eps, const uint16_t *w,
                                const int32_t *pos, const float *theta, double *y, double *s,
                                long M, long N, long K, long n_rot, long head_dim)
{
    int rc = thi_oracle_rmsnorm_qkv(x, gamma, eps, w, y, s, M, N, K);
    if (rc) return rc;
    return thi_oracle_rope_inplace(y, s, pos, theta, M, N, n_rot, head_dim);
}

/*
 * Decode attention, one new token per request against that request's own key/value cache
 * (Eq. 6: softmax(Q K^T / sqrt(d)) V per head; Sec. III-D.1: attention is run per request because
 * every request has its own cache).  Layout taken: q[B,Hq,D]; k, v[B,Hkv,S_max,D] (the positions of
 * one head are contiguous, as the per-head scheduling of Sec. III-C.2 streams them); request b uses
 * positions [0, len[b]).  Query head h reads key/value head h / (Hq/Hkv) (grouped-query attention).
 *   t_j   = scale * sum_d q[b,h,d] * k[b,g,j,d]
 *   p_j   = exp(t_j - max_j t) / sum_j exp(t_j - max_j t)      (the shift cancels: plain softmax)
 *   y[b,h,d] = sum_j p_j * v[b,g,j,d],    s[b,h,d] = sum_j p_j * |v[b,g,j,d]|
 * len[b] = 0 gives y = s = 0.  scale is the fp32 value the GPU entry point receives.
 */
int thi_oracle_decode_attention(const uint16_t *q, const uint16_t *k, const uint16_t *v, const int32_t *len,
                                float scale, double *y, double *s, long B, long Hq, long Hkv, long D, long S_max)
{
    if (B < 1 || Hq < 1 || Hkv < 1 || D < 1 || S_max < 1 || Hq % Hkv) return -2;
    const long group = Hq / Hkv;
    for (long b = 0; b < B; ++b)
        if (len[b] < 0 || len[b] > S_max) return -2;
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (long b = 0; b < B; ++b) {
        for (long h = 0; h < Hq; ++h) {
            const long L = len[b], g = h / group;
            double *yo = y + (b * Hq + h) * D;
            double *so = s ? s + (b * Hq + h) * D : NULL;
            for (long d = 0; d < D; ++d) { yo[d] = 0.0; if (so) so[d] = 0.0; }
            if (L == 0) continue;
            double *t = (double *)malloc((size_t)L * sizeof(double));
            if (!t) { failed = 1; continue; }
            const uint16_t *qh = q + (b * Hq + h) * D;
            const uint16_t *kh = k + ((b * Hkv + g) * S_max) * D;
            const uint16_t *vh = v + ((b * Hkv + g) * S_max) * D;
            double tmax = -INFINITY;
            for (long j = 0; j < L; ++j) {
                double acc = 0.0;
                for (long d = 0; d < D; ++d) acc += half_bits_to_double(qh[d]) * half_bits_to_double(kh[j * D + d]);
                t[j] = (double)scale * acc;
                if (t[j] > tmax) tmax = t[j];
            }
            double denom = 0.0;
            for (long j = 0; j < L; ++j) { t[j] = exp(t[j] - tmax); denom += t[j]; }
            for (long j = 0; j < L; ++j) {
                const double p = t[j] / denom;
                for (long d = 0; d < D; ++d) {
                    const double val = half_bits_to_double(vh[j * D + d]);
                    yo[d] += p * val;
                    if (so) so[d] += p * fabs(val);
                }
            }
            free(t);
        }
    }
    return failed ? -1 : 0;
}
