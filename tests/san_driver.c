/* Driver for the sanitizer run of the CPU oracle: every exported function once on a small ragged block, every
 * buffer a heap allocation of exactly the size the function is documented to touch, so that an access outside it,
 * a signed overflow, a bad shift or a misaligned access stops the run.  Built together with oracle/mesa_ref.c under
 * -fsanitize=address,undefined by tests/test_sanitizers.py; prints OK. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

float mesa_ref_half_to_float(uint16_t h);
uint16_t mesa_ref_float_to_half(float f);
float mesa_ref_bf16_to_float(uint16_t h);
uint16_t mesa_ref_float_to_bf16(float f);
void mesa_ref_philox4x32(const uint32_t ctr[4], const uint32_t key[2], int rounds, uint32_t out[4]);
float mesa_ref_sr_uniform(uint64_t seed, uint64_t offset, uint64_t e);
int mesa_ref_update_running_params(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner, float *alpha, float *beta, float lambda, int first_call);
int mesa_ref_update_running_params_sym(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner, float *alpha, float *beta, float lambda, int first_call);
int mesa_ref_update_running_scale_sym(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner, float *m, float lambda, int first_call);
int mesa_ref_update_running_params_fixed_beta(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner, float *alpha, float *beta, float lambda, int first_call, float beta_fixed);
int mesa_ref_group_minmax(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner, float *mn_out, float *mx_out);
int mesa_ref_quantize_headwise(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner, const float *alpha, const float *beta, int8_t *q, int mode, uint64_t seed, uint64_t offset);
int mesa_ref_quantize_sym(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner, const float *m, int8_t *q, int mode, uint64_t seed, uint64_t offset);
int mesa_ref_quantize_update_fused(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner, float *alpha, float *beta, float lambda, int8_t *q, int mode, uint64_t seed, uint64_t offset);
int mesa_ref_gelu_fwd_q(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner, float *alpha, float *beta, float lambda, double *y, int8_t *q, int mode, uint64_t seed, uint64_t offset);
int mesa_ref_dequantize(const int8_t *q, int64_t outer, int64_t groups, int64_t inner, const float *alpha, const float *beta, void *x_hat, int dt);
int mesa_ref_dequantize_sym(const int8_t *q, int64_t outer, int64_t groups, int64_t inner, const float *m, void *x_hat, int dt);
int mesa_ref_quantize_headwise_b4(const void *x, int dt, int64_t outer, int64_t groups, int64_t inner, const float *alpha, const float *beta, uint8_t *q4, int mode, uint64_t seed, uint64_t offset);
int mesa_ref_dequantize_b4(const uint8_t *q4, int64_t outer, int64_t groups, int64_t inner, const float *alpha, const float *beta, void *x_hat, int dt);
int mesa_ref_gelu_bwd_q_b4(const uint8_t *q4, int64_t outer, int64_t groups, int64_t inner, const float *alpha, const float *beta, const void *dy, int dt, double *dx);
int mesa_ref_softmax_fwd(const void *s, int dt, int64_t total_rows, int64_t cols, double *y);
int mesa_ref_layernorm_fwd(const void *x, int dt, int64_t M, int64_t D, const void *gamma, const void *bias, double eps, double *y, double *mean, double *rstd);
int mesa_ref_softmax_bwd_q(const int8_t *yq, int64_t B, int64_t H, int64_t rows, int64_t cols, const float *alpha, const float *beta, const void *dy, int dt, double *dx);
int mesa_ref_gelu_bwd_q(const int8_t *xq, int64_t outer, int64_t groups, int64_t inner, const float *alpha, const float *beta, const void *dy, int dt, double *dx);
int mesa_ref_relu_bwd_q(const int8_t *xq, int64_t outer, int64_t groups, int64_t inner, const float *alpha, const float *beta, const void *dy, int dt, double *dx);
int mesa_ref_layernorm_bwd_q(const int8_t *xq, int64_t M, int64_t D, int64_t G, const float *alpha, const float *beta, const float *mean, const float *rstd, const void *gamma, const void *dy, int dt, double *dx, double *dgamma, double *dbeta);
int mesa_ref_linear_dw_q(const int8_t *xq, int64_t M, int64_t K, int64_t G, const float *alpha, const float *beta, const void *dy, int64_t N_out, int dt, double *dW, double *db);
int mesa_ref_linear_dw_q_entries(const int8_t *xq, int64_t M, int64_t K, int64_t G, const float *alpha, const float *beta, const void *dy, int64_t N_out, int dt, const int64_t *n_idx, const int64_t *k_idx, int64_t count, double *out);
int mesa_ref_conv2d_dw_q(const int8_t *xq, const int64_t *geom, int64_t G, const float *alpha, const float *beta, const void *dy, int dt, double *dW, double *db);
int mesa_ref_conv2d_dw_q_entries(const int8_t *xq, const int64_t *geom, int64_t G, const float *alpha, const float *beta, const void *dy, int dt, const int64_t *idx, int64_t count, double *out);
int mesa_ref_attn_av_bwd_q(const int8_t *aq, const int8_t *vq, int64_t B, int64_t H, int64_t N, int64_t Dh, const float *alpha_a, const float *beta_a, const float *alpha_v, const float *beta_v, const void *dO, int dt, double *dA, double *dV);
int mesa_ref_attn_qk_bwd_q(const int8_t *qq, const int8_t *kq, int64_t B, int64_t H, int64_t N, int64_t Dh, const float *alpha_q, const float *beta_q, const float *alpha_k, const float *beta_k, const void *dS, int dt, double scale, double *dQ, double *dK);

static uint32_t lcg = 12345u;
static float rnd(void) { lcg = lcg * 1664525u + 1013904223u; return (float)((lcg >> 8) & 0xFFFF) / 32768.0f - 1.0f; }
#define NEW(T, n) ((T *)malloc(sizeof(T) * (size_t)(n)))

/* x of `n` elements in storage type dt (0 binary32, 1 binary16, 2 bfloat16), scaled */
static void *make_x(int dt, int64_t n, float scale)
{
    if (dt == 0) { float *p = NEW(float, n); for (int64_t i = 0; i < n; ++i) p[i] = rnd() * scale; return p; }
    uint16_t *p = NEW(uint16_t, n);
    for (int64_t i = 0; i < n; ++i) p[i] = dt == 1 ? mesa_ref_float_to_half(rnd() * scale) : mesa_ref_float_to_bf16(rnd() * scale);
    return p;
}

int main(void)
{
    /* conversions over every 16-bit pattern and a sweep of binary32 patterns, including infinities and nans */
    double acc = 0.0;
    for (uint32_t h = 0; h < 65536u; ++h) {
        float f = mesa_ref_half_to_float((uint16_t)h), g = mesa_ref_bf16_to_float((uint16_t)h);
        if (f == f) acc += (double)mesa_ref_float_to_half(f);
        if (g == g) acc += (double)mesa_ref_float_to_bf16(g);
    }
    for (uint32_t b = 0; b < 0xFFFF0000u; b += 65521u) {
        float f; memcpy(&f, &b, 4);
        acc += (double)mesa_ref_float_to_half(f) + (double)mesa_ref_float_to_bf16(f);
    }
    uint32_t ctr[4] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0, 0}, key[2] = {0xFFFFFFFFu, 0xFFFFFFFFu}, out[4];
    mesa_ref_philox4x32(ctr, key, 10, out);
    acc += (double)out[0] + (double)mesa_ref_sr_uniform(~0ull, ~0ull - 3, ~0ull);

    for (int dt = 0; dt < 3; ++dt) {
        const int64_t outer = 3, G = 3, inner = 19 * 19, n = outer * G * inner;   /* odd slabs */
        void *x = make_x(dt, n, 2.5f);
        float *a = NEW(float, G), *b = NEW(float, G), *m = NEW(float, G), *mn = NEW(float, G), *mx = NEW(float, G);
        int8_t *q = NEW(int8_t, n);
        double *d64 = NEW(double, n);
        void *dy = make_x(dt, n, 1.0f);
        void *xh = malloc((size_t)n * (dt == 0 ? 4 : 2));
        for (int first = 1; first >= 0; --first) {
            mesa_ref_update_running_params(x, dt, outer, G, inner, a, b, 0.9f, first);
            mesa_ref_update_running_params_sym(x, dt, outer, G, inner, a, b, 0.9f, first);
            mesa_ref_update_running_params_fixed_beta(x, dt, outer, G, inner, a, b, 0.9f, first, -0.17f);
            mesa_ref_update_running_scale_sym(x, dt, outer, G, inner, m, 0.9f, first);
            mesa_ref_update_running_params(x, dt, outer, G, inner, a, b, 0.9f, first);
        }
        mesa_ref_group_minmax(x, dt, outer, G, inner, mn, mx);
        for (int mode = 0; mode < 2; ++mode) {
            mesa_ref_quantize_sym(x, dt, outer, G, inner, m, q, mode, 7, 1ull << 40);
            mesa_ref_dequantize_sym(q, outer, G, inner, m, xh, dt);
            mesa_ref_quantize_headwise(x, dt, outer, G, inner, a, b, q, mode, 0xFFFFFFFFFFFFFFFFull, 0xFFFFFFFFFFFFFFF0ull);
            mesa_ref_quantize_update_fused(x, dt, outer, G, inner, a, b, 0.9f, q, mode, 3, 5);
            mesa_ref_gelu_fwd_q(x, dt, outer, G, inner, a, b, 0.9f, d64, q, mode, 3, 5);
        }
        /* four-bit codes: n is odd, so the last byte holds one code */
        uint8_t *q4 = NEW(uint8_t, (n + 1) / 2);
        for (int mode = 0; mode < 2; ++mode) {
            mesa_ref_quantize_headwise_b4(x, dt, outer, G, inner, a, b, q4, mode, 9, 1ull << 33);
            mesa_ref_dequantize_b4(q4, outer, G, inner, a, b, xh, dt);
            mesa_ref_gelu_bwd_q_b4(q4, outer, G, inner, a, b, dy, dt, d64);
        }
        acc += d64[n - 1];
        free(q4);
        mesa_ref_dequantize(q, outer, G, inner, a, b, xh, dt);
        mesa_ref_gelu_bwd_q(q, outer, G, inner, a, b, dy, dt, d64);
        mesa_ref_relu_bwd_q(q, outer, G, inner, a, b, dy, dt, d64);
        mesa_ref_softmax_bwd_q(q, outer, G, 19, 19, a, b, dy, dt, d64);
        mesa_ref_softmax_fwd(x, dt, outer * G * 19, 19, d64);
        acc += d64[n - 1];
        /* a constant group and a degenerate range */
        a[0] = 0.0f; m[0] = 0.0f;
        mesa_ref_quantize_headwise(x, dt, outer, G, inner, a, b, q, 1, 1, 1);
        mesa_ref_quantize_sym(x, dt, outer, G, inner, m, q, 1, 1, 1);
        /* empty inputs touch nothing */
        mesa_ref_quantize_headwise(NULL, dt, 0, G, inner, a, b, NULL, 0, 0, 0);
        mesa_ref_dequantize(NULL, outer, 0, inner, a, b, NULL, dt);
        free(x); free(a); free(b); free(m); free(mn); free(mx); free(q); free(d64); free(dy); free(xh);

        /* token matrices: LayerNorm forward / backward, Linear weight gradient */
        const int64_t Mr = 37, D = 24, Gc = 3, Nout = 10;
        void *t = make_x(dt, Mr * D, 3.0f), *gam = make_x(dt, D, 1.0f), *bias = make_x(dt, D, 1.0f), *dyt = make_x(dt, Mr * D, 1.0f);
        void *dyl = make_x(dt, Mr * Nout, 1.0f);
        double *y = NEW(double, Mr * D), *mean = NEW(double, Mr), *rstd = NEW(double, Mr);
        float *meanf = NEW(float, Mr), *rstdf = NEW(float, Mr), *ta = NEW(float, Gc), *tb = NEW(float, Gc);
        int8_t *tq = NEW(int8_t, Mr * D);
        double *dx = NEW(double, Mr * D), *dg = NEW(double, D), *dbt = NEW(double, D), *dW = NEW(double, Nout * D), *db = NEW(double, Nout);
        mesa_ref_layernorm_fwd(t, dt, Mr, D, gam, bias, 1e-5, y, mean, rstd);
        for (int64_t i = 0; i < Mr; ++i) { meanf[i] = (float)mean[i]; rstdf[i] = (float)rstd[i]; }
        mesa_ref_update_running_params(t, dt, Mr, Gc, D / Gc, ta, tb, 0.9f, 1);
        mesa_ref_quantize_headwise(t, dt, Mr, Gc, D / Gc, ta, tb, tq, 1, 11, 0);
        mesa_ref_layernorm_bwd_q(tq, Mr, D, Gc, ta, tb, meanf, rstdf, gam, dyt, dt, dx, dg, dbt);
        mesa_ref_linear_dw_q(tq, Mr, D, Gc, ta, tb, dyl, Nout, dt, dW, db);
        int64_t ni[3] = {0, Nout - 1, 4}, ki[3] = {D - 1, 0, 7};
        double ent[3];
        mesa_ref_linear_dw_q_entries(tq, Mr, D, Gc, ta, tb, dyl, Nout, dt, ni, ki, 3, ent);
        acc += dW[Nout * D - 1] + ent[2] + dg[D - 1] + dbt[0];
        free(t); free(gam); free(bias); free(dyt); free(dyl); free(y); free(mean); free(rstd); free(meanf); free(rstdf);
        free(ta); free(tb); free(tq); free(dx); free(dg); free(dbt); free(dW); free(db);

        /* convolution weight gradient: stride, padding and dilation all in play; OH = 4, OW = 10 */
        const int64_t geom[13] = {2, 4, 7, 9, 3, 3, 2, 2, 1, 1, 2, 1, 3};
        int8_t *cq = NEW(int8_t, 2 * 4 * 7 * 9);
        for (int64_t i = 0; i < 2 * 4 * 7 * 9; ++i) cq[i] = (int8_t)(i * 53 % 256 - 128);
        void *cdy = make_x(dt, 2 * 3 * 4 * 10, 1.0f);
        float ca[2] = {1.5f, 3.0f}, cb[2] = {-0.5f, 0.25f};
        double *cdW = NEW(double, 3 * 4 * 3 * 2), *cdb = NEW(double, 3), cent[2];
        int64_t cidx[8] = {0, 0, 0, 0, 2, 3, 2, 1};
        mesa_ref_conv2d_dw_q(cq, geom, 2, ca, cb, cdy, dt, cdW, cdb);
        mesa_ref_conv2d_dw_q_entries(cq, geom, 2, ca, cb, cdy, dt, cidx, 2, cent);
        acc += cdW[3 * 4 * 3 * 2 - 1] + cdb[2] + cent[1];
        free(cq); free(cdy); free(cdW); free(cdb);

        /* attention products */
        const int64_t B = 2, H = 2, N = 7, Dh = 5;
        int8_t *aq = NEW(int8_t, B * H * N * N), *c3 = NEW(int8_t, B * H * N * Dh);
        for (int64_t i = 0; i < B * H * N * N; ++i) aq[i] = (int8_t)(i * 37 % 256 - 128);
        for (int64_t i = 0; i < B * H * N * Dh; ++i) c3[i] = (int8_t)(i * 91 % 256 - 128);
        void *dO = make_x(dt, B * H * N * Dh, 1.0f), *dS = make_x(dt, B * H * N * N, 1.0f);
        float ha[2] = {1.0f, 2.0f}, hb[2] = {-0.5f, 0.0f};
        double *dA = NEW(double, B * H * N * N), *dV = NEW(double, B * H * N * Dh), *dQ = NEW(double, B * H * N * Dh), *dK = NEW(double, B * H * N * Dh);
        mesa_ref_attn_av_bwd_q(aq, c3, B, H, N, Dh, ha, hb, ha, hb, dO, dt, dA, dV);
        mesa_ref_attn_qk_bwd_q(c3, c3, B, H, N, Dh, ha, hb, ha, hb, dS, dt, 0.447, dQ, dK);
        acc += dA[B * H * N * N - 1] + dK[0];
        free(aq); free(c3); free(dO); free(dS); free(dA); free(dV); free(dQ); free(dK);
    }
    printf("OK %s\n", acc == acc ? "finite" : "nan");
    return 0;
}
