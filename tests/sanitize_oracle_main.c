/* Driver for the sanitizer build of the CPU oracle (tests/test_sanitize.py compiles this file together with
 * oracle/moss_oracle.c under -fsanitize=address,undefined and runs it): every exported oracle function once on
 * small, ragged and degenerate inputs, with heap buffers of exactly the documented sizes, so that an access
 * past a buffer, a signed overflow or a misaligned access in the oracle ends the run with a report. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { float s_base, s_cur; double cum_lr; int64_t step, last_rebase; float amax_seen; uint32_t overflow_count, clipped_count, reserved; } wstate;
typedef struct { float lr, beta1, beta2, eps, weight_decay, one_minus_beta1, one_minus_beta2, bias_corr1, bias_corr2, margin; int32_t interval; } adamw;

double moss_oracle_e4m3_decode(uint8_t);
uint8_t moss_oracle_e4m3_encode(double);
int moss_oracle_quant_act_2level(const uint16_t *, int64_t, int64_t, int64_t, int, int, uint8_t *, uint8_t *, float *);
int moss_oracle_quant_act_2level_given_max(const uint16_t *, int64_t, int64_t, int64_t, int, int, uint16_t, uint8_t *, uint8_t *, float *);
int moss_oracle_dequant(const uint8_t *, const uint8_t *, float, int64_t, int64_t, double *);
int moss_oracle_weight_init(const float *, int64_t, int64_t, wstate *, uint8_t *, uint8_t *);
int moss_oracle_weight_step(float *, float *, float *, const void *, int, int64_t, int64_t, const adamw *, wstate *, uint8_t *, uint8_t *);
int moss_oracle_gemm(int64_t, int64_t, int64_t, const uint8_t *, const uint8_t *, float, const uint8_t *, const uint8_t *, float, double *);
int moss_oracle_gemm_sampled(int64_t, int64_t, int64_t, const uint8_t *, const uint8_t *, float, const uint8_t *, const uint8_t *, float,
                             const int64_t *, const int64_t *, int64_t, double *);
int moss_oracle_row_norms(int64_t, int64_t, const uint8_t *, const uint8_t *, float, double *);
int moss_oracle_swiglu(const uint16_t *, const uint16_t *, int64_t, double *);
int moss_oracle_swiglu_backward(const uint16_t *, const uint16_t *, const uint16_t *, int64_t, double *, double *);
double moss_oracle_snr_db(const double *, const double *, int64_t);
int moss_oracle_rmsnorm(const uint16_t *, const uint16_t *, double, int64_t, int64_t, double *);
int moss_oracle_rmsnorm_backward(const uint16_t *, const uint16_t *, const uint16_t *, const uint16_t *, double, int64_t, int64_t, double *);
int moss_oracle_groupwise_fp8(const uint16_t *, int64_t, int64_t, int64_t, uint8_t *, float *, double *);

static uint64_t rs = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) { rs ^= rs << 13; rs ^= rs >> 7; rs ^= rs << 17; return (uint32_t)(rs >> 32); }
static uint16_t bf16_of(float f) { uint32_t u; memcpy(&u, &f, 4); return (uint16_t)((u + 0x7FFF + ((u >> 16) & 1)) >> 16); }
#define CHECK(c) do { if (!(c)) { printf("check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static int quant_case(int64_t rows, int64_t cols, int64_t ld, float scale)
{
    uint16_t *x = malloc(sizeof(uint16_t) * (size_t)(rows * ld));
    for (int64_t i = 0; i < rows * ld; i++) x[i] = bf16_of(scale * ((float)(rnd() % 2001) - 1000.0f) / 250.0f);
    uint16_t mx = 0;
    for (int64_t r = 0; r < rows; r++) for (int64_t c = 0; c < cols; c++) { uint16_t a = x[r * ld + c] & 0x7FFF; if (a > mx) mx = a; }
    for (int axis = 0; axis < 2; axis++) {
        if (axis == 1 && rows % 32) continue;
        int64_t outer = axis ? cols : rows, inner = axis ? rows : cols;
        uint8_t *q = malloc((size_t)(outer * inner)), *e = malloc((size_t)(outer * inner / 32)), *q2 = malloc((size_t)(outer * inner)), *e2 = malloc((size_t)(outer * inner / 32));
        double *dq = malloc(sizeof(double) * (size_t)(outer * inner)), *nrm = malloc(sizeof(double) * (size_t)outer);
        float s, s2;
        for (int mode = 0; mode < 2; mode++) {
            CHECK(moss_oracle_quant_act_2level(x, rows, cols, ld, axis, mode, q, e, &s) == 0);
            CHECK(moss_oracle_quant_act_2level_given_max(x, rows, cols, ld, axis, mode, mx, q2, e2, &s2) == 0);
            CHECK(s == s2 && !memcmp(q, q2, (size_t)(outer * inner)) && !memcmp(e, e2, (size_t)(outer * inner / 32)));
            CHECK(moss_oracle_dequant(q, e, s, outer, inner, dq) == 0);
            CHECK(moss_oracle_row_norms(outer, inner, q, e, s, nrm) == 0);
        }
        free(q); free(e); free(q2); free(e2); free(dq); free(nrm);
    }
    free(x);
    return 0;
}

int main(void)
{
    for (int c = 0; c < 256; c++) { double v = moss_oracle_e4m3_decode((uint8_t)c); if (!isnan(v)) CHECK(moss_oracle_e4m3_encode(v) == (uint8_t)c); }
    CHECK(moss_oracle_e4m3_encode(1e30) == 0x7E && moss_oracle_e4m3_encode(-1e30) == 0xFE && moss_oracle_e4m3_encode(-0.0) == 0x80);
    if (quant_case(1, 32, 32, 1.0f) || quant_case(7, 96, 104, 1.0f) || quant_case(64, 160, 160, 1e-30f) || quant_case(32, 32, 40, 0.0f) ||
        quant_case(96, 64, 64, 1e30f)) return 1;

    /* weight path: ragged size, FP32 and BF16 gradients, a re-scaling step */
    const int64_t rows = 5, cols = 12, n = rows * cols;
    float *w = malloc(sizeof(float) * n), *m = calloc(n, sizeof(float)), *v = calloc(n, sizeof(float)), *g = malloc(sizeof(float) * n);
    uint16_t *gb = malloc(sizeof(uint16_t) * n);
    uint8_t *wq = malloc(n), *wqt = malloc(n);
    for (int64_t i = 0; i < n; i++) w[i] = ((float)(rnd() % 2001) - 1000.0f) * 2e-5f;
    wstate st;
    CHECK(moss_oracle_weight_init(w, rows, cols, &st, wq, wqt) == 0);
    for (int t = 1; t <= 6; t++) {
        for (int64_t i = 0; i < n; i++) { g[i] = ((float)(rnd() % 2001) - 1000.0f) * 1e-6f; gb[i] = bf16_of(g[i]); }
        adamw a = {3e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, 0.1f, 0.05f, (float)(1.0 - pow(0.9, t)), (float)(1.0 - pow(0.95, t)), 1.0f, 3};
        CHECK(moss_oracle_weight_step(w, m, v, (t & 1) ? (const void *)g : (const void *)gb, !(t & 1), rows, cols, &a, &st, wq, (t & 2) ? wqt : NULL) == 0);
    }
    CHECK(st.step == 6 && st.last_rebase == 6);
    free(w); free(m); free(v); free(g); free(gb); free(wq); free(wqt);

    /* GEMM: with and without exponents, full and sampled */
    const int64_t M = 5, N = 3, K = 64;
    uint8_t *a = malloc(M * K), *b = malloc(N * K), *ae = malloc(M * K / 32), *be = malloc(N * K / 32);
    for (int64_t i = 0; i < M * K; i++) { a[i] = (uint8_t)rnd(); if ((a[i] & 0x7F) == 0x7F) a[i] = 0x30; }
    for (int64_t i = 0; i < N * K; i++) { b[i] = (uint8_t)rnd(); if ((b[i] & 0x7F) == 0x7F) b[i] = 0x30; }
    for (int64_t i = 0; i < M * K / 32; i++) ae[i] = (uint8_t)(100 + rnd() % 28);
    for (int64_t i = 0; i < N * K / 32; i++) be[i] = (uint8_t)(rnd() % 128);
    double *out = malloc(sizeof(double) * M * N), smp[4];
    int64_t ms[4] = {0, 4, 2, 4}, ns[4] = {0, 2, 1, 0};
    CHECK(moss_oracle_gemm(M, N, K, a, ae, 0.5f, b, be, 2.0f, out) == 0);
    CHECK(moss_oracle_gemm_sampled(M, N, K, a, ae, 0.5f, b, be, 2.0f, ms, ns, 4, smp) == 0);
    for (int i = 0; i < 4; i++) CHECK(smp[i] == out[ms[i] * N + ns[i]]);
    CHECK(moss_oracle_gemm(M, N, K, a, NULL, 0.5f, b, NULL, 2.0f, out) == 0);
    ms[1] = M;   /* out of range: must be refused, not read */
    CHECK(moss_oracle_gemm_sampled(M, N, K, a, ae, 0.5f, b, be, 2.0f, ms, ns, 4, smp) != 0);
    free(a); free(b); free(ae); free(be); free(out);

    /* SwiGLU and SNR */
    uint16_t gt[9], up[9], dh[9];
    double h[9], dg[9], du[9];
    for (int i = 0; i < 9; i++) { gt[i] = bf16_of((float)(i - 4) * 3.0f); up[i] = bf16_of((float)i * 0.5f); dh[i] = bf16_of(1e-3f * (float)(i + 1)); }
    CHECK(moss_oracle_swiglu(gt, up, 9, h) == 0 && moss_oracle_swiglu_backward(gt, up, dh, 9, dg, du) == 0);
    CHECK(moss_oracle_swiglu(gt, up, 0, h) == 0);
    /* RMSNorm and the comparison quantizers on exactly sized buffers */
    {
        const int64_t r = 3, c = 48;
        uint16_t *hh = malloc(sizeof(uint16_t) * r * c), *gg = malloc(sizeof(uint16_t) * c), *dd = malloc(sizeof(uint16_t) * r * c);
        double *yy = malloc(sizeof(double) * r * c), *dq = malloc(sizeof(double) * r * c);
        uint8_t *qq = malloc(r * c);
        float *sc = malloc(sizeof(float) * r * c / 16);
        for (int64_t i = 0; i < r * c; i++) { hh[i] = bf16_of(((float)(rnd() % 2001) - 1000.0f) / 300.0f); dd[i] = bf16_of(((float)(rnd() % 2001) - 1000.0f) * 1e-3f); }
        for (int64_t i = 0; i < c; i++) gg[i] = bf16_of(1.0f + (float)(i % 5) * 0.1f);
        CHECK(moss_oracle_rmsnorm(hh, gg, 1e-5, r, c, yy) == 0);
        CHECK(moss_oracle_rmsnorm_backward(hh, gg, dd, NULL, 1e-5, r, c, yy) == 0);
        CHECK(moss_oracle_rmsnorm_backward(hh, gg, dd, hh, 0.0, r, c, yy) == 0);
        CHECK(moss_oracle_groupwise_fp8(hh, r, c, 16, qq, sc, dq) == 0 && moss_oracle_groupwise_fp8(hh, r, c, 0, qq, sc, dq) == 0);
        CHECK(moss_oracle_groupwise_fp8(hh, r, c, 32, qq, NULL, dq) != 0);      /* 48 % 32 != 0: refused */
        free(hh); free(gg); free(dd); free(yy); free(dq); free(qq); free(sc);
    }
    double xs[3] = {3, 4, 0}, ds[3] = {3, 4, 1};
    CHECK(fabs(moss_oracle_snr_db(xs, ds, 3) - 13.979400086720377) < 1e-12);
    printf("oracle sanitizer run: ok\n");
    return 0;
}
