/*
 * MOSS CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct implementation of what the MOSS hot path
 * computes (arXiv 2511.05811): two-level microscaled FP8 quantization of
 * activations (Sec. 3.1, Eq. 2-3), per-tensor FP8 weights with the automatic
 * scaling rule fused into an AdamW step (Sec. 2.2 Eq. 1, Sec. 3.2 Eq. 10,
 * App. C), and the block-scaled FP8 GEMM with epilogue dequantization
 * (Sec. 3.1, Fig. 3b).
 *
 * Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
 * load this file.  It shares no code, header, table or constant generator
 * with the HIP library and includes no HIP header.  Every step is written in
 * the paper's order and notation; there is no blocking, fusion or reordering.
 * OpenMP is used only across independent rows / output entries.
 *
 * Every function here is pinned by tests/test_oracle_*.py ("-m 'not gpu'"):
 * exhaustive E4M3 tables against a library cast, exact rational brute force,
 * closed forms and invariants.  Parity-unpinned functions: none.  (The paper's
 * SNR *gaps* between schemes come from activations of a trained model and are
 * compared only softly on synthetic tensors; the functions that compute them
 * are pinned.)
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define MOSS_O_OK 0
#define MOSS_O_BAD_ARG 1
#define MOSS_O_NONFINITE 2

#define E4M3_MAX 448.0 /* Delta_max of E4M3, Sec. 3.1 below Eq. 2 */
#define K2 32          /* level-2 group size, Sec. 3.1 ("k2 = 32") */

/* ------------------------------------------------------------------ */
/* E4M3 ("FN" flavour of the OCP 8-bit format the paper cites in Sec. 2.1):
 * 1 sign, 4 exponent bits (bias 7), 3 mantissa bits, no infinities,
 * S.1111.111 is NaN, largest finite value 448, subnormal step 2^-9.     */

double moss_oracle_e4m3_decode(uint8_t code)
{
    int sign = code >> 7, ex = (code >> 3) & 0xF, man = code & 7;
    double v;
    if (ex == 0xF && man == 7) return NAN;
    if (ex == 0) v = ldexp((double)man, -9);              /* subnormal: man * 2^-9 */
    else         v = ldexp(1.0 + (double)man / 8.0, ex - 7);
    return sign ? -v : v;
}

/* Round-to-nearest, ties to even mantissa, |y| > 448 saturates to +-448.
 * The sign of y is kept (so -0 and negative values that round to zero give
 * 0x80).  y must not be NaN. */
uint8_t moss_oracle_e4m3_encode(double y)
{
    uint8_t sign = signbit(y) ? 0x80 : 0x00;
    double a = fabs(y);
    if (a > E4M3_MAX) return sign | 0x7E;
    if (a < ldexp(1.0, -6)) {
        /* subnormal range (and the step up to the first normal): grid 2^-9.
         * rint() is round-half-even in the default rounding mode; a result of
         * 8 is the code of 2^-6, the smallest normal.                      */
        double q = rint(ldexp(a, 9));
        return sign | (uint8_t)q;
    }
    int ex;
    (void)frexp(a, &ex);          /* a = f * 2^ex, f in [0.5,1) -> floor(log2 a) = ex-1 */
    ex -= 1;
    double q = rint(ldexp(a, 3 - ex)); /* a / 2^(ex-3) in [8,16) -> integer in [8,16] */
    if (q == 16.0) { q = 8.0; ex += 1; }
    return sign | (uint8_t)(((ex + 7) << 3) | ((int)q - 8));
}

/* ------------------------------------------------------------------ */
/* small helpers                                                        */

static double bf16_to_double(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* Round a double to 24 significant bits, ties to even, unbounded exponent. */
static double round_to_24_bits(double p)
{
    if (p == 0.0) return p;
    int ex;
    double f = frexp(p, &ex);          /* |f| in [0.5,1) */
    double r = rint(ldexp(f, 24));     /* integer with |r| in [2^23, 2^24] */
    return ldexp(r, ex - 24);
}

/* Level-2 exponent e_i = round(log2(amax_i / amax)) (Eq. 3), evaluated
 * exactly.  mode 0 (nearest, the paper's "closest power of two" in the log
 * domain): the unique integer k with 2^(2k-1) <= (amax_i/amax)^2 < 2^(2k+1).
 * mode 1 (ceil): the smallest k with amax_i <= 2^k * amax.  Squares of BF16
 * values and their power-of-two multiples are exact in double.  Result is
 * clamped to [-127, 0]; an all-zero group gives -127.                  */
static int local_exponent(double amax_i, double amax, int mode)
{
    if (amax_i == 0.0) return -127;
    int k = ilogb(amax_i) - ilogb(amax) - 2;
    if (mode == 0) {
        double r2 = amax_i * amax_i, a2 = amax * amax;
        while (!(r2 < ldexp(a2, 2 * k + 1))) k++;
    } else {
        while (!(amax_i <= ldexp(amax, k))) k++;
    }
    if (k < -127) k = -127;
    if (k > 0) k = 0;   /* cannot happen: amax_i <= amax */
    return k;
}

/* ------------------------------------------------------------------ */
/* Two-level microscaling quantizer (Sec. 3.1, Eq. 2-3 and the quantize /
 * dequantize maps Q = round(X / (s*ss_i)), DQ = Q*s*ss_i).
 *
 * x        BF16 bits, rows x cols, row stride ld (elements)
 * axis     0: groups of 32 along the columns (row-major outputs
 *             q[rows][cols], e[rows][cols/32]);
 *          1: groups of 32 along the rows, outputs stored transposed
 *             (q[cols][rows], e[cols][rows/32]).
 * exp_mode 0 nearest (Eq. 3), 1 ceil.
 * The global scale s is per tensor and does not depend on axis.        */
static int quant_with_max(const uint16_t *x, int64_t rows, int64_t cols, int64_t ld, int axis, int exp_mode,
                          double given_max, uint8_t *q, uint8_t *e, float *s_global);

int moss_oracle_quant_act_2level(const uint16_t *x, int64_t rows, int64_t cols, int64_t ld,
                                 int axis, int exp_mode,
                                 uint8_t *q, uint8_t *e, float *s_global)
{
    return quant_with_max(x, rows, cols, ld, axis, exp_mode, -1.0, q, e, s_global);
}

/* The same with the tensor maximum of Eq. 2 handed in by whoever produced X (BF16 magnitude bits)
 * instead of being searched for: it has to be at least max|X|; with exactly max|X| the result is that
 * of moss_oracle_quant_act_2level.                                                                  */
int moss_oracle_quant_act_2level_given_max(const uint16_t *x, int64_t rows, int64_t cols, int64_t ld,
                                           int axis, int exp_mode, uint16_t max_bf16_bits,
                                           uint8_t *q, uint8_t *e, float *s_global)
{
    double given = bf16_to_double((uint16_t)(max_bf16_bits & 0x7FFF));
    if (!isfinite(given)) return MOSS_O_NONFINITE;
    return quant_with_max(x, rows, cols, ld, axis, exp_mode, given, q, e, s_global);
}

static int quant_with_max(const uint16_t *x, int64_t rows, int64_t cols, int64_t ld, int axis, int exp_mode,
                          double given_max, uint8_t *q, uint8_t *e, float *s_global)
{
    if (!x || !q || !e || !s_global) return MOSS_O_BAD_ARG;
    if (rows <= 0 || cols <= 0 || ld < cols) return MOSS_O_BAD_ARG;
    if (axis == 0 && cols % K2) return MOSS_O_BAD_ARG;
    if (axis == 1 && rows % K2) return MOSS_O_BAD_ARG;

    /* level 1 (Eq. 2): s_i = amax_i / 448, and s = max_i s_i = amax / 448 */
    double amax = 0.0;
    for (int64_t r = 0; r < rows; r++)
        for (int64_t c = 0; c < cols; c++) {
            double v = fabs(bf16_to_double(x[r * ld + c]));
            if (!isfinite(v)) return MOSS_O_NONFINITE;
            if (v > amax) amax = v;
        }
    if (given_max >= 0.0) {
        if (given_max < amax) return MOSS_O_BAD_ARG;    /* not a bound of |X| */
        amax = given_max;
    }
    float s = 1.0f;                       /* all-zero tensor: s = 1 */
    if (amax > 0.0) s = (float)amax / 448.0f;   /* one IEEE single division */
    float inv_s = 1.0f / s;               /* one IEEE single division */
    /* Eq. 2 divides by a positive scale, so a zero input has code zero.  For a tensor whose
     * maximum is below 448 * 2^-128 the single-precision reciprocal overflows and 0 * inf
     * would be NaN: the largest finite single stands in for it (nonzero inputs still
     * saturate or round as their true quotient would within a factor the format cannot
     * resolve).                                                                            */
    if (!isfinite(inv_s)) inv_s = FLT_MAX;
    *s_global = s;

    int64_t n_outer = axis == 0 ? rows : cols;        /* index of the output row */
    int64_t n_inner = axis == 0 ? cols : rows;        /* length along the grouping axis */
    int64_t n_groups = n_inner / K2;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < n_outer; o++) {
        for (int64_t g = 0; g < n_groups; g++) {
            double xv[K2];
            double amax_i = 0.0;
            for (int j = 0; j < K2; j++) {
                int64_t i = g * K2 + j;
                int64_t r = axis == 0 ? o : i, c = axis == 0 ? i : o;
                xv[j] = bf16_to_double(x[r * ld + c]);
                if (fabs(xv[j]) > amax_i) amax_i = fabs(xv[j]);
            }
            /* level 2 (Eq. 3): ss_i = 2^{e_i}, stored as the E8M0 byte e_i + 127 */
            int e_i = local_exponent(amax_i, amax, exp_mode);
            e[o * n_groups + g] = (uint8_t)(e_i + 127);
            for (int j = 0; j < K2; j++) {
                /* y = x / (s * ss_i): one single-precision multiply by 1/s
                 * (exact product, rounded once to 24 bits), then the exact
                 * power-of-two step, then one rounding to E4M3.           */
                double p = round_to_24_bits(xv[j] * (double)inv_s);
                double y = ldexp(p, -e_i);
                q[o * n_inner + g * K2 + j] = moss_oracle_e4m3_encode(y);
            }
        }
    }
    return MOSS_O_OK;
}

/* DQ = Q * s * ss_i (Sec. 3.1) for a quantized [outer x inner] tensor. */
int moss_oracle_dequant(const uint8_t *q, const uint8_t *e, float s,
                        int64_t outer, int64_t inner, double *out)
{
    if (!q || !out || inner % K2) return MOSS_O_BAD_ARG;
    int64_t n_groups = inner / K2;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; o++)
        for (int64_t i = 0; i < inner; i++) {
            int ex = e ? (int)e[o * n_groups + i / K2] - 127 : 0;
            out[o * inner + i] = ldexp(moss_oracle_e4m3_decode(q[o * inner + i]), ex) * (double)s;
        }
    return MOSS_O_OK;
}

/* ------------------------------------------------------------------ */
/* Weight path: per-tensor FP8 weights with automatic scaling (Sec. 3.2).   */

typedef struct {
    float s_base;            /* s_0 of Eq. 10: amax(W)/448 at the last max-reduction */
    float s_cur;             /* scale used by the latest cast, s_t of Eq. 10 */
    double cum_lr;           /* sum of (margin * eta) since the last max-reduction ("eta * t") */
    int64_t step;            /* optimizer steps taken */
    int64_t last_rebase;     /* step of the last max-reduction */
    float amax_seen;         /* amax of the weights at the latest cast */
    uint32_t overflow_count; /* elements outside the range the scale covers, |w| > 448 * s_cur
                                (compared exactly), summed over all casts */
    uint32_t clipped_count;  /* elements whose code the saturation changed: |fl(w * fl(1/s))| > 464,
                                the midpoint above 448; summed over all casts */
    uint32_t reserved;       /* always 0 here (the device library keeps a flag word in this place) */
} moss_oracle_wstate;

typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    float one_minus_beta1, one_minus_beta2; /* caller-rounded (1-beta) */
    float bias_corr1, bias_corr2;           /* caller-rounded 1-beta^t */
    float margin;                           /* multiplies eta in Eq. 10; the paper uses 1 */
    int32_t interval;                       /* max-reduction every `interval` steps; <=0: never */
} moss_oracle_adamw_args;

/* Q_W = round_E4M3(W / s) with W/s evaluated as one single-precision multiply
 * by fl(1/s); s == 0 (all-zero tensor) maps everything to zero codes.     */
static void cast_weights(const float *w, int64_t n, float s, uint8_t *wq,
                         float *amax_out, uint32_t *overflow_add, uint32_t *clipped_add)
{
    float inv_s = s > 0.0f ? 1.0f / s : 0.0f;
    float amax = 0.0f;
    uint32_t over = 0, clipped = 0;
    /* The scale is meant to keep W / s inside [-448, 448] (Sec. 3.2, text under Eq. 10).  An
     * element breaks that when |w| > 448 * s; the product of a single and 448 is exact in
     * double, so the comparison is exact.                                                  */
    const double range = E4M3_MAX * (double)s;
    for (int64_t i = 0; i < n; i++) {
        float y = w[i] * inv_s;
        if (fabsf(w[i]) > amax) amax = fabsf(w[i]);
        if ((double)fabsf(w[i]) > range) over++;
        if (fabsf(y) > 464.0f) clipped++; /* beyond the values that round to 448 on their own */
        if (wq) wq[i] = moss_oracle_e4m3_encode((double)y);
    }
    *amax_out = amax;
    *overflow_add = over;
    *clipped_add = clipped;
}

static void transpose_u8(const uint8_t *src, int64_t rows, int64_t cols, uint8_t *dst)
{
    for (int64_t r = 0; r < rows; r++)
        for (int64_t c = 0; c < cols; c++) dst[c * rows + r] = src[r * cols + c];
}

/* Initialisation: s_0 = amax(W_0)/448 by one max-reduction (Sec. 3.2, text
 * under Eq. 10), then the first cast.  w is FP32 [rows x cols].            */
int moss_oracle_weight_init(const float *w, int64_t rows, int64_t cols,
                            moss_oracle_wstate *st, uint8_t *wq, uint8_t *wq_t)
{
    if (!w || !st || !wq || rows <= 0 || cols <= 0) return MOSS_O_BAD_ARG;
    int64_t n = rows * cols;
    float amax = 0.0f;
    for (int64_t i = 0; i < n; i++) {
        if (!isfinite(w[i])) return MOSS_O_NONFINITE;
        if (fabsf(w[i]) > amax) amax = fabsf(w[i]);
    }
    memset(st, 0, sizeof *st);
    st->s_base = amax / 448.0f;
    st->s_cur = st->s_base;
    uint32_t over, clipped;
    cast_weights(w, n, st->s_cur, wq, &st->amax_seen, &over, &clipped);
    st->overflow_count = over;
    st->clipped_count = clipped;
    if (wq_t) transpose_u8(wq, rows, cols, wq_t);
    return MOSS_O_OK;
}

/* One optimizer step with the cast fused in.
 *  1. AdamW (Eq. 1), FP32, this operation order, nothing contracted.
 *  2. predict (Eq. 10): cum_lr += margin*eta; s_t = s_0 + cum_lr/448.
 *  3. every `interval` steps re-scale from the true maximum (Sec. 3.2,
 *     last paragraph): s_0 = s_t = amax(W_new)/448, cum_lr = 0.
 *  4. cast W_new with s_t; record amax, the number of elements outside 448 * s_t and the
 *     number of elements the saturation changed.
 * g is FP32 (g_is_bf16 == 0) or BF16 bits (g_is_bf16 == 1).              */
int moss_oracle_weight_step(float *w, float *m, float *v, const void *g, int g_is_bf16,
                            int64_t rows, int64_t cols, const moss_oracle_adamw_args *a,
                            moss_oracle_wstate *st, uint8_t *wq, uint8_t *wq_t)
{
    if (!w || !m || !v || !g || !a || !st || !wq || rows <= 0 || cols <= 0) return MOSS_O_BAD_ARG;
    int64_t n = rows * cols;
    const float *g32 = (const float *)g;
    const uint16_t *g16 = (const uint16_t *)g;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; i++) {
        float gi = g_is_bf16 ? (float)bf16_to_double(g16[i]) : g32[i];
        float t1 = a->beta1 * m[i];
        float t2 = a->one_minus_beta1 * gi;
        float mi = t1 + t2;                              /* m_t */
        float t3 = a->beta2 * v[i];
        float t4 = a->one_minus_beta2 * gi;
        float t5 = t4 * gi;
        float vi = t3 + t5;                              /* v_t */
        float mhat = mi / a->bias_corr1;
        float vhat = vi / a->bias_corr2;
        float den = sqrtf(vhat);
        den = den + a->eps;
        float u = mhat / den;
        float wd = a->weight_decay * w[i];
        float upd = u + wd;
        upd = a->lr * upd;
        w[i] = w[i] - upd;                               /* W_{t+1} */
        m[i] = mi;
        v[i] = vi;
    }
    st->step += 1;
    st->cum_lr += (double)a->margin * (double)a->lr;
    st->s_cur = (float)((double)st->s_base + st->cum_lr / 448.0);
    if (a->interval > 0 && st->step % a->interval == 0) {
        float amax = 0.0f;
        for (int64_t i = 0; i < n; i++)
            if (fabsf(w[i]) > amax) amax = fabsf(w[i]);
        st->s_base = amax / 448.0f;
        st->s_cur = st->s_base;
        st->cum_lr = 0.0;
        st->last_rebase = st->step;
    }
    uint32_t over, clipped;
    cast_weights(w, n, st->s_cur, wq, &st->amax_seen, &over, &clipped);
    st->overflow_count += over;
    st->clipped_count += clipped;
    if (wq_t) transpose_u8(wq, rows, cols, wq_t);
    return MOSS_O_OK;
}

/* ------------------------------------------------------------------ */
/* GEMM (Sec. 3.1, Fig. 3b): Q_y = Q_b x (Q_a * ss_a), dequantized in the
 * epilogue by the two FP32 scales.  Here both operands may carry level-2
 * exponents (a NULL exponent pointer is the artificial scale 1):
 *   out[m,n] = a_s*b_s * sum_k dec(a[m,k]) 2^(ae[m,k/32]-127) dec(b[n,k]) 2^(be[n,k/32]-127)
 * a is [M x K], b is [N x K], both K-contiguous; FP64 throughout.        */

static double gemm_entry(int64_t K, const uint8_t *a_row, const uint8_t *ae_row,
                         const uint8_t *b_row, const uint8_t *be_row)
{
    double acc = 0.0;
    for (int64_t k = 0; k < K; k++) {
        double av = moss_oracle_e4m3_decode(a_row[k]);
        double bv = moss_oracle_e4m3_decode(b_row[k]);
        int ea = ae_row ? (int)ae_row[k / K2] - 127 : 0;
        int eb = be_row ? (int)be_row[k / K2] - 127 : 0;
        acc += ldexp(av, ea) * ldexp(bv, eb);
    }
    return acc;
}

int moss_oracle_gemm(int64_t M, int64_t N, int64_t K,
                     const uint8_t *a_q, const uint8_t *a_e, float a_s,
                     const uint8_t *b_q, const uint8_t *b_e, float b_s, double *out)
{
    if (!a_q || !b_q || !out || M <= 0 || N <= 0 || K <= 0 || K % K2) return MOSS_O_BAD_ARG;
    int64_t G = K / K2;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; m++)
        for (int64_t n = 0; n < N; n++)
            out[m * N + n] = (double)a_s * (double)b_s *
                             gemm_entry(K, a_q + m * K, a_e ? a_e + m * G : NULL,
                                        b_q + n * K, b_e ? b_e + n * G : NULL);
    return MOSS_O_OK;
}

/* The same sum for a list of (m, n) pairs only: lets the oracle check sampled
 * outputs of GEMMs too large to recompute in full.                         */
int moss_oracle_gemm_sampled(int64_t M, int64_t N, int64_t K,
                             const uint8_t *a_q, const uint8_t *a_e, float a_s,
                             const uint8_t *b_q, const uint8_t *b_e, float b_s,
                             const int64_t *ms, const int64_t *ns, int64_t count, double *out)
{
    if (!a_q || !b_q || !out || !ms || !ns || K <= 0 || K % K2) return MOSS_O_BAD_ARG;
    int64_t G = K / K2;
    for (int64_t i = 0; i < count; i++)
        if (ms[i] < 0 || ms[i] >= M || ns[i] < 0 || ns[i] >= N) return MOSS_O_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; i++) {
        int64_t m = ms[i], n = ns[i];
        out[i] = (double)a_s * (double)b_s *
                 gemm_entry(K, a_q + m * K, a_e ? a_e + m * G : NULL,
                            b_q + n * K, b_e ? b_e + n * G : NULL);
    }
    return MOSS_O_OK;
}

/* 2-norms of the dequantized rows (global scale folded in): the tolerance of
 * the GEMM comparison is 1e-3 * |a_row| * |b_row| per output.              */
int moss_oracle_row_norms(int64_t R, int64_t K, const uint8_t *q, const uint8_t *e, float s,
                          double *norms)
{
    if (!q || !norms || K % K2) return MOSS_O_BAD_ARG;
    int64_t G = K / K2;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; r++) {
        double acc = 0.0;
        for (int64_t k = 0; k < K; k++) {
            int ex = e ? (int)e[r * G + k / K2] - 127 : 0;
            double v = ldexp(moss_oracle_e4m3_decode(q[r * K + k]), ex) * (double)s;
            acc += v * v;
        }
        norms[r] = sqrt(acc);
    }
    return MOSS_O_OK;
}

/* ------------------------------------------------------------------ */
/* The producer on the input side of the down projection (the paper leaves the non-linear
 * layers in BF16, Sec. 4.1): SwiGLU of a LLaMA feed-forward block,
 *      h = silu(g) * u,   silu(g) = g / (1 + exp(-g)),
 * from BF16 gate and up projections, in double.  Backward for an upstream gradient dh:
 *      d_up = dh * silu(g),   d_gate = dh * u * sig(g) * (1 + g * (1 - sig(g))),   sig(g) = 1 / (1 + exp(-g)).
 * The outputs are the exact doubles: rounding them to BF16 (and taking the maximum of the rounded
 * magnitudes that the quantizer wants) is left to the caller, who knows which rounding he compares with. */
int moss_oracle_swiglu(const uint16_t *gate, const uint16_t *up, int64_t n, double *h)
{
    if (!gate || !up || !h || n < 0) return MOSS_O_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; i++) {
        double g = bf16_to_double(gate[i]), u = bf16_to_double(up[i]);
        h[i] = g / (1.0 + exp(-g)) * u;
    }
    return MOSS_O_OK;
}

int moss_oracle_swiglu_backward(const uint16_t *gate, const uint16_t *up, const uint16_t *dh, int64_t n,
                                double *d_gate, double *d_up)
{
    if (!gate || !up || !dh || !d_gate || !d_up || n < 0) return MOSS_O_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; i++) {
        double g = bf16_to_double(gate[i]), u = bf16_to_double(up[i]), d = bf16_to_double(dh[i]);
        double sig = 1.0 / (1.0 + exp(-g));
        d_up[i] = d * (g * sig);
        d_gate[i] = d * u * (sig * (1.0 + g * (1.0 - sig)));
    }
    return MOSS_O_OK;
}

/* ------------------------------------------------------------------ */
/* The producer in front of the QKV and gate / up projections' quantizers (non-linear layers stay in
 * BF16, Sec. 4.1): RMSNorm of a LLaMA block over each row of h [rows x cols],
 *      y[r, c] = h[r, c] / sqrt(mean_c(h[r, :]^2) + eps) * gamma[c],
 * from BF16 h and gamma, in double.  Backward for an upstream gradient dy, with the gradient that
 * reaches h directly over the residual connection added in (d_res, may be NULL):
 *      g = dy * gamma,  n = h / sqrt(mean(h^2) + eps),
 *      d_h = d_res + (g - n * mean_c(g * n)) / sqrt(mean(h^2) + eps).
 * (The gradient of gamma is not part of the path: it never meets a quantizer.)  Outputs are exact
 * doubles; rounding to BF16 is left to the caller.                                                 */
int moss_oracle_rmsnorm(const uint16_t *h, const uint16_t *gamma, double eps, int64_t rows, int64_t cols, double *y)
{
    if (!h || !gamma || !y || rows <= 0 || cols <= 0 || !(eps >= 0.0)) return MOSS_O_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; r++) {
        double ss = 0.0;
        for (int64_t c = 0; c < cols; c++) {
            double v = bf16_to_double(h[r * cols + c]);
            ss += v * v;
        }
        const double rms = sqrt(ss / (double)cols + eps);
        for (int64_t c = 0; c < cols; c++)
            y[r * cols + c] = bf16_to_double(h[r * cols + c]) / rms * bf16_to_double(gamma[c]);
    }
    return MOSS_O_OK;
}

int moss_oracle_rmsnorm_backward(const uint16_t *h, const uint16_t *gamma, const uint16_t *dy, const uint16_t *d_res,
                                 double eps, int64_t rows, int64_t cols, double *d_h)
{
    if (!h || !gamma || !dy || !d_h || rows <= 0 || cols <= 0 || !(eps >= 0.0)) return MOSS_O_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; r++) {
        double ss = 0.0;
        for (int64_t c = 0; c < cols; c++) {
            double v = bf16_to_double(h[r * cols + c]);
            ss += v * v;
        }
        const double rms = sqrt(ss / (double)cols + eps);
        double dot = 0.0;                                   /* sum_c g n */
        for (int64_t c = 0; c < cols; c++) {
            double g = bf16_to_double(dy[r * cols + c]) * bf16_to_double(gamma[c]);
            dot += g * (bf16_to_double(h[r * cols + c]) / rms);
        }
        const double mean_gn = dot / (double)cols;
        for (int64_t c = 0; c < cols; c++) {
            double g = bf16_to_double(dy[r * cols + c]) * bf16_to_double(gamma[c]);
            double n = bf16_to_double(h[r * cols + c]) / rms;
            double res = d_res ? bf16_to_double(d_res[r * cols + c]) : 0.0;
            d_h[r * cols + c] = res + (g - n * mean_gn) / rms;
        }
    }
    return MOSS_O_OK;
}

/* ------------------------------------------------------------------ */
/* The two schemes the paper compares two-level microscaling with (Sec. 3.1, Proof 1: per-tensor
 * quantization, Eq. 5, and per-group quantization, Eq. 6; the activation-SNR table of Sec. 4.5.2 uses
 * groups of 128): one FP32 scale per `group` consecutive elements of a row, s_g = max|X_g| / 448
 * (1 for an all-zero group), codes round(x / s_g) in E4M3, dequantized value code * s_g.
 * group == 0 means one scale for the whole tensor.  x / s_g is evaluated in double (exact to well
 * below an E4M3 rounding step) and rounded once.  dq receives the dequantized values, scales (may
 * be NULL) the rows * cols / group scales (one for group == 0).                                  */
int moss_oracle_groupwise_fp8(const uint16_t *x, int64_t rows, int64_t cols, int64_t group,
                              uint8_t *q, float *scales, double *dq)
{
    if (!x || !q || !dq || rows <= 0 || cols <= 0 || group < 0) return MOSS_O_BAD_ARG;
    if (group > 0 && cols % group) return MOSS_O_BAD_ARG;
    const int64_t n = rows * cols, g = group > 0 ? group : n;
    for (int64_t i = 0; i < n; i++)
        if (!isfinite(bf16_to_double(x[i]))) return MOSS_O_NONFINITE;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < n / g; b++) {
        double amax = 0.0;
        for (int64_t i = b * g; i < (b + 1) * g; i++) {
            double v = fabs(bf16_to_double(x[i]));
            if (v > amax) amax = v;
        }
        float s = amax > 0.0 ? (float)amax / 448.0f : 1.0f;
        if (scales) scales[b] = s;
        for (int64_t i = b * g; i < (b + 1) * g; i++) {
            q[i] = moss_oracle_e4m3_encode(bf16_to_double(x[i]) / (double)s);
            dq[i] = moss_oracle_e4m3_decode(q[i]) * (double)s;
        }
    }
    return MOSS_O_OK;
}

/* Quantization SNR in dB (Sec. 3.1, Eq. 4): signal power over noise power,
 * 10 log10( sum x^2 / sum (dq - x)^2 ) (the expectations of Eq. 4 over the same n elements;
 * the 1/n cancel).                                                       */
double moss_oracle_snr_db(const double *x, const double *dq, int64_t n)
{
    double ps = 0.0, pn = 0.0;
    for (int64_t i = 0; i < n; i++) {
        ps += x[i] * x[i];
        pn += (dq[i] - x[i]) * (dq[i] - x[i]);
    }
    return 10.0 * log10(ps / pn);
}

int moss_oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
