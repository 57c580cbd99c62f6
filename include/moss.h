/*
 * moss.h -- C ABI of the MI355X (gfx950) implementation of the MOSS FP8 hot path
 * (arXiv 2511.05811): two-level microscaled FP8 quantization of activations and
 * gradients, per-tensor FP8 weights with automatic scaling fused into the AdamW
 * step, and the block-scaled FP8 GEMMs of a linear layer.
 *
 * Conventions for every entry point
 *  - Every tensor pointer is a DEVICE pointer owned by the caller; the library
 *    allocates nothing and keeps no hidden state besides cached device properties
 *    and the one process-wide setting of moss_quant_set_poll_limit.
 *    Pointers to `moss_adamw_args` are HOST pointers (read during the call).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *    work is enqueued asynchronously on it; nothing synchronizes with the host.
 *  - Scales travel as device scalars, so chaining quantizer -> GEMM needs no host
 *    round trip.
 *  - Argument errors are detected on the host before anything is launched and are
 *    returned as a negative-free status code (never an abort, never an exception).
 *  - Inputs must be finite.  Tensor base pointers and leading dimensions must be
 *    16-byte aligned unless stated otherwise.
 *  - `workspace` is device scratch of at least the size the matching
 *    *_workspace_bytes() call reports; contents need not be initialised and are
 *    clobbered.  Two calls that share a workspace must be ordered on one stream.
 */
#ifndef MOSS_H
#define MOSS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOSS_OK = 0,
    MOSS_ERR_NULL = 1,        /* a required pointer is NULL */
    MOSS_ERR_SHAPE = 2,       /* a size is non-positive or not a multiple of the group size */
    MOSS_ERR_ALIGN = 3,       /* a pointer or leading dimension is not 16-byte aligned */
    MOSS_ERR_WORKSPACE = 4,   /* workspace missing or too small */
    MOSS_ERR_UNSUPPORTED = 5, /* flag / dtype combination not implemented */
    MOSS_ERR_HIP = 6          /* the HIP runtime reported an error (launch, query) */
} moss_status;

const char *moss_status_string(int status);

/* Number of compute units of the current device (0 if no device is usable). */
int moss_device_cu_count(void);

/* ---- element types of operands that come in more than one type -------------- */
#define MOSS_DT_BF16 0
#define MOSS_DT_F32 1

/* ---------------------------------------------------------------------------
 * Two-level microscaling quantizer  (paper Sec. 3.1, Eq. 2 and Eq. 3, and the
 * quantize / dequantize maps Q = round(X / (s ss_i)),  DQ = Q s ss_i).
 *
 *   x        BF16 [rows x cols], row stride `ld` elements.
 *   s        one FP32 global scale per tensor:  s = amax(X) / 448  (s = 1 for an
 *            all-zero tensor); written to *s_global (device).
 *   ss_i     one power of two per group of 32 elements, ss_i = 2^(e_i),
 *            e_i = round(log2(amax_i / amax)) in [-127, 0]  (MOSS_EXP_NEAREST, the
 *            paper's "closest power of two"), or the ceiling (MOSS_EXP_CEIL, which
 *            never saturates a code).  Stored as the E8M0 byte e_i + 127; an
 *            all-zero group stores byte 0.
 *   codes    E4M3 (max 448) of  y = fl32(x * fl32(1/s)) * 2^(-e_i), rounded to
 *            nearest even, saturated to +-448, sign kept (fl32(1/s) is capped at
 *            FLT_MAX, so a zero input has code zero whatever the scale).
 *
 * MOSS_Q_ROW: groups run along the columns (the inner dimension of Y = X W^T and
 *             of dX = dY W): q_row [rows x cols], e_row [rows x cols/32].
 * MOSS_Q_COL: groups run along the rows (the inner dimension of dW = dY^T X), and
 *             the outputs are stored transposed so that the groups are contiguous:
 *             q_col [cols x rows], e_col [cols x rows/32].
 * Both flags may be set in one call; both outputs then share the one global scale.
 *
 * Requirements: cols % 32 == 0; rows % 32 == 0 if MOSS_Q_COL; ld >= cols, ld % 8 == 0.
 * Outputs are dense (no padding).  Returns MOSS_OK or an argument / HIP error.
 * ------------------------------------------------------------------------- */
#define MOSS_Q_ROW 1u
#define MOSS_Q_COL 2u
#define MOSS_EXP_NEAREST 0u
#define MOSS_EXP_CEIL 4u
/* Optional promise about `workspace` (moss_quant_act_2level only): it was zero-filled before its first use
 * and since then nothing but completed calls of moss_quant_act_2level has written to it.  The one-launch
 * path (tensors of up to 64 MiB) then skips the small launch that clears its meeting words -- the kernel
 * leaves them at zero itself.  Without the flag the workspace's contents need not be initialised.  A wrong
 * promise gives a wrong global scale or a slow call, never an access out of bounds or a hang.           */
#define MOSS_WS_KEPT 8u

size_t moss_quant_workspace_bytes(int64_t rows, int64_t cols, unsigned flags);

int moss_quant_act_2level(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld, unsigned flags,
                          uint8_t *q_row, uint8_t *e_row, uint8_t *q_col, uint8_t *e_col,
                          float *s_global, void *workspace, size_t workspace_bytes, void *stream);

/* The same call for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch (partial maxima, meeting
 * words) lives in a 16 KiB array in the library's device data segment, one copy per GPU, held until the
 * process ends; the call allocates nothing and frees nothing.  Arguments, outputs and errors as for
 * moss_quant_act_2level; MOSS_ERR_WORKSPACE if a shape ever needed more scratch than the array holds
 * (the quantizer's scratch does not grow with the shape, so every accepted shape fits); MOSS_ERR_HIP
 * if the array's address cannot be resolved.  The first call on a device resolves that address (a host
 * query, make it outside a capture).  All calls on one GPU share the one array: calls that overlap on a
 * GPU (different streams, different threads) race; order them on one stream.  The array is zero when
 * the library is loaded and every kernel that uses its meeting words clears them before it ends, so a
 * tensor of up to 64 MiB takes exactly one launch here.  MOSS_WS_KEPT is accepted and has no effect.  */
int moss_quant_act_2level_noalloc(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld, unsigned flags,
                                  uint8_t *q_row, uint8_t *e_row, uint8_t *q_col, uint8_t *e_col,
                                  float *s_global, void *stream);

/* Mid-sized and large tensors are quantized by one launch whose workgroups meet once, through
 * a few words of the workspace, to agree on the global maximum (Sec. 3.1: one FP32 scale per
 * tensor).  A workgroup polls for the result at most `polls` times before it computes the
 * maximum from X by itself, so the kernel ends even if its workgroups cannot all run at once;
 * the outputs are the same on either path.  Process-wide, takes effect from the next call; the
 * default is 32768.  0 makes every workgroup that finds the result not yet published take the
 * slow path (used by the tests).  The one-launch kernel assumes the device to itself: when other
 * kernels occupy compute units at the same time (calls on several streams at once) part of its
 * grid may have to wait for them, and workgroups then fall back to the slow path after the
 * bound -- correct, but slow; quantizer calls that must overlap other work should be
 * serialised on one stream. */
void moss_quant_set_poll_limit(unsigned polls);

/* The same quantizer for a tensor whose producer already knows a bound of |X| (Sec. 3.1, Eq. 2:
 * the global scale is the largest of the group scales, s = max|X| / 448; a kernel that writes X can
 * keep the running maximum of what it writes, and the search for it, one extra pass over X, falls
 * away).
 *   x_absmax_bits  device pointer to one 32-bit word: the BF16 bit pattern, sign bit cleared, of a
 *                  value >= max|X| (what an unsigned atomic maximum over `bits & 0x7FFF` of every
 *                  element written leaves; moss_swiglu_bf16 below writes such a word).  With
 *                  exactly max|X| every output equals that of moss_quant_act_2level; with a larger
 *                  bound the outputs are Eq. 2-3 evaluated with the bound in place of max|X|; with
 *                  a smaller value or a non-finite pattern the outputs are unspecified.
 * Everything else as above; no workspace; one launch, X is read once.                           */
int moss_quant_act_2level_given_max(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld, unsigned flags,
                                    const uint32_t *x_absmax_bits,
                                    uint8_t *q_row, uint8_t *e_row, uint8_t *q_col, uint8_t *e_col,
                                    float *s_global, void *stream);

/* ---------------------------------------------------------------------------
 * SwiGLU, the BF16 producer in front of the down projection's quantizer (the paper keeps the
 * non-linear layers in BF16, Sec. 4.1; fusing the search for max|X| into the producer is what
 * makes the quantizer of Sec. 3.1 a single pass over its input):
 *      h = silu(gate) * up,   silu(g) = g / (1 + exp(-g)),
 * evaluated in FP32 and rounded once to BF16 (round to nearest even; the FP32 evaluation is
 * within ~2^-18 relative of the exact value, so h is the correctly rounded BF16 value except
 * where the exact value lies that close to a rounding boundary, and then it is the BF16
 * neighbour: |h - exact| <= (1/2 + 2^-9) BF16 ulp).  *h_absmax_bits receives the largest `bits & 0x7FFF` over the h written: exactly
 * max|h| as a BF16 bit pattern, ready for moss_quant_act_2level_given_max.
 *
 * Backward, for an upstream gradient dh (BF16):
 *      d_up = dh * silu(gate),   d_gate = dh * up * sig(gate) * (1 + gate * (1 - sig(gate))),
 * sig(g) = 1 / (1 + exp(-g)), both rounded once to BF16, each with its own maximum word.
 *
 * gate, up, dh, h, d_gate, d_up: BF16 [rows x cols], all with row stride `ld` elements
 * (ld >= cols, ld % 8 == 0, cols % 8 == 0, 16-byte aligned); non-finite inputs are not supported.
 * The maximum words are device memory, written (not accumulated) by the call.                     */
int moss_swiglu_bf16(const void *gate, const void *up, int64_t rows, int64_t cols, int64_t ld,
                     void *h, uint32_t *h_absmax_bits, void *stream);
int moss_swiglu_bf16_backward(const void *gate, const void *up, const void *dh, int64_t rows, int64_t cols, int64_t ld,
                              void *d_gate, void *d_up, uint32_t *d_gate_absmax_bits, uint32_t *d_up_absmax_bits,
                              void *stream);

/* ---------------------------------------------------------------------------
 * RMSNorm, the BF16 producer in front of the quantizers of the QKV and of the gate / up projections
 * (non-linear layers stay in BF16, Sec. 4.1; as for SwiGLU above, the point is the maximum word that
 * lets the quantizer of Sec. 3.1 skip its search pass).  Over each row of h [rows x cols]:
 *      y = h / sqrt(mean(h^2) + eps) * gamma.
 * Forward, optionally fused with the residual add in front of the norm: with delta != NULL,
 * h = x + delta is rounded to BF16 and written to h_out, and the norm is taken over those rounded
 * values; with delta == NULL, h = x (h_out is ignored).  y is rounded once to BF16 from an FP32
 * evaluation (|y - exact| <= (1/2 + 2^-9) BF16 ulp); *y_absmax_bits receives max|y| as written.
 *
 * Backward, fused with the gradient that reaches h directly over the residual connection
 * (d_res, NULL for none):
 *      g = dy * gamma,  n = h / sqrt(mean(h^2) + eps),
 *      d_h = d_res + (g - n * mean(g * n)) / sqrt(mean(h^2) + eps),
 * rounded once to BF16, with its maximum word (d_h is the O projection's dY in a pre-norm block).
 * The gradient of gamma is not produced (it never meets a quantizer).
 *
 * x, delta, h, h_out, y, dy, d_res, d_h: BF16 [rows x cols], row stride `ld` elements; gamma: BF16 [cols].
 * Requirements: cols % 8 == 0, cols <= 16384 (a row is held in one workgroup's registers, else
 * MOSS_ERR_UNSUPPORTED), ld >= cols, ld % 8 == 0, eps >= 0, 16-byte aligned pointers, finite inputs.
 * The maximum words are device memory, written (not accumulated) by the call.                      */
int moss_add_rmsnorm_bf16(const void *x, const void *delta, const void *gamma, float eps, int64_t rows, int64_t cols,
                          int64_t ld, void *h_out, void *y, uint32_t *y_absmax_bits, void *stream);
int moss_rmsnorm_bf16_backward(const void *h, const void *gamma, const void *dy, const void *d_res, float eps,
                               int64_t rows, int64_t cols, int64_t ld, void *d_h, uint32_t *d_h_absmax_bits,
                               void *stream);

/* ---------------------------------------------------------------------------
 * Per-tensor FP8 weights with automatic scaling  (paper Sec. 3.2, Eq. 10 and the
 * interval re-scaling of its last paragraph; AdamW as in Sec. 2.2 Eq. 1; App. C).
 *
 * The state is a small plain struct in DEVICE memory that the caller owns and may
 * copy out / back in to checkpoint a run.
 * ------------------------------------------------------------------------- */
typedef struct {
    float s_base;            /* s_0: amax(W)/448 at the last max-reduction */
    float s_cur;             /* s_t: scale of the latest cast (Eq. 10) */
    double cum_lr;           /* sum of margin*lr since the last max-reduction ("eta t") */
    int64_t step;            /* optimizer steps taken */
    int64_t last_rebase;     /* step of the last max-reduction */
    float amax_seen;         /* amax of the weights at the latest cast (free by-product) */
    uint32_t overflow_count; /* elements outside the range the scale covers, |w| > 448 s_cur (compared
                                exactly), summed over all casts since the initialisation.  A predicted
                                scale that holds its bound adds nothing; the exact scale fl(amax/448) of
                                the initialisation or of a re-scaling step may round below amax/448,
                                and then counts the largest elements although nothing is clipped */
    uint32_t clipped_count;  /* elements whose code the saturating cast changed: |fl(w fl(1/s))| > 464,
                                i.e. beyond the values that round to 448 by themselves; same sum */
    uint32_t flags;          /* MOSS_WSTATE_* bits, sticky until the next initialisation */
} moss_wscale_state;

/* moss_weight_autoscale_cast was called with args->step != state.step + 1: the caller's step count,
 * which decides when the scale is re-based, has drifted from the state's. */
#define MOSS_WSTATE_STEP_MISMATCH 1u

typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    float one_minus_beta1, one_minus_beta2; /* 1-beta, rounded to FP32 by the caller */
    float bias_corr1, bias_corr2;           /* 1-beta^t, rounded to FP32 by the caller */
    float margin;                           /* multiplies lr in the prediction; the paper's rule is 1 */
    int32_t interval;                       /* max-reduction every `interval` steps; <= 0: never */
    int64_t step;                           /* number t of the step this call performs (1-based);
                                               must equal state.step + 1 (the state lives on the
                                               device, so the call cannot check it: a mismatch sets
                                               MOSS_WSTATE_STEP_MISMATCH in state.flags) */
} moss_adamw_args;

size_t moss_weight_workspace_bytes(int64_t rows, int64_t cols);

/* Initialisation: s_0 = amax(W_0)/448 by one max-reduction, state reset, first cast.
 *   w      [rows x cols] dense, FP32 (MOSS_DT_F32) or BF16 (MOSS_DT_BF16); not modified.
 *   wq     E4M3 codes [rows x cols]:  round(fl32(w * fl32(1/s)))  (all zero if s == 0).
 *   wq_t   optional [cols x rows] byte transpose of wq (the K-contiguous operand of
 *          dX = dY W); may be NULL.
 * Requirements: rows * cols % 4 == 0.                                             */
int moss_weight_autoscale_init(const void *w, int w_dtype, int64_t rows, int64_t cols,
                               moss_wscale_state *state, uint8_t *wq, uint8_t *wq_t,
                               void *workspace, size_t workspace_bytes, void *stream);

/* One optimizer step with scale prediction and the FP8 cast fused in: a single
 * streaming pass reads W, m, v, g, applies AdamW in FP32
 *     m = b1 m + (1-b1) g;  v = b2 v + ((1-b2) g) g;
 *     W = W - lr ( (m/bc1) / (sqrt(v/bc2) + eps) + wd W )
 * (each operation rounded once, nothing contracted), writes W, m, v and the E4M3
 * codes of the NEW weights under the predicted scale
 *     cum_lr += margin*lr;   s_t = (float)(s_base + cum_lr/448)
 * without any max-reduction pass.  amax(W_new) and the number of clipped elements
 * are produced on the way.  If args->interval > 0 and args->step % interval == 0 the
 * scale is re-based instead: s_base = s_t = amax(W_new)/448, cum_lr = 0, and the
 * cast is redone with it (one extra pass over W on that step only).
 *   w, m, v  FP32 [rows x cols], updated in place.
 *   g        gradient, FP32 or BF16 (g_dtype).
 * Requirements: rows * cols % 4 == 0.                                             */
int moss_weight_autoscale_cast(float *w, float *m, float *v, const void *g, int g_dtype,
                               int64_t rows, int64_t cols, const moss_adamw_args *args,
                               moss_wscale_state *state, uint8_t *wq, uint8_t *wq_t,
                               void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * Block-scaled FP8 GEMM with epilogue dequantization (paper Sec. 3.1, Fig. 3b:
 * Q_y = Q_w x (Q_x * ss_x), then one multiply by s_x s_W outside the main loop).
 *
 *   out[m,n] (+)= a_s*b_s * sum_k  dec(a_q[m,k]) 2^(a_e[m,k/32]-127)
 *                                 * dec(b_q[n,k]) 2^(b_e[n,k/32]-127)
 *
 *   a_q [M x K], b_q [N x K]   E4M3 codes, both K-contiguous, dense.
 *   a_e [M x K/32], b_e [N x K/32]  E8M0 bytes, or NULL for the artificial unit
 *                               scale the paper gives per-tensor weights.
 *   a_s, b_s                    device FP32 scalars (global / per-tensor scales).
 *   out  [M x N], row stride ld_out elements, BF16 or FP32 (out_dtype);
 *        accumulate != 0 adds into an FP32 `out` (dW accumulation), else overwrites.
 * The three GEMMs of a linear layer are three calls:
 *   Y  = X W^T   : a = (Xq_row, ex_row, s_x),   b = (Wq,   NULL, s_W)   M=T, N=out, K=in
 *   dX = dY W    : a = (dYq_row, edy_row, s_dy), b = (Wq^T, NULL, s_W)   M=T, N=in,  K=out
 *   dW = dY^T X  : a = (dYq_col, edy_col, s_dy), b = (Xq_col, ex_col, s_x) M=out, N=in, K=T
 * FP32 accumulation on the block-scaled FP8 matrix cores; the level-2 exponents are
 * applied by the matrix instruction itself.
 * Requirements: K % 32 == 0; ld_out >= N; accumulate only with MOSS_DT_F32.
 * ------------------------------------------------------------------------- */
/* The GEMM needs no scratch today: moss_gemm_workspace_bytes returns 0 and `workspace` / `workspace_bytes` are
 * not looked at (pass NULL and 0); the arguments are reserved for a split-K variant. */
size_t moss_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);

int moss_gemm_fp8_mx(int64_t M, int64_t N, int64_t K,
                     const uint8_t *a_q, const uint8_t *a_e, const float *a_s,
                     const uint8_t *b_q, const uint8_t *b_e, const float *b_s,
                     void *out, int out_dtype, int64_t ld_out, int accumulate,
                     void *workspace, size_t workspace_bytes, void *stream);

/* Comparison baseline only (not part of the MOSS path): the same tiling on the BF16
 * matrix cores, out[m,n] = sum_k a[m,k] b[n,k], BF16 in, FP32 accumulate, BF16 out.
 * a [M x K], b [N x K] dense; K % 32 == 0.                                        */
int moss_gemm_bf16_baseline(int64_t M, int64_t N, int64_t K, const void *a_bf16, const void *b_bf16,
                            void *out_bf16, int64_t ld_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOSS_H */
