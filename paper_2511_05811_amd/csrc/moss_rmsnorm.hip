// RMSNorm forward (optionally fused with the residual add in front of it) and backward (fused with the
// residual-path gradient) in BF16, each output that feeds a quantizer with the maximum of its magnitudes:
// the producer in front of the quantizers of the QKV and gate / up projections (forward) and of the
// O projection's dY (backward).  The paper keeps the non-linear layers in BF16 (Sec. 4.1); what this adds
// is the tensor maximum of Sec. 3.1, Eq. 2 as a by-product of writing the tensor, so that
// moss_quant_act_2level_given_max needs no search pass.
//
// Bound: HBM.  A workgroup takes whole rows (grid-stride): every thread holds its 16-byte chunks of the row
// in registers between the row's reduction (sum of squares; in the backward also sum of dy gamma h) and the
// output, so every input is read once.  Arithmetic in FP32 (sums of a few thousand terms: relative error
// ~1e-6, far below half a BF16 step), one rounding to BF16 per output by V_CVT_PK_BF16_F32.  The maximum is
// taken over the bit patterns actually written and merged into the caller's word by one atomic per
// workgroup; a one-thread kernel clears the word first (no memset: the call can be captured into a graph).
#include "moss_internal.h"

namespace moss {
namespace {

constexpr int kRnThreads = 256;
constexpr int kRnMaxChunks = 8;      // 16-byte chunks per thread: rows of up to 256 * 8 * 8 = 16384 elements

typedef unsigned short rn_u16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 rn_bf16x2 __attribute__((ext_vector_type(2)));
typedef float rn_f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t rn_pk_max_u16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(rn_u16x2, a), __builtin_bit_cast(rn_u16x2, b)));
}
__device__ __forceinline__ uint32_t rn_pack(float a, float b)     // two FP32 -> two BF16 (RNE), a in the low half
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(rn_f32x2{a, b}, rn_bf16x2));
}
__device__ __forceinline__ float rn_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float rn_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// sums of a and b over the workgroup, returned to every thread
__device__ __forceinline__ void block_sum2(float &a, float &b, float (*red)[2])
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_xor(a, off, 64);
        b += __shfl_xor(b, off, 64);
    }
    __syncthreads();                       // (the previous row's readers are done with red)
    if ((threadIdx.x & 63) == 0) {
        red[threadIdx.x >> 6][0] = a;
        red[threadIdx.x >> 6][1] = b;
    }
    __syncthreads();
    a = red[0][0]; b = red[0][1];
#pragma unroll
    for (int i = 1; i < kRnThreads / kWave; i++) {
        a += red[i][0];
        b += red[i][1];
    }
}

__device__ __forceinline__ void merge_max(uint32_t m, uint32_t *word, uint32_t *red)
{
    m = (m & 0xFFFFu) > (m >> 16) ? (m & 0xFFFFu) : (m >> 16);
    m = wave_max_u32(m);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kRnThreads / kWave; i++) m = red[i] > m ? red[i] : m;
        if (m) __hip_atomic_fetch_max(word, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__global__ void k_rmsnorm_clear(uint32_t *a)
{
    if (threadIdx.x == 0) *a = 0;
}

// h = x + delta (if ADD), y = h / sqrt(mean(h^2) + eps) * gamma over each row.  The norm is taken over the
// BF16 values of h that are stored, so y is a function of the stored h alone.
template <bool ADD, int CHUNKS>
__global__ __launch_bounds__(kRnThreads) void k_add_rmsnorm(const uint16_t *__restrict__ x, const uint16_t *__restrict__ delta,
                                                            const uint16_t *__restrict__ gamma, float eps, int64_t rows,
                                                            int chunks_per_row, int64_t ld, float inv_cols,
                                                            uint16_t *__restrict__ h_out, uint16_t *__restrict__ y,
                                                            uint32_t *__restrict__ y_max)
{
    __shared__ float red[kRnThreads / kWave][2];
    __shared__ uint32_t redm[kRnThreads / kWave];
    uint32_t m = 0;
    uint4 gm[CHUNKS];
#pragma unroll
    for (int k = 0; k < CHUNKS; k++) {
        const int c = threadIdx.x + k * kRnThreads;
        gm[k] = c < chunks_per_row ? *reinterpret_cast<const uint4 *>(gamma + (int64_t)c * 8) : make_uint4(0, 0, 0, 0);
    }
    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        uint4 hv[CHUNKS];
        float ss = 0.0f, unused = 0.0f;
#pragma unroll
        for (int k = 0; k < CHUNKS; k++) {
            const int c = threadIdx.x + k * kRnThreads;
            hv[k] = make_uint4(0, 0, 0, 0);
            if (c < chunks_per_row) {
                const int64_t off = r * ld + (int64_t)c * 8;
                hv[k] = ld_stream16(x + off);
                if (ADD) {
                    const uint4 d = ld_stream16(delta + off);
                    const uint32_t a[4] = {hv[k].x, hv[k].y, hv[k].z, hv[k].w}, b[4] = {d.x, d.y, d.z, d.w};
                    uint32_t o[4];
#pragma unroll
                    for (int w = 0; w < 4; w++) o[w] = rn_pack(rn_lo(a[w]) + rn_lo(b[w]), rn_hi(a[w]) + rn_hi(b[w]));
                    hv[k] = make_uint4(o[0], o[1], o[2], o[3]);
                    st_stream16(h_out + off, hv[k]);
                }
            }
            const uint32_t a[4] = {hv[k].x, hv[k].y, hv[k].z, hv[k].w};
#pragma unroll
            for (int w = 0; w < 4; w++) ss += rn_lo(a[w]) * rn_lo(a[w]) + rn_hi(a[w]) * rn_hi(a[w]);
        }
        block_sum2(ss, unused, red);
        const float inv = 1.0f / sqrtf(ss * inv_cols + eps);
#pragma unroll
        for (int k = 0; k < CHUNKS; k++) {
            const int c = threadIdx.x + k * kRnThreads;
            if (c >= chunks_per_row) continue;
            const uint32_t a[4] = {hv[k].x, hv[k].y, hv[k].z, hv[k].w}, g[4] = {gm[k].x, gm[k].y, gm[k].z, gm[k].w};
            uint32_t o[4];
#pragma unroll
            for (int w = 0; w < 4; w++) {
                o[w] = rn_pack((rn_lo(a[w]) * inv) * rn_lo(g[w]), (rn_hi(a[w]) * inv) * rn_hi(g[w]));
                m = rn_pk_max_u16(m, o[w] & 0x7FFF7FFFu);
            }
            st_stream16(y + r * ld + (int64_t)c * 8, make_uint4(o[0], o[1], o[2], o[3]));
        }
    }
    merge_max(m, y_max, redm);
}

// d_h = d_res + (g - n mean(g n)) / rms with g = dy gamma, n = h / rms, rms = sqrt(mean(h^2) + eps).
// With S = sum(dy gamma h): mean(g n) = S / (rms cols), so d_h = d_res + (g - h S / (rms^2 cols)) / rms.
template <bool RES, int CHUNKS>
__global__ __launch_bounds__(kRnThreads) void k_rmsnorm_backward(const uint16_t *__restrict__ h, const uint16_t *__restrict__ gamma,
                                                                 const uint16_t *__restrict__ dy, const uint16_t *__restrict__ d_res,
                                                                 float eps, int64_t rows, int chunks_per_row, int64_t ld,
                                                                 float inv_cols, uint16_t *__restrict__ d_h,
                                                                 uint32_t *__restrict__ dh_max)
{
    __shared__ float red[kRnThreads / kWave][2];
    __shared__ uint32_t redm[kRnThreads / kWave];
    uint32_t m = 0;
    uint4 gm[CHUNKS];
#pragma unroll
    for (int k = 0; k < CHUNKS; k++) {
        const int c = threadIdx.x + k * kRnThreads;
        gm[k] = c < chunks_per_row ? *reinterpret_cast<const uint4 *>(gamma + (int64_t)c * 8) : make_uint4(0, 0, 0, 0);
    }
    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        uint4 hv[CHUNKS], gv[CHUNKS];        // h, and g = dy * gamma as FP32 pairs would not fit: keep dy and redo the product
        float ss = 0.0f, sg = 0.0f;
#pragma unroll
        for (int k = 0; k < CHUNKS; k++) {
            const int c = threadIdx.x + k * kRnThreads;
            hv[k] = gv[k] = make_uint4(0, 0, 0, 0);
            if (c < chunks_per_row) {
                const int64_t off = r * ld + (int64_t)c * 8;
                hv[k] = ld_stream16(h + off);
                gv[k] = ld_stream16(dy + off);
            }
            const uint32_t a[4] = {hv[k].x, hv[k].y, hv[k].z, hv[k].w}, d[4] = {gv[k].x, gv[k].y, gv[k].z, gv[k].w};
            const uint32_t g[4] = {gm[k].x, gm[k].y, gm[k].z, gm[k].w};
#pragma unroll
            for (int w = 0; w < 4; w++) {
                ss += rn_lo(a[w]) * rn_lo(a[w]) + rn_hi(a[w]) * rn_hi(a[w]);
                sg += (rn_lo(d[w]) * rn_lo(g[w])) * rn_lo(a[w]) + (rn_hi(d[w]) * rn_hi(g[w])) * rn_hi(a[w]);
            }
        }
        block_sum2(ss, sg, red);
        const float inv = 1.0f / sqrtf(ss * inv_cols + eps);
        const float coef = (sg * inv_cols) * (inv * inv);       // S / (rms^2 cols)
#pragma unroll
        for (int k = 0; k < CHUNKS; k++) {
            const int c = threadIdx.x + k * kRnThreads;
            if (c >= chunks_per_row) continue;
            const int64_t off = r * ld + (int64_t)c * 8;
            const uint32_t a[4] = {hv[k].x, hv[k].y, hv[k].z, hv[k].w}, d[4] = {gv[k].x, gv[k].y, gv[k].z, gv[k].w};
            const uint32_t g[4] = {gm[k].x, gm[k].y, gm[k].z, gm[k].w};
            uint32_t rs[4] = {0, 0, 0, 0};
            if (RES) {
                const uint4 t = ld_stream16(d_res + off);
                rs[0] = t.x; rs[1] = t.y; rs[2] = t.z; rs[3] = t.w;
            }
            uint32_t o[4];
#pragma unroll
            for (int w = 0; w < 4; w++) {
                float lo = ((rn_lo(d[w]) * rn_lo(g[w])) - rn_lo(a[w]) * coef) * inv;
                float hi = ((rn_hi(d[w]) * rn_hi(g[w])) - rn_hi(a[w]) * coef) * inv;
                if (RES) {
                    lo += rn_lo(rs[w]);
                    hi += rn_hi(rs[w]);
                }
                o[w] = rn_pack(lo, hi);
                m = rn_pk_max_u16(m, o[w] & 0x7FFF7FFFu);
            }
            st_stream16(d_h + off, make_uint4(o[0], o[1], o[2], o[3]));
        }
    }
    merge_max(m, dh_max, redm);
}

int check_rows(int64_t rows, int64_t cols, int64_t ld, float eps)
{
    if (rows <= 0 || cols <= 0 || cols % 8 || ld < cols || !(eps >= 0.0f)) return MOSS_ERR_SHAPE;
    if (cols > (int64_t)kRnThreads * kRnMaxChunks * 8) return MOSS_ERR_UNSUPPORTED;     // a row has to fit the workgroup's registers
    if (ld % 8) return MOSS_ERR_ALIGN;
    return MOSS_OK;
}

int rows_grid(int64_t rows)
{
    int cus = moss_internal_cu_count();
    if (cus <= 0) cus = 256;
    const int64_t cap = (int64_t)cus * 8;
    return (int)(rows < cap ? rows : cap);
}

}  // namespace
}  // namespace moss

extern "C" int moss_add_rmsnorm_bf16(const void *x, const void *delta, const void *gamma, float eps, int64_t rows, int64_t cols,
                                     int64_t ld, void *h_out, void *y, uint32_t *y_absmax_bits, void *stream)
{
    using namespace moss;
    if (!x || !gamma || !y || !y_absmax_bits || (delta && !h_out)) return MOSS_ERR_NULL;
    int rc = check_rows(rows, cols, ld, eps);
    if (rc) return rc;
    if (!moss_aligned16(x) || !moss_aligned16(gamma) || !moss_aligned16(y) || ((uintptr_t)y_absmax_bits & 3)) return MOSS_ERR_ALIGN;
    if (delta && (!moss_aligned16(delta) || !moss_aligned16(h_out))) return MOSS_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int cpr = (int)(cols / 8), chunks = (cpr + kRnThreads - 1) / kRnThreads;
    const float inv_cols = 1.0f / (float)cols;
    const dim3 grid(rows_grid(rows)), block(kRnThreads);
    hipLaunchKernelGGL(k_rmsnorm_clear, dim3(1), dim3(64), 0, st, y_absmax_bits);
    MOSS_LAUNCH_CHECK();
#define MOSS_RN_FWD(A, C)                                                                                                    \
    hipLaunchKernelGGL((k_add_rmsnorm<A, C>), grid, block, 0, st, (const uint16_t *)x, (const uint16_t *)delta,                \
                       (const uint16_t *)gamma, eps, rows, cpr, ld, inv_cols, (uint16_t *)h_out, (uint16_t *)y, y_absmax_bits)
    if (delta) {
        if (chunks <= 1) MOSS_RN_FWD(true, 1); else if (chunks <= 2) MOSS_RN_FWD(true, 2); else if (chunks <= 4) MOSS_RN_FWD(true, 4); else MOSS_RN_FWD(true, 8);
    } else {
        if (chunks <= 1) MOSS_RN_FWD(false, 1); else if (chunks <= 2) MOSS_RN_FWD(false, 2); else if (chunks <= 4) MOSS_RN_FWD(false, 4); else MOSS_RN_FWD(false, 8);
    }
#undef MOSS_RN_FWD
    MOSS_LAUNCH_CHECK();
    return MOSS_OK;
}

extern "C" int moss_rmsnorm_bf16_backward(const void *h, const void *gamma, const void *dy, const void *d_res, float eps,
                                          int64_t rows, int64_t cols, int64_t ld, void *d_h, uint32_t *d_h_absmax_bits,
                                          void *stream)
{
    using namespace moss;
    if (!h || !gamma || !dy || !d_h || !d_h_absmax_bits) return MOSS_ERR_NULL;
    int rc = check_rows(rows, cols, ld, eps);
    if (rc) return rc;
    if (!moss_aligned16(h) || !moss_aligned16(gamma) || !moss_aligned16(dy) || !moss_aligned16(d_h)) return MOSS_ERR_ALIGN;
    if ((d_res && !moss_aligned16(d_res)) || ((uintptr_t)d_h_absmax_bits & 3)) return MOSS_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int cpr = (int)(cols / 8), chunks = (cpr + kRnThreads - 1) / kRnThreads;
    const float inv_cols = 1.0f / (float)cols;
    const dim3 grid(rows_grid(rows)), block(kRnThreads);
    hipLaunchKernelGGL(k_rmsnorm_clear, dim3(1), dim3(64), 0, st, d_h_absmax_bits);
    MOSS_LAUNCH_CHECK();
#define MOSS_RN_BWD(R, C)                                                                                                    \
    hipLaunchKernelGGL((k_rmsnorm_backward<R, C>), grid, block, 0, st, (const uint16_t *)h, (const uint16_t *)gamma,           \
                       (const uint16_t *)dy, (const uint16_t *)d_res, eps, rows, cpr, ld, inv_cols, (uint16_t *)d_h,            \
                       d_h_absmax_bits)
    if (d_res) {
        if (chunks <= 1) MOSS_RN_BWD(true, 1); else if (chunks <= 2) MOSS_RN_BWD(true, 2); else if (chunks <= 4) MOSS_RN_BWD(true, 4); else MOSS_RN_BWD(true, 8);
    } else {
        if (chunks <= 1) MOSS_RN_BWD(false, 1); else if (chunks <= 2) MOSS_RN_BWD(false, 2); else if (chunks <= 4) MOSS_RN_BWD(false, 4); else MOSS_RN_BWD(false, 8);
    }
#undef MOSS_RN_BWD
    MOSS_LAUNCH_CHECK();
    return MOSS_OK;
}
