// SwiGLU forward and backward in BF16, each output with the maximum of its magnitudes: the producer
// in front of the quantizer of the down projection (forward) and of the gate / up projections' dY
// (backward).  The paper keeps the non-linear layers in BF16 (Sec. 4.1); what this adds is the tensor
// maximum of Sec. 3.1, Eq. 2 as a by-product of writing the tensor, so that the quantizer of these
// tensors (172 MiB each at LLaMA-7B sizes and 8192 tokens: too large to be kept on chip between a
// search for the maximum and the conversion) reads them once.
//
// Bound: HBM (2 or 3 BF16 tensors in, 1 or 2 out).  Every thread handles 16-byte chunks of eight
// elements; arithmetic in FP32 with the hardware's exp2 and reciprocal approximations (1 ulp each),
// one rounding to BF16 (round to nearest even) by V_CVT_PK_BF16_F32.  The maximum is taken over the
// bit patterns actually written (unsigned maximum of the 15 magnitude bits), folded per wave and per
// workgroup, and merged into the caller's word by one atomic per workgroup; a one-thread kernel clears
// the word first (no memset, so the call can be captured into a graph).
#include "moss_internal.h"

namespace moss {
namespace {

constexpr int kSwThreads = 256;
constexpr int kSwUnroll = 2;

typedef unsigned short sw_u16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 sw_bf16x2 __attribute__((ext_vector_type(2)));
typedef float sw_f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t sw_pk_max_u16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(sw_u16x2, a), __builtin_bit_cast(sw_u16x2, b)));
}
// two FP32 -> two BF16 (round to nearest even), a in the low half
__device__ __forceinline__ uint32_t sw_pack(float a, float b)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(sw_f32x2{a, b}, sw_bf16x2));
}
__device__ __forceinline__ float lo_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// sig(g) = 1 / (1 + exp(-g)); exp(-g) = 2^(-g log2 e) overflows to +inf for g < -88.7, which gives 0
__device__ __forceinline__ float sigmoid(float g)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.44269504088896340736f));
}

__device__ __forceinline__ void fold_max(uint32_t m, uint32_t *word, uint32_t *red)
{
    m = (m & 0xFFFFu) > (m >> 16) ? (m & 0xFFFFu) : (m >> 16);
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kSwThreads / kWave; i++) m = red[i] > m ? red[i] : m;
        if (m) __hip_atomic_fetch_max(word, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
}

__global__ void k_swiglu_clear(uint32_t *a, uint32_t *b)
{
    if (threadIdx.x == 0) {
        *a = 0;
        if (b) *b = 0;
    }
}

__device__ __forceinline__ int64_t chunk_offset(int64_t id, int chunks_per_row, int64_t ld, int dense)
{
    if (dense) return id * 8;
    const int64_t row = id / chunks_per_row;
    return row * ld + (id - row * chunks_per_row) * 8;
}

__global__ __launch_bounds__(kSwThreads) void k_swiglu(const uint16_t *__restrict__ gate, const uint16_t *__restrict__ up,
                                                       int64_t n_chunks, int chunks_per_row, int64_t ld, int dense,
                                                       uint16_t *__restrict__ h, uint32_t *__restrict__ h_max)
{
    __shared__ uint32_t red[kSwThreads / kWave];
    uint32_t m = 0;
    const int64_t stride = (int64_t)gridDim.x * kSwThreads * kSwUnroll;
    for (int64_t id0 = (int64_t)blockIdx.x * kSwThreads * kSwUnroll + threadIdx.x; id0 < n_chunks; id0 += stride) {
        uint4 g[kSwUnroll], u[kSwUnroll];
        int64_t off[kSwUnroll];
#pragma unroll
        for (int k = 0; k < kSwUnroll; k++) {
            const int64_t id = id0 + (int64_t)k * kSwThreads;
            off[k] = -1;
            if (id < n_chunks) {
                off[k] = chunk_offset(id, chunks_per_row, ld, dense);
                g[k] = ld_stream16(gate + off[k]);
                u[k] = ld_stream16(up + off[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < kSwUnroll; k++) {
            if (off[k] < 0) continue;
            const uint32_t gw[4] = {g[k].x, g[k].y, g[k].z, g[k].w}, uw[4] = {u[k].x, u[k].y, u[k].z, u[k].w};
            uint32_t o[4];
#pragma unroll
            for (int w = 0; w < 4; w++) {
                const float g0 = lo_f32(gw[w]), g1 = hi_f32(gw[w]);
                o[w] = sw_pack((g0 * sigmoid(g0)) * lo_f32(uw[w]), (g1 * sigmoid(g1)) * hi_f32(uw[w]));
                m = sw_pk_max_u16(m, o[w] & 0x7FFF7FFFu);
            }
            st_stream16(h + off[k], make_uint4(o[0], o[1], o[2], o[3]));
        }
    }
    fold_max(m, h_max, red);
}

__global__ __launch_bounds__(kSwThreads) void k_swiglu_backward(const uint16_t *__restrict__ gate, const uint16_t *__restrict__ up,
                                                                const uint16_t *__restrict__ dh, int64_t n_chunks,
                                                                int chunks_per_row, int64_t ld, int dense,
                                                                uint16_t *__restrict__ d_gate, uint16_t *__restrict__ d_up,
                                                                uint32_t *__restrict__ dg_max, uint32_t *__restrict__ du_max)
{
    __shared__ uint32_t red[kSwThreads / kWave];
    uint32_t mg = 0, mu = 0;
    const int64_t stride = (int64_t)gridDim.x * kSwThreads;
    for (int64_t id = (int64_t)blockIdx.x * kSwThreads + threadIdx.x; id < n_chunks; id += stride) {
        const int64_t off = chunk_offset(id, chunks_per_row, ld, dense);
        const uint4 g = ld_stream16(gate + off), u = ld_stream16(up + off), d = ld_stream16(dh + off);
        const uint32_t gw[4] = {g.x, g.y, g.z, g.w}, uw[4] = {u.x, u.y, u.z, u.w}, dw[4] = {d.x, d.y, d.z, d.w};
        uint32_t og[4], ou[4];
#pragma unroll
        for (int w = 0; w < 4; w++) {
            float rg[2], ru[2];
#pragma unroll
            for (int e = 0; e < 2; e++) {
                const float gv = e ? hi_f32(gw[w]) : lo_f32(gw[w]), uv = e ? hi_f32(uw[w]) : lo_f32(uw[w]);
                const float dv = e ? hi_f32(dw[w]) : lo_f32(dw[w]);
                const float sg = sigmoid(gv);
                ru[e] = dv * (gv * sg);
                rg[e] = (dv * uv) * (sg * (1.0f + gv * (1.0f - sg)));
            }
            og[w] = sw_pack(rg[0], rg[1]);
            ou[w] = sw_pack(ru[0], ru[1]);
            mg = sw_pk_max_u16(mg, og[w] & 0x7FFF7FFFu);
            mu = sw_pk_max_u16(mu, ou[w] & 0x7FFF7FFFu);
        }
        st_stream16(d_gate + off, make_uint4(og[0], og[1], og[2], og[3]));
        st_stream16(d_up + off, make_uint4(ou[0], ou[1], ou[2], ou[3]));
    }
    fold_max(mg, dg_max, red);
    fold_max(mu, du_max, red);
}

int check_common(int64_t rows, int64_t cols, int64_t ld)
{
    if (rows <= 0 || cols <= 0 || cols % 8 || ld < cols) return MOSS_ERR_SHAPE;
    if (rows * (cols / 8) >= ((int64_t)1 << 40)) return MOSS_ERR_SHAPE;
    if (ld % 8) return MOSS_ERR_ALIGN;
    return MOSS_OK;
}

int grid_for(int64_t n_chunks, int per_thread)
{
    const int64_t want = (n_chunks + (int64_t)kSwThreads * per_thread - 1) / ((int64_t)kSwThreads * per_thread);
    int cus = moss_internal_cu_count();
    if (cus <= 0) cus = 256;
    const int64_t cap = (int64_t)cus * 16;       // a few waves' worth of workgroups per compute unit, grid-stride beyond
    return (int)(want < cap ? want : cap);
}

}  // namespace
}  // namespace moss

extern "C" int moss_swiglu_bf16(const void *gate, const void *up, int64_t rows, int64_t cols, int64_t ld,
                                void *h, uint32_t *h_absmax_bits, void *stream)
{
    using namespace moss;
    if (!gate || !up || !h || !h_absmax_bits) return MOSS_ERR_NULL;
    int rc = check_common(rows, cols, ld);
    if (rc) return rc;
    if (!moss_aligned16(gate) || !moss_aligned16(up) || !moss_aligned16(h) || ((uintptr_t)h_absmax_bits & 3)) return MOSS_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int chunks_per_row = (int)(cols / 8);
    const int64_t n_chunks = rows * chunks_per_row;
    hipLaunchKernelGGL(k_swiglu_clear, dim3(1), dim3(64), 0, st, h_absmax_bits, (uint32_t *)nullptr);
    MOSS_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_swiglu, dim3(grid_for(n_chunks, kSwUnroll)), dim3(kSwThreads), 0, st, (const uint16_t *)gate,
                       (const uint16_t *)up, n_chunks, chunks_per_row, ld, (int)(ld == cols), (uint16_t *)h, h_absmax_bits);
    MOSS_LAUNCH_CHECK();
    return MOSS_OK;
}

extern "C" int moss_swiglu_bf16_backward(const void *gate, const void *up, const void *dh, int64_t rows, int64_t cols,
                                         int64_t ld, void *d_gate, void *d_up, uint32_t *d_gate_absmax_bits,
                                         uint32_t *d_up_absmax_bits, void *stream)
{
    using namespace moss;
    if (!gate || !up || !dh || !d_gate || !d_up || !d_gate_absmax_bits || !d_up_absmax_bits) return MOSS_ERR_NULL;
    int rc = check_common(rows, cols, ld);
    if (rc) return rc;
    if (!moss_aligned16(gate) || !moss_aligned16(up) || !moss_aligned16(dh) || !moss_aligned16(d_gate) || !moss_aligned16(d_up))
        return MOSS_ERR_ALIGN;
    if (((uintptr_t)d_gate_absmax_bits & 3) || ((uintptr_t)d_up_absmax_bits & 3)) return MOSS_ERR_ALIGN;
    if (d_gate_absmax_bits == d_up_absmax_bits) return MOSS_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    const int chunks_per_row = (int)(cols / 8);
    const int64_t n_chunks = rows * chunks_per_row;
    hipLaunchKernelGGL(k_swiglu_clear, dim3(1), dim3(64), 0, st, d_gate_absmax_bits, d_up_absmax_bits);
    MOSS_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_swiglu_backward, dim3(grid_for(n_chunks, 1)), dim3(kSwThreads), 0, st, (const uint16_t *)gate,
                       (const uint16_t *)up, (const uint16_t *)dh, n_chunks, chunks_per_row, ld, (int)(ld == cols),
                       (uint16_t *)d_gate, (uint16_t *)d_up, d_gate_absmax_bits, d_up_absmax_bits);
    MOSS_LAUNCH_CHECK();
    return MOSS_OK;
}
