// Two-level microscaling quantizer for gfx950 (paper Sec. 3.1, Eq. 1-2).
//
// Pass 1 (k_amax_bf16) streams X once and leaves one partial |x| maximum per
// workgroup in the workspace.  Pass 2 (k_quant_row / k_quant_col) folds the
// partials into the global scale s = amax/448 and then, per group of 32 values,
// derives the power-of-two local scale from integer / exact FP32 comparisons and
// emits E4M3 codes of (x * 2^-e) * (1/s).  Magnitudes of finite BF16 values order
// like their low 15 bits, so every maximum is an integer maximum and is exact.
#include "moss_internal.h"

namespace moss {

constexpr int kQuantThreads = 256;
constexpr int kMaxPartials = 2048;

// max of the eight 15-bit magnitudes held in a 16-byte chunk
__device__ __forceinline__ uint32_t chunk_absmax(const uint4 &r)
{
    uint32_t m = 0;
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
        uint32_t lo = w[i] & 0x7FFFu, hi = (w[i] >> 16) & 0x7FFFu;
        m = lo > m ? lo : m;
        m = hi > m ? hi : m;
    }
    return m;
}

__global__ __launch_bounds__(kQuantThreads) void k_amax_bf16(const uint16_t *__restrict__ x, int64_t n_chunks,
                                                             int chunks_per_row, int64_t ld, int dense,
                                                             uint32_t *__restrict__ partial)
{
    __shared__ uint32_t red[kQuantThreads / kWave];
    uint32_t m = 0;
    const int64_t stride = (int64_t)gridDim.x * kQuantThreads;
    for (int64_t id = (int64_t)blockIdx.x * kQuantThreads + threadIdx.x; id < n_chunks; id += stride) {
        int64_t off;
        if (dense) {
            off = id * 8;
        } else {
            int64_t row = id / chunks_per_row;
            off = row * ld + (id - row * chunks_per_row) * 8;
        }
        uint4 r = *reinterpret_cast<const uint4 *>(x + off);
        uint32_t c = chunk_absmax(r);
        m = c > m ? c : m;
    }
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kQuantThreads / kWave; i++) m = red[i] > m ? red[i] : m;
        partial[blockIdx.x] = m;
    }
}

struct GlobalScale {
    float s, inv_s;   // s = amax/448 (1 for an all-zero tensor), inv_s = fl(1/s)
    float frac;       // amax = frac * 2^expo, frac in [0.5, 1)
    int expo;
    bool zero;
};

// Every workgroup folds the (few) partial maxima itself: cheaper than another launch.
__device__ __forceinline__ GlobalScale fold_global_scale(const uint32_t *partial, int n_partial, uint32_t *red)
{
    uint32_t m = 0;
    for (int i = threadIdx.x; i < n_partial; i += blockDim.x) {
        uint32_t p = partial[i];
        m = p > m ? p : m;
    }
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    const int nw = blockDim.x >> 6;
    m = red[0];
    for (int i = 1; i < nw; i++) m = red[i] > m ? red[i] : m;
    GlobalScale g;
    float amax = bf16_bits_to_f32(m);
    g.zero = (m == 0);
    g.s = g.zero ? 1.0f : amax / kE4M3Max;
    g.inv_s = 1.0f / g.s;
    g.frac = __builtin_amdgcn_frexp_mantf(amax);
    g.expo = __builtin_amdgcn_frexp_expf(amax);
    return g;
}

// e = round(log2(a/amax)) (or its ceiling), clamped to [-127, 0]; a = 15-bit BF16
// magnitude bits.  With a = f_a 2^ea and amax = f_A 2^eA (f in [0.5,1), at most 8
// significant bits) the candidates are ea-eA-1, ea-eA, ea-eA+1 and the choice needs
// only products of two 8-bit significands, exact in FP32:
//   nearest: +1 if f_a^2 >= 2 f_A^2, -1 if 2 f_a^2 < f_A^2;   ceil: +1 if f_a > f_A.
template <bool CEIL>
__device__ __forceinline__ int local_exponent(uint32_t a_bits, const GlobalScale &g)
{
    if (a_bits == 0) return -127;
    float a = bf16_bits_to_f32(a_bits);
    float fa = __builtin_amdgcn_frexp_mantf(a);
    int k = __builtin_amdgcn_frexp_expf(a) - g.expo;
    if (CEIL) {
        k += (fa > g.frac) ? 1 : 0;
    } else {
        float fa2 = fa * fa, fA2 = g.frac * g.frac;
        k += (fa2 >= 2.0f * fA2) ? 1 : 0;
        k -= (2.0f * fa2 < fA2) ? 1 : 0;
    }
    k = k < -127 ? -127 : k;
    return k > 0 ? 0 : k;
}

// 2^(-e) for e in [-127, 0] as an FP32 bit pattern
__device__ __forceinline__ float pow2_neg(int e) { return __uint_as_float((uint32_t)(127 - e) << 23); }

__device__ __forceinline__ uint32_t quad_max_u32(uint32_t v)
{
    uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
    v = o > v ? o : v;
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);           // quad_perm [2,3,0,1]
    return o > v ? o : v;
}

// Row grouping: a group is 64 contiguous bytes = the 16-byte chunks of four
// neighbouring lanes.  Each thread handles kRowUnroll chunks that are one block
// stride apart so that all its loads are in flight together.
constexpr int kRowUnroll = 4;

template <bool CEIL>
__global__ __launch_bounds__(kQuantThreads) void k_quant_row(const uint16_t *__restrict__ x, int64_t n_chunks,
                                                             int chunks_per_row, int64_t ld, int dense,
                                                             const uint32_t *__restrict__ partial, int n_partial,
                                                             uint8_t *__restrict__ q, uint8_t *__restrict__ e,
                                                             float *__restrict__ s_global)
{
    __shared__ uint32_t red[kQuantThreads / kWave];
    const GlobalScale g = fold_global_scale(partial, n_partial, red);
    if (blockIdx.x == 0 && threadIdx.x == 0) *s_global = g.s;

    const int64_t base = (int64_t)blockIdx.x * (kQuantThreads * kRowUnroll) + threadIdx.x;
    uint4 raw[kRowUnroll];
#pragma unroll
    for (int u = 0; u < kRowUnroll; u++) {
        int64_t id = base + (int64_t)u * kQuantThreads;
        raw[u] = make_uint4(0, 0, 0, 0);
        if (id < n_chunks) {
            int64_t off;
            if (dense) {
                off = id * 8;
            } else {
                int64_t row = id / chunks_per_row;
                off = row * ld + (id - row * chunks_per_row) * 8;
            }
            raw[u] = *reinterpret_cast<const uint4 *>(x + off);
        }
    }
#pragma unroll
    for (int u = 0; u < kRowUnroll; u++) {
        int64_t id = base + (int64_t)u * kQuantThreads;
        // the four lanes of a quad hold one group; n_chunks % 4 == 0 keeps quads uniform
        uint32_t gmax = quad_max_u32(chunk_absmax(raw[u]));
        int ex = local_exponent<CEIL>(gmax, g);
        float p2 = pow2_neg(ex);
        const uint32_t w[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
        uint32_t out[2];
#pragma unroll
        for (int h = 0; h < 2; h++) {
            float y0 = (bf16_bits_to_f32(w[2 * h] & 0xFFFFu) * p2) * g.inv_s;
            float y1 = (__uint_as_float(w[2 * h] & 0xFFFF0000u) * p2) * g.inv_s;
            float y2 = (bf16_bits_to_f32(w[2 * h + 1] & 0xFFFFu) * p2) * g.inv_s;
            float y3 = (__uint_as_float(w[2 * h + 1] & 0xFFFF0000u) * p2) * g.inv_s;
            out[h] = cvt4_e4m3_sat(y0, y1, y2, y3);
        }
        if (id < n_chunks) {
            *reinterpret_cast<uint2 *>(q + id * 8) = make_uint2(out[0], out[1]);
            if ((threadIdx.x & 3) == 0) e[id >> 2] = (uint8_t)(ex + 127);
        }
    }
}

// Column grouping (groups of 32 along the rows, outputs transposed).  One wave owns a
// 128-column stripe; each lane owns two neighbouring columns, so a wave-wide 4-byte
// load covers 256 contiguous bytes of one row and a whole group lives in one lane's
// registers (no cross-lane reduction).  A lane walks kColGroups consecutive row groups
// so that its 32-byte code stores fill complete 128-byte lines of the transposed output.
constexpr int kColGroups = 4;

template <bool CEIL>
__global__ __launch_bounds__(kWave) void k_quant_col(const uint16_t *__restrict__ x, int64_t rows, int64_t cols,
                                                     int64_t ld, const uint32_t *__restrict__ partial, int n_partial,
                                                     uint8_t *__restrict__ q, uint8_t *__restrict__ e,
                                                     float *__restrict__ s_global, int write_scale)
{
    __shared__ uint32_t red[1];
    const GlobalScale g = fold_global_scale(partial, n_partial, red);
    if (write_scale && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *s_global = g.s;

    const int64_t c0 = (int64_t)blockIdx.x * 128 + 2 * threadIdx.x;
    if (c0 >= cols) return;
    const int64_t n_groups = rows / kGroup;
    const int64_t g_begin = (int64_t)blockIdx.y * kColGroups;
    for (int gi = 0; gi < kColGroups; gi++) {
        const int64_t grp = g_begin + gi;
        if (grp >= n_groups) break;
        const uint16_t *src = x + grp * kGroup * ld + c0;
        uint32_t v[kGroup];
#pragma unroll
        for (int j = 0; j < kGroup; j++) v[j] = *reinterpret_cast<const uint32_t *>(src + j * ld);
        uint32_t m0 = 0, m1 = 0;
#pragma unroll
        for (int j = 0; j < kGroup; j++) {
            uint32_t lo = v[j] & 0x7FFFu, hi = (v[j] >> 16) & 0x7FFFu;
            m0 = lo > m0 ? lo : m0;
            m1 = hi > m1 ? hi : m1;
        }
        const int ex0 = local_exponent<CEIL>(m0, g), ex1 = local_exponent<CEIL>(m1, g);
        const float p0 = pow2_neg(ex0), p1 = pow2_neg(ex1);
        uint32_t o0[8], o1[8];
#pragma unroll
        for (int j = 0; j < 8; j++) {
            float a0 = (bf16_bits_to_f32(v[4 * j] & 0xFFFFu) * p0) * g.inv_s;
            float a1 = (bf16_bits_to_f32(v[4 * j + 1] & 0xFFFFu) * p0) * g.inv_s;
            float a2 = (bf16_bits_to_f32(v[4 * j + 2] & 0xFFFFu) * p0) * g.inv_s;
            float a3 = (bf16_bits_to_f32(v[4 * j + 3] & 0xFFFFu) * p0) * g.inv_s;
            o0[j] = cvt4_e4m3_sat(a0, a1, a2, a3);
            float b0 = (__uint_as_float(v[4 * j] & 0xFFFF0000u) * p1) * g.inv_s;
            float b1 = (__uint_as_float(v[4 * j + 1] & 0xFFFF0000u) * p1) * g.inv_s;
            float b2 = (__uint_as_float(v[4 * j + 2] & 0xFFFF0000u) * p1) * g.inv_s;
            float b3 = (__uint_as_float(v[4 * j + 3] & 0xFFFF0000u) * p1) * g.inv_s;
            o1[j] = cvt4_e4m3_sat(b0, b1, b2, b3);
        }
        uint8_t *d0 = q + c0 * rows + grp * kGroup;
        uint8_t *d1 = d0 + rows;
        reinterpret_cast<uint4 *>(d0)[0] = make_uint4(o0[0], o0[1], o0[2], o0[3]);
        reinterpret_cast<uint4 *>(d0)[1] = make_uint4(o0[4], o0[5], o0[6], o0[7]);
        reinterpret_cast<uint4 *>(d1)[0] = make_uint4(o1[0], o1[1], o1[2], o1[3]);
        reinterpret_cast<uint4 *>(d1)[1] = make_uint4(o1[4], o1[5], o1[6], o1[7]);
        e[c0 * n_groups + grp] = (uint8_t)(ex0 + 127);
        e[(c0 + 1) * n_groups + grp] = (uint8_t)(ex1 + 127);
    }
}

}  // namespace moss

extern "C" size_t moss_quant_workspace_bytes(int64_t rows, int64_t cols, unsigned flags)
{
    (void)rows; (void)cols; (void)flags;
    return (size_t)moss::kMaxPartials * sizeof(uint32_t);
}

extern "C" int moss_quant_act_2level(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld, unsigned flags,
                                     uint8_t *q_row, uint8_t *e_row, uint8_t *q_col, uint8_t *e_col,
                                     float *s_global, void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace moss;
    const bool want_row = flags & MOSS_Q_ROW, want_col = flags & MOSS_Q_COL, ceil_mode = flags & MOSS_EXP_CEIL;
    if (flags & ~(MOSS_Q_ROW | MOSS_Q_COL | MOSS_EXP_CEIL)) return MOSS_ERR_UNSUPPORTED;
    if (!want_row && !want_col) return MOSS_ERR_UNSUPPORTED;
    if (!x_bf16 || !s_global) return MOSS_ERR_NULL;
    if (want_row && (!q_row || !e_row)) return MOSS_ERR_NULL;
    if (want_col && (!q_col || !e_col)) return MOSS_ERR_NULL;
    if (rows <= 0 || cols <= 0 || cols % kGroup || ld < cols) return MOSS_ERR_SHAPE;
    if (want_col && rows % kGroup) return MOSS_ERR_SHAPE;
    if (rows * (cols / 8) >= ((int64_t)1 << 40)) return MOSS_ERR_SHAPE;
    if (ld % 8 || !moss_aligned16(x_bf16)) return MOSS_ERR_ALIGN;
    if (want_row && !moss_aligned16(q_row)) return MOSS_ERR_ALIGN;
    if (want_col && !moss_aligned16(q_col)) return MOSS_ERR_ALIGN;
    if (!moss_aligned16(workspace) || ((uintptr_t)s_global & 3)) return MOSS_ERR_ALIGN;
    if (!workspace || workspace_bytes < moss_quant_workspace_bytes(rows, cols, flags)) return MOSS_ERR_WORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    const uint16_t *x = (const uint16_t *)x_bf16;
    uint32_t *partial = (uint32_t *)workspace;
    const int chunks_per_row = (int)(cols / 8);
    const int64_t n_chunks = rows * chunks_per_row;
    const int dense = (ld == cols);

    int64_t want_blocks = (n_chunks + kQuantThreads * 4 - 1) / (kQuantThreads * 4);
    const int n_partial = (int)(want_blocks < kMaxPartials ? want_blocks : kMaxPartials);
    hipLaunchKernelGGL(k_amax_bf16, dim3(n_partial), dim3(kQuantThreads), 0, st, x, n_chunks, chunks_per_row, ld, dense,
                       partial);
    MOSS_LAUNCH_CHECK();

    if (want_row) {
        const int64_t per_block = (int64_t)kQuantThreads * kRowUnroll;
        const int64_t blocks = (n_chunks + per_block - 1) / per_block;
        if (blocks > 0x7FFFFFFF) return MOSS_ERR_SHAPE;
        if (ceil_mode)
            hipLaunchKernelGGL(k_quant_row<true>, dim3((unsigned)blocks), dim3(kQuantThreads), 0, st, x, n_chunks,
                               chunks_per_row, ld, dense, partial, n_partial, q_row, e_row, s_global);
        else
            hipLaunchKernelGGL(k_quant_row<false>, dim3((unsigned)blocks), dim3(kQuantThreads), 0, st, x, n_chunks,
                               chunks_per_row, ld, dense, partial, n_partial, q_row, e_row, s_global);
        MOSS_LAUNCH_CHECK();
    }
    if (want_col) {
        const int64_t gx = (cols + 127) / 128;
        const int64_t gy = (rows / kGroup + kColGroups - 1) / kColGroups;
        if (gy > 65535) return MOSS_ERR_SHAPE;
        const int write_scale = want_row ? 0 : 1;
        if (ceil_mode)
            hipLaunchKernelGGL(k_quant_col<true>, dim3((unsigned)gx, (unsigned)gy), dim3(kWave), 0, st, x, rows, cols, ld,
                               partial, n_partial, q_col, e_col, s_global, write_scale);
        else
            hipLaunchKernelGGL(k_quant_col<false>, dim3((unsigned)gx, (unsigned)gy), dim3(kWave), 0, st, x, rows, cols, ld,
                               partial, n_partial, q_col, e_col, s_global, write_scale);
        MOSS_LAUNCH_CHECK();
    }
    return MOSS_OK;
}
