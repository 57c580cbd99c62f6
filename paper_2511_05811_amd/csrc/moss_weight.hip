// Per-tensor FP8 weights with automatic scaling for gfx950 (paper Sec. 3.2, Eq. 10;
// AdamW of Sec. 2.2 Eq. 1; App. C).
//
// The optimizer step is one streaming pass: each workgroup derives the predicted
// scale s_t = s_base + cum_lr/448 from the device-resident state (O(1), no
// max-reduction), applies AdamW to its slice, writes W, m, v and the E4M3 codes of the
// new weights, and leaves one partial amax / clipped-element count per workgroup in
// the workspace.  A one-workgroup epilogue kernel folds the partials into the state.
// Partials instead of atomics keep the result independent of scheduling.
#include "moss_internal.h"

#pragma clang fp contract(off)

namespace moss {

constexpr int kWThreads = 256;
constexpr int kWMaxBlocks = 4096;   // grid cap of the flat (1-D) kernels
constexpr int kWTile = 128;         // tile edge of the 2-D kernel that also emits the transposed codes
// |y| <= 464 rounds to 448 by itself (464 is the midpoint to the next grid point, tie to
// even); beyond it the saturating cast changes the result: that is a clipped element.
constexpr float kClip = 464.0f;

struct WPartials {
    float *amax;      // [slots]
    uint32_t *over;   // [slots] elements outside 448 s
    uint32_t *clip;   // [slots] elements the saturation changed
};

// per-thread running by-products of a cast
struct WCounts {
    float amax = 0.0f;
    uint32_t over = 0, clip = 0;
};

// The scale is meant to keep |w| / s within 448 (Sec. 3.2, text under Eq. 10); an element is out of
// range when |w| > 448 s, compared exactly.  448 s has up to 27 significant bits, but for a single w
// "w > 448 s" is the same as "w > the largest single that does not exceed 448 s", so one
// double product per workgroup leaves a single-precision comparison per element.
__device__ __forceinline__ float range_limit(float s)
{
    const double exact = 448.0 * (double)s;
    float t = (float)exact;
    if ((double)t > exact) t = __uint_as_float(__float_as_uint(t) - 1u);
    return t;
}

__device__ __forceinline__ void count4(WCounts &c, const float4 &wv, float y0, float y1, float y2, float y3, float limit)
{
    c.over += (fabsf(wv.x) > limit) + (fabsf(wv.y) > limit) + (fabsf(wv.z) > limit) + (fabsf(wv.w) > limit);
    c.clip += (fabsf(y0) > kClip) + (fabsf(y1) > kClip) + (fabsf(y2) > kClip) + (fabsf(y3) > kClip);
}

// one slot per workgroup of the largest grid a call may launch
__host__ __device__ inline int64_t partial_slots(int64_t rows, int64_t cols)
{
    const int64_t tiles = ((rows + kWTile - 1) / kWTile) * ((cols + kWTile - 1) / kWTile);
    return tiles > kWMaxBlocks ? tiles : kWMaxBlocks;
}

__device__ __forceinline__ WPartials ws_partials(void *ws, int64_t slots)
{
    WPartials p;
    p.amax = reinterpret_cast<float *>(ws);
    p.over = reinterpret_cast<uint32_t *>(ws) + slots;
    p.clip = reinterpret_cast<uint32_t *>(ws) + 2 * slots;
    return p;
}

// Block-wide max / sums; the result is valid in thread 0 only.
__device__ __forceinline__ void block_reduce(WCounts &c)
{
    __shared__ float r_amax[kWThreads / kWave];
    __shared__ uint32_t r_over[kWThreads / kWave], r_clip[kWThreads / kWave];
    c.amax = wave_max_f32(c.amax);
    c.over = wave_sum_u32(c.over);
    c.clip = wave_sum_u32(c.clip);
    if ((threadIdx.x & 63) == 0) {
        r_amax[threadIdx.x >> 6] = c.amax;
        r_over[threadIdx.x >> 6] = c.over;
        r_clip[threadIdx.x >> 6] = c.clip;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kWThreads / kWave; i++) {
            c.amax = fmaxf(c.amax, r_amax[i]);
            c.over += r_over[i];
            c.clip += r_clip[i];
        }
    }
}

__device__ __forceinline__ void block_reduce_store(WCounts c, void *ws, int64_t slots)
{
    block_reduce(c);
    if (threadIdx.x == 0) {
        WPartials p = ws_partials(ws, slots);
        const int64_t b = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
        p.amax[b] = c.amax;
        p.over[b] = c.over;
        p.clip[b] = c.clip;
    }
}

__device__ __forceinline__ float4 load_as_f32x4(const void *p, int64_t i4, bool bf16)
{
    if (bf16) {
        uint2 r = ld_stream8(reinterpret_cast<const uint2 *>(p) + i4);
        return make_float4(bf16_bits_to_f32(r.x & 0xFFFFu), __uint_as_float(r.x & 0xFFFF0000u),
                           bf16_bits_to_f32(r.y & 0xFFFFu), __uint_as_float(r.y & 0xFFFF0000u));
    }
    return ld_stream_f4(reinterpret_cast<const float4 *>(p) + i4);
}

struct AdamW {
    float lr, beta1, beta2, eps, wd, omb1, omb2, bc1, bc2;
};

// One AdamW element update; every operation is a single correctly rounded FP32
// operation in the order of Eq. 1 of the paper (no FMA contraction; the build asks for
// IEEE division and square root).
__device__ __forceinline__ void adamw_elem(float &w, float &m, float &v, float g, const AdamW &a)
{
    float mi = a.beta1 * m + a.omb1 * g;
    float vi = a.beta2 * v + (a.omb2 * g) * g;
    float mhat = mi / a.bc1;
    float vhat = vi / a.bc2;
    float den = sqrtf(vhat) + a.eps;
    float u = mhat / den;
    float upd = a.lr * (u + a.wd * w);
    w = w - upd;
    m = mi;
    v = vi;
}

// Scale the cast of this call uses.  predict != 0: Eq. 10 from the state before the
// step; predict == 0: the scale already stored in the state (after init / re-base).
__device__ __forceinline__ float scale_for_cast(const moss_wscale_state *st, int predict, double lr_term)
{
    if (!predict) return st->s_cur;
    double cum = st->cum_lr + lr_term;
    return (float)((double)st->s_base + cum / 448.0);
}

template <bool G_BF16, bool DO_CAST>
__global__ __launch_bounds__(kWThreads) void k_adamw_cast(float *__restrict__ w, float *__restrict__ m,
                                                          float *__restrict__ v, const void *__restrict__ g,
                                                          int64_t n4, AdamW a, double lr_term,
                                                          const moss_wscale_state *__restrict__ st,
                                                          uint8_t *__restrict__ wq, void *ws, int64_t slots)
{
    float inv_s = 0.0f, limit = 0.0f;
    if (DO_CAST) {
        float s = scale_for_cast(st, 1, lr_term);
        inv_s = s > 0.0f ? 1.0f / s : 0.0f;
        limit = range_limit(s);
    }
    WCounts cnt;
    const int64_t stride = (int64_t)gridDim.x * kWThreads;
    for (int64_t i = (int64_t)blockIdx.x * kWThreads + threadIdx.x; i < n4; i += stride) {
        float4 wv = ld_stream_f4(reinterpret_cast<float4 *>(w) + i);
        float4 mv = ld_stream_f4(reinterpret_cast<float4 *>(m) + i);
        float4 vv = ld_stream_f4(reinterpret_cast<float4 *>(v) + i);
        float4 gv = load_as_f32x4(g, i, G_BF16);
        adamw_elem(wv.x, mv.x, vv.x, gv.x, a);
        adamw_elem(wv.y, mv.y, vv.y, gv.y, a);
        adamw_elem(wv.z, mv.z, vv.z, gv.z, a);
        adamw_elem(wv.w, mv.w, vv.w, gv.w, a);
        st_stream_f4(reinterpret_cast<float4 *>(w) + i, wv);
        st_stream_f4(reinterpret_cast<float4 *>(m) + i, mv);
        st_stream_f4(reinterpret_cast<float4 *>(v) + i, vv);
        cnt.amax = fmaxf(cnt.amax, fmaxf(fmaxf(fabsf(wv.x), fabsf(wv.y)), fmaxf(fabsf(wv.z), fabsf(wv.w))));
        if (DO_CAST) {
            float y0 = wv.x * inv_s, y1 = wv.y * inv_s, y2 = wv.z * inv_s, y3 = wv.w * inv_s;
            count4(cnt, wv, y0, y1, y2, y3, limit);
            st_stream4(reinterpret_cast<uint32_t *>(wq) + i, cvt4_e4m3_sat(y0, y1, y2, y3));
        }
    }
    block_reduce_store(cnt, ws, slots);
}

template <bool W_BF16>
__global__ __launch_bounds__(kWThreads) void k_weight_amax(const void *__restrict__ w, int64_t n4, void *ws, int64_t slots)
{
    WCounts cnt;
    const int64_t stride = (int64_t)gridDim.x * kWThreads;
    for (int64_t i = (int64_t)blockIdx.x * kWThreads + threadIdx.x; i < n4; i += stride) {
        float4 wv = load_as_f32x4(w, i, W_BF16);
        cnt.amax = fmaxf(cnt.amax, fmaxf(fmaxf(fabsf(wv.x), fabsf(wv.y)), fmaxf(fabsf(wv.z), fabsf(wv.w))));
    }
    block_reduce_store(cnt, ws, slots);
}

template <bool W_BF16>
__global__ __launch_bounds__(kWThreads) void k_weight_cast(const void *__restrict__ w, int64_t n4,
                                                           const moss_wscale_state *__restrict__ st,
                                                           uint8_t *__restrict__ wq, void *ws, int64_t slots)
{
    const float s = scale_for_cast(st, 0, 0.0);
    const float inv_s = s > 0.0f ? 1.0f / s : 0.0f;
    const float limit = range_limit(s);
    WCounts cnt;
    const int64_t stride = (int64_t)gridDim.x * kWThreads;
    for (int64_t i = (int64_t)blockIdx.x * kWThreads + threadIdx.x; i < n4; i += stride) {
        float4 wv = load_as_f32x4(w, i, W_BF16);
        cnt.amax = fmaxf(cnt.amax, fmaxf(fmaxf(fabsf(wv.x), fabsf(wv.y)), fmaxf(fabsf(wv.z), fabsf(wv.w))));
        float y0 = wv.x * inv_s, y1 = wv.y * inv_s, y2 = wv.z * inv_s, y3 = wv.w * inv_s;
        count4(cnt, wv, y0, y1, y2, y3, limit);
        st_stream4(reinterpret_cast<uint32_t *>(wq) + i, cvt4_e4m3_sat(y0, y1, y2, y3));
    }
    block_reduce_store(cnt, ws, slots);
}

// 2-D variant used when the transposed codes are wanted as well: a workgroup owns a
// 128 x 128 tile, walks it 8 rows at a time (32 lanes x float4 = one 512-byte row piece),
// writes the codes row-major (128 bytes per row) and collects them transposed in LDS;
// at the end 8 lanes write the 128 bytes of each transposed row.  STEP: apply AdamW first
// (fused optimizer step), otherwise cast only, with the scale already in the state.
template <bool STEP, bool SRC_BF16>
__global__ __launch_bounds__(kWThreads) void k_weight_tile(float *__restrict__ w, float *__restrict__ m,
                                                           float *__restrict__ v, const void *__restrict__ src,
                                                           int64_t rows, int64_t cols, AdamW a, double lr_term,
                                                           const moss_wscale_state *__restrict__ st,
                                                           uint8_t *__restrict__ wq, uint8_t *__restrict__ wq_t,
                                                           void *ws, int64_t slots)
{
    constexpr int kPitch = kWTile + 4;
    __shared__ __attribute__((aligned(16))) uint8_t tt[kWTile][kPitch];   // [column][row]
    const float s = scale_for_cast(st, STEP ? 1 : 0, lr_term);
    const float inv_s = s > 0.0f ? 1.0f / s : 0.0f;
    const float limit = range_limit(s);
    const int tid = threadIdx.x, rl = tid >> 5, c4 = (tid & 31) * 4;
    const int64_t r0 = (int64_t)blockIdx.y * kWTile, c0 = (int64_t)blockIdx.x * kWTile;
    const int64_t col = c0 + c4;
    WCounts cnt;
#pragma unroll 4
    for (int it = 0; it < 16; it++) {
        const int rr = it * 8 + rl;
        const int64_t row = r0 + rr;
        uint32_t code = 0;
        if (row < rows && col < cols) {          // cols % 4 == 0: a float4 is inside or outside as a whole
            const int64_t i4 = (row * cols + col) >> 2;
            float4 wv;
            if (STEP) {
                wv = ld_stream_f4(reinterpret_cast<float4 *>(w) + i4);
                float4 mv = ld_stream_f4(reinterpret_cast<float4 *>(m) + i4);
                float4 vv = ld_stream_f4(reinterpret_cast<float4 *>(v) + i4);
                float4 gv = load_as_f32x4(src, i4, SRC_BF16);
                adamw_elem(wv.x, mv.x, vv.x, gv.x, a);
                adamw_elem(wv.y, mv.y, vv.y, gv.y, a);
                adamw_elem(wv.z, mv.z, vv.z, gv.z, a);
                adamw_elem(wv.w, mv.w, vv.w, gv.w, a);
                st_stream_f4(reinterpret_cast<float4 *>(w) + i4, wv);
                st_stream_f4(reinterpret_cast<float4 *>(m) + i4, mv);
                st_stream_f4(reinterpret_cast<float4 *>(v) + i4, vv);
            } else {
                wv = load_as_f32x4(src, i4, SRC_BF16);
            }
            cnt.amax = fmaxf(cnt.amax, fmaxf(fmaxf(fabsf(wv.x), fabsf(wv.y)), fmaxf(fabsf(wv.z), fabsf(wv.w))));
            const float y0 = wv.x * inv_s, y1 = wv.y * inv_s, y2 = wv.z * inv_s, y3 = wv.w * inv_s;
            count4(cnt, wv, y0, y1, y2, y3, limit);
            code = cvt4_e4m3_sat(y0, y1, y2, y3);
            st_stream4(reinterpret_cast<uint32_t *>(wq) + i4, code);
        }
        tt[c4][rr] = (uint8_t)code;
        tt[c4 + 1][rr] = (uint8_t)(code >> 8);
        tt[c4 + 2][rr] = (uint8_t)(code >> 16);
        tt[c4 + 3][rr] = (uint8_t)(code >> 24);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; k++) {
        const int idx = tid + k * kWThreads, c = idx >> 3, piece = idx & 7;
        if (c0 + c < cols && r0 + piece * 16 < rows) {   // rows % 16 == 0: a 16-row piece is whole
            const uint32_t *p = reinterpret_cast<const uint32_t *>(&tt[c][piece * 16]);
            st_stream16(wq_t + (c0 + c) * rows + r0 + piece * 16, make_uint4(p[0], p[1], p[2], p[3]));
        }
    }
    block_reduce_store(cnt, ws, slots);
}

enum FinalizeMode {
    kFinInit = 0,     // after k_weight_amax at initialisation: reset state, s_base = s_cur = amax/448
    kFinStep = 1,     // after a fused step: advance step / cum_lr / s_cur, record amax, add overflow
    kFinRebase = 2,   // after an AdamW-only pass on a re-scaling step: s_base = s_cur = amax/448
    kFinCastOnly = 3  // after a cast-only pass: record amax, add overflow
};

// `step`: the step number the caller says this call performs (only looked at by the two modes that
// advance the step count): a caller whose count has drifted from the state's is flagged in the state.
__global__ __launch_bounds__(kWThreads) void k_weight_finalize(moss_wscale_state *st, void *ws, int64_t slots,
                                                               int n_partial, int mode, double lr_term, int64_t step)
{
    WPartials p = ws_partials(ws, slots);
    WCounts c;
    for (int i = threadIdx.x; i < n_partial; i += kWThreads) {
        c.amax = fmaxf(c.amax, p.amax[i]);
        c.over += p.over[i];
        c.clip += p.clip[i];
    }
    block_reduce(c);
    if (threadIdx.x != 0) return;
    const float amax = c.amax;
    const uint32_t over = c.over, clip = c.clip;
    if ((mode == kFinStep || mode == kFinRebase) && st->step + 1 != step) st->flags |= MOSS_WSTATE_STEP_MISMATCH;
    if (mode == kFinInit) {
        st->s_base = amax / kE4M3Max;
        st->s_cur = st->s_base;
        st->cum_lr = 0.0;
        st->step = 0;
        st->last_rebase = 0;
        st->amax_seen = amax;
        st->overflow_count = 0;
        st->clipped_count = 0;
        st->flags = 0;
    } else if (mode == kFinStep) {
        double cum = st->cum_lr + lr_term;
        st->cum_lr = cum;
        st->s_cur = (float)((double)st->s_base + cum / 448.0);
        st->step += 1;
        st->amax_seen = amax;
        st->overflow_count += over;
        st->clipped_count += clip;
    } else if (mode == kFinRebase) {
        st->step += 1;
        st->s_base = amax / kE4M3Max;
        st->s_cur = st->s_base;
        st->cum_lr = 0.0;
        st->last_rebase = st->step;
        st->amax_seen = amax;
    } else {
        st->amax_seen = amax;
        st->overflow_count += over;
        st->clipped_count += clip;
    }
}

// Byte transpose [rows x cols] -> [cols x rows] through a padded LDS tile.
constexpr int kTT = 64;
__global__ __launch_bounds__(256) void k_transpose_u8(const uint8_t *__restrict__ src, int64_t rows, int64_t cols,
                                                      uint8_t *__restrict__ dst)
{
    __shared__ uint8_t tile[kTT][kTT + 4];
    const int64_t r0 = (int64_t)blockIdx.y * kTT, c0 = (int64_t)blockIdx.x * kTT;
    for (int i = threadIdx.x; i < kTT * kTT; i += 256) {
        int r = i / kTT, c = i % kTT;
        if (r0 + r < rows && c0 + c < cols) tile[r][c] = src[(r0 + r) * cols + c0 + c];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kTT * kTT; i += 256) {
        int c = i / kTT, r = i % kTT;
        if (r0 + r < rows && c0 + c < cols) dst[(c0 + c) * rows + r0 + r] = tile[r][c];
    }
}

static int grid_for(int64_t n4)
{
    int64_t per_block = (int64_t)kWThreads * 4;   // >= 4 vectors per thread before striding
    int64_t blocks = (n4 + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;
    return (int)(blocks < kWMaxBlocks ? blocks : kWMaxBlocks);
}

static int launch_transpose(const uint8_t *src, int64_t rows, int64_t cols, uint8_t *dst, hipStream_t st)
{
    int64_t gx = (cols + kTT - 1) / kTT, gy = (rows + kTT - 1) / kTT;
    if (gy > 65535) return MOSS_ERR_SHAPE;
    hipLaunchKernelGGL(k_transpose_u8, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, st, src, rows, cols, dst);
    MOSS_LAUNCH_CHECK();
    return MOSS_OK;
}

}  // namespace moss

extern "C" size_t moss_weight_workspace_bytes(int64_t rows, int64_t cols)
{
    if (rows <= 0 || cols <= 0) return 0;
    return (size_t)moss::partial_slots(rows, cols) * (sizeof(float) + 2 * sizeof(uint32_t));
}

static int check_weight_common(int64_t rows, int64_t cols, const void *state, const void *wq, const void *wq_t,
                               const void *ws, size_t ws_bytes)
{
    if (!state || !wq) return MOSS_ERR_NULL;
    if (rows <= 0 || cols <= 0 || (rows * cols) % 4) return MOSS_ERR_SHAPE;
    if (!moss_aligned16(wq) || ((uintptr_t)state & 7)) return MOSS_ERR_ALIGN;
    if (wq_t && !moss_aligned16(wq_t)) return MOSS_ERR_ALIGN;
    if (!ws || ws_bytes < moss_weight_workspace_bytes(rows, cols)) return MOSS_ERR_WORKSPACE;
    if (!moss_aligned16(ws)) return MOSS_ERR_ALIGN;
    return MOSS_OK;
}

namespace moss {

// the 2-D kernel needs whole float4 per row and whole 16-row pieces per transposed row
static bool tile_path_ok(int64_t rows, int64_t cols) { return cols % 4 == 0 && rows % 16 == 0; }

struct WLaunch {
    int64_t rows, cols, n4, slots;
    int grid1d;
    dim3 grid2d;
    hipStream_t st;
    void *ws;
    moss_wscale_state *state;
};

static int finalize(const WLaunch &L, int n_partial, int mode, double lr_term, int64_t step = 0)
{
    hipLaunchKernelGGL(k_weight_finalize, dim3(1), dim3(kWThreads), 0, L.st, L.state, L.ws, L.slots, n_partial, mode, lr_term,
                       step);
    MOSS_LAUNCH_CHECK();
    return MOSS_OK;
}

// cast (and transposed copy) of the weights under the scale stored in the state
static int cast_only(const WLaunch &L, const void *w, bool bf16, uint8_t *wq, uint8_t *wq_t)
{
    const AdamW none{};
    if (wq_t && tile_path_ok(L.rows, L.cols)) {
        if (bf16)
            hipLaunchKernelGGL((k_weight_tile<false, true>), L.grid2d, dim3(kWThreads), 0, L.st, nullptr, nullptr, nullptr, w,
                               L.rows, L.cols, none, 0.0, L.state, wq, wq_t, L.ws, L.slots);
        else
            hipLaunchKernelGGL((k_weight_tile<false, false>), L.grid2d, dim3(kWThreads), 0, L.st, nullptr, nullptr, nullptr, w,
                               L.rows, L.cols, none, 0.0, L.state, wq, wq_t, L.ws, L.slots);
        MOSS_LAUNCH_CHECK();
        return finalize(L, (int)(L.grid2d.x * L.grid2d.y), kFinCastOnly, 0.0);
    }
    if (bf16)
        hipLaunchKernelGGL(k_weight_cast<true>, dim3(L.grid1d), dim3(kWThreads), 0, L.st, w, L.n4, L.state, wq, L.ws, L.slots);
    else
        hipLaunchKernelGGL(k_weight_cast<false>, dim3(L.grid1d), dim3(kWThreads), 0, L.st, w, L.n4, L.state, wq, L.ws, L.slots);
    MOSS_LAUNCH_CHECK();
    int rc = finalize(L, L.grid1d, kFinCastOnly, 0.0);
    if (rc) return rc;
    if (wq_t) return launch_transpose(wq, L.rows, L.cols, wq_t, L.st);
    return MOSS_OK;
}

static int make_launch(WLaunch &L, int64_t rows, int64_t cols, moss_wscale_state *state, void *ws, void *stream)
{
    L.rows = rows; L.cols = cols; L.n4 = rows * cols / 4; L.slots = partial_slots(rows, cols);
    L.grid1d = grid_for(L.n4);
    const int64_t gx = (cols + kWTile - 1) / kWTile, gy = (rows + kWTile - 1) / kWTile;
    if (gy > 65535 || gx > 0x7FFFFFFF) return MOSS_ERR_SHAPE;
    L.grid2d = dim3((unsigned)gx, (unsigned)gy);
    L.st = (hipStream_t)stream; L.ws = ws; L.state = state;
    return MOSS_OK;
}

}  // namespace moss

extern "C" int moss_weight_autoscale_init(const void *w, int w_dtype, int64_t rows, int64_t cols,
                                          moss_wscale_state *state, uint8_t *wq, uint8_t *wq_t,
                                          void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace moss;
    if (!w) return MOSS_ERR_NULL;
    if (w_dtype != MOSS_DT_F32 && w_dtype != MOSS_DT_BF16) return MOSS_ERR_UNSUPPORTED;
    int rc = check_weight_common(rows, cols, state, wq, wq_t, workspace, workspace_bytes);
    if (rc) return rc;
    if (!moss_aligned16(w)) return MOSS_ERR_ALIGN;
    WLaunch L;
    if ((rc = make_launch(L, rows, cols, state, workspace, stream))) return rc;
    const bool bf16 = w_dtype == MOSS_DT_BF16;
    if (bf16)
        hipLaunchKernelGGL(k_weight_amax<true>, dim3(L.grid1d), dim3(kWThreads), 0, L.st, w, L.n4, workspace, L.slots);
    else
        hipLaunchKernelGGL(k_weight_amax<false>, dim3(L.grid1d), dim3(kWThreads), 0, L.st, w, L.n4, workspace, L.slots);
    MOSS_LAUNCH_CHECK();
    if ((rc = finalize(L, L.grid1d, kFinInit, 0.0))) return rc;
    return cast_only(L, w, bf16, wq, wq_t);
}

extern "C" int moss_weight_autoscale_cast(float *w, float *m, float *v, const void *g, int g_dtype,
                                          int64_t rows, int64_t cols, const moss_adamw_args *args,
                                          moss_wscale_state *state, uint8_t *wq, uint8_t *wq_t,
                                          void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace moss;
    if (!w || !m || !v || !g || !args) return MOSS_ERR_NULL;
    if (g_dtype != MOSS_DT_F32 && g_dtype != MOSS_DT_BF16) return MOSS_ERR_UNSUPPORTED;
    int rc = check_weight_common(rows, cols, state, wq, wq_t, workspace, workspace_bytes);
    if (rc) return rc;
    if (!moss_aligned16(w) || !moss_aligned16(m) || !moss_aligned16(v) || ((uintptr_t)g & 7)) return MOSS_ERR_ALIGN;
    if (g_dtype == MOSS_DT_F32 && !moss_aligned16(g)) return MOSS_ERR_ALIGN;
    if (args->step < 1) return MOSS_ERR_SHAPE;

    WLaunch L;
    if ((rc = make_launch(L, rows, cols, state, workspace, stream))) return rc;
    AdamW a{args->lr, args->beta1, args->beta2, args->eps, args->weight_decay,
            args->one_minus_beta1, args->one_minus_beta2, args->bias_corr1, args->bias_corr2};
    const double lr_term = (double)args->margin * (double)args->lr;
    const bool rebase = args->interval > 0 && (args->step % args->interval) == 0;
    const bool gb = g_dtype == MOSS_DT_BF16;
    const dim3 g1(L.grid1d), blk(kWThreads);

    if (rebase) {
        // AdamW alone (it yields amax(W_new)), re-base the scale from it, then cast with the new scale
        if (gb)
            hipLaunchKernelGGL((k_adamw_cast<true, false>), g1, blk, 0, L.st, w, m, v, g, L.n4, a, lr_term, state, wq, workspace, L.slots);
        else
            hipLaunchKernelGGL((k_adamw_cast<false, false>), g1, blk, 0, L.st, w, m, v, g, L.n4, a, lr_term, state, wq, workspace, L.slots);
        MOSS_LAUNCH_CHECK();
        if ((rc = finalize(L, L.grid1d, kFinRebase, lr_term, args->step))) return rc;
        return cast_only(L, w, false, wq, wq_t);
    }
    if (wq_t && tile_path_ok(rows, cols)) {
        if (gb)
            hipLaunchKernelGGL((k_weight_tile<true, true>), L.grid2d, blk, 0, L.st, w, m, v, g, rows, cols, a, lr_term, state, wq, wq_t, workspace, L.slots);
        else
            hipLaunchKernelGGL((k_weight_tile<true, false>), L.grid2d, blk, 0, L.st, w, m, v, g, rows, cols, a, lr_term, state, wq, wq_t, workspace, L.slots);
        MOSS_LAUNCH_CHECK();
        return finalize(L, (int)(L.grid2d.x * L.grid2d.y), kFinStep, lr_term, args->step);
    }
    if (gb)
        hipLaunchKernelGGL((k_adamw_cast<true, true>), g1, blk, 0, L.st, w, m, v, g, L.n4, a, lr_term, state, wq, workspace, L.slots);
    else
        hipLaunchKernelGGL((k_adamw_cast<false, true>), g1, blk, 0, L.st, w, m, v, g, L.n4, a, lr_term, state, wq, workspace, L.slots);
    MOSS_LAUNCH_CHECK();
    if ((rc = finalize(L, L.grid1d, kFinStep, lr_term, args->step))) return rc;
    if (wq_t) return launch_transpose(wq, rows, cols, wq_t, L.st);
    return MOSS_OK;
}
