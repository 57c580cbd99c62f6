// Two-level microscaling quantizer for gfx950 (paper Sec. 3.1, Eq. 2-3).
//
// Codes can only be emitted once the maximum of the whole tensor is known (s = amax/448), so
// every path sees X, agrees on the maximum, and then, per group of 32 values, derives the
// power-of-two local scale from integer / exact FP32 comparisons and emits the E4M3 codes of
// (x * 2^-e) * (1/s).  Magnitudes of finite BF16 values order like their low 15 bits, so every
// maximum is an integer maximum and is exact.
//
//  * One launch (k_quant_persist): tensors of up to four 128 x 128 tiles per workgroup of a
//    co-resident grid stay in registers between the maximum and the codes; X is read once.
//  * Two launches: k_amax_bf16 leaves one partial maximum per workgroup in the workspace, and
//    k_quant_row (row groups alone) or k_quant_tile (column groups, or both groupings from one
//    fetch of X) folds the partials and converts.
#include <atomic>

#include "moss_internal.h"

namespace moss {

constexpr int kQuantThreads = 256;
constexpr int kMaxPartials = 2048;

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// lane-wise maximum of two pairs of 16-bit unsigned values (one packed instruction)
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}

constexpr uint32_t kMagMask = 0x7FFF7FFFu;   // the 15 magnitude bits of both BF16 halves of a word

// max of the eight 15-bit magnitudes held in a 16-byte chunk
__device__ __forceinline__ uint32_t chunk_absmax(const uint4 &r)
{
    const uint32_t p = pk_max_u16(pk_max_u16(r.x & kMagMask, r.y & kMagMask), pk_max_u16(r.z & kMagMask, r.w & kMagMask));
    const uint32_t lo = p & 0xFFFFu, hi = p >> 16;
    return lo > hi ? lo : hi;
}

constexpr int kAmaxUnroll = 4;

__global__ __launch_bounds__(kQuantThreads) void k_amax_bf16(const uint16_t *__restrict__ x, int64_t n_chunks,
                                                             int chunks_per_row, int64_t ld, int dense,
                                                             uint32_t *__restrict__ partial)
{
    __shared__ uint32_t red[kQuantThreads / kWave];
    uint32_t m = 0;
    // kAmaxUnroll independent 16-byte loads per thread and trip keep enough bytes in flight
    const int64_t stride = (int64_t)gridDim.x * kQuantThreads * kAmaxUnroll;
    for (int64_t id0 = (int64_t)blockIdx.x * kQuantThreads * kAmaxUnroll + threadIdx.x; id0 < n_chunks; id0 += stride) {
        uint4 r[kAmaxUnroll];
#pragma unroll
        for (int u = 0; u < kAmaxUnroll; u++) {
            const int64_t id = id0 + (int64_t)u * kQuantThreads;
            r[u] = make_uint4(0, 0, 0, 0);
            if (id < n_chunks) {
                int64_t off;
                if (dense) {
                    off = id * 8;
                } else {
                    int64_t row = id / chunks_per_row;
                    off = row * ld + (id - row * chunks_per_row) * 8;
                }
                r[u] = ld_stream16(x + off);
            }
        }
#pragma unroll
        for (int u = 0; u < kAmaxUnroll; u++) {
            uint32_t c = chunk_absmax(r[u]);
            m = c > m ? c : m;
        }
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
    float s, inv_s;   // s = amax/448 (1 for an all-zero tensor), inv_s = fl(1/s), at most FLT_MAX
    float frac;       // amax = frac * 2^expo, frac in [0.5, 1)
    int expo;
    bool zero;
    // Integer form of the local exponent, for a tensor maximum that is a normal BF16 number (see fast_group)
    bool fast;
    int add;          // added to a group maximum's bit pattern before its exponent field is read
    int ebase;        // 127 - exponent field of the tensor maximum
    uint32_t fbits;   // bit pattern of inv_s with 127 added to its exponent field (may leave the finite range)
    int wide_at;      // groups whose byte is <= wide_at need the two-product form (-1 or less: none)
};

template <bool CEIL>
__device__ __forceinline__ GlobalScale make_global_scale(uint32_t amax_bits);

// Every workgroup folds the (few) partial maxima itself: cheaper than another launch.
template <bool CEIL>
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
    return make_global_scale<CEIL>(m);
}

// The exponent of a group with maximum a under the tensor maximum A is round(log2(a / A)) (Eq. 3), or
// its ceiling.  For normal BF16 numbers a = 2^(Ea-127) (128 + ma) / 128, A likewise, so it is
// Ea - EA + c with c in {-1, 0, +1} decided by the 7-bit mantissas alone:
//   nearest: +1 iff (128 + ma)^2 >= 2 (128 + mA)^2,  -1 iff 2 (128 + ma)^2 < (128 + mA)^2
//            (for a given mA only one of the two can happen: the first for mA <= 52, the second for mA >= 54);
//   ceiling: +1 iff ma > mA.
// Either way c = +1 is "ma >= some threshold T", c = -1 is "ma < T": adding 128 - T (or -T) to the 15-bit
// pattern of a carries into (borrows from) its exponent field exactly when c applies, and
//   Ea - EA + c = ((a + add) >> 7) - EA
// with one constant per tensor.  Zero groups and groups whose maximum is a BF16 subnormal do not fit this
// form and are handled apart.
template <bool CEIL>
__device__ __forceinline__ GlobalScale make_global_scale(uint32_t m)
{
    m = (uint32_t)__builtin_amdgcn_readfirstlane((int)m);   // the same in every lane: keep what follows in scalar registers
    GlobalScale g;
    float amax = bf16_bits_to_f32(m);
    g.zero = (m == 0);
    g.s = g.zero ? 1.0f : amax / kE4M3Max;
    g.inv_s = fminf(1.0f / g.s, __FLT_MAX__);   // finite, so that zero inputs keep code zero
    g.frac = __builtin_amdgcn_frexp_mantf(amax);
    g.expo = __builtin_amdgcn_frexp_expf(amax);
    const int mA = (int)(m & 127u), EA = (int)(m >> 7), M = 128 + mA;
    g.fast = EA >= 1;
    if (CEIL) {
        g.add = 127 - mA;
    } else {
        int t = (int)((float)M * 1.41421356f);               // ceil(sqrt(2) M), fixed up in integers
        while (t * t < 2 * M * M) t++;
        while ((t - 1) * (t - 1) >= 2 * M * M) t--;
        if (t <= 255) {
            g.add = 256 - t;                                   // +1 iff 128 + ma >= t
        } else {
            int u = (int)((float)M * 0.70710678f);             // ceil(M / sqrt(2))
            while (2 * u * u < M * M) u++;
            while (2 * (u - 1) * (u - 1) >= M * M) u--;
            g.add = 128 - u;                                   // -1 iff 128 + ma < u
        }
    }
    g.ebase = 127 - EA;
    const uint32_t ib = __float_as_uint(g.inv_s);
    g.fbits = ib + (127u << 23);
    g.wide_at = (int)(ib >> 23) - 128;
    return g;
}

// Exponent byte and factor 2^-e * (1/s) of a group with maximum bit pattern a (zero or a normal number) in
// the integer form: 2^-e * (1/s) is inv_s with -e added to its exponent field (finite unless byte <= g.wide_at,
// which the caller checks through min_fbyte).  A zero group stores byte 0 and multiplies its zeros by 1/s.
__device__ __forceinline__ void fast_group(uint32_t a, const GlobalScale &g, uint32_t &byte, float &factor, uint32_t &min_fbyte)
{
    int k = (int)((a + (uint32_t)g.add) >> 7) + g.ebase;
    k = k < 0 ? 0 : k;
    const bool z = a == 0;
    byte = z ? 0u : (uint32_t)k;
    const uint32_t fb = z ? 127u : (uint32_t)k;
    min_fbyte = fb < min_fbyte ? fb : min_fbyte;
    factor = __uint_as_float(g.fbits - (fb << 23));
}

// The general form (any finite a, any tensor maximum): e = round(log2(a/amax)) (or its ceiling), clamped
// to [-127, 0]; a = 15-bit BF16 magnitude bits.  With a = f_a 2^ea and amax = f_A 2^eA (f in [0.5,1), at most 8
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

// The code of x in a group with exponent e is cast((x * 2^-e) * (1/s)) (Sec. 3.1, Eq. 2).  The
// first product is exact, so x * (2^-e * (1/s)) rounds to the same value whenever that
// single factor is finite; it is not for groups of tiny nonzero values under a small
// global maximum, which take the two-product form.  An all-zero group (e = -127) gets the
// factor 0: its codes are signed zeros either way.
// group_factor returns that single factor, or NaN / infinity where the two-product form is needed.
__device__ __forceinline__ float group_factor(uint32_t a_bits, int ex, const GlobalScale &g)
{
    return a_bits == 0 ? g.inv_s * 0.0f : pow2_neg(ex) * g.inv_s;
}

__device__ __forceinline__ bool factor_is_wide(float fused) { return !(fused < __builtin_inff()); }

// 2^(-e) from the stored exponent byte e + 127
__device__ __forceinline__ float pow2_neg_of_byte(uint32_t byte) { return __uint_as_float((254u - byte) << 23); }

template <bool FUSED>
__device__ __forceinline__ float scaled(float x, float fused, uint32_t ebyte, float inv_s)
{
    return FUSED ? x * fused : (x * pow2_neg_of_byte(ebyte)) * inv_s;
}

// Saturation of the cast.  The converter turns values beyond +-448 into the NaN code unless the wave's
// FP16_OVFL mode bit is set, in which case it saturates to the largest finite code by itself: the kernels
// set the bit once (converter_saturates) instead of clamping every value first (one instruction per value
// and grouping saved; the exhaustive all-BF16-values test covers the behaviour).  The mode bit lives and dies
// with the wave, and these kernels have no other instruction that it affects.
__device__ __forceinline__ float clamp448(float y) { return y; }
__device__ __forceinline__ void converter_saturates()
{
    __builtin_amdgcn_s_setreg((1 - 1) << 11 | 23 << 6 | 1, 1);   // hwreg(MODE, offset 23, 1 bit) = 1
}

// four FP32 values -> four E4M3 bytes (a in the lowest byte), saturating
__device__ __forceinline__ uint32_t cvt4_sat(float a, float b, float c, float d)
{
    int r = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a), clamp448(b), 0, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(c), clamp448(d), r, true);
    return (uint32_t)r;
}

__device__ __forceinline__ uint32_t quad_max_u32(uint32_t v)
{
    uint32_t o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
    v = o > v ? o : v;
    o = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);           // quad_perm [2,3,0,1]
    return o > v ? o : v;
}

// E4M3 codes of the 8 values of a 16-byte chunk that share one group factor
template <bool FUSED>
__device__ __forceinline__ uint2 row_codes(const uint4 &r, float fused, uint32_t ebyte, float inv_s)
{
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
    uint32_t out[2];
#pragma unroll
    for (int h = 0; h < 2; h++) {
        const float y0 = scaled<FUSED>(bf16_bits_to_f32(w[2 * h] & 0xFFFFu), fused, ebyte, inv_s);
        const float y1 = scaled<FUSED>(__uint_as_float(w[2 * h] & 0xFFFF0000u), fused, ebyte, inv_s);
        const float y2 = scaled<FUSED>(bf16_bits_to_f32(w[2 * h + 1] & 0xFFFFu), fused, ebyte, inv_s);
        const float y3 = scaled<FUSED>(__uint_as_float(w[2 * h + 1] & 0xFFFF0000u), fused, ebyte, inv_s);
        out[h] = cvt4_sat(y0, y1, y2, y3);
    }
    return make_uint2(out[0], out[1]);
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
    converter_saturates();
    const GlobalScale g = fold_global_scale<CEIL>(partial, n_partial, red);
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
            raw[u] = ld_stream16(x + off);
        }
    }
    float f[kRowUnroll];
    uint32_t eb[kRowUnroll], gmax[kRowUnroll];
    uint32_t sub_min = ~0u, min_fb = 255u;
#pragma unroll
    for (int u = 0; u < kRowUnroll; u++) {
        // the four lanes of a quad hold one group; n_chunks % 4 == 0 keeps quads uniform
        gmax[u] = quad_max_u32(chunk_absmax(raw[u]));
        sub_min = gmax[u] - 1u < sub_min ? gmax[u] - 1u : sub_min;     // (a zero group wraps to the largest value)
        fast_group(gmax[u], g, eb[u], f[u], min_fb);
    }
    // the integer form does not cover a subnormal tensor or group maximum, nor factors beyond the finite range
    bool any_wide = false;
    if (__any(!g.fast || sub_min < 127u || (int)min_fb <= g.wide_at)) {
        bool wide = false;
#pragma unroll
        for (int u = 0; u < kRowUnroll; u++) {
            const int ex = local_exponent<CEIL>(gmax[u], g);
            eb[u] = (uint32_t)(ex + 127);
            f[u] = group_factor(gmax[u], ex, g);
            wide |= factor_is_wide(f[u]);
        }
        any_wide = __any(wide);
    }
#pragma unroll
    for (int u = 0; u < kRowUnroll; u++) {
        const int64_t id = base + (int64_t)u * kQuantThreads;
        const uint2 out = any_wide ? row_codes<false>(raw[u], f[u], eb[u], g.inv_s) : row_codes<true>(raw[u], f[u], eb[u], g.inv_s);
        if (id < n_chunks) {
            st_stream8(q + id * 8, out);
            if ((threadIdx.x & 3) == 0) e[id >> 2] = (uint8_t)eb[u];
        }
    }
}

// Column grouping (groups of 32 along the rows, outputs stored transposed), optionally fused
// with the row grouping so that X is fetched once for both outputs.
//
// A workgroup owns a 128 x 128 tile, one wave per 32-row group.  Lane (rl = lane / 16,
// ch = lane % 16) holds rows 8 rl .. 8 rl + 7 of the group and the 8 columns of chunk ch, so
//  * every global load is 16 bytes per lane and a wave instruction fetches four full
//    256-byte row pieces;
//  * a column group lives in the four lanes {ch, ch+16, ch+32, ch+48}: its maximum is a packed
//    in-register maximum over 8 rows and two cross-lane steps -- no LDS, no barrier;
//  * a row group (32 columns of one row) lives in a quad of lanes, as in k_quant_row;
//  * a lane ends up with 8 consecutive rows of each of its columns = one 8-byte piece of a
//    transposed output row; the pieces are collected in LDS and, after the only barrier,
//    8 lanes write the 128 bytes of each transposed row.
constexpr int kTile = 128;
constexpr int kTilePitch = kTile + 8;   // bytes per staged output row (8-byte aligned pieces, some bank spread)

// LDS of a workgroup that converts tiles: the transposed codes of the tile, and the exponent bytes of the tile's
// 128 x 4 row groups and 4 x 128 column groups, which leave as one 4-byte store per row / per column (single-byte
// stores from every lane cost several times the cache-line visits and were ~3.5 us of a 64 MiB tensor's 42 us).
struct TileLds {
    __attribute__((aligned(16))) uint8_t tt[kTile][kTilePitch];   // transposed codes [column][row]
    __attribute__((aligned(8))) uint8_t te[4][kTile];             // row-group exponents [column group of the tile][row]
    __attribute__((aligned(8))) uint8_t tc[4][kTile];             // column-group exponents [row group of the tile][column]
    uint32_t redo;                                                // bit k: the workgroup's tile k needs the general form
};

// The converter writes two bytes of its destination and keeps the other two, so its destination is also an
// input.  For the first write into a word that input is dead weight: handing it a register that is free
// anyway (one of the operands) saves the move that a zero would need.
__device__ __forceinline__ uint32_t cvt_lo_fresh(float a, float b)
{
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)__float_as_uint(a), false);
}
__device__ __forceinline__ uint32_t cvt_hi(float a, float b, uint32_t word)
{
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)word, true);
}

// What a lane needs to know about its part of a tile: byte offsets from wave-uniform tile bases (32 bits are
// enough inside a tile: the host checks 128 * row pitch < 2^31), and which of its rows / columns exist.
struct LanePlace {
    uint32_t q_row_off;    // from q_row + r0 * cols + c0 to this lane's first row, this lane's 8 columns
    bool col_ok;           // this lane's 8 columns exist (cols % 32 == 0: all or none)
    int n_ok;              // how many of this lane's 8 rows exist
};

// Codes of one lane's 8 x 8 values for both groupings.  Rows are taken two at a time: the
// converter packs two values into two neighbouring bytes, so feeding it the same column
// of two consecutive rows builds the transposed 8-row pieces without any byte shuffling.
// rbytes / cbytes hold the 8 row-group and the 8 column-group exponent bytes (needed by the two-product form).
// FULL: every row and column of the tile exists, nothing is predicated.
template <bool ROW, bool COL, bool FUSED, bool FULL>
__device__ __forceinline__ void tile_codes(const uint4 (&raw)[8], const float (&rf)[8], const uint32_t (&rbytes)[2],
                                           const float (&cf)[8], const uint32_t (&cbytes)[2], float inv_s, int n_ok,
                                           uint8_t *__restrict__ q_row_tile, uint32_t q_row_off, uint32_t cols,
                                           uint32_t (&pieces)[8][2])
{
#pragma unroll
    for (int pr = 0; pr < 4; pr++) {
        float x[2][8];
#pragma unroll
        for (int k = 0; k < 2; k++) {
            const uint4 &r = raw[2 * pr + k];
            const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
            for (int d = 0; d < 4; d++) {
                x[k][2 * d] = bf16_bits_to_f32(w[d] & 0xFFFFu);
                x[k][2 * d + 1] = __uint_as_float(w[d] & 0xFFFF0000u);
            }
        }
        if (ROW) {
#pragma unroll
            for (int k = 0; k < 2; k++) {
                const int it = 2 * pr + k;
                const uint32_t eb = (rbytes[it >> 2] >> (8 * (it & 3))) & 0xFFu;
                float y[8];
#pragma unroll
                for (int j = 0; j < 8; j++) y[j] = clamp448(scaled<FUSED>(x[k][j], rf[it], eb, inv_s));
                const uint2 out = make_uint2(cvt_hi(y[2], y[3], cvt_lo_fresh(y[0], y[1])), cvt_hi(y[6], y[7], cvt_lo_fresh(y[4], y[5])));
                // (codes are stored through the caches: the GEMM that follows reads them, and inside a training step this
                // measured 2 % faster for the quantizer than streaming stores; X itself is streamed)
                if (FULL || it < n_ok) *reinterpret_cast<uint2 *>(q_row_tile + (q_row_off + (uint32_t)it * cols)) = out;
            }
        }
        if (!COL) continue;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const uint32_t eb = (cbytes[j >> 2] >> (8 * (j & 3))) & 0xFFu;
            const float a = clamp448(scaled<FUSED>(x[0][j], cf[j], eb, inv_s));
            const float b = clamp448(scaled<FUSED>(x[1][j], cf[j], eb, inv_s));
            uint32_t &word = pieces[j][pr >> 1];
            if (pr & 1)
                word = cvt_hi(a, b, word);
            else
                word = cvt_lo_fresh(a, b);
        }
    }
}

// Group maxima of a lane's part of a tile: rmax[it] = maximum of the row group that holds this lane's 8 columns
// of row it (a quad of lanes shares it), cmax[j] = maximum of the column group of this lane's column j over the
// wave's 32 rows (this lane's 8 rows and those of the lanes 16, 32 and 48 further on).
template <bool ROW, bool COL>
__device__ __forceinline__ void tile_group_maxima(const uint4 (&raw)[8], uint32_t (&rmax)[8], uint32_t (&cmax)[8])
{
    uint32_t pm[4] = {0, 0, 0, 0};
#pragma unroll
    for (int it = 0; it < 8; it++) {
        const uint32_t m0 = raw[it].x & kMagMask, m1 = raw[it].y & kMagMask, m2 = raw[it].z & kMagMask,
                       m3 = raw[it].w & kMagMask;
        if (COL) {
            pm[0] = pk_max_u16(pm[0], m0);
            pm[1] = pk_max_u16(pm[1], m1);
            pm[2] = pk_max_u16(pm[2], m2);
            pm[3] = pk_max_u16(pm[3], m3);
        }
        if (ROW) {
            const uint32_t p = pk_max_u16(pk_max_u16(m0, m1), pk_max_u16(m2, m3));
            const uint32_t lo = p & 0xFFFFu, hi = p >> 16;
            rmax[it] = quad_max_u32(lo > hi ? lo : hi);
        }
    }
    if (COL) {
#pragma unroll
        for (int d = 0; d < 4; d++) {
            pm[d] = pk_max_u16(pm[d], (uint32_t)__shfl_xor((int)pm[d], 16, 64));
            pm[d] = pk_max_u16(pm[d], (uint32_t)__shfl_xor((int)pm[d], 32, 64));
        }
#pragma unroll
        for (int j = 0; j < 8; j++) cmax[j] = (pm[j >> 1] >> (16 * (j & 1))) & 0xFFFFu;
    }
}

struct TileShape {
    int64_t rows, cols, ld;
};

__device__ __forceinline__ bool tile_is_full(const TileShape &sh, int64_t r0, int64_t c0)
{
    return r0 + kTile <= sh.rows && c0 + kTile <= sh.cols;
}

// This lane's 8 x 16 bytes of the tile whose first element is (r0, c0); zeros outside X.
__device__ __forceinline__ void load_tile(uint4 (&raw)[8], const uint16_t *__restrict__ x, const TileShape &sh, int64_t r0,
                                          int64_t c0)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, rl = lane >> 4, ch = lane & 15;
    const uint16_t *tile = x + r0 * sh.ld + c0;                                      // wave-uniform
    const uint32_t ld = (uint32_t)sh.ld;
    const uint32_t off = (uint32_t)(wave * kGroup + rl * 8) * ld + (uint32_t)ch * 8;  // elements, < 2^31 (host check)
    if (tile_is_full(sh, r0, c0)) {
#pragma unroll
        for (int it = 0; it < 8; it++) raw[it] = ld_stream16(tile + (off + (uint32_t)it * ld));
    } else {
        const bool ok = c0 + ch * 8 < sh.cols;
        const int64_t rbase = r0 + wave * kGroup + rl * 8;
#pragma unroll
        for (int it = 0; it < 8; it++) {
            raw[it] = make_uint4(0, 0, 0, 0);
            if (ok && rbase + it < sh.rows) raw[it] = ld_stream16(tile + (off + (uint32_t)it * ld));
        }
    }
}

// largest 15-bit magnitude among this lane's 64 values
__device__ __forceinline__ uint32_t tile_absmax(const uint4 (&raw)[8])
{
    uint32_t pm = 0;
#pragma unroll
    for (int it = 0; it < 8; it++)
        pm = pk_max_u16(pm, pk_max_u16(pk_max_u16(raw[it].x & kMagMask, raw[it].y & kMagMask),
                                       pk_max_u16(raw[it].z & kMagMask, raw[it].w & kMagMask)));
    const uint32_t lo = pm & 0xFFFFu, hi = pm >> 16;
    return lo > hi ? lo : hi;
}

// Exponents and codes of one 128 x 128 tile from the registers that hold it, in one of two forms.
//   FAST: for tiles that lie wholly inside X.  Nothing is predicated, the exponents come from the integer
//         form (fast_group) and every code from one multiplication by 2^-e (1/s).  That form does not cover
//         a subnormal tensor or group maximum, nor a factor beyond the finite range (tiny nonzero groups under
//         a small global maximum): the return value says whether this wave met one, and the tile then has to
//         be done again in the general form (what was stored is overwritten).
//   general (!FAST): any tile, any finite data: predicated accesses, local_exponent, two-product codes.
// The two forms never sit side by side in a loop body: a kernel runs the fast form over its tiles and the
// general form afterwards for the (rare) tiles that need it, so that the fast form's registers stay few.
// The body contains one workgroup barrier; the LDS staging area stays in use until the caller's next barrier.
template <bool ROW, bool COL, bool CEIL, bool FAST>
__device__ __forceinline__ bool quant_tile_body(const uint4 (&raw)[8], const TileShape &sh, int64_t r0, int64_t c0,
                                                const GlobalScale &g, uint8_t *__restrict__ q_row,
                                                uint8_t *__restrict__ e_row, uint8_t *__restrict__ q_col,
                                                uint8_t *__restrict__ e_col, TileLds &lds)
{
    constexpr bool FULL = FAST;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, rl = lane >> 4, ch = lane & 15;
    const int64_t rows = sh.rows, cols = sh.cols;
    const int row_in_tile = wave * kGroup + rl * 8;              // first of this lane's 8 rows
    const bool ok = FULL || (c0 + ch * 8 < cols && r0 + row_in_tile < rows);     // cols % 32 == 0: whole column chunks
    const int64_t left = rows - (r0 + row_in_tile);
    const int n_ok = FULL ? 8 : (!ok ? 0 : (left < 8 ? (int)left : 8));         // (always 0 or 8 with COL: rows % 32 == 0)
    const int64_t n_rgroups = rows / kGroup, n_cgroups = cols / kGroup;

    // group maxima, then exponent bytes and factors
    float rf[8], cf[8];
    uint32_t rbytes[2] = {0, 0}, cbytes[2] = {0, 0};
    bool redo = false;
    {
        uint32_t rmax[8], cmax[8];
        tile_group_maxima<ROW, COL>(raw, rmax, cmax);
        if (FAST) {
            uint32_t sub_min = ~0u, min_fb = 255u;
#pragma unroll
            for (int i = 0; i < 8; i++) {
                uint32_t byte;
                if (ROW) {
                    sub_min = rmax[i] - 1u < sub_min ? rmax[i] - 1u : sub_min;   // (a zero group wraps to the largest value)
                    fast_group(rmax[i], g, byte, rf[i], min_fb);
                    rbytes[i >> 2] |= byte << (8 * (i & 3));
                }
                if (COL) {
                    sub_min = cmax[i] - 1u < sub_min ? cmax[i] - 1u : sub_min;
                    fast_group(cmax[i], g, byte, cf[i], min_fb);
                    cbytes[i >> 2] |= byte << (8 * (i & 3));
                }
            }
            redo = __any(!g.fast || sub_min < 127u || (int)min_fb <= g.wide_at);
        } else {
#pragma unroll
            for (int i = 0; i < 8; i++) {
                rf[i] = cf[i] = 0.0f;     // (not used by the two-product form)
                if (ROW) rbytes[i >> 2] |= (uint32_t)(local_exponent<CEIL>(rmax[i], g) + 127) << (8 * (i & 3));
                if (COL) cbytes[i >> 2] |= (uint32_t)(local_exponent<CEIL>(cmax[i], g) + 127) << (8 * (i & 3));
            }
        }
    }

    // exponent bytes into LDS: the first lane of a quad holds its row group's bytes of 8 consecutive rows, the
    // first 16 lanes of a wave the bytes of their 8 columns for the wave's row group
    if (ROW && (lane & 3) == 0) *reinterpret_cast<uint2 *>(&lds.te[ch >> 2][row_in_tile]) = make_uint2(rbytes[0], rbytes[1]);
    if (COL && rl == 0) *reinterpret_cast<uint2 *>(&lds.tc[wave][ch * 8]) = make_uint2(cbytes[0], cbytes[1]);

    uint32_t pieces[8][2];
    uint8_t *q_row_tile = ROW ? q_row + r0 * cols + c0 : nullptr;                       // wave-uniform
    const uint32_t q_row_off = (uint32_t)row_in_tile * (uint32_t)cols + (uint32_t)ch * 8;
    tile_codes<ROW, COL, FAST, FULL>(raw, rf, rbytes, cf, cbytes, g.inv_s, n_ok, q_row_tile, q_row_off, (uint32_t)cols, pieces);

    // the 8 rows of this lane form one 8-byte piece of each of its 8 transposed rows
    if (COL) {
#pragma unroll
        for (int j = 0; j < 8; j++)
            *reinterpret_cast<uint2 *>(&lds.tt[ch * 8 + j][row_in_tile]) = make_uint2(pieces[j][0], pieces[j][1]);
    }
    __syncthreads();
    if (COL) {
        uint8_t *q_col_tile = q_col + c0 * rows + r0;                                    // wave-uniform
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const int idx = tid + k * kQuantThreads, c = idx >> 3, piece = idx & 7;
            if (FULL || (c0 + c < cols && r0 + piece * 16 < rows)) {
                const uint32_t *src = reinterpret_cast<const uint32_t *>(&lds.tt[c][piece * 16]);
                *reinterpret_cast<uint4 *>(q_col_tile + ((uint32_t)c * (uint32_t)rows + (uint32_t)piece * 16)) = make_uint4(src[0], src[1], src[2], src[3]);
            }
        }
    }
    // Exponent bytes: threads 0..127 each own a row of the tile (its 4 row-group bytes are neighbours in e_row),
    // threads 128..255 a column (its 4 column-group bytes are neighbours in e_col).
    if (ROW && tid < kTile) {
        const int r = tid;
        const uint32_t word = (uint32_t)lds.te[0][r] | (uint32_t)lds.te[1][r] << 8 | (uint32_t)lds.te[2][r] << 16 | (uint32_t)lds.te[3][r] << 24;
        uint8_t *dst = e_row + (r0 + r) * n_cgroups + (c0 >> 5);
        if (FULL && (n_cgroups & 3) == 0) {
            *reinterpret_cast<uint32_t *>(dst) = word;
        } else if (r0 + r < rows) {
#pragma unroll
            for (int q = 0; q < 4; q++)
                if (c0 + q * kGroup < cols) dst[q] = (uint8_t)(word >> (8 * q));
        }
    }
    if (COL && tid >= kTile) {
        const int c = tid - kTile;
        const uint32_t word = (uint32_t)lds.tc[0][c] | (uint32_t)lds.tc[1][c] << 8 | (uint32_t)lds.tc[2][c] << 16 | (uint32_t)lds.tc[3][c] << 24;
        uint8_t *dst = e_col + (c0 + c) * n_rgroups + (r0 >> 5);
        if (FULL && (n_rgroups & 3) == 0) {
            *reinterpret_cast<uint32_t *>(dst) = word;
        } else if (c0 + c < cols) {
#pragma unroll
            for (int q = 0; q < 4; q++)
                if (r0 + q * kGroup < rows) dst[q] = (uint8_t)(word >> (8 * q));
        }
    }
    return redo;
}

// Workgroup -> tile.  A tile leaves 4 exponent bytes per row and per column, pieces of memory lines that its
// neighbours complete.  Workgroups are handed to the 8 XCDs in turn (workgroup id modulo 8) and each XCD has an
// L2 of its own, so the tiles are dealt out in squares of kTileSquare x kTileSquare, a square to an XCD: the
// pieces of a line then meet in one L2 and leave it as whole 32-byte sectors instead of one write-back each.
constexpr int kXcds = 8;
constexpr int kTileSquare = 8;

__host__ __device__ inline int64_t tile_grid_size(int64_t tiles_x, int64_t tiles_y)
{
    const int64_t squares = ((tiles_x + kTileSquare - 1) / kTileSquare) * ((tiles_y + kTileSquare - 1) / kTileSquare);
    return (squares + kXcds - 1) / kXcds * kXcds * (kTileSquare * kTileSquare);
}

// false: this workgroup's place in the grid lies outside the tensor (squares over the edge, padding of the grid)
__device__ __forceinline__ bool tile_of_workgroup(uint32_t id, int tiles_x, int tiles_y, int &tx, int &ty)
{
    const uint32_t xcd = id % kXcds, k = id / kXcds;
    const uint32_t square = k / (kTileSquare * kTileSquare) * kXcds + xcd, j = k % (kTileSquare * kTileSquare);
    const uint32_t squares_x = (uint32_t)(tiles_x + kTileSquare - 1) / kTileSquare;
    ty = (int)(square / squares_x * kTileSquare + j / kTileSquare);
    tx = (int)(square % squares_x * kTileSquare + j % kTileSquare);
    return tx < tiles_x && ty < tiles_y;
}

template <bool ROW, bool CEIL>
__global__ __launch_bounds__(kQuantThreads, 4) void k_quant_tile(const uint16_t *__restrict__ x, int64_t rows, int64_t cols,
                                                                 int64_t ld, int tiles_x, int tiles_y,
                                                                 const uint32_t *__restrict__ partial,
                                                                 int n_partial, uint8_t *__restrict__ q_row,
                                                                 uint8_t *__restrict__ e_row, uint8_t *__restrict__ q_col,
                                                                 uint8_t *__restrict__ e_col, float *__restrict__ s_global)
{
    __shared__ uint32_t red[kQuantThreads / kWave];
    __shared__ TileLds lds;

    int tx, ty;
    if (!tile_of_workgroup(blockIdx.x, tiles_x, tiles_y, tx, ty)) return;     // (the whole workgroup, before any barrier)
    converter_saturates();
    if (threadIdx.x == 0) lds.redo = 0;
    const GlobalScale g = fold_global_scale<CEIL>(partial, n_partial, red);
    if (blockIdx.x == 0 && threadIdx.x == 0) *s_global = g.s;                 // (workgroup 0 has tile (0, 0))

    const TileShape sh = {rows, cols, ld};
    const int64_t r0 = (int64_t)ty * kTile, c0 = (int64_t)tx * kTile;
    uint4 raw[8];
    load_tile(raw, x, sh, r0, c0);
    bool general = true;
    if (tile_is_full(sh, r0, c0)) {        // (lds.redo was cleared before the barrier inside fold_global_scale)
        if (quant_tile_body<ROW, true, CEIL, true>(raw, sh, r0, c0, g, q_row, e_row, q_col, e_col, lds) && (threadIdx.x & 63) == 0)
            atomicOr(&lds.redo, 1u);
        __syncthreads();
        general = lds.redo != 0;
    }
    if (general) quant_tile_body<ROW, true, CEIL, false>(raw, sh, r0, c0, g, q_row, e_row, q_col, e_col, lds);
}

// ---------------------------------------------------------------------------------------------
// One-launch variant for tensors of up to kKeep tiles per workgroup of a co-resident grid (two
// workgroups per compute unit; 64 MiB of BF16 on 256 compute units).  A workgroup loads its
// tiles once and keeps them in registers between the maximum and the codes, so X is fetched
// from memory once instead of twice: 128 KiB of registers per workgroup hold the tensor, the
// other half of the register file does the arithmetic.
//
// Between the walks the workgroups agree on the global maximum through a few words of the
// workspace.  Only relaxed device-scope atomics are used, no fences: a release or acquire fence
// at device scope writes back / invalidates the whole L2 of the XCD and cost ~60 us per launch
// here.  Everything that travels is a single word that carries its own validity:
//   1. a workgroup merges its maximum into its group's word (atomic max) and only then -- the
//      second atomic's operand depends on the first one's return value -- counts itself in;
//   2. the workgroup that completes a group's count takes the group's word (all merges into it
//      were performed before their senders counted in), merges it into the global word and
//      counts the group in the same way;
//   3. the workgroup that completes the count of groups takes the global word and publishes
//      0x80000000 | maximum in one flag word per group, which the group's members poll.
// The poll is bounded: a workgroup that does not see its flag within poll_limit polls (the grid
// was not co-resident after all) computes the global maximum from X by itself, so every wave
// ends whatever the scheduler does, and the outputs are the same either way.
//
// The words start at zero and the kernel leaves them at zero: whoever completes a count is the
// last user of that count and of the maximum beside it and clears both; a flag is cleared by
// the last of its group's members and its publisher to be done with it (one more count per
// group, taken off the critical path: its result is looked at when the workgroup's tiles are
// finished).  A caller whose words are known to be zero can therefore skip the clearing launch.
constexpr int kKeep = 4;
constexpr uint32_t kPollLimit = 1u << 15;
constexpr int kSyncGroups = 8;
constexpr int kSyncStride = 32;                                    // words: every word on a 128-byte line of its own
constexpr int kSyncWords = (4 * kSyncGroups + 2) * kSyncStride;    // group maxima, group counts, flags, flag users, global max, global count

__global__ void k_quant_sync_reset(uint32_t *sync)
{
    for (int i = threadIdx.x; i < kSyncWords; i += blockDim.x) sync[i] = 0;
}

__device__ __forceinline__ uint32_t relaxed_load(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// v if `after` has arrived (it always has a value below 2^31 here): ties the issue of the next
// atomic to the completion of the previous one without a fence
__device__ __forceinline__ uint32_t after_value(uint32_t v, uint32_t after) { return v + (after >> 31); }

template <bool ROW, bool COL, bool CEIL>
__global__ __launch_bounds__(kQuantThreads, 2) void k_quant_persist(const uint16_t *__restrict__ x, int64_t rows,
                                                                    int64_t cols, int64_t ld, int tiles_x, int n_tiles,
                                                                    uint32_t *sync, uint32_t poll_limit,
                                                                    uint8_t *__restrict__ q_row,
                                                                    uint8_t *__restrict__ e_row,
                                                                    uint8_t *__restrict__ q_col,
                                                                    uint8_t *__restrict__ e_col,
                                                                    float *__restrict__ s_global)
{
    __shared__ uint32_t red[kQuantThreads / kWave + 1];
    __shared__ TileLds lds;

    converter_saturates();
    if (threadIdx.x == 0) lds.redo = 0;      // (read only behind the barriers of the meeting point)
    const TileShape sh = {rows, cols, ld};
    const int G = (int)gridDim.x, first = (int)blockIdx.x;
    auto origin = [&](int t, int64_t &r0, int64_t &c0) {
        const int ty = t / tiles_x;
        r0 = (int64_t)ty * kTile;
        c0 = (int64_t)(t - ty * tiles_x) * kTile;
    };

    // a workgroup's (up to kKeep) tiles are neighbours in a tile row: up to 1 KiB of every row of X in one place
    const int per_group = (n_tiles + G - 1) / G;
    auto kept_tile = [&](int k) { return k < per_group ? first * per_group + k : n_tiles; };
    // walk 1: maximum of |x| over this workgroup's tiles
    uint4 keep[kKeep][8];
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < kKeep; k++) {
        const int t = kept_tile(k);
        if (t < n_tiles) {
            int64_t r0, c0;
            origin(t, r0, c0);
            load_tile(keep[k], x, sh, r0, c0);
        } else {
#pragma unroll
            for (int it = 0; it < 8; it++) keep[k][it] = make_uint4(0, 0, 0, 0);
        }
    }
#pragma unroll
    for (int k = 0; k < kKeep; k++) {
        const uint32_t c = tile_absmax(keep[k]);
        m = c > m ? c : m;
    }
    // meeting point
    uint32_t members = 0, my_use = 0;        // (thread 0's)
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kQuantThreads / kWave; i++) m = red[i] > m ? red[i] : m;
        uint32_t *grp_max = sync, *grp_cnt = sync + kSyncGroups * kSyncStride, *flags = sync + 2 * kSyncGroups * kSyncStride;
        uint32_t *users = sync + 3 * kSyncGroups * kSyncStride;
        uint32_t *all_max = sync + 4 * kSyncGroups * kSyncStride, *all_cnt = all_max + kSyncStride;
        const int grp = first % kSyncGroups, n_grp = G < kSyncGroups ? G : kSyncGroups;
        members = (uint32_t)((G - grp + kSyncGroups - 1) / kSyncGroups);
        uint32_t old = atomicMax(&grp_max[grp * kSyncStride], m);
        if (atomicAdd(&grp_cnt[grp * kSyncStride], after_value(1u, old)) == members - 1) {
            const uint32_t gm = atomicExch(&grp_max[grp * kSyncStride], 0u);    // the group's maximum; word and count left at zero
            __hip_atomic_store(&grp_cnt[grp * kSyncStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            old = atomicMax(all_max, gm);
            if (atomicAdd(all_cnt, after_value(1u, old)) == (uint32_t)n_grp - 1) {
                const uint32_t am = atomicExch(all_max, 0u);
                __hip_atomic_store(all_cnt, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                uint32_t was[kSyncGroups];
#pragma unroll
                for (int i = 0; i < kSyncGroups; i++)
                    if (i < n_grp) was[i] = atomicExch(&flags[i * kSyncStride], 0x80000000u | am);
                // the publisher is one more user of every flag: counted in once the flag is out
#pragma unroll
                for (int i = 0; i < kSyncGroups; i++)
                    if (i < n_grp && atomicAdd(&users[i * kSyncStride], after_value(1u, was[i])) == (uint32_t)((G - i + kSyncGroups - 1) / kSyncGroups)) {
                        __hip_atomic_store(&flags[i * kSyncStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        __hip_atomic_store(&users[i * kSyncStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
            }
        }
        uint32_t polls = 0, flag;
        while (true) {
            flag = relaxed_load(&flags[grp * kSyncStride]);
            if (flag != 0 || polls >= poll_limit) break;
            polls++;
            __builtin_amdgcn_s_sleep(8);
        }
        my_use = atomicAdd(&users[grp * kSyncStride], 1u);      // done with the flag, seen or not
        red[kQuantThreads / kWave] = flag;
    }
    __syncthreads();
    uint32_t amax_bits = red[kQuantThreads / kWave];
    if (amax_bits != 0) {
        amax_bits &= 0x7FFFu;
    } else {
        // the flag did not come in time: take the maximum over all of X here
        uint32_t mm = 0;
        for (int t = 0; t < n_tiles; t++) {
            uint4 ra[8];
            int64_t r0, c0;
            origin(t, r0, c0);
            load_tile(ra, x, sh, r0, c0);
            const uint32_t c = tile_absmax(ra);
            mm = c > mm ? c : mm;
        }
        mm = wave_max_u32(mm);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mm;
        __syncthreads();
        amax_bits = red[0];
        for (int i = 1; i < kQuantThreads / kWave; i++) amax_bits = red[i] > amax_bits ? red[i] : amax_bits;
    }
    const GlobalScale g = make_global_scale<CEIL>(amax_bits);
    if (first == 0 && threadIdx.x == 0) *s_global = g.s;

    // walk 2: codes and exponents from the registers, in the fast form
    uint32_t edge = 0;       // tiles that reach beyond X: left to the general form
#pragma unroll
    for (int k = 0; k < kKeep; k++) {
        const int t = kept_tile(k);
        if (t < n_tiles) {
            int64_t r0, c0;
            origin(t, r0, c0);
            if (tile_is_full(sh, r0, c0)) {
                if (quant_tile_body<ROW, COL, CEIL, true>(keep[k], sh, r0, c0, g, q_row, e_row, q_col, e_col, lds) &&
                    (threadIdx.x & 63) == 0)
                    atomicOr(&lds.redo, 1u << k);
                __syncthreads();
            } else {
                edge |= 1u << k;
            }
        }
    }
    // walk 3 (rare): the tiles the fast form does not cover, fetched again and done in the general form
    __syncthreads();
    const uint32_t again = lds.redo | edge;
#pragma unroll 1
    for (int k = 0; k < kKeep; k++) {
        if (!((again >> k) & 1u)) continue;
        int64_t r0, c0;
        origin(kept_tile(k), r0, c0);
        uint4 ra[8];
        load_tile(ra, x, sh, r0, c0);
        quant_tile_body<ROW, COL, CEIL, false>(ra, sh, r0, c0, g, q_row, e_row, q_col, e_col, lds);
        __syncthreads();
    }
    // the last of a flag's users (the group's members and the publisher) leaves flag and count at zero
    if (threadIdx.x == 0 && my_use == members) {
        const int grp = first % kSyncGroups;
        uint32_t *flags = sync + 2 * kSyncGroups * kSyncStride, *users = sync + 3 * kSyncGroups * kSyncStride;
        __hip_atomic_store(&flags[grp * kSyncStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&users[grp * kSyncStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

}  // namespace moss

namespace {

std::atomic<uint32_t> g_poll_limit{moss::kPollLimit};

using PersistFn = void (*)(const uint16_t *, int64_t, int64_t, int64_t, int, int, uint32_t *, uint32_t, uint8_t *, uint8_t *,
                           uint8_t *, uint8_t *, float *);

PersistFn persist_kernel(bool row, bool col, bool ceil_mode)
{
    using namespace moss;
    if (row && col) return ceil_mode ? k_quant_persist<true, true, true> : k_quant_persist<true, true, false>;
    if (col) return ceil_mode ? k_quant_persist<false, true, true> : k_quant_persist<false, true, false>;
    return ceil_mode ? k_quant_persist<true, false, true> : k_quant_persist<true, false, false>;
}

// Workgroups of the one-launch kernel that one compute unit holds at a time, at most 2 (0: do not use it).
int persist_groups_per_cu(PersistFn fn, int variant)
{
    // (a property of the kernel's register and LDS use on gfx950, the same on every device of the process)
    static std::atomic<int> cached[8] = {{-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}};
    int v = cached[variant].load();
    if (v < 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void *>(fn), moss::kQuantThreads, 0) !=
            hipSuccess) {
            (void)hipGetLastError();
            n = 0;
        }
        v = n > 2 ? 2 : n;
        cached[variant].store(v);
    }
    return v;
}

}  // namespace

extern "C" void moss_quant_set_poll_limit(unsigned polls) { g_poll_limit.store(polls); }

extern "C" size_t moss_quant_workspace_bytes(int64_t rows, int64_t cols, unsigned flags)
{
    (void)rows; (void)cols; (void)flags;
    return (size_t)(moss::kMaxPartials + moss::kSyncWords) * sizeof(uint32_t);
}

// The launch that converts: k_quant_row for the row grouping alone, k_quant_tile as soon as the transposed
// grouping is wanted.  `partial` holds n_partial candidate maxima (BF16 magnitude bits) that every workgroup folds.
static int launch_codes(const uint16_t *x, int64_t rows, int64_t cols, int64_t ld, bool want_row, bool want_col,
                        bool ceil_mode, const uint32_t *partial, int n_partial, uint8_t *q_row, uint8_t *e_row,
                        uint8_t *q_col, uint8_t *e_col, float *s_global, hipStream_t st)
{
    using namespace moss;
    const int chunks_per_row = (int)(cols / 8);
    const int64_t n_chunks = rows * chunks_per_row;
    const int dense = (ld == cols);
    if (want_row && !want_col) {
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
        const int64_t gx = (cols + kTile - 1) / kTile, gy = (rows + kTile - 1) / kTile;
        if (gx > (1 << 24) || gy > (1 << 24) || tile_grid_size(gx, gy) > 0x7FFFFFFF) return MOSS_ERR_SHAPE;
        const dim3 grid((unsigned)tile_grid_size(gx, gy)), block(kQuantThreads);
#define MOSS_LAUNCH_TILE(R, C)                                                                                          \
    hipLaunchKernelGGL((k_quant_tile<R, C>), grid, block, 0, st, x, rows, cols, ld, (int)gx, (int)gy, partial, n_partial,  \
                       q_row, e_row, q_col, e_col, s_global)
        if (want_row) { if (ceil_mode) MOSS_LAUNCH_TILE(true, true); else MOSS_LAUNCH_TILE(true, false); }
        else          { if (ceil_mode) MOSS_LAUNCH_TILE(false, true); else MOSS_LAUNCH_TILE(false, false); }
#undef MOSS_LAUNCH_TILE
        MOSS_LAUNCH_CHECK();
    }
    return MOSS_OK;
}

// What both quantizer entry points with a search for the maximum check before anything is launched
// (the workspace apart).
static int quant_check_args(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld, unsigned flags,
                            const uint8_t *q_row, const uint8_t *e_row, const uint8_t *q_col, const uint8_t *e_col,
                            const float *s_global)
{
    using namespace moss;
    const bool want_row = flags & MOSS_Q_ROW, want_col = flags & MOSS_Q_COL;
    if (flags & ~(MOSS_Q_ROW | MOSS_Q_COL | MOSS_EXP_CEIL | MOSS_WS_KEPT)) return MOSS_ERR_UNSUPPORTED;
    if (!want_row && !want_col) return MOSS_ERR_UNSUPPORTED;
    if (!x_bf16 || !s_global) return MOSS_ERR_NULL;
    if (want_row && (!q_row || !e_row)) return MOSS_ERR_NULL;
    if (want_col && (!q_col || !e_col)) return MOSS_ERR_NULL;
    if (rows <= 0 || cols <= 0 || cols % kGroup || ld < cols) return MOSS_ERR_SHAPE;
    if (want_col && rows % kGroup) return MOSS_ERR_SHAPE;
    if (rows * (cols / 8) >= ((int64_t)1 << 40)) return MOSS_ERR_SHAPE;
    if (ld >= ((int64_t)1 << 24) || (want_col && rows >= ((int64_t)1 << 24))) return MOSS_ERR_SHAPE;   // 32-bit offsets inside a tile
    if (ld % 8 || !moss_aligned16(x_bf16)) return MOSS_ERR_ALIGN;
    if (want_row && (!moss_aligned16(q_row) || ((uintptr_t)e_row & 3))) return MOSS_ERR_ALIGN;
    if (want_col && (!moss_aligned16(q_col) || ((uintptr_t)e_col & 3))) return MOSS_ERR_ALIGN;
    if ((uintptr_t)s_global & 3) return MOSS_ERR_ALIGN;
    return MOSS_OK;
}

// moss_quant_act_2level with its scratch (partial maxima, then the meeting words of the one-launch kernel) at
// `workspace`, wherever that memory comes from.  Arguments already checked.
static int quant_with_workspace(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld, unsigned flags,
                                uint8_t *q_row, uint8_t *e_row, uint8_t *q_col, uint8_t *e_col,
                                float *s_global, void *workspace, bool words_are_zero, void *stream)
{
    using namespace moss;
    const bool want_row = flags & MOSS_Q_ROW, want_col = flags & MOSS_Q_COL, ceil_mode = flags & MOSS_EXP_CEIL;

    hipStream_t st = (hipStream_t)stream;
    const uint16_t *x = (const uint16_t *)x_bf16;
    uint32_t *partial = (uint32_t *)workspace;
    const int chunks_per_row = (int)(cols / 8);
    const int64_t n_chunks = rows * chunks_per_row;
    const int dense = (ld == cols);

    // Tensors of one to kKeep tiles per workgroup: one launch that keeps X in registers between the
    // maximum and the codes.
    {
        const int64_t tiles_x = (cols + kTile - 1) / kTile, tiles_y = (rows + kTile - 1) / kTile;
        const int64_t n_tiles = tiles_x * tiles_y;
        const int variant = (want_row ? 1 : 0) | (want_col ? 2 : 0) | (ceil_mode ? 4 : 0);
        PersistFn fn = persist_kernel(want_row, want_col, ceil_mode);
        const int per_cu = persist_groups_per_cu(fn, variant);
        const int64_t grid = (int64_t)per_cu * moss_internal_cu_count();
        if (per_cu > 0 && n_tiles >= grid && n_tiles <= grid * kKeep) {
            uint32_t *sync = partial + kMaxPartials;
            if (!words_are_zero) {       // (the kernel leaves them at zero itself)
                hipLaunchKernelGGL(k_quant_sync_reset, dim3(1), dim3(kQuantThreads), 0, st, sync);
                MOSS_LAUNCH_CHECK();
            }
            hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(kQuantThreads), 0, st, x, rows, cols, ld, (int)tiles_x,
                               (int)n_tiles, sync, g_poll_limit.load(), q_row, e_row, q_col, e_col, s_global);
            MOSS_LAUNCH_CHECK();
            return MOSS_OK;
        }
    }

    int64_t want_blocks = (n_chunks + kQuantThreads * kAmaxUnroll - 1) / (kQuantThreads * kAmaxUnroll);
    const int n_partial = (int)(want_blocks < kMaxPartials ? want_blocks : kMaxPartials);
    hipLaunchKernelGGL(k_amax_bf16, dim3(n_partial), dim3(kQuantThreads), 0, st, x, n_chunks, chunks_per_row, ld, dense,
                       partial);
    MOSS_LAUNCH_CHECK();

    return launch_codes(x, rows, cols, ld, want_row, want_col, ceil_mode, partial, n_partial, q_row, e_row, q_col, e_col,
                        s_global, st);
}

extern "C" int moss_quant_act_2level(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld, unsigned flags,
                                     uint8_t *q_row, uint8_t *e_row, uint8_t *q_col, uint8_t *e_col,
                                     float *s_global, void *workspace, size_t workspace_bytes, void *stream)
{
    const int rc = quant_check_args(x_bf16, rows, cols, ld, flags, q_row, e_row, q_col, e_col, s_global);
    if (rc != MOSS_OK) return rc;
    if (!moss_aligned16(workspace)) return MOSS_ERR_ALIGN;
    if (!workspace || workspace_bytes < moss_quant_workspace_bytes(rows, cols, flags)) return MOSS_ERR_WORKSPACE;
    return quant_with_workspace(x_bf16, rows, cols, ld, flags, q_row, e_row, q_col, e_col, s_global, workspace,
                                (flags & MOSS_WS_KEPT) != 0, stream);
}

// ---------------------------------------------------------------------------------------------
// The entry point for callers that cannot allocate.  Its scratch is an array in the library's own
// device data segment: every GPU the library runs on holds a copy (16 KiB, until the process ends) at an
// address of its own, which the host learns once per device from hipGetSymbolAddress.  In host code the
// array's name is only a handle for that query, never an address to hand to a kernel.
namespace {

constexpr size_t kScratchBytes = 16 * 1024;
static __device__ __align__(256) uint8_t scratch[kScratchBytes];

std::atomic<void *> g_scratch_ptr[64];   // per device: where that device's copy of `scratch` lives

// Address of the current device's copy of the array (asked for on the first call on that device).
int scratch_of_current_device(void **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return MOSS_ERR_HIP;
    }
    void *p = g_scratch_ptr[dev].load();
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return MOSS_ERR_HIP;
        }
        g_scratch_ptr[dev].store(p);   // racing first calls store the same address
    }
    *out = p;
    return MOSS_OK;
}

}  // namespace

extern "C" int moss_quant_act_2level_noalloc(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld, unsigned flags,
                                             uint8_t *q_row, uint8_t *e_row, uint8_t *q_col, uint8_t *e_col,
                                             float *s_global, void *stream)
{
    int rc = quant_check_args(x_bf16, rows, cols, ld, flags, q_row, e_row, q_col, e_col, s_global);
    if (rc != MOSS_OK) return rc;
    // the scratch a shape needs must fit the array (today it does not grow with the shape, so this only
    // fails if the two ever drift apart)
    if (moss_quant_workspace_bytes(rows, cols, flags) > kScratchBytes) return MOSS_ERR_WORKSPACE;
    void *ws = nullptr;
    rc = scratch_of_current_device(&ws);
    if (rc != MOSS_OK) return rc;
    // The partial maxima are written before they are read.  The meeting words of the one-launch path have
    // to start at zero: the array is zero when the library is loaded, only this entry point writes to it,
    // and the one-launch kernel clears every word it used before it ends, so no clearing launch is needed.
    return quant_with_workspace(x_bf16, rows, cols, ld, flags, q_row, e_row, q_col, e_col, s_global, ws, true, stream);
}

extern "C" int moss_quant_act_2level_given_max(const void *x_bf16, int64_t rows, int64_t cols, int64_t ld, unsigned flags,
                                               const uint32_t *x_absmax_bits, uint8_t *q_row, uint8_t *e_row,
                                               uint8_t *q_col, uint8_t *e_col, float *s_global, void *stream)
{
    using namespace moss;
    const bool want_row = flags & MOSS_Q_ROW, want_col = flags & MOSS_Q_COL, ceil_mode = flags & MOSS_EXP_CEIL;
    if (flags & ~(MOSS_Q_ROW | MOSS_Q_COL | MOSS_EXP_CEIL)) return MOSS_ERR_UNSUPPORTED;
    if (!want_row && !want_col) return MOSS_ERR_UNSUPPORTED;
    if (!x_bf16 || !s_global || !x_absmax_bits) return MOSS_ERR_NULL;
    if (want_row && (!q_row || !e_row)) return MOSS_ERR_NULL;
    if (want_col && (!q_col || !e_col)) return MOSS_ERR_NULL;
    if (rows <= 0 || cols <= 0 || cols % kGroup || ld < cols) return MOSS_ERR_SHAPE;
    if (want_col && rows % kGroup) return MOSS_ERR_SHAPE;
    if (rows * (cols / 8) >= ((int64_t)1 << 40)) return MOSS_ERR_SHAPE;
    if (ld >= ((int64_t)1 << 24) || (want_col && rows >= ((int64_t)1 << 24))) return MOSS_ERR_SHAPE;   // 32-bit offsets inside a tile
    if (ld % 8 || !moss_aligned16(x_bf16)) return MOSS_ERR_ALIGN;
    if (want_row && (!moss_aligned16(q_row) || ((uintptr_t)e_row & 3))) return MOSS_ERR_ALIGN;
    if (want_col && (!moss_aligned16(q_col) || ((uintptr_t)e_col & 3))) return MOSS_ERR_ALIGN;
    if (((uintptr_t)s_global & 3) || ((uintptr_t)x_absmax_bits & 3)) return MOSS_ERR_ALIGN;
    // the producer's word takes the place of the partial maxima: one candidate, nothing to search
    return launch_codes((const uint16_t *)x_bf16, rows, cols, ld, want_row, want_col, ceil_mode, x_absmax_bits, 1, q_row,
                        e_row, q_col, e_col, s_global, (hipStream_t)stream);
}
