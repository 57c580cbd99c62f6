// Internal helpers shared by the HIP translation units of libmoss_hip.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moss.h"

#define MOSS_HIP_TRY(expr)                       \
    do {                                         \
        if ((expr) != hipSuccess) {              \
            (void)hipGetLastError();             \
            return MOSS_ERR_HIP;                 \
        }                                        \
    } while (0)

#define MOSS_LAUNCH_CHECK()                      \
    do {                                         \
        if (hipGetLastError() != hipSuccess) return MOSS_ERR_HIP; \
    } while (0)

static inline bool moss_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int moss_internal_cu_count();

// 256 x 256 tile fast path of the block-scaled GEMM; MOSS_ERR_UNSUPPORTED if the shape or
// operands do not qualify (the caller falls back to the general kernel).
int moss_internal_gemm_big(int64_t M, int64_t N, int64_t K, const uint8_t *a_q, const uint8_t *a_e, const float *a_s,
                           const uint8_t *b_q, const uint8_t *b_e, const float *b_s, void *out, int out_f32,
                           int64_t ld_out, int accumulate, hipStream_t st);

namespace moss {

constexpr int kWave = 64;
constexpr int kGroup = 32;          // level-2 group size k2 (paper Sec. 3.1)
constexpr float kE4M3Max = 448.0f;  // Delta_max of E4M3 (paper Sec. 3.1)

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// Two FP32 values -> two E4M3 bytes in the low half of the result.  The hardware
// converter rounds to nearest even; values are clamped to +-448 first so that the
// cast saturates instead of producing the NaN code.
__device__ __forceinline__ uint32_t cvt2_e4m3_sat(float a, float b)
{
    a = __builtin_amdgcn_fmed3f(a, kE4M3Max, -kE4M3Max);
    b = __builtin_amdgcn_fmed3f(b, kE4M3Max, -kE4M3Max);
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false) & 0xFFFFu;
}

// Four FP32 values -> four E4M3 bytes (a in the lowest byte).
__device__ __forceinline__ uint32_t cvt4_e4m3_sat(float a, float b, float c, float d)
{
    a = __builtin_amdgcn_fmed3f(a, kE4M3Max, -kE4M3Max);
    b = __builtin_amdgcn_fmed3f(b, kE4M3Max, -kE4M3Max);
    c = __builtin_amdgcn_fmed3f(c, kE4M3Max, -kE4M3Max);
    d = __builtin_amdgcn_fmed3f(d, kE4M3Max, -kE4M3Max);
    int r = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, r, true);
    return (uint32_t)r;
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

__device__ __forceinline__ float wave_max_f32(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

}  // namespace moss
