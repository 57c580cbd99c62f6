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

// Streaming ("nontemporal") global accesses for data that is touched once per kernel: they
// do not allocate in the last-level cache, so a stream does not have to evict the dirty
// lines earlier kernels left there.  Measured on a cold 64-256 MB read: 5.1-6.5 TB/s against
// 2.7-3.0 TB/s with ordinary loads.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 ld_stream16(const void *p)
{
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint2 ld_stream8(const void *p)
{
    const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(p));
    return make_uint2(t.x, t.y);
}
__device__ __forceinline__ float4 ld_stream_f4(const void *p)
{
    const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void st_stream16(void *p, uint4 v)
{
    __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4 *>(p));
}
__device__ __forceinline__ void st_stream8(void *p, uint2 v)
{
    __builtin_nontemporal_store(u32x2{v.x, v.y}, reinterpret_cast<u32x2 *>(p));
}
__device__ __forceinline__ void st_stream4(void *p, uint32_t v) { __builtin_nontemporal_store(v, reinterpret_cast<uint32_t *>(p)); }
__device__ __forceinline__ void st_stream_f4(void *p, float4 v)
{
    __builtin_nontemporal_store(f32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4 *>(p));
}

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
