// Large-tile block-scaled FP8 GEMM for gfx950: the fast path of moss_gemm_fp8_mx
// (paper Sec. 3.1, Fig. 3b: only matrix-core instructions in the main loop, level-2
// exponents applied by the instruction, FP32 scales once in the epilogue).
//
// Shape of the kernel
//  * 256 x 256 output tile per workgroup of 4 waves (2 x 2), 128 x 128 per wave held as
//    4 x 4 accumulators of V_MFMA_SCALE_F32_32X32X64_F8F6F4 (256 accumulator registers).
//  * K advances in stages of 64 bytes.  A ring of four LDS stages (32 KiB each: 256 rows
//    of a and 256 rows of b) is filled by direct global->LDS loads that never touch
//    registers, issued three stages ahead of the stage being multiplied.
//  * Fragments are double buffered in registers: while the 16 matrix instructions of
//    stage t run, the fragments of stage t+1 are read from LDS.
//  * One barrier per stage.  Before it each wave waits until all of its loads except the
//    ones issued during this stage have landed (s_waitcnt vmcnt), so after the barrier
//    stages <= t+2 are visible to every wave.
//  * E8M0 scale bytes travel the same way: one dword (4 groups = 128 K) per row and
//    stage pair, copied to a small LDS ring and read back as one register per fragment.
//
// Operand layout of the instruction (measured with one-hot operands): lane (r = lane%32,
// h = lane/32) supplies for row r the bytes K[16h, 16h+16) in its first four source
// registers and K[32+16h, 32+16h+16) in the last four; K block B (32 wide) of row r is
// scaled by the selected byte of lane r+32B's scale register.
//
// LDS stage layout: row r = 64 bytes = four 16-byte chunks, chunk c stored at slot
// c ^ ((r >> 2) & 3): the 16 rows a quarter-wave reads with one 16-byte access then hit
// 16 different 16-byte bank groups, and a wave-wide global->LDS load still writes 1 KiB
// of consecutive LDS (16 rows) while each lane fetches the chunk that belongs there.
#include "moss_internal.h"

namespace moss {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kBT = 256;                     // tile edge (rows of a and rows of b per workgroup)
constexpr int kStageK = 64;                  // bytes of K per stage
constexpr int kStages = 4;
constexpr int kStageBytes = 2 * kBT * kStageK;        // a then b: 32 KiB
constexpr int kScaleSlotBytes = 2 * kBT * 4;          // a then b: one dword per row
constexpr int kScaleSlots = 4;
constexpr int kScaleBase = kStages * kStageBytes;     // 128 KiB
constexpr int kBigLdsBytes = kScaleBase + kScaleSlots * kScaleSlotBytes;   // 136 KiB

extern __shared__ __attribute__((aligned(1024))) uint8_t big_smem[];

// wave-wide direct global->LDS copy: every lane moves 16 bytes from base + off to
// lds_addr + 16 * lane (lds_addr is wave-uniform and goes through M0)
__device__ __forceinline__ void dma16(const uint8_t *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(off), "s"(base), "s"(lds_addr) : "memory");
}
__device__ __forceinline__ void dma4(const uint8_t *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dword %0, %1"
                 :: "v"(off), "s"(base), "s"(lds_addr) : "memory");
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

__device__ __forceinline__ void stage_barrier()
{
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

struct Frags {
    v8i a[4], b[4];
};

template <bool HAS_BE>
__global__ __launch_bounds__(256, 1) void k_gemm_mx_big(int64_t M, int64_t N, int64_t K,
                                                        const uint8_t *__restrict__ a_q, const uint8_t *__restrict__ a_e,
                                                        const float *__restrict__ a_s,
                                                        const uint8_t *__restrict__ b_q, const uint8_t *__restrict__ b_e,
                                                        const float *__restrict__ b_s,
                                                        void *__restrict__ out, int out_f32, int64_t ld_out, int accumulate,
                                                        int tiles_m, int tiles_n)
{
    constexpr int NSC = HAS_BE ? 2 : 1;   // scale copies per stage pair and wave
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int i32 = lane & 31, h = lane >> 5;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)big_smem;

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): give every XCD a
    // contiguous range of tiles, walked in bands of 4 tile rows so that the 32 tiles an XCD
    // works on at a time form a compact 4 x 8 block sharing a and b rows in that L2.
    const int total = tiles_m * tiles_n;
    int pid = blockIdx.x;
    {
        const int per = (total + 7) >> 3, xcd = pid & 7, idx = pid >> 3;
        const int full = total - (per - 1) * 8;          // XCDs that own `per` tiles (others per-1)
        int start = xcd < full ? xcd * per : full * per + (xcd - full) * (per - 1);
        if (total % 8 == 0) start = xcd * per;
        pid = start + idx;
    }
    constexpr int GM = 4;
    const int band = pid / (GM * tiles_n), rem = pid % (GM * tiles_n);
    const int band_rows = (tiles_m - band * GM) < GM ? (tiles_m - band * GM) : GM;
    // (the divisions run on the vector unit: tell the compiler the results are wave-uniform so
    // that everything derived from them lives in scalar registers)
    const int tm = __builtin_amdgcn_readfirstlane(band * GM + rem % band_rows);
    const int tn = __builtin_amdgcn_readfirstlane(rem / band_rows);
    const int64_t m0 = (int64_t)tm * kBT, n0 = (int64_t)tn * kBT;

    // ---- global -> LDS copy plan: per stage a wave copies 64 rows of a and 64 rows of b in
    // four + four wave-wide 16-byte copies of 16 rows each
    const int G = (int)(K >> 5);
    uint32_t a_off[4], b_off[4];
#pragma unroll
    for (int s = 0; s < 4; s++) {
        const int r = wave * 64 + s * 16 + (lane >> 2);
        const int c = (lane & 3) ^ ((r >> 2) & 3);
        int64_t ra = m0 + r, rb = n0 + r;
        ra = (ra < M ? ra : M - 1) - m0;
        rb = (rb < N ? rb : N - 1) - n0;
        a_off[s] = (uint32_t)(ra * K + c * 16);
        b_off[s] = (uint32_t)(rb * K + c * 16);
    }
    uint32_t ae_off, be_off;
    {
        const int r = wave * 64 + lane;
        int64_t ra = m0 + r, rb = n0 + r;
        ra = (ra < M ? ra : M - 1) - m0;
        rb = (rb < N ? rb : N - 1) - n0;
        ae_off = (uint32_t)(ra * G);
        be_off = (uint32_t)(rb * G);
    }
    const uint8_t *a_base = a_q + m0 * K, *b_base = b_q + n0 * K;
    const uint8_t *ae_base = a_e + m0 * G, *be_base = HAS_BE ? b_e + n0 * G : nullptr;

    auto issue_stage = [&](int u) {   // u = stage index (wave-uniform)
        const uint32_t slot = lds0 + (uint32_t)(u & (kStages - 1)) * kStageBytes + (uint32_t)wave * 64 * kStageK;
        const uint8_t *ab = a_base + (int64_t)u * kStageK, *bb = b_base + (int64_t)u * kStageK;
#pragma unroll
        for (int s = 0; s < 4; s++) dma16(ab, a_off[s], slot + s * 16 * kStageK);
#pragma unroll
        for (int s = 0; s < 4; s++) dma16(bb, b_off[s], slot + kBT * kStageK + s * 16 * kStageK);
    };
    auto issue_scales = [&](int p) {  // p = stage-pair index: groups 4p .. 4p+3 of every row
        const uint32_t slot = lds0 + kScaleBase + (uint32_t)(p & (kScaleSlots - 1)) * kScaleSlotBytes + (uint32_t)wave * 256;
        dma4(ae_base + (int64_t)p * 4, ae_off, slot);
        if (HAS_BE) dma4(be_base + (int64_t)p * 4, be_off, slot + kBT * 4);
    };

    // ---- LDS -> register fragment plan
    const int gi = (i32 >> 2) & 3;
    const int rd_lo = i32 * kStageK + ((h ^ gi) << 4);
    const int rd_hi = i32 * kStageK + (((2 + h) ^ gi) << 4);
    auto read_frags = [&](Frags &f, int u) {
        const uint8_t *sa = big_smem + (u & (kStages - 1)) * kStageBytes + wm * 128 * kStageK;
        const uint8_t *sb = big_smem + (u & (kStages - 1)) * kStageBytes + kBT * kStageK + wn * 128 * kStageK;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            uint4 lo = *reinterpret_cast<const uint4 *>(sa + i * 32 * kStageK + rd_lo);
            uint4 hi = *reinterpret_cast<const uint4 *>(sa + i * 32 * kStageK + rd_hi);
            f.a[i] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        }
#pragma unroll
        for (int j = 0; j < 4; j++) {
            uint4 lo = *reinterpret_cast<const uint4 *>(sb + j * 32 * kStageK + rd_lo);
            uint4 hi = *reinterpret_cast<const uint4 *>(sb + j * 32 * kStageK + rd_hi);
            f.b[j] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        }
    };
    // scale registers of a stage pair: byte 0 / byte 2 = this lane's group in the first /
    // second stage of the pair (lanes of the upper half shift their dword down by one byte)
    auto read_scales = [&](int (&sa)[4], int (&sb)[4], int p) {
        const uint8_t *base = big_smem + kScaleBase + (p & (kScaleSlots - 1)) * kScaleSlotBytes;
#pragma unroll
        for (int i = 0; i < 4; i++)
            sa[i] = (int)(*reinterpret_cast<const uint32_t *>(base + (wm * 128 + i * 32 + i32) * 4) >> (8 * h));
#pragma unroll
        for (int j = 0; j < 4; j++)
            sb[j] = HAS_BE ? (int)(*reinterpret_cast<const uint32_t *>(base + kBT * 4 + (wn * 128 + j * 32 + i32) * 4) >> (8 * h))
                           : 0x7F7F7F7F;
    };

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

    const int T = (int)(K / kStageK);   // even and >= 8 (host checks K % 128 == 0, K >= 512)

    // prologue: stages 0, 1, 2 and the scales of pairs 0, 1 in flight
    issue_scales(0);
    issue_stage(0);
    issue_stage(1);
    issue_scales(1);
    issue_stage(2);
    wait_vmcnt<8 + NSC>();            // everything but pair 1's scales and stage 2 has landed
    stage_barrier();

    Frags fe, fo;                     // fragments of the even / odd stage
    int sa_cur[4], sb_cur[4], sa_nxt[4], sb_nxt[4];
    read_frags(fe, 0);
    read_scales(sa_cur, sb_cur, 0);

#define MOSS_MFMA_STAGE(F, OPSEL)                                                                           \
    _Pragma("unroll") for (int i = 0; i < 4; i++) _Pragma("unroll") for (int j = 0; j < 4; j++)            \
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(F.b[j], F.a[i], acc[i][j], 0, 0, OPSEL, \
                                                                    sb_cur[j], OPSEL, sa_cur[i]);

    // steady state: iteration t issues stage t+3, reads the fragments of stage t+1 and
    // multiplies stage t
    int t = 0;
    for (; t + 4 < T; t += 2) {
        issue_stage(t + 3);
        read_frags(fo, t + 1);
        MOSS_MFMA_STAGE(fe, 0)
        wait_vmcnt<8>();              // stage t+2 (and older) landed; stage t+3 may be in flight
        stage_barrier();

        issue_scales((t + 4) >> 1);
        issue_stage(t + 4);
        read_frags(fe, t + 2);
        read_scales(sa_nxt, sb_nxt, (t + 2) >> 1);
        MOSS_MFMA_STAGE(fo, 2)
        wait_vmcnt<8 + NSC>();        // stage t+3 landed
        stage_barrier();
#pragma unroll
        for (int i = 0; i < 4; i++) { sa_cur[i] = sa_nxt[i]; sb_cur[i] = sb_nxt[i]; }
    }
    // t == T-4: last stage to issue is T-1
    issue_stage(t + 3);
    read_frags(fo, t + 1);
    MOSS_MFMA_STAGE(fe, 0)
    wait_vmcnt<8>();
    stage_barrier();
    read_frags(fe, t + 2);
    read_scales(sa_nxt, sb_nxt, (t + 2) >> 1);
    MOSS_MFMA_STAGE(fo, 2)
    wait_vmcnt<0>();
    stage_barrier();
#pragma unroll
    for (int i = 0; i < 4; i++) { sa_cur[i] = sa_nxt[i]; sb_cur[i] = sb_nxt[i]; }
    // t == T-2: nothing left to issue
    read_frags(fo, t + 3);
    MOSS_MFMA_STAGE(fe, 0)
    MOSS_MFMA_STAGE(fo, 2)
#undef MOSS_MFMA_STAGE

    // ---- epilogue: one multiply by s_a * s_b, then the store.  Accumulator register v of
    // lane (i32, h) in fragment (i, j) is out[m, n] with m = .. + i32 and
    // n = .. + 8 (v / 4) + 4 h + v % 4: four consecutive n per register quad.
    const float scale = (*a_s) * (*b_s);
    const bool vec_ok = (ld_out % 4 == 0);
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int64_t m = m0 + wm * 128 + i * 32 + i32;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; j++) {
#pragma unroll
            for (int qd = 0; qd < 4; qd++) {
                const int64_t n = n0 + wn * 128 + j * 32 + qd * 8 + 4 * h;
                if (n >= N) continue;
                const float r0 = acc[i][j][4 * qd] * scale, r1 = acc[i][j][4 * qd + 1] * scale;
                const float r2 = acc[i][j][4 * qd + 2] * scale, r3 = acc[i][j][4 * qd + 3] * scale;
                if (out_f32) {
                    float *o = reinterpret_cast<float *>(out) + m * ld_out + n;
                    if (vec_ok && n + 3 < N) {
                        float4 v = make_float4(r0, r1, r2, r3);
                        if (accumulate) {
                            const float4 p = *reinterpret_cast<const float4 *>(o);
                            v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
                        }
                        *reinterpret_cast<float4 *>(o) = v;
                    } else {
                        const float r[4] = {r0, r1, r2, r3};
                        for (int e = 0; e < 4 && n + e < N; e++) o[e] = accumulate ? o[e] + r[e] : r[e];
                    }
                } else {
                    uint16_t *o = reinterpret_cast<uint16_t *>(out) + m * ld_out + n;
                    if (vec_ok && n + 3 < N) {
                        *reinterpret_cast<uint2 *>(o) = make_uint2(bf16_rne(r0) | (bf16_rne(r1) << 16),
                                                                   bf16_rne(r2) | (bf16_rne(r3) << 16));
                    } else {
                        const float r[4] = {r0, r1, r2, r3};
                        for (int e = 0; e < 4 && n + e < N; e++) o[e] = (uint16_t)bf16_rne(r[e]);
                    }
                }
            }
        }
    }
}

}  // namespace moss

// Returns MOSS_ERR_UNSUPPORTED when the shape does not fit the fast path (the caller then
// uses the general kernel).
int moss_internal_gemm_big(int64_t M, int64_t N, int64_t K, const uint8_t *a_q, const uint8_t *a_e, const float *a_s,
                           const uint8_t *b_q, const uint8_t *b_e, const float *b_s, void *out, int out_f32,
                           int64_t ld_out, int accumulate, hipStream_t st)
{
    using namespace moss;
    if (!a_e || K % 128 || K < 512 || K > (1 << 22)) return MOSS_ERR_UNSUPPORTED;
    if ((int64_t)kBT * K >= ((int64_t)1 << 32)) return MOSS_ERR_UNSUPPORTED;
    const int64_t tiles_m = (M + kBT - 1) / kBT, tiles_n = (N + kBT - 1) / kBT;
    if (tiles_m * tiles_n > 0x7FFFFFF) return MOSS_ERR_UNSUPPORTED;
    static bool attr_set[2] = {false, false};
    const int which = b_e ? 1 : 0;
    if (!attr_set[which]) {
        hipError_t e = b_e ? hipFuncSetAttribute((const void *)k_gemm_mx_big<true>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsBytes)
                           : hipFuncSetAttribute((const void *)k_gemm_mx_big<false>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsBytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return MOSS_ERR_UNSUPPORTED;
        }
        attr_set[which] = true;
    }
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
    if (b_e)
        hipLaunchKernelGGL(k_gemm_mx_big<true>, grid, block, kBigLdsBytes, st, M, N, K, a_q, a_e, a_s, b_q, b_e, b_s, out,
                           out_f32, ld_out, accumulate, (int)tiles_m, (int)tiles_n);
    else
        hipLaunchKernelGGL(k_gemm_mx_big<false>, grid, block, kBigLdsBytes, st, M, N, K, a_q, a_e, a_s, b_q, b_e, b_s, out,
                           out_f32, ld_out, accumulate, (int)tiles_m, (int)tiles_n);
    if (hipGetLastError() != hipSuccess) return MOSS_ERR_HIP;
    return MOSS_OK;
}
