// Large-tile block-scaled FP8 GEMM for gfx950: the fast path of moss_gemm_fp8_mx
// (paper Sec. 3.1, Fig. 3b: only matrix-core instructions in the main loop, level-2
// exponents applied by the instruction, FP32 scales once in the epilogue).
//
// Shape of the kernel
//  * 256 x 256 output tile per workgroup of 4 waves (2 x 2), 128 x 128 per wave held as
//    4 x 4 accumulators of V_MFMA_SCALE_F32_32X32X64_F8F6F4 (256 accumulator registers).
//  * K advances in stages of 128 bytes = one full 128-byte cache line per tile row.  (The
//    texture path costs about the same per line touched whether 64 or 128 bytes of it are
//    used: 64-byte rows cap the feed rate near 27 B/clk/CU, full lines reach ~62, and the
//    kernel needs 32 B/clk/CU at full matrix-core rate.)
//  * Two LDS stage slots of 64 KiB (256 rows of a, 256 rows of b) filled by direct
//    global->LDS loads that never touch registers.  A stage is multiplied in two substeps
//    of K = 64; fragments are double buffered in registers, so the fragments of the next
//    substep are read from LDS while the 16 matrix instructions of the current one run.
//  * The loads of stage P+2 are issued during substep 1 of stage P (their slot is free from
//    then on), one copy after each matrix instruction, and have to land by the end of
//    substep 0 of stage P+1: one to two substeps (1024 matrix-core cycles each) of latency
//    hiding with 64 KiB in flight.
//  * One barrier per stage, at the end of substep 0; before it every wave waits for its
//    own outstanding loads (stage P+1) and LDS reads.
//  * E8M0 scale bytes travel the same way in blocks of 16 bytes (16 groups = K 512) per
//    row into a small LDS ring; a lane reads one dword per fragment and stage and the
//    instruction's byte selector picks the group of the substep.
//  * Epilogue: accumulators times s_a*s_b are staged through LDS (row stride padded by 16
//    bytes) so that every global store instruction writes whole 256-byte row pieces.
//
// Operand layout of the instruction (measured with one-hot operands): lane (r = lane%32,
// h = lane/32) supplies for row r the bytes K[16h, 16h+16) in its first four source
// registers and K[32+16h, 32+16h+16) in the last four; K block B (32 wide) of row r is
// scaled by the selected byte of lane r+32B's scale register.
//
// LDS stage layout: row r = 128 bytes = eight 16-byte chunks, chunk c stored at slot
// c ^ ((r >> 1) & 7): the 16 rows a quarter-wave reads with one 16-byte access then hit
// 16 different 16-byte bank groups, and a wave-wide global->LDS load still writes 1 KiB
// of consecutive LDS (8 rows) while each lane fetches the chunk that belongs there.
#include <type_traits>

#include "moss_internal.h"

namespace moss {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kBT = 256;                     // tile edge (rows of a and rows of b per workgroup)
constexpr int kStageK = 128;                 // bytes of K per stage (one cache line per row)
constexpr int kSlotBytes = 2 * kBT * kStageK;          // a then b: 64 KiB
constexpr int kScaleSlotBytes = 2 * kBT * 16;          // a then b, 16 exponent bytes (K 512) per row: 8 KiB
constexpr int kScaleBase = 2 * kSlotBytes;             // 128 KiB
constexpr int kBigLdsBytes = kScaleBase + 2 * kScaleSlotBytes;   // 144 KiB
constexpr int kEpiRowBytes = 256 + 16;       // 128 BF16 (or 64 FP32) of one row + padding (keeps 16-byte alignment)
constexpr int kEpiWaveBytes = 128 * kEpiRowBytes;      // 34 KiB per wave, 136 KiB in all
static_assert(4 * kEpiWaveBytes <= kBigLdsBytes, "epilogue staging must fit");

extern __shared__ __attribute__((aligned(1024))) uint8_t big_smem[];

// wave-wide direct global->LDS copy: every lane moves 16 bytes from base + off to
// lds_addr + 16 * lane (lds_addr is wave-uniform and goes through M0)
__device__ __forceinline__ void dma16(const uint8_t *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(off), "s"(base), "s"(lds_addr) : "memory");
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

__device__ __forceinline__ void wait_lds_and_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
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
        const int q = total >> 3, r = total & 7, xcd = pid & 7, idx = pid >> 3;
        pid = (xcd < r ? xcd * (q + 1) : r * (q + 1) + (xcd - r) * q) + idx;
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
    // eight + eight wave-wide copies of 8 full rows (8 x 128 B = 1 KiB of LDS) each
    const int G = (int)(K >> 5);
    uint32_t a_off[8], b_off[8];
#pragma unroll
    for (int s = 0; s < 8; s++) {
        const int r = wave * 64 + s * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        int64_t ra = m0 + r, rb = n0 + r;
        ra = (ra < M ? ra : M - 1) - m0;
        rb = (rb < N ? rb : N - 1) - n0;
        a_off[s] = (uint32_t)(ra * K + c * 16);
        b_off[s] = (uint32_t)(rb * K + c * 16);
    }
    uint32_t ae_off, be_off;   // scale copies: lane = row, 16 bytes of that row's exponent bytes
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

    // copy number idx (0..15) of stage P: 0..7 = 8-row pieces of a, 8..15 = of b
    auto issue_piece = [&](int P, int idx) {
        const uint32_t slot = lds0 + (uint32_t)(P & 1) * kSlotBytes + (uint32_t)wave * 64 * kStageK;
        if (idx < 8) dma16(a_base + (int64_t)P * kStageK, a_off[idx], slot + idx * 8 * kStageK);
        else dma16(b_base + (int64_t)P * kStageK, b_off[idx - 8], slot + kBT * kStageK + (idx - 8) * 8 * kStageK);
    };
    auto issue_stage = [&](int P) {   // P = stage index (wave-uniform)
#pragma unroll
        for (int idx = 0; idx < 16; idx++) issue_piece(P, idx);
    };
    // First exponent byte of scale block blk: blocks are 16 groups wide; the last one is
    // shifted back so that its 16-byte copy ends exactly at the end of the row.
    auto scale_block_start = [&](int blk) { const int st = blk * 16; return st + 16 <= G ? st : G - 16; };
    auto issue_scales = [&](int blk) {
        const uint32_t slot = lds0 + kScaleBase + (uint32_t)(blk & 1) * kScaleSlotBytes + (uint32_t)wave * 64 * 16;
        const int st = scale_block_start(blk);
        dma16(ae_base + st, ae_off, slot);
        if (HAS_BE) dma16(be_base + st, be_off, slot + kBT * 16);
    };

    // ---- LDS -> register fragment plan (substep s of a stage = chunks 4s .. 4s+3 of a row)
    const int sw = (i32 >> 1) & 7;
    auto read_frags = [&](Frags &f, int P, int s) {
        const uint8_t *sa = big_smem + (P & 1) * kSlotBytes + (wm * 128 + i32) * kStageK;
        const uint8_t *sb = big_smem + (P & 1) * kSlotBytes + kBT * kStageK + (wn * 128 + i32) * kStageK;
        const int lo_off = ((4 * s + h) ^ sw) << 4, hi_off = ((4 * s + 2 + h) ^ sw) << 4;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            uint4 lo = *reinterpret_cast<const uint4 *>(sa + i * 32 * kStageK + lo_off);
            uint4 hi = *reinterpret_cast<const uint4 *>(sa + i * 32 * kStageK + hi_off);
            f.a[i] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        }
#pragma unroll
        for (int j = 0; j < 4; j++) {
            uint4 lo = *reinterpret_cast<const uint4 *>(sb + j * 32 * kStageK + lo_off);
            uint4 hi = *reinterpret_cast<const uint4 *>(sb + j * 32 * kStageK + hi_off);
            f.b[j] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        }
    };
    // scale registers of stage P: byte 0 / byte 2 = this lane's group in substep 0 / 1 (lanes
    // of the upper half shift their dword down by one byte, see shift_scales)
    auto read_scales = [&](int (&sa)[4], int (&sb)[4], int P) {
        const int blk = P >> 2;
        const int dw = (4 * P - scale_block_start(blk));          // byte offset of the stage's dword
        const uint8_t *base = big_smem + kScaleBase + (blk & 1) * kScaleSlotBytes + dw;
#pragma unroll
        for (int i = 0; i < 4; i++) sa[i] = (int)*reinterpret_cast<const uint32_t *>(base + (wm * 128 + i * 32 + i32) * 16);
#pragma unroll
        for (int j = 0; j < 4; j++)
            sb[j] = HAS_BE ? (int)*reinterpret_cast<const uint32_t *>(base + kBT * 16 + (wn * 128 + j * 32 + i32) * 16)
                           : 0x7F7F7F7F;
    };
    auto shift_scales = [&](int (&dst_a)[4], int (&dst_b)[4], const int (&sa)[4], const int (&sb)[4]) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            dst_a[i] = (int)((uint32_t)sa[i] >> (8 * h));
            dst_b[i] = (int)((uint32_t)sb[i] >> (8 * h));
        }
    };

    v16f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

    const int T = (int)(K / kStageK);   // >= 4 (host checks K % 128 == 0, K >= 512)

    // prologue: scale block 0, stages 0 and 1 in flight; wait for all but stage 1
    issue_scales(0);
    issue_stage(0);
    issue_stage(1);
    wait_vmcnt<16>();
    wait_lds_and_barrier();

    Frags fe, fo;                     // fragments of substep 0 / substep 1
    int sa_cur[4], sb_cur[4], sa_raw[4], sb_raw[4];
    read_frags(fe, 0, 0);
    read_scales(sa_raw, sb_raw, 0);
    shift_scales(sa_cur, sb_cur, sa_raw, sb_raw);

#define MOSS_MFMA_SUBSTEP(F, OPSEL)                                                                         \
    __builtin_amdgcn_sched_barrier(0);                                                                      \
    _Pragma("unroll") for (int i = 0; i < 4; i++) _Pragma("unroll") for (int j = 0; j < 4; j++)            \
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(F.b[j], F.a[i], acc[i][j], 0, 0, OPSEL, \
                                                                    sb_cur[j], OPSEL, sa_cur[i]);           \
    __builtin_amdgcn_sched_barrier(0);

    // One stage.  The order inside a substep is pinned (scheduling barriers): first the LDS
    // reads for the next substep, then the 16 matrix instructions of the current one, so that
    // the reads complete under the matrix work.  NEXT: a stage P+1 exists; ISSUE: so does P+2.
    auto stage = [&](int P, auto next_tag, auto issue_tag) {
        constexpr bool NEXT = decltype(next_tag)::value, ISSUE = decltype(issue_tag)::value;
        // substep 0: multiply K[0,64) of stage P while fetching the fragments of K[64,128)
        read_frags(fo, P, 1);
        MOSS_MFMA_SUBSTEP(fe, 0)
        if constexpr (NEXT) {
            wait_vmcnt<0>();          // this wave's part of stage P+1 (and its scales) has landed
            wait_lds_and_barrier();   // ... and everyone is done reading stage P's slot
            // substep 1: fetch the first fragments of stage P+1 and refill the freed slot with
            // stage P+2.  The 16 copies are spread between the 16 matrix instructions: issued in
            // one burst they would block this wave's instruction stream (and with it the matrix
            // pipe) until the texture path has taken them all.
            if constexpr (ISSUE) {
                if (((P + 2) & 3) == 0) issue_scales((P + 2) >> 2);
            }
            read_frags(fe, P + 1, 0);
            read_scales(sa_raw, sb_raw, P + 1);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int idx = 0; idx < 16; idx++) {
            const int i = idx >> 2, j = idx & 3;
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fo.b[j], fo.a[i], acc[i][j], 0, 0, 2, sb_cur[j], 2,
                                                                        sa_cur[i]);
            if constexpr (ISSUE) issue_piece(P + 2, idx);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (NEXT) shift_scales(sa_cur, sb_cur, sa_raw, sb_raw);
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    int P = 0;
    for (; P + 2 < T; P++) stage(P, yes{}, yes{});
    stage(P, yes{}, no{});
    stage(P + 1, no{}, no{});
#undef MOSS_MFMA_SUBSTEP

    // ---- epilogue.  Accumulator register v of lane (i32, h) in fragment (i, j) is out[m, n]
    // with m = .. + 32 i + i32 and n = .. + 32 j + 8 (v / 4) + 4 h + v % 4.  Scale, convert, stage
    // the wave's 128 x 128 block through its private LDS region and store whole row pieces.
    const float scale = (*a_s) * (*b_s);
    wait_lds_and_barrier();           // all fragment reads are done: LDS can be reused
    uint8_t *stg = big_smem + wave * kEpiWaveBytes;
    const int64_t mw = m0 + wm * 128, nw = n0 + wn * 128;
    const bool vec_ok = (ld_out % 8 == 0);
    if (!out_f32) {
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 4; j++)
#pragma unroll
                for (int qd = 0; qd < 4; qd++) {
                    const uint32_t lo = bf16_rne(acc[i][j][4 * qd] * scale) | (bf16_rne(acc[i][j][4 * qd + 1] * scale) << 16);
                    const uint32_t hi = bf16_rne(acc[i][j][4 * qd + 2] * scale) | (bf16_rne(acc[i][j][4 * qd + 3] * scale) << 16);
                    *reinterpret_cast<uint2 *>(stg + (i * 32 + i32) * kEpiRowBytes + (j * 32 + qd * 8 + 4 * h) * 2) = make_uint2(lo, hi);
                }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        // 16 lanes cover one 256-byte row piece, a wave instruction covers 4 rows
        uint16_t *o = reinterpret_cast<uint16_t *>(out);
        const int rr = lane >> 4, cc = (lane & 15) * 8;
#pragma unroll 4
        for (int it = 0; it < 32; it++) {
            const int row = it * 4 + rr;
            const int64_t m = mw + row, n = nw + cc;
            if (m >= M || n >= N) continue;
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + row * kEpiRowBytes + cc * 2);
            uint16_t *dst = o + m * ld_out + n;
            if (vec_ok && n + 7 < N) {
                *reinterpret_cast<uint4 *>(dst) = v;
            } else {
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
                for (int e = 0; e < 8 && n + e < N; e++) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
            }
        }
    } else {
        // FP32 output: two passes of 64 columns (a 256-byte row piece is 64 floats)
        float *o = reinterpret_cast<float *>(out);
        const int rr = lane >> 4, cc = (lane & 15) * 4;
#pragma unroll
        for (int half = 0; half < 2; half++) {
            if (half) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int jj = 0; jj < 2; jj++)
#pragma unroll
                    for (int qd = 0; qd < 4; qd++) {
                        const int j = half * 2 + jj;
                        *reinterpret_cast<float4 *>(stg + (i * 32 + i32) * kEpiRowBytes + (jj * 32 + qd * 8 + 4 * h) * 4) =
                            make_float4(acc[i][j][4 * qd] * scale, acc[i][j][4 * qd + 1] * scale,
                                        acc[i][j][4 * qd + 2] * scale, acc[i][j][4 * qd + 3] * scale);
                    }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll 4
            for (int it = 0; it < 32; it++) {
                const int row = it * 4 + rr;
                const int64_t m = mw + row, n = nw + half * 64 + cc;
                if (m >= M || n >= N) continue;
                float4 v = *reinterpret_cast<const float4 *>(stg + row * kEpiRowBytes + cc * 4);
                float *dst = o + m * ld_out + n;
                if (vec_ok && n + 3 < N) {
                    if (accumulate) {
                        const float4 p = *reinterpret_cast<const float4 *>(dst);
                        v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
                    }
                    *reinterpret_cast<float4 *>(dst) = v;
                } else {
                    const float r[4] = {v.x, v.y, v.z, v.w};
                    for (int e = 0; e < 4 && n + e < N; e++) dst[e] = accumulate ? dst[e] + r[e] : r[e];
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
