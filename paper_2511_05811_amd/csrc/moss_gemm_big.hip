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
//    of K = 64; fragments are double buffered in registers: substep 1's are read from LDS
//    behind the 16 matrix instructions of substep 0, one 16-byte read each, the next stage's
//    first ones behind the second half of substep 1's (see the barriers below).
//  * The loads of stage P+2 are issued during substep 1 of stage P (their slot is free from
//    then on), one copy after each matrix instruction, and have to land by the middle of
//    substep 1 of stage P+1: two to three substeps (1024 matrix-core cycles each) of latency
//    hiding with 64 KiB in flight.
//  * Two barriers per stage.  The first, at the end of substep 0, only says that every wave
//    has read the stage's last fragments, so the slot may be refilled.  The second sits in the
//    middle of substep 1: before it every wave waits for its own copies of stage P+1, behind it
//    the first fragments of stage P+1 are read, two 16-byte reads per matrix instruction.
//    (With a single barrier at the end of substep 0 that also waited for the copies, they had
//    one to two substeps; an L2 miss takes longer, and inside a training step, where every
//    GEMM starts on cold operands, the later wait is worth 5 % of the GEMM time.)
//  * E8M0 scale bytes travel the same way in blocks of 16 bytes (16 groups = K 512) per
//    row into a small LDS ring; a lane reads one dword per fragment and stage and the
//    instruction's byte selector picks the group of the substep.
//  * Epilogue: accumulators times s_a*s_b are staged through the wave's own part of the last
//    stage slot (16-byte chunks XOR-swizzled by row) so that every global store instruction
//    writes whole 256-byte row pieces.
//  * Persistent workgroups, one per compute unit; the first two stages of a workgroup's next
//    tile are already in flight while it writes out the current one.
//  * A second instantiation with half the rows of a (128 x 256 tile, 64 x 128 per wave) serves
//    problems with too few full tiles for the machine.
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
#include <atomic>
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
constexpr int kDummyBase = kScaleBase + 2 * kScaleSlotBytes;     // 144 KiB: 1 KiB per wave that nobody reads
constexpr int kBigLdsBytes = kDummyBase + 4 * 1024;              // 148 KiB

extern __shared__ __attribute__((aligned(1024))) uint8_t big_smem[];

// wave-wide direct global->LDS copy: every lane moves 16 bytes from base + off to
// lds_addr + 16 * lane (lds_addr is wave-uniform and goes through M0)
__device__ __forceinline__ void dma16(const uint8_t *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(off), "s"(base), "s"(lds_addr) : "memory", "m0");
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

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// two FP32 -> two BF16 (round to nearest even), a in the low half: one V_CVT_PK_BF16_F32
__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

struct Frags {
    v8i a[4], b[4];
};

// The block-scaled matrix instruction as volatile inline assembly: volatile asm statements keep
// their program order, which is what pins "one matrix instruction, one LDS read, one global->LDS
// copy" in the main loop (compiler scheduling hints did not survive: all 16 matrix instructions
// of a substep were emitted first and the memory instructions after them in one burst).
// SEL = 0 / 2 picks scale byte 0 / 2 of both scale registers.  Independent accumulators back to
// back need no wait states; the places where results are consumed add their own (see callers).
template <int SEL>
__device__ __forceinline__ void mfma_scaled(v16f &acc, const v8i &x, const v8i &y, int sx, int sy)
{
    if (SEL == 0)
        asm volatile("v_mfma_scale_f32_32x32x64_f8f6f4 %0, %1, %2, %0, %3, %4 op_sel_hi:[0,0,0]"
                     : "+a"(acc) : "v"(x), "v"(y), "v"(sx), "v"(sy));
    else
        asm volatile("v_mfma_scale_f32_32x32x64_f8f6f4 %0, %1, %2, %0, %3, %4 op_sel_hi:[1,1,0]"
                     : "+a"(acc) : "v"(x), "v"(y), "v"(sx), "v"(sy));
}
__device__ __forceinline__ void pin() { asm volatile("" ::: "memory"); }

// What a wave needs to know about one output tile: wave-uniform bases (scalar registers) and
// its lanes' byte offsets for the global->LDS copies.
struct TileCtx {
    int64_t m0, n0;
    const uint8_t *a_base, *b_base, *ae_base, *be_base;
    uint32_t a_off[8], b_off[8], ae_off, be_off;
};

// MI = 32-row fragments of a per wave: 4 gives the 256 x 256 tile described above, 2 a 128 x 256
// tile (64 x 128 per wave, half the accumulators) for problems with too few full tiles to fill
// the machine.  The narrower tile reads 1.5 times the LDS bytes per matrix instruction.
template <bool HAS_BE, int MI>
__global__ __launch_bounds__(256, 1) void k_gemm_mx_big(int64_t M, int64_t N, int64_t K,
                                                        const uint8_t *__restrict__ a_q, const uint8_t *__restrict__ a_e,
                                                        const float *__restrict__ a_s,
                                                        const uint8_t *__restrict__ b_q, const uint8_t *__restrict__ b_e,
                                                        const float *__restrict__ b_s,
                                                        void *__restrict__ out, int out_f32, int64_t ld_out, int accumulate,
                                                        int tiles_m, int tiles_n)
{
    constexpr int kMT = MI * 64;             // rows of a per tile
    constexpr int kRowsA = kMT / 4;          // rows of a a wave copies per stage (64 or 32), in kPiecesA pieces of 8
    constexpr int kPiecesA = kRowsA / 8;
    constexpr int kPiecesD = kPiecesA + 8;   // copies per stage and wave (a, then b)
    constexpr int kNM = MI * 4;              // matrix instructions per substep
    constexpr int kPiecesR = 2 * MI + 8;     // 16-byte fragment reads per substep (a fragments, then b fragments)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int i32 = lane & 31, h = lane >> 5;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)big_smem;
    const int G = (int)(K >> 5);
    const int T = (int)(K / kStageK);   // stages per tile, >= 4 (host checks K % 128 == 0, K >= 512)
    const int NB = (T + 3) >> 2;        // scale blocks per tile
    const int total = tiles_m * tiles_n;
    const int n_my_tiles = (total - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;

    // The k-th tile of this (persistent) workgroup.  Workgroups are dealt round-robin to the 8
    // XCDs (each with its own L2) and gridDim.x is a multiple of 8 whenever a workgroup has more
    // than one tile, so tile number blockIdx.x + k gridDim.x stays on this XCD.  Every XCD gets a
    // contiguous range of tiles, walked in bands of 4 tile rows: the 32 tiles an XCD works on at a
    // time form a compact 4 x 8 block sharing a and b rows in that L2.
    auto make_ctx = [&](int k, TileCtx &c) {
        int pid = (int)blockIdx.x + k * (int)gridDim.x;
        {
            const int q = total >> 3, r = total & 7, xcd = pid & 7, idx = pid >> 3;
            pid = (xcd < r ? xcd * (q + 1) : r * (q + 1) + (xcd - r) * q) + idx;
        }
        constexpr int GM = 4;
        const int band = pid / (GM * tiles_n), rem = pid % (GM * tiles_n);
        const int band_rows = (tiles_m - band * GM) < GM ? (tiles_m - band * GM) : GM;
        // (the divisions run on the vector unit: tell the compiler the results are wave-uniform
        // so that everything derived from them lives in scalar registers)
        const int tm = __builtin_amdgcn_readfirstlane(band * GM + rem % band_rows);
        const int tn = __builtin_amdgcn_readfirstlane(rem / band_rows);
        c.m0 = (int64_t)tm * kMT;
        c.n0 = (int64_t)tn * kBT;
        // per stage a wave copies kRowsA rows of a and 64 rows of b in wave-wide copies of 8 full rows
        // (8 x 128 B = 1 KiB of LDS) each; rows beyond the matrix repeat the last row.  In LDS a wave's
        // rows of a start at row 64 wave whatever kRowsA is (the swizzle only looks at the low row bits).
#pragma unroll
        for (int s = 0; s < 8; s++) {
            const int r = wave * 64 + s * 8 + (lane >> 3);
            const int ch = (lane & 7) ^ ((r >> 1) & 7);
            int64_t ra = c.m0 + wave * kRowsA + s * 8 + (lane >> 3), rb = c.n0 + r;
            ra = (ra < M ? ra : M - 1) - c.m0;
            rb = (rb < N ? rb : N - 1) - c.n0;
            c.a_off[s] = (uint32_t)(ra * K + ch * 16);
            c.b_off[s] = (uint32_t)(rb * K + ch * 16);
        }
        {   // scale copies: lane = row, 16 of that row's exponent bytes
            const int r = wave * 64 + lane;
            int64_t ra = c.m0 + r, rb = c.n0 + r;
            ra = (ra < M ? ra : M - 1) - c.m0;
            rb = (rb < N ? rb : N - 1) - c.n0;
            c.ae_off = (uint32_t)(ra * G);
            c.be_off = (uint32_t)(rb * G);
        }
        c.a_base = a_q + c.m0 * K;
        c.b_base = b_q + c.n0 * K;
        c.ae_base = a_e + c.m0 * G;
        c.be_base = HAS_BE ? b_e + c.n0 * G : nullptr;
    };

    // all copies of stage P of tile c into the stage slot `par`: first the 8-row pieces of a, then the eight of b
    auto issue_stage = [&](const TileCtx &c, int P, int par) {
        const uint32_t slot = lds0 + (uint32_t)par * kSlotBytes + (uint32_t)wave * 64 * kStageK;
#pragma unroll
        for (int idx = 0; idx < kPiecesA; idx++) dma16(c.a_base + (int64_t)P * kStageK, c.a_off[idx], slot + idx * 8 * kStageK);
#pragma unroll
        for (int idx = 0; idx < 8; idx++) dma16(c.b_base + (int64_t)P * kStageK, c.b_off[idx], slot + kBT * kStageK + idx * 8 * kStageK);
    };
    // First exponent byte of scale block blk: blocks are 16 groups wide; the last one is
    // shifted back so that its 16-byte copy ends exactly at the end of the row.
    auto scale_block_start = [&](int blk) { const int st = blk * 16; return st + 16 <= G ? st : G - 16; };
    auto issue_scales = [&](const TileCtx &c, int blk, int spar) {
        const uint32_t slot = lds0 + kScaleBase + (uint32_t)spar * kScaleSlotBytes + (uint32_t)wave * 64 * 16;
        const int st = scale_block_start(blk);
        dma16(c.ae_base + st, c.ae_off, slot);
        if (HAS_BE) dma16(c.be_base + st, c.be_off, slot + kBT * 16);
    };

    // ---- LDS -> register fragment plan (substep s of a stage = chunks 4s .. 4s+3 of a row)
    const int sw = (i32 >> 1) & 7;
    // piece idx (0 .. kPiecesR-1) of the fragments of substep s of the stage in slot `par`: fragment
    // idx/2 (first the MI of a, then the 4 of b), low or high four registers
    auto read_piece = [&](Frags &f, int par, int s, int idx) {
        const int fr = idx >> 1, half = idx & 1;
        const int ra = wm * (kMT / 2) + fr * 32;                       // first tile row of the a fragment
        const uint8_t *base = big_smem + par * kSlotBytes +
                              (fr < MI ? ((ra / kRowsA) * 64 + ra % kRowsA + i32) * kStageK
                                       : kBT * kStageK + (wn * 128 + (fr - MI) * 32 + i32) * kStageK);
        const uint4 v = *reinterpret_cast<const uint4 *>(base + (((4 * s + 2 * half + h) ^ sw) << 4));
        v8i &dst = fr < MI ? f.a[fr] : f.b[fr - MI];
        dst[4 * half + 0] = (int)v.x; dst[4 * half + 1] = (int)v.y; dst[4 * half + 2] = (int)v.z; dst[4 * half + 3] = (int)v.w;
    };
    // LDS byte offset (from the scale area) of the dword that holds the four exponent bytes of stage P, for a
    // tile whose scale block 0 sits in scale slot parity sp0
    auto scale_dword_offset = [&](int P, int sp0) {
        const int blk = P >> 2;
        return (uint32_t)(((sp0 + blk) & 1) * kScaleSlotBytes + 4 * P - scale_block_start(blk));
    };
    // raw scale dwords of the stage at that offset
    auto read_scales = [&](int (&sa)[MI], int (&sb)[4], uint32_t off) {
        const uint8_t *base = big_smem + kScaleBase + off;
#pragma unroll
        for (int i = 0; i < MI; i++) sa[i] = (int)*reinterpret_cast<const uint32_t *>(base + (wm * (kMT / 2) + i * 32 + i32) * 16);
#pragma unroll
        for (int j = 0; j < 4; j++)
            sb[j] = HAS_BE ? (int)*reinterpret_cast<const uint32_t *>(base + kBT * 16 + (wn * 128 + j * 32 + i32) * 16)
                           : 0x7F7F7F7F;
    };
    // byte 0 / byte 2 of a scale register = this lane's group in substep 0 / 1: lanes of the
    // upper half shift their dword down by one byte.  There is one register set per substep, and
    // each is rewritten in the middle of the other substep, when the matrix instructions that
    // read it have long retired and its next readers are eight instructions away: rewriting
    // registers that matrix instructions in flight still name cost ~190 cycles per stage.  (The
    // shifts are volatile asm so that they stay where they are put.)
    const int sh8 = 8 * h;
    auto shift_scales = [&](int (&dst_a)[MI], int (&dst_b)[4], const int (&sa)[MI], const int (&sb)[4]) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            if (i < MI) asm volatile("v_lshrrev_b32 %0, %1, %2" : "=v"(dst_a[i]) : "v"(sh8), "v"(sa[i]));
            asm volatile("v_lshrrev_b32 %0, %1, %2" : "=v"(dst_b[i]) : "v"(sh8), "v"(sb[i]));
        }
    };

    v16f acc[MI][4];
    Frags fe, fo;                     // fragments of substep 0 / substep 1
    int sa0[MI], sb0[4], sa1[MI], sb1[4], sa_raw[MI], sb_raw[4];   // scales of substep 0 / substep 1, raw dwords

    TileCtx cx;
    make_ctx(0, cx);
    // prologue: scale block 0, stages 0 and 1 of the first tile in flight
    issue_scales(cx, 0, 0);
    issue_stage(cx, 0, 0);
    issue_stage(cx, 1, 1);

    const float scale = (*a_s) * (*b_s);

    for (int ti = 0; ti < n_my_tiles; ti++) {
        const bool has_next = ti + 1 < n_my_tiles;
        const int g0 = ti * T, sp0 = (ti * NB) & 1;      // global stage / scale block numbers of this tile's first
        // Stage 0 and scale block 0 of this tile were issued two stages ago (or by the prologue),
        // stage 1 just now: wait for all but the latter, then fetch the first fragments.
        wait_vmcnt<kPiecesD>();
        wait_lds_and_barrier();
#pragma unroll
        for (int idx = 0; idx < kPiecesR; idx++) read_piece(fe, g0 & 1, 0, idx);
        read_scales(sa_raw, sb_raw, scale_dword_offset(0, sp0));
        shift_scales(sa0, sb0, sa_raw, sb_raw);
        asm volatile("s_nop 4" ::: "memory");    // vector ALU write -> scale operand of a matrix instruction
#pragma unroll
        for (int i = 0; i < MI; i++)
#pragma unroll
            for (int j = 0; j < 4; j++)
#pragma unroll
                for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

        // The stages of this tile.  There is exactly one copy of a stage's matrix instructions in the
        // kernel (everything optional around them hangs on wave-uniform flags), so the accumulator
        // registers never have to move.  The instruction order is pinned by the volatile asm statements
        // and the compiler barriers between them: in substep 0 each matrix instruction is followed by one
        // (narrow tile: one or two) 16-byte LDS read of substep 1's fragments, in substep 1 by the global->LDS
        // copies of the stage after next and, in its second half, by the reads of the next stage's first fragments.  With one wave per SIMD a burst of memory
        // instructions would block this wave's issue -- and so the matrix pipe -- until the LDS /
        // texture queues had taken them all.
        const int64_t m0 = cx.m0, n0 = cx.n0;
        for (int P = 0; P < T; P++) {
            const int par = (g0 + P) & 1;            // this stage's slot; the next stage sits in par ^ 1
            // Everything the middle of the stage and substep 1 need to know is worked out in the shadow of
            // the first matrix instructions of substep 0 (the empty asm statements fence the scalar code in
            // between them: with one wave per SIMD whatever runs between two substeps leaves the matrix
            // pipe idle):
            //   next  : there is a stage P+1 in this tile (the epilogue, not this loop, hands over to the next tile)
            //   own   : slot `par` is refilled with stage P+2 of this tile
            //   issue : ... or with stage 0 of the next tile; when there is nothing to refill (the last stage, and
            //           the one before it for the last tile) the copies still run, aimed at stage T-1 again and at
            //           an LDS area nobody reads, which keeps the loop free of branches
            int fl = 0, iP = 0, Pl = 0;
            uint32_t sc_off = 0, dst_a = 0, dst_b = 0, dstep = 0;
            const uint8_t *a_src = nullptr, *b_src = nullptr;
            // substep 0: multiply K[0,64) while fetching the fragments of K[64,128)
#pragma unroll
            for (int idx = 0; idx < kNM; idx++) {
                const int i = idx >> 2, j = idx & 3;
                mfma_scaled<0>(acc[i][j], fe.b[j], fe.a[i], sb0[j], sa0[i]);
#pragma unroll
                for (int p = idx * kPiecesR / kNM; p < (idx + 1) * kPiecesR / kNM; p++) read_piece(fo, par, 1, p);
                // (a chain of fenced pieces, one behind each of the first matrix instructions)
                if (idx == 0) {
                    Pl = P;
                    asm volatile("" : "+s"(Pl));
                    const bool own = Pl + 2 < T, issue = own || (Pl + 2 == T && has_next);
                    iP = own ? Pl + 2 : (issue ? 0 : T - 1);
                    fl = T - Pl < 3 ? T - Pl : 3;                      // stages left in this tile, capped: 1, 2 or 3
                }
                if (idx == 1) {
                    asm volatile("" : "+s"(fl), "+s"(iP), "+s"(Pl));
                    sc_off = scale_dword_offset(Pl + 1, sp0);
                }
                if (idx == 2) {
                    asm volatile("" : "+s"(sc_off), "+s"(iP));
                    a_src = cx.a_base + (int64_t)iP * kStageK;
                    b_src = cx.b_base + (int64_t)iP * kStageK;
                }
                if (idx == 3) {
                    asm volatile("" : "+s"(a_src), "+s"(b_src), "+s"(fl));
                    const bool issue = fl == 3 || (fl == 2 && has_next);
                    const uint32_t slot = lds0 + (uint32_t)par * kSlotBytes + (uint32_t)wave * 64 * kStageK;
                    const uint32_t dummy = lds0 + kDummyBase + (uint32_t)wave * 1024;
                    dst_a = issue ? slot : dummy;
                    dst_b = issue ? slot + kBT * kStageK : dummy;
                    dstep = issue ? 8 * kStageK : 0;
                }
                if (idx == 4) asm volatile("" : "+s"(dst_a), "+s"(dst_b), "+s"(dstep));
                if (idx == kNM / 2) shift_scales(sa1, sb1, sa_raw, sb_raw);     // this stage's scales for substep 1
                pin();
            }
            const bool next = fl >= 2, own = fl == 3, issue = own || (next && has_next);
            if (next) wait_lds_and_barrier();    // everyone is done reading this stage's slot: it may be refilled
            if (issue && !own) {                 // from here on cx describes the next tile
                make_ctx(ti + 1, cx);
                a_src = cx.a_base;
                b_src = cx.b_base;
            }
            // substep 1: multiply K[64,128) and refill the slot.  Stage P+1 is only waited for in the middle of
            // the substep (its copies have had a stage and a quarter by then); the first fragments of stage
            // P+1 are fetched behind that second barrier, two reads per matrix instruction.
            pin();
            uint32_t cur = dst_a;
            constexpr int kBB = kNM / 2;                         // the matrix instruction the second barrier follows
            constexpr int kBefore = kBB * kPiecesD / kNM;        // copies of this substep issued before it
#pragma unroll
            for (int idx = 0; idx < kNM; idx++) {
                const int i = idx >> 2, j = idx & 3;
                mfma_scaled<2>(acc[i][j], fo.b[j], fo.a[i], sb1[j], sa1[i]);
                if (idx == kBB && next) {
                    wait_vmcnt<kBefore>();    // this wave's part of stage P+1 (and its scales) has landed
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                    read_scales(sa_raw, sb_raw, sc_off);
                }
                if (idx >= kBB) {
#pragma unroll
                    for (int p = (idx - kBB) * kPiecesR / (kNM - kBB); p < (idx - kBB + 1) * kPiecesR / (kNM - kBB); p++)
                        read_piece(fe, par ^ 1, 0, p);     // (after the last stage: read and never used)
                }
#pragma unroll
                for (int p = idx * kPiecesD / kNM; p < (idx + 1) * kPiecesD / kNM; p++) {
                    if (p == kPiecesA) cur = dst_b;
                    if (p < kPiecesA) dma16(a_src, cx.a_off[p], cur);
                    else dma16(b_src, cx.b_off[p - kPiecesA], cur);
                    cur += dstep;
                }
                if (idx == kBB + (kNM - kBB) / 2 && next) shift_scales(sa0, sb0, sa_raw, sb_raw);   // the next stage's, for its substep 0
            }
            // the next scale block, behind this substep's copies (the wait above counts back from the newest copy)
            if (issue && (iP & 3) == 0) issue_scales(cx, iP >> 2, own ? (sp0 + (iP >> 2)) & 1 : (sp0 + NB) & 1);
        }
        // (stage 1 of the next tile belongs into the last stage's slot, which the epilogue uses first:
        // it is issued after the epilogue)
        asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");   // let the last matrix instructions retire

        // ---- epilogue.  Accumulator register v of lane (i32, h) in fragment (i, j) is out[m, n] with
        // m = .. + 32 i + i32 and n = .. + 32 j + 8 (v / 4) + 4 h + v % 4.  Scale, convert, and stage
        // 16 KiB at a time through the two 8 KiB pieces of the last stage's slot that this wave itself
        // fills by copies (rows 64 wave .. of the a and of the b half), then store whole 256-byte row
        // pieces.  Inside a 256-byte staged row the 16-byte chunk c sits at c ^ (row & 15).
        wait_lds_and_barrier();   // every wave is done reading the last stage's fragments
        const int epar = (g0 + T - 1) & 1;
        uint8_t *pieceA = big_smem + epar * kSlotBytes + wave * 64 * kStageK;
        uint8_t *pieceB = pieceA + kBT * kStageK;
        const int64_t mw = m0 + wm * (kMT / 2), nw = n0 + wn * 128;
        if (!out_f32) {
            uint16_t *o = reinterpret_cast<uint16_t *>(out);
#pragma unroll
            for (int rnd = 0; rnd < MI / 2; rnd++) {
#pragma unroll
                for (int ii = 0; ii < 2; ii++) {
                    const int i = 2 * rnd + ii;
                    uint8_t *pc = (ii ? pieceB : pieceA) + i32 * 256 + 8 * h;
#pragma unroll
                    for (int j = 0; j < 4; j++)
#pragma unroll
                        for (int qd = 0; qd < 4; qd++) {
                            const uint32_t lo = pack_bf16(acc[i][j][4 * qd] * scale, acc[i][j][4 * qd + 1] * scale);
                            const uint32_t hi = pack_bf16(acc[i][j][4 * qd + 2] * scale, acc[i][j][4 * qd + 3] * scale);
                            *reinterpret_cast<uint2 *>(pc + (((j * 4 + qd) ^ (i32 & 15)) << 4)) = make_uint2(lo, hi);
                        }
                }
                // 16 lanes cover one 256-byte row piece (128 BF16), a wave instruction covers 4 rows
                const int cc = lane & 15;
#pragma unroll 4
                for (int k = 0; k < 16; k++) {
                    const int rl = 4 * k + (lane >> 4), ii = rl >> 5, rr = rl & 31;
                    const uint4 v = *reinterpret_cast<const uint4 *>((ii ? pieceB : pieceA) + rr * 256 + ((cc ^ (rr & 15)) << 4));
                    const int64_t m = mw + (2 * rnd + ii) * 32 + rr, n = nw + cc * 8;
                    // (N % 8 == 0 and ld_out % 8 == 0 on this path: a piece is inside or outside as a whole)
                    // (streaming store: a BF16 output is an activation or gradient for a later layer, and leaving
                    // it out of the last-level cache keeps the operands of the GEMMs in flight there)
                    if (m < M && n < N) st_stream16(o + m * ld_out + n, v);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // staged rows consumed before they are overwritten
            }
        } else {
            float *o = reinterpret_cast<float *>(out);
#pragma unroll
            for (int i = 0; i < MI; i++) {      // one 32-row block per round: 32 rows x 512 B, halves in the two pieces
#pragma unroll
                for (int j = 0; j < 4; j++)
#pragma unroll
                    for (int qd = 0; qd < 4; qd++)
                        *reinterpret_cast<float4 *>(((j >> 1) ? pieceB : pieceA) + i32 * 256 +
                                                    ((((j & 1) * 8 + qd * 2 + h) ^ (i32 & 15)) << 4)) =
                            make_float4(acc[i][j][4 * qd] * scale, acc[i][j][4 * qd + 1] * scale,
                                        acc[i][j][4 * qd + 2] * scale, acc[i][j][4 * qd + 3] * scale);
                // 32 lanes cover one 512-byte row (128 floats), a wave instruction covers 2 rows
                const int l32 = lane & 31, cc = l32 & 15;
#pragma unroll 4
                for (int k = 0; k < 16; k++) {
                    const int rr = 2 * k + (lane >> 5);
                    float4 v = *reinterpret_cast<const float4 *>(((l32 >> 4) ? pieceB : pieceA) + rr * 256 + ((cc ^ (rr & 15)) << 4));
                    const int64_t m = mw + i * 32 + rr, n = nw + l32 * 4;
                    if (m >= M || n >= N) continue;
                    float *dst = o + m * ld_out + n;
                    if (accumulate) {
                        const float4 p = *reinterpret_cast<const float4 *>(dst);
                        v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
                    }
                    *reinterpret_cast<float4 *>(dst) = v;
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
        }
        // the pieces are free again: fill them with this wave's part of stage 1 of the next tile
        if (has_next) issue_stage(cx, 1, epar);
    }
    wait_vmcnt<0>();   // no copy into LDS may be outstanding when the wave ends
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
    if (N % 8 || ld_out % 8) return MOSS_ERR_UNSUPPORTED;      // the epilogue stores whole 16-byte pieces
    if ((int64_t)kBT * K >= ((int64_t)1 << 32)) return MOSS_ERR_UNSUPPORTED;
    int cus = moss_internal_cu_count();
    cus = cus >= 8 ? cus & ~7 : 8;
    // 256 x 256 tiles when they fill the machine, else 128 x 256 (twice the tiles, each at a somewhat
    // lower rate).  Time in units of one full tile on all compute units: rounds of full tiles, or rounds
    // of half tiles at 0.78 each (a half tile takes 0.76 of the time of a full one: 67 us against 88 us
    // for M = 4096, N = 2048, K = 7168), so the narrow tile pays only where it saves whole rounds.
    const int64_t tiles_n = (N + kBT - 1) / kBT;
    const int64_t full = ((M + kBT - 1) / kBT) * tiles_n, half = ((M + kBT / 2 - 1) / (kBT / 2)) * tiles_n;
    const double t_full = (double)((full + cus - 1) / cus), t_half = 0.78 * (double)((half + cus - 1) / cus);
    const bool narrow = t_half < t_full;
    const int64_t tiles_m = narrow ? (M + kBT / 2 - 1) / (kBT / 2) : (M + kBT - 1) / kBT;
    if (tiles_m * tiles_n > 0x7FFFFFF) return MOSS_ERR_UNSUPPORTED;
    using Kern = void (*)(int64_t, int64_t, int64_t, const uint8_t *, const uint8_t *, const float *, const uint8_t *,
                          const uint8_t *, const float *, void *, int, int64_t, int, int, int);
    static const Kern kerns[4] = {k_gemm_mx_big<false, 4>, k_gemm_mx_big<true, 4>, k_gemm_mx_big<false, 2>,
                                  k_gemm_mx_big<true, 2>};
    static std::atomic<bool> attr_done[64][4];   // the LDS size attribute is set once per device and kernel (setting it
                                                 // twice from racing threads is harmless: same value)
    const int which = (b_e ? 1 : 0) | (narrow ? 2 : 0);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MOSS_ERR_HIP;
    std::atomic<bool>(&attr_set)[4] = attr_done[dev];
    if (!attr_set[which].load()) {
        if (hipFuncSetAttribute((const void *)kerns[which], hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsBytes) !=
            hipSuccess) {
            (void)hipGetLastError();
            return MOSS_ERR_UNSUPPORTED;
        }
        attr_set[which].store(true);
    }
    // persistent workgroups: one per compute unit (rounded down to a multiple of 8 so that the tiles
    // of a workgroup stay on one XCD), or one per tile if there are fewer tiles
    const int64_t total = tiles_m * tiles_n;
    // No more workgroups than the rounds need: 1376 tiles take 6 rounds on 256 compute units and on 232
    // alike, and under the power limit the idle units' share goes into the clock of the busy ones.
    const int64_t rounds = (total + cus - 1) / cus;
    int64_t wgs = (total + rounds - 1) / rounds;
    wgs = (wgs + 7) & ~(int64_t)7;
    if (wgs > cus) wgs = cus;
    const dim3 grid((unsigned)(total < cus ? total : wgs)), block(256);
    hipLaunchKernelGGL(kerns[which], grid, block, kBigLdsBytes, st, M, N, K, a_q, a_e, a_s, b_q, b_e, b_s, out, out_f32,
                       ld_out, accumulate, (int)tiles_m, (int)tiles_n);
    if (hipGetLastError() != hipSuccess) return MOSS_ERR_HIP;
    return MOSS_OK;
}
