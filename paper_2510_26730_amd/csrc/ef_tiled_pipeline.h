// The LDS operand pipeline of the matrix-core bound kernels (tiled expert FFN halves, Gram tiles of the
// token distances): a workgroup of four waves owns a 256 x 256 output tile, a wave 128 x 128 (4 x 4 MFMA
// 32x32x16 accumulators); both operands arrive as 1 KiB operand fragments (32 rows x 16 k), eight of each
// per k-step, through kTileStages LDS stage buffers filled by direct global -> LDS loads kTileStages - 1 stages ahead of
// the one that feeds the matrix cores, one barrier per stage.
//
// The macros below are written against names the using kernel defines: lds (the stage buffers), src (per
// thread source of its 8 fragment quarters per stage), acc[4][4], wave, lane, nstage, AOFF, BOFF, lds_base,
// kSwapOperands and HALF.
#pragma once
#include "ef_device.h"

namespace ef {

constexpr int kTileKS = 2;               // MFMA k-steps (16 columns each) per LDS stage
constexpr int kStageFrags = 16 * kTileKS;  // fragments per stage: per k-step 8 of each operand
constexpr int kTileStages = 4;           // LDS stage buffers (five, all of a compute unit's LDS, measured 1-3 % slower)
// s_waitcnt immediate "vmcnt <= n, do not wait on expcnt / lgkmcnt" (gfx9 encoding: vmcnt[3:0] in bits
// 3:0 and vmcnt[5:4] in bits 15:14, expcnt in 6:4, lgkmcnt in 11:8)
constexpr int tiled_wait_vm(int n) { return ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8) | (n & 15); }
static_assert(kStageFrags / 4 == 8, "the wait counts assume 8 loads per wave per stage");
// prologue: kTileStages - 1 stages are issued; the first has landed when at most the others' loads are outstanding
constexpr int kWaitVmFirst = tiled_wait_vm(8 * (kTileStages - 2));
// main loop, before the barrier of stage st: stage st+1 has landed when at most the loads of the stages issued
// after it (st+2 .. st+kTileStages-2 and half of stage st+kTileStages-1) are outstanding
constexpr int kWaitVmNext = tiled_wait_vm(8 * (kTileStages - 3) + 4);
static_assert(8 * (kTileStages - 2) < 64, "vmcnt is a 6-bit counter");

// ------------------------------------------------------------------------------------------
// A direct global -> LDS load of 64 lanes x 16 bytes into LDS byte offset `lds_off` (wave-uniform,
// passed through M0).  It is issued as inline assembly: the compiler then keeps it where the source
// puts it relative to the LDS reads and adds no waits of its own for it, so every vmcnt wait on these
// loads in this file is explicit.
#define EF_TILED_DMA(gptr, lds_off)                                                                  \
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_off) : "memory")
// ring buffer of stage st (the first stage of the wave's range sits in buffer 0)
#define EF_TILED_BUF(st) ((int)((unsigned)((st) - ring0_) % (unsigned)kTileStages))
// LDS byte offset of fragment slot q*4 + wave of the buffer of stage st
#define EF_TILED_DST(st, q) (lds_base + ((EF_TILED_BUF(st) * kStageFrags + (q) * 4 + wave) << 10))
// all of a wave's loads of one stage in a burst (prologue only).  Every wave issues kStageFrags/4 loads
// per stage, unconditionally (past the end the last stage is re-read, in bounds), so "my loads of
// stage st have landed" is a constant wait count.
#define EF_TILED_ISSUE(st)                                                                           \
    {                                                                                                \
        const int stc_ = min((st), nstage - 1);                                                      \
        _Pragma("unroll") for (int q = 0; q < kStageFrags / 4; ++q)                                  \
            EF_TILED_DMA(src[q] + (size_t)stc_ * kTileKS * 64, EF_TILED_DST(st, q));                 \
    }
// HALF: operands are fp16 fragments instead of bf16; accumulation is fp32 either way.  The second half always
// runs in fp16 (activations and the W2 section of a blob are fp16, see mfma32h); the first half does in
// contexts with 4-bit experts (tokens and the dequantised weights are fp16 there), otherwise it runs in bf16.
typedef _Float16 tiled_half8 __attribute__((ext_vector_type(8)));
typedef _Float16 tiled_half2 __attribute__((ext_vector_type(2)));
template <bool HALF>
__device__ __forceinline__ floatx16 tiled_mfma(u32x4_t a, u32x4_t b, floatx16 c) {
    if constexpr (HALF)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(tiled_half8, a),
                                                      __builtin_bit_cast(tiled_half8, b), c, 0, 0, 0);
    else
        return mfma32v(a, b, c);
}

#define EF_TILED_READ(a, b, cur, ks)                                                              \
    {                                                                                                \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) a[i] = lds[cur][(ks) * 16 + AOFF + i][lane];     \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) b[j] = lds[cur][(ks) * 16 + 8 + BOFF + j][lane]; \
    }
// One k-step: 16 MFMAs on the current fragments (ac, bc) while the 8 fragments of the next k-step are
// read from LDS into (an, bn) and half of the wave's loads of stage `st` are issued: four rounds of
// four MFMAs with an LDS read after the first, second and fourth (the eight reads fill the first ten
// MFMA slots, so the last one is issued six MFMAs before the next k-step waits for it) and a
// global -> LDS load after the third.  A wave that issues its loads in a burst stalls at the issue
// until the CU's address path (about 64 bytes per clock) has taken them, and its matrix core idles
// meanwhile; one load per four MFMAs (128 clocks, four waves) stays below that rate.
//
// NLA / NLB (literals 0..4): only the first NLA operand-A fragments and the first NLB operand-B fragments
// of the wave are live; the MFMAs and LDS reads of the others are left out.  The token tiles are one of
// the two operands, and the last token panel of a group is rarely full: the kernels are limited by power,
// so matrix-core work on tiles that do not exist costs real throughput.  Loads and barriers are the same in
// every variant (the waves of a workgroup run different ones side by side).
// kSwapOperands (a constant of the kernel): the product is formed transposed, operand-B fragment first.  The two
// operand layouts are mirror images (lane 32*g + i holds row / column i, k-group g), so the same fragments serve.
#define EF_TILED_MF(ac, bc, r, j, NLA, NLB)                                                          \
    if ((r) < (NLA) && (j) < (NLB))                                                                  \
        acc[r][j] = kSwapOperands ? tiled_mfma<HALF>(bc[j], ac[r], acc[r][j]) : tiled_mfma<HALF>(ac[r], bc[j], acc[r][j]);
#define EF_TILED_RA(an, buf, ks, r, NLA) if ((r) < (NLA)) an[r] = lds[buf][(ks) * 16 + AOFF + (r)][lane];
#define EF_TILED_RB(bn, buf, ks, r, NLB) if ((r) < (NLB)) bn[r] = lds[buf][(ks) * 16 + 8 + BOFF + (r)][lane];
#define EF_TILED_ROUND(ac, bc, r, x0, x1, x3, st, half, NLA, NLB)                                    \
    EF_TILED_MF(ac, bc, r, 0, NLA, NLB)                                                              \
    x0 __builtin_amdgcn_sched_barrier(0);                                                            \
    EF_TILED_MF(ac, bc, r, 1, NLA, NLB)                                                              \
    x1 __builtin_amdgcn_sched_barrier(0);                                                            \
    EF_TILED_MF(ac, bc, r, 2, NLA, NLB)                                                              \
    EF_TILED_DMA(src[(half) * 4 + (r)] + (size_t)stc_ * kTileKS * 64, EF_TILED_DST(st, (half) * 4 + (r))); \
    __builtin_amdgcn_sched_barrier(0);                                                               \
    EF_TILED_MF(ac, bc, r, 3, NLA, NLB)                                                              \
    x3 __builtin_amdgcn_sched_barrier(0);
#define EF_TILED_STEP(ac, bc, an, bn, buf, ks, st, half, NLA, NLB)                                   \
    {                                                                                                \
        const int stc_ = min((st), nstage - 1);                                                      \
        EF_TILED_ROUND(ac, bc, 0, EF_TILED_RA(an, buf, ks, 0, NLA), EF_TILED_RB(bn, buf, ks, 0, NLB), \
                       EF_TILED_RA(an, buf, ks, 1, NLA), st, half, NLA, NLB)                         \
        EF_TILED_ROUND(ac, bc, 1, EF_TILED_RB(bn, buf, ks, 1, NLB), EF_TILED_RA(an, buf, ks, 2, NLA), \
                       EF_TILED_RB(bn, buf, ks, 2, NLB), st, half, NLA, NLB)                         \
        EF_TILED_ROUND(ac, bc, 2, EF_TILED_RA(an, buf, ks, 3, NLA), EF_TILED_RB(bn, buf, ks, 3, NLB), , st, half, \
                       NLA, NLB)                                                                     \
        EF_TILED_ROUND(ac, bc, 3, , , , st, half, NLA, NLB)                                          \
    }
// The main loop over stages [first, last): stage st feeds the matrix cores while the loads of stages
// st+1 .. st+kTileStages-2 are in flight and those of stage st+kTileStages-1 are being issued; one barrier per stage.
#define EF_TILED_LOOP(first, last, NLA, NLB)                                                         \
    for (int st = (first); st < (last); ++st) {                                                      \
        const int cur = EF_TILED_BUF(st), nxt = EF_TILED_BUF(st + 1);                                \
        /* the buffer of stage st+kTileStages-1 held stage st-1, whose last reads every wave */      \
        /* finished before the barrier of the previous iteration */                                  \
        EF_TILED_STEP(a0, b0, a1, b1, cur, 1, st + kTileStages - 1, 0, NLA, NLB)                     \
        /* stage st+1 must have landed */                                                            \
        __builtin_amdgcn_s_waitcnt(kWaitVmNext);                                                     \
        __syncthreads();                                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                           \
        EF_TILED_STEP(a1, b1, a0, b0, nxt, 0, st + kTileStages - 1, 1, NLA, NLB)                     \
    }
#define EF_TILED_PROLOGUE(first)                                                                     \
    static_assert(kTileKS == 2, "the loop alternates two fragment register sets");                   \
    u32x4_t a0[4], b0[4], a1[4], b1[4];                                                              \
    const int ring0_ = (first);                                                                      \
    _Pragma("unroll") for (int ps_ = 0; ps_ < kTileStages - 1; ++ps_) EF_TILED_ISSUE((first) + ps_)  \
    __builtin_amdgcn_s_waitcnt(kWaitVmFirst); /* my part of the first stage has landed */            \
    __syncthreads();                          /* ... and everybody else's */                         \
    EF_TILED_READ(a0, b0, 0, 0)
// `live` (wave-uniform, 0..4): live token tiles of the wave; they are operand B in the first half ...
#define EF_TILED_PIPELINE_TILES_B(first, last, live)                                                 \
    EF_TILED_PROLOGUE(first)                                                                         \
    switch (live) {                                                                                  \
        case 4: EF_TILED_LOOP(first, last, 4, 4) break;                                              \
        case 3: EF_TILED_LOOP(first, last, 4, 3) break;                                              \
        case 2: EF_TILED_LOOP(first, last, 4, 2) break;                                              \
        case 1: EF_TILED_LOOP(first, last, 4, 1) break;                                              \
        default: EF_TILED_LOOP(first, last, 4, 0) break;                                             \
    }                                                                                                \
    __builtin_amdgcn_s_waitcnt(0);
// ... and operand A in the second
#define EF_TILED_PIPELINE_TILES_A(first, last, live)                                                 \
    EF_TILED_PROLOGUE(first)                                                                         \
    switch (live) {                                                                                  \
        case 4: EF_TILED_LOOP(first, last, 4, 4) break;                                              \
        case 3: EF_TILED_LOOP(first, last, 3, 4) break;                                              \
        case 2: EF_TILED_LOOP(first, last, 2, 4) break;                                              \
        case 1: EF_TILED_LOOP(first, last, 1, 4) break;                                              \
        default: EF_TILED_LOOP(first, last, 0, 4) break;                                             \
    }                                                                                                \
    __builtin_amdgcn_s_waitcnt(0);

// a wave with a 2 x 2 share of a 128 x 128 tile (operand-A slots AOFF, AOFF + 1, operand-B slots BOFF, BOFF + 1)
#define EF_TILED_PIPELINE_2X2(first, last)                                                           \
    EF_TILED_PROLOGUE(first)                                                                         \
    EF_TILED_LOOP(first, last, 2, 2)                                                                 \
    __builtin_amdgcn_s_waitcnt(0);

}  // namespace ef
