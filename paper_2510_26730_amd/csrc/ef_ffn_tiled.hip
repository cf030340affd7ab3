// Grouped SwiGLU expert FFN for groups with many tokens (prefill): matrix-core bound.
//
// When an expert sees hundreds of tokens every weight fragment is reused by many token tiles and
// the two FFN halves are dense contractions: 256 x 256 output tiles per workgroup, 128 x 128 per
// wave (4 x 4 MFMA 32x32x16 accumulators), operands staged through LDS.  All three operands
// (expert weights, packed tokens, activations) are already stored as 1 KiB operand fragments, so
// the global -> LDS copy is a plain contiguous copy and an LDS operand read is 64 lanes x 16
// consecutive bytes (no bank conflicts, no swizzle).  Four LDS stage buffers are filled by direct
// global -> LDS loads three stages ahead of the one feeding the matrix cores, one barrier per stage.
// Workgroups that share a weight panel (same rows, different token panels) have consecutive ids,
// so the panel is fetched from HBM once and served to the others by L2 / MALL.
#include "ef_device.h"
#include "ef_kernels.h"

namespace ef {

constexpr int kTileKS = 2;               // MFMA k-steps (16 columns each) per LDS stage
constexpr int kStageFrags = 16 * kTileKS;  // fragments per stage: per k-step 8 of each operand
constexpr int kTileStages = 4;           // LDS stage buffers (power of two)
// s_waitcnt immediate "vmcnt <= 16, do not wait on expcnt / lgkmcnt" (gfx9 encoding: vmcnt[3:0] in bits
// 3:0 and vmcnt[5:4] in bits 15:14, expcnt in 6:4, lgkmcnt in 11:8)
constexpr int kWaitVm16 = (1 << 14) | (0x7 << 4) | (0xF << 8) | 0;
constexpr int kWaitVm12 = (0 << 14) | (0x7 << 4) | (0xF << 8) | 12;
static_assert(kStageFrags / 4 == 8, "the wait count assumes 8 loads per wave per stage");

// Index of a workgroup within its group -> (weight panel np, token panel mp).  Workgroups with the
// same index mod 8 land on one XCD; consecutive ones there walk the token panels of
// kTiledPanelBlock weight panels, so the panels an XCD works on at one time share its L2.
// Returns false for the padding workgroups past the last weight panel.
__device__ __forceinline__ bool tiled_panel(int local, int rot, int npanels, int mpanels, int &np, int &mp) {
    // `rot`: the XCD that takes the group's first panel block.  Groups whose panels do not fill a round of
    // eight XCDs would otherwise all start on XCD 0 and overfill its 32 compute units while others idle.
    const int xcd = (local - rot) & 7, j = local >> 3;
    const int pb = tiled_panel_block(npanels);
    const int blk = pb * mpanels;
    const int jb = j / blk, jj = j - jb * blk;
    np = (jb * 8 + xcd) * pb + jj / mpanels;
    mp = jj % mpanels;
    return np < npanels;
}

// ------------------------------------------------------------------------------------------
// The LDS pipeline shared by both kernels (they name their locals alike: lds, src, acc, wave, lane,
// nstage, AOFF, BOFF).
//
// A direct global -> LDS load of 64 lanes x 16 bytes into LDS byte offset `lds_off` (wave-uniform,
// passed through M0).  It is issued as inline assembly: the compiler then keeps it where the source
// puts it relative to the LDS reads and adds no waits of its own for it, so every vmcnt wait on these
// loads in this file is explicit.
#define EF_TILED_DMA(gptr, lds_off)                                                                  \
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_off) : "memory")
// LDS byte offset of fragment slot q*4 + wave of the buffer of stage st
#define EF_TILED_DST(st, q) (lds_base + ((((st) & (kTileStages - 1)) * kStageFrags + (q) * 4 + wave) << 10))
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
// st+1 and st+2 are in flight and those of stage st+3 are being issued; one barrier per stage.
#define EF_TILED_LOOP(first, last, NLA, NLB)                                                         \
    for (int st = (first); st < (last); ++st) {                                                      \
        const int cur = st & (kTileStages - 1), nxt = (st + 1) & (kTileStages - 1);                  \
        /* the buffer of stage st+3 held stage st-1, whose last reads every wave finished before */  \
        /* the barrier of the previous iteration */                                                  \
        EF_TILED_STEP(a0, b0, a1, b1, cur, 1, st + 3, 0, NLA, NLB)                                   \
        /* stage st+1 must have landed: of the loads issued after it (stage st+2 and half of */      \
        /* stage st+3) all 12 may still be outstanding */                                            \
        __builtin_amdgcn_s_waitcnt(kWaitVm12);                                                       \
        __syncthreads();                                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                           \
        EF_TILED_STEP(a1, b1, a0, b0, nxt, 0, st + 3, 1, NLA, NLB)                                   \
    }
#define EF_TILED_PROLOGUE(first)                                                                     \
    static_assert(kTileKS == 2, "the loop alternates two fragment register sets");                   \
    u32x4_t a0[4], b0[4], a1[4], b1[4];                                                              \
    EF_TILED_ISSUE(first)                                                                            \
    EF_TILED_ISSUE((first) + 1)                                                                      \
    EF_TILED_ISSUE((first) + 2)                                                                      \
    __builtin_amdgcn_s_waitcnt(kWaitVm16); /* my part of the first stage has landed */               \
    __syncthreads();                       /* ... and everybody else's */                            \
    EF_TILED_READ(a0, b0, (first) & (kTileStages - 1), 0)
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

// ------------------------------------------------------------------------------------------
// first half, tiled: act = silu(X W1^T) * (X W3^T) for (group, 4 row blocks, 8 token tiles)
// operand A slots 0..7 = W1/W3 fragments of row blocks rb0..rb0+3 (slot = 2*rbl + which),
// operand B slots 8..15 = packed-token fragments of tiles t0..t0+7
// ------------------------------------------------------------------------------------------
template <bool HALF>
__global__ __launch_bounds__(256, 1) void ffn_gate_up_tiled_kernel(GroupTable gt, const uint4 *__restrict__ xp,
                                                                    uint4 *__restrict__ act, int d) {
    constexpr bool kSwapOperands = false;
    __shared__ __attribute__((aligned(16))) u32x4_t lds[kTileStages][kStageFrags][64];
    const int wg = blockIdx.x;
    int grp = 0;
    while (grp + 1 < gt.n_groups && gt.wg_start[grp + 1] <= wg) ++grp;
    const int local = wg - gt.wg_start[grp];
    const int F = gt.F[grp];
    const int ntiles = gt.n_tiles[grp];
    const int mpanels = (ntiles + 7) >> 3;
    int np, mp;
    if (!tiled_panel(local, gt.xcd_rot[grp], F >> 7, mpanels, np, mp)) return;
    const int rb0 = np * 4, t0 = mp * 8;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS DMA targets go through M0
    const int wf = wave & 1, wt = wave >> 1;
    const int nkb = d >> 4;
    const int nstage = nkb / kTileKS;

    // per-thread source of its 8 fragment quarters per stage: fragment q*4 + wave of the stage
    const u32x4_t *src[kStageFrags / 4];
#pragma unroll
    for (int q = 0; q < kStageFrags / 4; ++q) {
        const int fi = q * 4 + wave;              // 0 .. kStageFrags-1
        const int ks = fi >> 4, slot = fi & 15;
        const uint4 *p;
        if (slot < 8) {
            const int rbl = slot >> 1, which = slot & 1;
            p = reinterpret_cast<const uint4 *>(gt.blob[grp]) + ((size_t)(rb0 + rbl) * 2 + which) * nkb * 64;
        } else {
            const int tile = min(t0 + (slot - 8), ntiles - 1);
            p = xp + (size_t)(gt.tile_start[grp] + tile) * nkb * 64;
        }
        src[q] = reinterpret_cast<const u32x4_t *>(p + (size_t)ks * 64 + lane);
    }

    floatx16 acc[4][4];   // [operand-A fragment: W1 rb, W3 rb, W1 rb+1, W3 rb+1][token tile]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) zero16(acc[i][j]);

    const int AOFF = wf * 4, BOFF = wt * 4;
    const unsigned lds_base = (unsigned)(size_t)&lds[0][0][0];   // LDS byte offset: the low half of its flat address
    // token tiles t0 + 4*wt .. +3 of this wave that exist (wave-uniform)
    const int live = max(0, min(4, ntiles - (t0 + BOFF)));
    EF_TILED_PIPELINE_TILES_B(0, nstage, live)

    // epilogue: act fragments (paired order) of row blocks rb0 + 2*wf + {0,1}, tiles t0 + 4*wt + j
    const int nkb2 = F >> 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int tile = t0 + wt * 4 + j;
        if (tile >= ntiles) continue;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int rb = rb0 + wf * 2 + h;
            uint4 *dst = act + gt.act_off[grp] + ((size_t)tile * nkb2 + rb * 2) * 64 + lane;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                uint32_t pk[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float g0 = acc[2 * h][j][8 * s + 2 * q], g1 = acc[2 * h][j][8 * s + 2 * q + 1];
                    const float v0 = g0 / (1.f + __expf(-g0)) * acc[2 * h + 1][j][8 * s + 2 * q];
                    const float v1 = g1 / (1.f + __expf(-g1)) * acc[2 * h + 1][j][8 * s + 2 * q + 1];
                    pk[q] = pack_act2(v0, v1);
                }
                dst[(size_t)s * 64] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
            }
        }
    }
}

hipError_t launch_ffn_gate_up_tiled(const GroupTable &gt, int total_wgs, const void *xp, void *act, int d,
                                    bool f16, hipStream_t s) {
    if (total_wgs <= 0) return hipSuccess;
    // the kernel's index mapping and the grid must come from the same workgroup count per group
    for (int i = 0; i < gt.n_groups; ++i)
        if (gt.wg_start[i + 1] - gt.wg_start[i] != ffn_gate_up_tiled_wgs(gt.F[i], gt.n_tiles[i]) ||
            !ffn_tiled_ok(d, gt.F[i], gt.n_tiles[i]))
            return hipErrorInvalidValue;
    if (gt.wg_start[gt.n_groups] != total_wgs) return hipErrorInvalidValue;
    if (f16)
        hipLaunchKernelGGL(ffn_gate_up_tiled_kernel<true>, dim3(total_wgs), dim3(256), 0, s, gt,
                           reinterpret_cast<const uint4 *>(xp), reinterpret_cast<uint4 *>(act), d);
    else
        hipLaunchKernelGGL(ffn_gate_up_tiled_kernel<false>, dim3(total_wgs), dim3(256), 0, s, gt,
                           reinterpret_cast<const uint4 *>(xp), reinterpret_cast<uint4 *>(act), d);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// second half, tiled: Y = act W2^T for (group, 8 token tiles, 8 column blocks)
// operand A slots 0..7 = activation fragments of tiles t0..t0+7,
// operand B slots 8..15 = W2 fragments of column blocks cb0..cb0+7
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 1) void ffn_down_tiled_kernel(GroupTable gt, const uint4 *__restrict__ act,
                                                                 float *__restrict__ Y, int d, int ksg_all,
                                                                 int split_grp, int split_ksg, long long y_plane) {
    // Y^T = W2 act^T: a lane then ends with one token (its index mod 32) and four consecutive output columns per
    // accumulator quad, which is one 16-byte store; with the product the other way round a lane holds one
    // column of four consecutive tokens and the tile leaves in 4-byte stores, four times as many instructions
    constexpr bool kSwapOperands = true;
    constexpr bool HALF = true;   // fp16 activations and W2 fragments
    __shared__ __attribute__((aligned(16))) u32x4_t lds[kTileStages][kStageFrags][64];
    const int wg = blockIdx.x;
    int grp = 0;
    while (grp + 1 < gt.n_groups && gt.wg_start[grp + 1] <= wg) ++grp;
    const int local = wg - gt.wg_start[grp];
    const int F = gt.F[grp];
    const int ntiles = gt.n_tiles[grp];
    const int mpanels = (ntiles + 7) >> 3;
    // K slices across workgroups (one Y plane each, summed by the un-permute) when the tiles alone
    // would leave most of the chip idle; neighbouring workgroups take the slices of one tile.  One group of the
    // launch (the last one) may have a slice count of its own: shorter workgroups that fill the launch's last,
    // partly empty round over the compute units
    const int ksg = grp == split_grp ? split_ksg : ksg_all;
    const int kslice = local % ksg;
    int np, mp;
    if (!tiled_panel(local / ksg, gt.xcd_rot[grp], d >> 8, mpanels, np, mp)) return;
    const int cb0 = np * 8, t0 = mp * 8;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS DMA targets go through M0
    const int wc = wave & 1, wt = wave >> 1;
    const int nkb = F >> 4;
    const int nstage = nkb / kTileKS;
    const int s0 = (int)((long long)kslice * nstage / ksg), s1 = (int)((long long)(kslice + 1) * nstage / ksg);

    const u32x4_t *src[kStageFrags / 4];
#pragma unroll
    for (int q = 0; q < kStageFrags / 4; ++q) {
        const int fi = q * 4 + wave;
        const int ks = fi >> 4, slot = fi & 15;
        const uint4 *p;
        if (slot < 8) {
            const int tile = min(t0 + slot, ntiles - 1);
            p = act + gt.act_off[grp] + (size_t)tile * nkb * 64;
        } else {
            p = reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(gt.blob[grp]) + (size_t)4 * d * F) +
                (size_t)(cb0 + slot - 8) * nkb * 64;
        }
        src[q] = reinterpret_cast<const u32x4_t *>(p + (size_t)ks * 64 + lane);
    }

    floatx16 acc[4][4];   // [token tile][column block]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) zero16(acc[i][j]);

    const int AOFF = wt * 4, BOFF = wc * 4;
    const unsigned lds_base = (unsigned)(size_t)&lds[0][0][0];   // LDS byte offset: the low half of its flat address
    // token tiles t0 + 4*wt .. +3 of this wave that exist (wave-uniform)
    const int live = max(0, min(4, ntiles - (t0 + AOFF)));
    EF_TILED_PIPELINE_TILES_A(s0, s1, live)

    const int g = lane >> 5;
    float *Yp = Y + (size_t)kslice * y_plane;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int tile = t0 + wt * 4 + i;
        if (tile >= ntiles) continue;
        const int tl = tile * kTile + (lane & 31);
        if (tl >= gt.count[grp]) continue;
        float *row = Yp + (size_t)(gt.row_offset[grp] + tl) * d;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = (cb0 + wc * 4 + j) * 32 + 4 * g;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<float4 *>(row + col + 8 * q) =
                    make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        }
    }
}

hipError_t launch_ffn_down_tiled(const GroupTable &gt, int total_wgs, int ksg, int split_grp, int split_ksg,
                                 const void *act, float *y, long long y_plane, int d, hipStream_t s) {
    if (total_wgs <= 0) return hipSuccess;
    if (ksg < 1 || (split_grp >= 0 && (split_grp >= gt.n_groups || split_ksg < 1))) return hipErrorInvalidValue;
    for (int i = 0; i < gt.n_groups; ++i) {
        const int ks = i == split_grp ? split_ksg : ksg;
        if (gt.wg_start[i + 1] - gt.wg_start[i] != ffn_down_tiled_wgs(d, gt.n_tiles[i]) * ks ||
            !ffn_tiled_ok(d, gt.F[i], gt.n_tiles[i]) || gt.F[i] / 32 < ks)
            return hipErrorInvalidValue;
    }
    if (gt.wg_start[gt.n_groups] != total_wgs) return hipErrorInvalidValue;
    hipLaunchKernelGGL(ffn_down_tiled_kernel, dim3(total_wgs), dim3(256), 0, s, gt,
                       reinterpret_cast<const uint4 *>(act), y, d, ksg, split_grp, split_ksg, y_plane);
    return hipGetLastError();
}

}  // namespace ef
