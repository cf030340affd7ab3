// Grouped SwiGLU expert FFN for groups with many tokens (prefill): matrix-core bound.
//
// When an expert sees hundreds of tokens every weight fragment is reused by many token tiles and
// the two FFN halves are dense contractions: 256 x 256 output tiles per workgroup, 128 x 128 per
// wave (4 x 4 MFMA 32x32x16 accumulators), operands staged through LDS.  All three operands
// (expert weights, packed tokens, activations) are already stored as 1 KiB operand fragments, so
// the global -> LDS copy is a plain contiguous copy and an LDS operand read is 64 lanes x 16
// consecutive bytes (no bank conflicts, no swizzle).  The LDS stage buffers (four) are filled by direct
// global -> LDS loads three stages ahead of the one feeding the matrix cores, one barrier per stage.
// Workgroups that share a weight panel (same rows, different token panels) have consecutive ids,
// so the panel is fetched from HBM once and served to the others by L2 / MALL.
#include "ef_device.h"
#include "ef_kernels.h"
#include "ef_tiled_pipeline.h"

namespace ef {

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
