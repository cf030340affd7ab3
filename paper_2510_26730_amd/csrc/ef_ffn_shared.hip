// Grouped SwiGLU expert FFN for groups of a few token tiles (3 to 7: too many for one pass of the plain
// weight-streaming kernels, too few for the matrix-core tiled ones).
//
// The plain streaming kernels give every wave its own copy of the token (or activation) fragments: with
// TT token tiles per pass a wave fetches TT KiB of them from L2 for every 2 KiB of weights, and at four
// tiles that traffic, not HBM, bounds the kernel.  Here the four waves of a workgroup work on the same
// token tiles and share those fragments through an LDS ring: each wave loads a quarter of a stage's
// fragments and every wave reads all of them from LDS, so L2 serves them once per workgroup.  Weights
// still stream straight from HBM into operand registers (1 KiB fragments, nontemporal), a register ring
// of three stages per wave, one barrier per stage of four k-blocks.
#include "ef_device.h"
#include "ef_kernels.h"

namespace ef {

constexpr int kShDepth = 3;   // register ring: stages in flight per wave (one workgroup per CU); the variants that
                              // fit two workgroups per CU (<= 256 registers) keep two stages
constexpr int kShLds = 4;     // LDS ring of shared token / activation fragments (stages, power of two)

// ------------------------------------------------------------------------------------------
// first half: act = silu(X W1^T) * (X W3^T).  Workgroup = (group, pass of TT token tiles, four
// consecutive 32-row blocks of F), wave = one row block, whole K range in stages of four k-blocks.
// ------------------------------------------------------------------------------------------
template <int TT, int D, int OCC>
__global__ __launch_bounds__(256, OCC) void ffn_gate_up_shared_kernel(GroupTable gt, const uint4 *__restrict__ xp,
                                                                    uint4 *__restrict__ act, int d) {
    __shared__ __attribute__((aligned(16))) u32x4_t xs[kShLds][TT * 4][64];
    const int wg = blockIdx.x;
    int grp = 0;
    while (grp + 1 < gt.n_groups && gt.wg_start[grp + 1] <= wg) ++grp;
    const int local = wg - gt.wg_start[grp];
    const int F = gt.F[grp];
    const int rbw = (F >> 5) >> 2;               // workgroups per pass (F is a multiple of 128)
    const int pass = local / rbw;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rb = (local % rbw) * 4 + wave;
    int ntl = gt.n_tiles[grp] - pass * TT;
    if (ntl > TT) ntl = TT;
    const int nkb = d >> 4, nq = d >> 6;         // d is a multiple of 64: whole stages

    const uint4 *w1 = reinterpret_cast<const uint4 *>(gt.blob[grp]) + (size_t)rb * 2 * nkb * 64 + lane;
    const uint4 *w3 = w1 + (size_t)nkb * 64;
    // this wave's share of the token fragments of a stage: k-block `wave` of each tile (tiles past the
    // group's last one repeat it; their results are dropped)
    const uint4 *xsrc[TT];
#pragma unroll
    for (int u = 0; u < TT; ++u)
        xsrc[u] = xp + (size_t)(gt.tile_start[grp] + pass * TT + min(u, ntl - 1)) * nkb * 64 + lane;

    floatx16 G[TT], U[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) { zero16(G[tt]); zero16(U[tt]); }

    u32x4_t wa[D][4], wb[D][4], xr[D][TT];
    // every load is unconditional (past the end the last stage is re-read, in bounds).  The token fragments are
    // requested before the weights: they are handed to the workgroup one stage before the weights of their
    // stage are used, and loads return in issue order, so waiting for them must not mean waiting for those weights
#define EF_SHU_LOAD(slot, kq)                                                                            \
    {                                                                                                    \
        const int kc_ = min((kq), nq - 1);                                                               \
        _Pragma("unroll") for (int u = 0; u < TT; ++u)                                                   \
            xr[slot][u] = *reinterpret_cast<const u32x4_t *>(xsrc[u] + (size_t)(4 * kc_ + wave) * 64);   \
        __builtin_amdgcn_sched_barrier(0);                                                               \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                  \
            wa[slot][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(w1 + (size_t)(4 * kc_ + j) * 64)); \
            wb[slot][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(w3 + (size_t)(4 * kc_ + j) * 64)); \
        }                                                                                                \
    }
#define EF_SHU_SHARE(slot, st)                                                                           \
    {                                                                                                    \
        _Pragma("unroll") for (int u = 0; u < TT; ++u) xs[(st) & (kShLds - 1)][u * 4 + wave][lane] = xr[slot][u]; \
    }
#define EF_SHU_COMPUTE(slot, st)                                                                         \
    {                                                                                                    \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                  \
            _Pragma("unroll") for (int tt = 0; tt < TT; ++tt) {                                          \
                const u32x4_t xb_ = xs[(st) & (kShLds - 1)][tt * 4 + j][lane];                           \
                G[tt] = mfma32v(wa[slot][j], xb_, G[tt]);                                                \
                U[tt] = mfma32v(wb[slot][j], xb_, U[tt]);                                                \
            }                                                                                            \
        }                                                                                                \
    }
    // one stage: hand the next stage's token fragments to the workgroup, compute this one, refill the
    // register slot just used, barrier (the next stage's fragments are visible; this stage's LDS
    // buffer is overwritten three stages from now)
#define EF_SHU_STAGE(slot, next_slot, st)                                                                \
    {                                                                                                    \
        EF_SHU_SHARE(next_slot, (st) + 1)                                                                \
        EF_SHU_COMPUTE(slot, st)                                                                         \
        EF_SHU_LOAD(slot, (st) + D)                                                                      \
        __syncthreads();                                                                                 \
    }
#pragma unroll
    for (int ring_ = 0; ring_ < D; ++ring_) EF_SHU_LOAD(ring_, ring_)
    EF_SHU_SHARE(0, 0)
    __syncthreads();
    int st = 0;
    for (; st + D <= nq; st += D) {
#pragma unroll
        for (int ring_ = 0; ring_ < D; ++ring_) EF_SHU_STAGE(ring_, (ring_ + 1) % D, st + ring_)
    }
#pragma unroll
    for (int ring_ = 0; ring_ < D - 1; ++ring_)
        if (st + ring_ < nq) EF_SHU_STAGE(ring_, ring_ + 1, st + ring_)
#undef EF_SHU_LOAD
#undef EF_SHU_SHARE
#undef EF_SHU_COMPUTE
#undef EF_SHU_STAGE

    // a lane holds 16 F-values of one token: the two paired-order fragments the second half consumes
    const int nkb2 = F >> 4;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        if (tt >= ntl) break;
        uint4 *dst = act + gt.act_off[grp] + ((size_t)(pass * TT + tt) * nkb2 + rb * 2) * 64 + lane;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            uint32_t pk[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float g0 = G[tt][8 * s + 2 * q], g1 = G[tt][8 * s + 2 * q + 1];
                const float v0 = g0 / (1.f + __expf(-g0)) * U[tt][8 * s + 2 * q];
                const float v1 = g1 / (1.f + __expf(-g1)) * U[tt][8 * s + 2 * q + 1];
                pk[q] = pack_act2(v0, v1);
            }
            dst[(size_t)s * 64] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        }
    }
}

hipError_t launch_ffn_gate_up_shared(const GroupTable &gt, int total_wgs, int tiles_per_pass, int occ, const void *xp,
                                     void *act, int d, hipStream_t s) {
    if (total_wgs <= 0) return hipSuccess;
    if (d % 64 != 0) return hipErrorInvalidValue;
    for (int i = 0; i < gt.n_groups; ++i)
        if (gt.F[i] % 128 != 0 || gt.n_tiles[i] <= 0 ||
            gt.wg_start[i + 1] - gt.wg_start[i] != ffn_gate_up_shared_wgs(gt.F[i], gt.n_tiles[i], tiles_per_pass))
            return hipErrorInvalidValue;
    if (gt.wg_start[gt.n_groups] != total_wgs) return hipErrorInvalidValue;
    const uint4 *x = reinterpret_cast<const uint4 *>(xp);
    uint4 *a = reinterpret_cast<uint4 *>(act);
    if (tiles_per_pass == 2)
        hipLaunchKernelGGL((ffn_gate_up_shared_kernel<2, kShDepth, 1>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else if (tiles_per_pass == 4 && occ == 2)
        hipLaunchKernelGGL((ffn_gate_up_shared_kernel<4, 2, 2>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else if (tiles_per_pass == 4)
        hipLaunchKernelGGL((ffn_gate_up_shared_kernel<4, kShDepth, 1>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// second half: Y = act W2^T.  Workgroup = (group, pass of TT token tiles, eight consecutive
// 32-column blocks of d, one of `ksg` K-slices), wave = two column blocks.  Activations (fp16) are operand
// A (rows = tokens), shared through LDS; W2 fragments (fp16) operand B (a lane holds one output column).
// Each K-slice writes its own partial Y plane; the un-permute sums the planes in order.
// ------------------------------------------------------------------------------------------
template <int TT, int D, int OCC>
__global__ __launch_bounds__(256, OCC) void ffn_down_shared_kernel(GroupTable gt, const uint4 *__restrict__ act,
                                                                 float *__restrict__ Y, int d, int ksg,
                                                                 long long y_plane) {
    constexpr int CBW = 2;
    __shared__ __attribute__((aligned(16))) u32x4_t as[kShLds][TT * 4][64];
    const int wg = blockIdx.x;
    int grp = 0;
    while (grp + 1 < gt.n_groups && gt.wg_start[grp + 1] <= wg) ++grp;
    const int local = wg - gt.wg_start[grp];
    const int ncb = d >> 5, ncq = (ncb + 7) >> 3;
    const int kslice = local % ksg;
    const int cq = (local / ksg) % ncq, pass = (local / ksg) / ncq;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cb0 = cq * 8 + wave * CBW;
    const bool valid = cb0 < ncb;                 // d is a multiple of 64: both column blocks or none
    const int cbc = valid ? cb0 : 0;              // waves past the last column load block 0 and drop the result
    const int F = gt.F[grp];
    const int nkb = F >> 4, nq = F >> 6;          // F is a multiple of 128: whole stages
    const int q0 = (int)((long long)kslice * nq / ksg), q1 = (int)((long long)(kslice + 1) * nq / ksg);
    int ntl = gt.n_tiles[grp] - pass * TT;
    if (ntl > TT) ntl = TT;

    const size_t cb_stride = (size_t)nkb * 64;
    const uint4 *w2 = reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(gt.blob[grp]) +
                                                      (size_t)4 * d * F) + (size_t)cbc * cb_stride + lane;
    const uint4 *asrc[TT];
#pragma unroll
    for (int u = 0; u < TT; ++u)
        asrc[u] = act + gt.act_off[grp] + (size_t)(pass * TT + min(u, ntl - 1)) * nkb * 64 + lane;

    floatx16 acc[CBW][TT];
#pragma unroll
    for (int cw = 0; cw < CBW; ++cw)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) zero16(acc[cw][tt]);

    u32x4_t wq[D][CBW][4], ar[D][TT];
#define EF_SHD_LOAD(slot, kq)                                                                            \
    {                                                                                                    \
        const int kc_ = min((kq), nq - 1);                                                               \
        _Pragma("unroll") for (int u = 0; u < TT; ++u)                                                   \
            ar[slot][u] = *reinterpret_cast<const u32x4_t *>(asrc[u] + (size_t)(4 * kc_ + wave) * 64);   \
        __builtin_amdgcn_sched_barrier(0);                                                               \
        _Pragma("unroll") for (int cw = 0; cw < CBW; ++cw)                                               \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                \
                wq[slot][cw][j] = __builtin_nontemporal_load(                                            \
                    reinterpret_cast<const u32x4_t *>(w2 + cw * cb_stride + (size_t)(4 * kc_ + j) * 64)); \
    }
#define EF_SHD_SHARE(slot, st)                                                                           \
    {                                                                                                    \
        _Pragma("unroll") for (int u = 0; u < TT; ++u) as[(st) & (kShLds - 1)][u * 4 + wave][lane] = ar[slot][u]; \
    }
#define EF_SHD_COMPUTE(slot, st)                                                                         \
    {                                                                                                    \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                  \
            _Pragma("unroll") for (int tt = 0; tt < TT; ++tt) {                                          \
                const u32x4_t af_ = as[(st) & (kShLds - 1)][tt * 4 + j][lane];                           \
                _Pragma("unroll") for (int cw = 0; cw < CBW; ++cw)                                       \
                    acc[cw][tt] = mfma32h(wq[slot][cw][j], af_, acc[cw][tt]);                            \
            }                                                                                            \
        }                                                                                                \
    }
#define EF_SHD_STAGE(slot, next_slot, st)                                                                \
    {                                                                                                    \
        EF_SHD_SHARE(next_slot, (st) + 1)                                                                \
        EF_SHD_COMPUTE(slot, st)                                                                         \
        EF_SHD_LOAD(slot, (st) + D)                                                                      \
        __syncthreads();                                                                                 \
    }
#pragma unroll
    for (int ring_ = 0; ring_ < D; ++ring_) EF_SHD_LOAD(ring_, q0 + ring_)
    EF_SHD_SHARE(0, q0)
    __syncthreads();
    int st = q0;
    for (; st + D <= q1; st += D) {
#pragma unroll
        for (int ring_ = 0; ring_ < D; ++ring_) EF_SHD_STAGE(ring_, (ring_ + 1) % D, st + ring_)
    }
#pragma unroll
    for (int ring_ = 0; ring_ < D - 1; ++ring_)
        if (st + ring_ < q1) EF_SHD_STAGE(ring_, ring_ + 1, st + ring_)
#undef EF_SHD_LOAD
#undef EF_SHD_SHARE
#undef EF_SHD_COMPUTE
#undef EF_SHD_STAGE

    if (!valid) return;
    const int g = lane >> 5;
    float *Yp = Y + (size_t)kslice * y_plane;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        if (tt >= ntl) break;
        // the product is formed transposed (W2 fragment first: the operand layouts are mirror images), so a lane
        // holds token lane % 32 and four consecutive output columns per accumulator quad: 16-byte stores
        const int tl = (pass * TT + tt) * kTile + (lane & 31);
        if (tl >= gt.count[grp]) continue;
        float *row = Yp + (size_t)(gt.row_offset[grp] + tl) * d;
#pragma unroll
        for (int cw = 0; cw < CBW; ++cw) {
            const int col = (cb0 + cw) * 32 + 4 * g;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<float4 *>(row + col + 8 * q) =
                    make_float4(acc[cw][tt][4 * q], acc[cw][tt][4 * q + 1], acc[cw][tt][4 * q + 2], acc[cw][tt][4 * q + 3]);
        }
    }
}

hipError_t launch_ffn_down_shared(const GroupTable &gt, int total_wgs, int tiles_per_pass, int occ, int ksg, const void *act,
                                  float *y, long long y_plane, int d, hipStream_t s) {
    if (total_wgs <= 0) return hipSuccess;
    if (d % 64 != 0 || ksg < 1) return hipErrorInvalidValue;
    for (int i = 0; i < gt.n_groups; ++i)
        if (gt.F[i] % 128 != 0 || gt.n_tiles[i] <= 0 ||
            gt.wg_start[i + 1] - gt.wg_start[i] != ffn_down_shared_wgs(d, gt.n_tiles[i], tiles_per_pass, ksg))
            return hipErrorInvalidValue;
    if (gt.wg_start[gt.n_groups] != total_wgs) return hipErrorInvalidValue;
    const uint4 *a = reinterpret_cast<const uint4 *>(act);
    if (tiles_per_pass == 2)
        hipLaunchKernelGGL((ffn_down_shared_kernel<2, kShDepth, 1>), dim3(total_wgs), dim3(256), 0, s, gt, a, y, d, ksg, y_plane);
    else if (tiles_per_pass == 4 && occ == 2)
        hipLaunchKernelGGL((ffn_down_shared_kernel<4, 2, 2>), dim3(total_wgs), dim3(256), 0, s, gt, a, y, d, ksg, y_plane);
    else if (tiles_per_pass == 4)
        hipLaunchKernelGGL((ffn_down_shared_kernel<4, kShDepth, 1>), dim3(total_wgs), dim3(256), 0, s, gt, a, y, d, ksg, y_plane);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ef
