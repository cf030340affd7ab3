// Grouped SwiGLU expert FFN over the cache slots: token permutation into operand tiles, the two
// weight-streaming matrix-core kernels, and the weighted un-permute.
//
// Both FFN halves are bound by streaming the active experts' weights from HBM whenever an expert
// sees few tokens (decode); every weight fragment is then used exactly once.  The kernels are
// therefore built around long, contiguous, software-pipelined 1 KiB fragment streams per wave and
// enough waves in flight; the matrix cores only have to keep up.
#include <hip/hip_ext.h>

#include "ef_device.h"
#include "ef_kernels.h"

namespace ef {

// ------------------------------------------------------------------------------------------
// token permutation into per-expert groups, written directly in operand-fragment order:
// xp[tile][kb][lane (g,i)] = 8 bf16 of row i of the tile, columns kb*16 + 8g .. +8.
// grid = (tiles, column chunks); a workgroup copies a 32-row x (16*kb_per_wg)-column panel.
// ------------------------------------------------------------------------------------------
// eight bf16 -> eight fp16 (exact for 2^-14 <= |x| < 65504): the 4-bit FFN kernels run the matrix cores in fp16
__device__ __forceinline__ uint4 bf16x8_to_f16x8(uint4 v) {
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float lo = __builtin_bit_cast(float, w[q] << 16), hi = __builtin_bit_cast(float, w[q] & 0xFFFF0000u);
        w[q] = __builtin_bit_cast(uint32_t, half2v{(_Float16)lo, (_Float16)hi});
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

__global__ __launch_bounds__(256) void pack_x_kernel(PackTable pt, const uint16_t *__restrict__ h, int d, int k,
                                                     const int32_t *__restrict__ perm, uint4 *__restrict__ xp,
                                                     int kb_per_wg, int f16) {
    const int tile = blockIdx.x;
    int grp = 0;
    while (grp + 1 < pt.n_groups && pt.tile_start[grp + 1] <= tile) ++grp;
    const int local = tile - pt.tile_start[grp];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g = lane >> 5, i = lane & 31;
    const int r = local * kTile + i;
    const bool valid = r < pt.count[grp];
    int token = 0;
    if (valid) token = pt.row_offset[grp] < 0 ? r : perm[pt.row_offset[grp] + r] / k;
    const uint4 *src = reinterpret_cast<const uint4 *>(h + (size_t)token * d);
    const int nkb = d >> 4;
    uint4 *dst = xp + (size_t)tile * nkb * 64 + lane;
    const int kb0 = blockIdx.y * kb_per_wg;
    const int kb1 = min(nkb, kb0 + kb_per_wg);
    // Rows past the group's count are left as they are: every FFN kernel keeps tokens in separate
    // operand columns (rows), so whatever such a row holds only reaches outputs that are never
    // written.  Groups of a few tokens would otherwise spend most of this kernel storing zeros.
    if (!valid) return;
    for (int kb = kb0 + wave; kb < kb1; kb += 4) {
        const uint4 v = src[kb * 2 + g];
        dst[(size_t)kb * 64] = f16 ? bf16x8_to_f16x8(v) : v;
    }
}

hipError_t launch_pack_x(const PackTable &pt, int total_tiles, const uint16_t *h, int d, int k,
                         const int32_t *perm, void *xp, bool f16, hipStream_t s) {
    if (total_tiles <= 0) return hipSuccess;
    const int nkb = d >> 4;
    // enough workgroups to fill the chip at small tile counts, at least 8 fragments per workgroup
    int chunks = 1;
    while (total_tiles * chunks < 1024 && nkb / (chunks * 2) >= 8) chunks *= 2;
    const int kb_per_wg = (nkb + chunks - 1) / chunks;
    hipLaunchKernelGGL(pack_x_kernel, dim3(total_tiles, chunks), dim3(256), 0, s, pt, h, d, k, perm,
                       reinterpret_cast<uint4 *>(xp), kb_per_wg, f16 ? 1 : 0);
    return hipGetLastError();
}

// The same packing planned on the device: the tile -> (group, local tile) table is derived from the
// per-expert counts the grouping kernel left in device memory (experts in id order, 32-row tiles,
// the dense shared FFN last), so the launch needs nothing from the host and can be enqueued
// before the host has read the counts.  grid.x is an upper bound of the tile count; surplus
// workgroups exit.
__global__ __launch_bounds__(256) void pack_x_dev_kernel(const int32_t *__restrict__ counts,
                                                         const int32_t *__restrict__ offsets, int E, int has_shared,
                                                         int T, const uint16_t *__restrict__ h, int d, int k,
                                                         const int32_t *__restrict__ perm, uint4 *__restrict__ xp,
                                                         int kb_per_wg, int f16) {
    const int tile = blockIdx.x;
    // every wave finds the tile's group on its own: lane e holds the tile count of expert e (E <= 64), an
    // inclusive scan across the lanes gives the first tile after each expert, a ballot the expert
    const int ln = threadIdx.x & 63;
    const int my_nt = ln < E ? (counts[ln] + kTile - 1) / kTile : 0;
    int incl = my_nt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(incl, off);
        if (ln >= off) incl += o;
    }
    const unsigned long long owns = __ballot(ln < E && tile >= incl - my_nt && tile < incl);
    const int routed_tiles = __shfl(incl, 63);
    const int grp = owns ? __ffsll((long long)owns) - 1 : -1;
    const int first = grp >= 0 ? __shfl(incl - my_nt, grp) : routed_tiles;
    int count, row_offset;
    if (grp >= 0) {
        count = counts[grp];
        row_offset = offsets[grp];
    } else {
        if (!has_shared || tile - first >= (T + kTile - 1) / kTile) return;
        count = T;
        row_offset = -1;
    }
    const int local = tile - first;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g = lane >> 5, i = lane & 31;
    const int r = local * kTile + i;
    const bool valid = r < count;
    int token = 0;
    if (valid) token = row_offset < 0 ? r : perm[row_offset + r] / k;
    const uint4 *src = reinterpret_cast<const uint4 *>(h + (size_t)token * d);
    const int nkb = d >> 4;
    uint4 *dst = xp + (size_t)tile * nkb * 64 + lane;
    const int kb0 = blockIdx.y * kb_per_wg;
    const int kb1 = min(nkb, kb0 + kb_per_wg);
    // Rows past the group's count are left as they are: every FFN kernel keeps tokens in separate
    // operand columns (rows), so whatever such a row holds only reaches outputs that are never
    // written.  Groups of a few tokens would otherwise spend most of this kernel storing zeros.
    if (!valid) return;
    for (int kb = kb0 + wave; kb < kb1; kb += 4) {
        const uint4 v = src[kb * 2 + g];
        dst[(size_t)kb * 64] = f16 ? bf16x8_to_f16x8(v) : v;
    }
}

hipError_t launch_pack_x_dev(const int32_t *counts, const int32_t *offsets, int E, bool has_shared, int T,
                             int max_tiles, const uint16_t *h, int d, int k, const int32_t *perm, void *xp,
                             bool f16, hipStream_t s) {
    if (max_tiles <= 0) return hipSuccess;
    const int nkb = d >> 4;
    int chunks = 1;
    while (max_tiles * chunks < 1024 && nkb / (chunks * 2) >= 8) chunks *= 2;
    const int kb_per_wg = (nkb + chunks - 1) / chunks;
    hipLaunchKernelGGL(pack_x_dev_kernel, dim3(max_tiles, chunks), dim3(256), 0, s, counts, offsets, E,
                       has_shared ? 1 : 0, T, h, d, k, perm, reinterpret_cast<uint4 *>(xp), kb_per_wg, f16 ? 1 : 0);
    return hipGetLastError();
}

// K loop of the first FFN half for NTL live token tiles: three register stages of UNR fragments per
// operand; stages c+1 and c+2 are in flight while stage c feeds the matrix cores.  Every load is
// unconditional (the last prefetch re-reads the final stage, in bounds).
template <int TT, int NTL, int UNR>
__device__ __forceinline__ void up_stream(const uint4 *__restrict__ w1, const uint4 *__restrict__ w3,
                                          const uint4 *__restrict__ x0, int nkb, int k0, int k1,
                                          floatx16 (&G)[TT], floatx16 (&U)[TT]) {
    u32x4_t a1A[UNR], a3A[UNR], xA[NTL][UNR], a1B[UNR], a3B[UNR], xB[NTL][UNR], a1C[UNR], a3C[UNR], xC[NTL][UNR];
#define EF_UP_LOAD(a1, a3, x, kb)                                                                        \
    {                                                                                                    \
        _Pragma("unroll") for (int u = 0; u < UNR; ++u) {                                                \
            a1[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(w1 + (size_t)((kb) + u) * 64)); \
            a3[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(w3 + (size_t)((kb) + u) * 64)); \
        }                                                                                                \
        _Pragma("unroll") for (int tt = 0; tt < NTL; ++tt)                                               \
            _Pragma("unroll") for (int u = 0; u < UNR; ++u)                                              \
                x[tt][u] = *reinterpret_cast<const u32x4_t *>(x0 + ((size_t)tt * nkb + (kb) + u) * 64);  \
    }
#define EF_UP_COMPUTE(a1, a3, x)                                                                         \
    {                                                                                                    \
        _Pragma("unroll") for (int u = 0; u < UNR; ++u)                                                  \
            _Pragma("unroll") for (int tt = 0; tt < NTL; ++tt) {                                         \
                G[tt] = mfma32v(a1[u], x[tt][u], G[tt]);                                                 \
                U[tt] = mfma32v(a3[u], x[tt][u], U[tt]);                                                 \
            }                                                                                            \
    }
    const int nfull = (k1 - k0) / UNR;
    int kb = k0;
    if (nfull > 0) {
        const int last = k0 + (nfull - 1) * UNR;
        EF_UP_LOAD(a1A, a3A, xA, kb)
        EF_UP_LOAD(a1B, a3B, xB, min(kb + UNR, last))
        int c = 0;
        for (; c + 3 <= nfull; c += 3) {   // three register stages: two are always in flight
            EF_UP_LOAD(a1C, a3C, xC, kb + 2 * UNR)
            EF_UP_COMPUTE(a1A, a3A, xA)
            EF_UP_LOAD(a1A, a3A, xA, min(kb + 3 * UNR, last))
            EF_UP_COMPUTE(a1B, a3B, xB)
            EF_UP_LOAD(a1B, a3B, xB, min(kb + 4 * UNR, last))
            EF_UP_COMPUTE(a1C, a3C, xC)
            kb += 3 * UNR;
        }
        if (c < nfull) {
            EF_UP_COMPUTE(a1A, a3A, xA)
            kb += UNR;
        }
        if (c + 1 < nfull) {
            EF_UP_COMPUTE(a1B, a3B, xB)
            kb += UNR;
        }
    }
    for (; kb < k1; ++kb) {
        const uint4 b1 = load_stream(w1 + (size_t)kb * 64), b3 = load_stream(w3 + (size_t)kb * 64);
#pragma unroll
        for (int tt = 0; tt < NTL; ++tt) {
            const uint4 xv = x0[((size_t)tt * nkb + kb) * 64];
            G[tt] = mfma32(b1, xv, G[tt]);
            U[tt] = mfma32(b3, xv, U[tt]);
        }
    }
#undef EF_UP_LOAD
#undef EF_UP_COMPUTE
}

// ------------------------------------------------------------------------------------------
// first half: act = silu(X W1^T) * (X W3^T).
//
// Work unit of a wave: (group, 32 F-rows "rb", pass of TT token tiles, K slice).  Weights are
// operand A (rows = F index), packed tokens operand B (columns = tokens), so a lane ends with 16
// F-values of one token: exactly the two paired-order fragments the second half consumes.
// A workgroup is 4 waves = (4/KS row blocks) x (KS K-slices); K-slices are summed in a fixed
// order through LDS before the non-linear epilogue.  Loads are double-buffered in registers:
// the fragments of chunk c+1 are in flight while chunk c feeds the matrix cores.
// ------------------------------------------------------------------------------------------
template <int TT, int KS>
__global__ __launch_bounds__(256) void ffn_gate_up_kernel(GroupTable gt, const uint4 *__restrict__ xp,
                                                          uint4 *__restrict__ act, int d) {
    constexpr int RBW = 4 / KS;
    constexpr int UNR = (TT == 1) ? 4 : (TT == 2) ? 2 : 1;   // fragments per operand per pipeline stage (register budget)
    constexpr int REGION = TT * 2 * 16 * 64;  // floats of one wave's partial (G and U of TT tiles)
    __shared__ float red[(KS > 1) ? 2 * REGION : 1];

    const int wg = blockIdx.x;
    int grp = 0;
    while (grp + 1 < gt.n_groups && gt.wg_start[grp + 1] <= wg) ++grp;
    const int local = wg - gt.wg_start[grp];
    const int F = gt.F[grp];
    const int nrb = F >> 5, rbw = (nrb + RBW - 1) / RBW;
    const int pass = local / rbw;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rbl = wave / KS, ks = wave % KS;
    const int rb = (local % rbw) * RBW + rbl;
    const bool active = rb < nrb;
    int ntl = gt.n_tiles[grp] - pass * TT;
    if (ntl > TT) ntl = TT;
    const int nkb = d >> 4;
    const int k0 = (int)((long long)ks * nkb / KS), k1 = (int)((long long)(ks + 1) * nkb / KS);

    floatx16 G[TT], U[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) { zero16(G[tt]); zero16(U[tt]); }

    if (active) {
        const uint4 *w1 = reinterpret_cast<const uint4 *>(gt.blob[grp]) + (size_t)rb * 2 * nkb * 64 + lane;
        const uint4 *w3 = w1 + (size_t)nkb * 64;
        const uint4 *x0 = xp + (size_t)(gt.tile_start[grp] + pass * TT) * nkb * 64 + lane;
        // the number of live token tiles is wave-uniform: pick a loop whose loads are unconditional,
        // so the compiler knows how many are in flight and waits only for the oldest stage
        if (TT == 1 || ntl == 1) up_stream<TT, 1, UNR>(w1, w3, x0, nkb, k0, k1, G, U);
        else if (TT == 2 || ntl == 2) up_stream<TT, 2, UNR>(w1, w3, x0, nkb, k0, k1, G, U);
        else if (ntl == 3) up_stream<TT, (TT > 2 ? 3 : TT), UNR>(w1, w3, x0, nkb, k0, k1, G, U);
        else up_stream<TT, TT, UNR>(w1, w3, x0, nkb, k0, k1, G, U);
    }

    // fixed-order sum of the K-slices: (p0 + p2) + (p1 + p3) for KS = 4, p0 + p1 for KS = 2
    if (KS > 1) {
        auto put = [&](float *r) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    r[((tt * 2 + 0) * 16 + v) * 64 + lane] = G[tt][v];
                    r[((tt * 2 + 1) * 16 + v) * 64 + lane] = U[tt][v];
                }
        };
        auto add = [&](const float *r) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    G[tt][v] += r[((tt * 2 + 0) * 16 + v) * 64 + lane];
                    U[tt][v] += r[((tt * 2 + 1) * 16 + v) * 64 + lane];
                }
        };
        if (KS == 4) {
            if (ks >= 2) put(red + (ks - 2) * REGION);
            __syncthreads();
            if (ks < 2) add(red + ks * REGION);
            __syncthreads();
            if (ks == 1) put(red);
            __syncthreads();
            if (ks == 0) add(red);
        } else {
            if (ks == 1) put(red + rbl * REGION);
            __syncthreads();
            if (ks == 0) add(red + rbl * REGION);
        }
    }

    if (active && ks == 0) {
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
}

template <int TT>
static hipError_t launch_up_tt(const GroupTable &gt, int total_wgs, int ks, const uint4 *x, uint4 *a, int d,
                               hipStream_t s) {
    if (ks == 1) hipLaunchKernelGGL((ffn_gate_up_kernel<TT, 1>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else if (ks == 2) hipLaunchKernelGGL((ffn_gate_up_kernel<TT, 2>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else if (ks == 4) hipLaunchKernelGGL((ffn_gate_up_kernel<TT, 4>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_ffn_gate_up(const GroupTable &gt, int total_wgs, int tiles_per_pass, int ks, const void *xp,
                              void *act, int d, hipStream_t s) {
    if (total_wgs <= 0) return hipSuccess;
    const uint4 *x = reinterpret_cast<const uint4 *>(xp);
    uint4 *a = reinterpret_cast<uint4 *>(act);
    if (tiles_per_pass == 1) return launch_up_tt<1>(gt, total_wgs, ks, x, a, d, s);
    if (tiles_per_pass == 2) return launch_up_tt<2>(gt, total_wgs, ks, x, a, d, s);
    if (tiles_per_pass == 4) return launch_up_tt<4>(gt, total_wgs, ks, x, a, d, s);
    return hipErrorInvalidValue;
}

// K loop of the second FFN half for NTL live token tiles and CBW column blocks per wave (same
// three-stage pipeline as up_stream).  An activation fragment is loaded once and multiplied with
// CBW weight fragments: activations come from L2 and are shared by every column block of the
// group, so blocking over columns cuts that traffic and leaves the fetch paths to the weights.
template <int TT, int NTL, int CBW, int UNR>
__device__ __forceinline__ void down_stream(const uint4 *__restrict__ w2, size_t cb_stride,
                                            const uint4 *__restrict__ a0, int nkb, int k0, int k1,
                                            floatx16 (&acc)[CBW][TT]) {
    u32x4_t bA[CBW][UNR], aA[NTL][UNR], bB[CBW][UNR], aB[NTL][UNR], bC[CBW][UNR], aC[NTL][UNR];
#define EF_DN_LOAD(b, a, kb)                                                                             \
    {                                                                                                    \
        _Pragma("unroll") for (int cw = 0; cw < CBW; ++cw)                                               \
            _Pragma("unroll") for (int u = 0; u < UNR; ++u)                                              \
                b[cw][u] = __builtin_nontemporal_load(                                                   \
                    reinterpret_cast<const u32x4_t *>(w2 + cw * cb_stride + (size_t)((kb) + u) * 64));   \
        _Pragma("unroll") for (int tt = 0; tt < NTL; ++tt)                                               \
            _Pragma("unroll") for (int u = 0; u < UNR; ++u)                                              \
                a[tt][u] = *reinterpret_cast<const u32x4_t *>(a0 + ((size_t)tt * nkb + (kb) + u) * 64);  \
    }
#define EF_DN_COMPUTE(b, a)                                                                              \
    {                                                                                                    \
        _Pragma("unroll") for (int u = 0; u < UNR; ++u)                                                  \
            _Pragma("unroll") for (int tt = 0; tt < NTL; ++tt)                                           \
                _Pragma("unroll") for (int cw = 0; cw < CBW; ++cw)                                       \
                    acc[cw][tt] = mfma32h(b[cw][u], a[tt][u], acc[cw][tt]);                              \
    }
    const int nfull = (k1 - k0) / UNR;
    int kb = k0;
    if (nfull > 0) {
        const int last = k0 + (nfull - 1) * UNR;
        EF_DN_LOAD(bA, aA, kb)
        EF_DN_LOAD(bB, aB, min(kb + UNR, last))
        int c = 0;
        for (; c + 3 <= nfull; c += 3) {
            EF_DN_LOAD(bC, aC, kb + 2 * UNR)
            EF_DN_COMPUTE(bA, aA)
            EF_DN_LOAD(bA, aA, min(kb + 3 * UNR, last))
            EF_DN_COMPUTE(bB, aB)
            EF_DN_LOAD(bB, aB, min(kb + 4 * UNR, last))
            EF_DN_COMPUTE(bC, aC)
            kb += 3 * UNR;
        }
        if (c < nfull) {
            EF_DN_COMPUTE(bA, aA)
            kb += UNR;
        }
        if (c + 1 < nfull) {
            EF_DN_COMPUTE(bB, aB)
            kb += UNR;
        }
    }
    for (; kb < k1; ++kb) {
#pragma unroll
        for (int cw = 0; cw < CBW; ++cw) {
            const u32x4_t b = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4_t *>(w2 + cw * cb_stride + (size_t)kb * 64));
#pragma unroll
            for (int tt = 0; tt < NTL; ++tt)
                acc[cw][tt] = mfma32h(b, *reinterpret_cast<const u32x4_t *>(a0 + ((size_t)tt * nkb + kb) * 64),
                                      acc[cw][tt]);
        }
    }
#undef EF_DN_LOAD
#undef EF_DN_COMPUTE
}

// ------------------------------------------------------------------------------------------
// second half: Y = act W2^T.  A workgroup owns (group, pass of TT token tiles, CBW*32 output
// columns, one of `ksg` K-slices); its four waves split that slice again and are summed in a fixed
// order, (p0 + p2) + (p1 + p3), through LDS.  Each K-slice writes its own partial Y plane; the
// un-permute sums the planes in order.  The product is formed transposed (W2 fragment first: the operand
// layouts are mirror images), so a lane ends with one token and groups of four consecutive output columns:
// 16-byte LDS accesses in the reduction and 16-byte stores to Y.  Both operands fp16 (see mfma32h).
// ------------------------------------------------------------------------------------------
template <int TT>
__global__ __launch_bounds__(256, 2) void ffn_down_kernel(GroupTable gt, const uint4 *__restrict__ act,
                                                       float *__restrict__ Y, int d, int ksg,
                                                       long long y_plane) {
    constexpr int CBW = kDownColBlocks;
    constexpr int UNR = TT > 2 ? 1 : 2;
    constexpr int TH = TT > 2 ? 2 : TT;          // token tiles per round of the epilogue (LDS budget)
    constexpr int REGION = CBW * TH * 4 * 64;    // 16-byte units of one wave's partial of one round
    __shared__ __attribute__((aligned(16))) float4 red[4 * REGION];
    const int wg = blockIdx.x;
    int grp = 0;
    while (grp + 1 < gt.n_groups && gt.wg_start[grp + 1] <= wg) ++grp;
    const int local = wg - gt.wg_start[grp];
    const int ncbw = (d >> 5) / CBW;
    const int kslice = local % ksg;
    const int cb0 = ((local / ksg) % ncbw) * CBW, pass = (local / ksg) / ncbw;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int F = gt.F[grp];
    const int nkb = F >> 4;
    const int part = kslice * 4 + wave, nparts = ksg * 4;
    const int k0 = (int)((long long)part * nkb / nparts), k1 = (int)((long long)(part + 1) * nkb / nparts);
    int ntl = gt.n_tiles[grp] - pass * TT;
    if (ntl > TT) ntl = TT;
    const size_t cb_stride = (size_t)nkb * 64;
    const uint4 *w2 = reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(gt.blob[grp]) +
                                                      (size_t)4 * d * F) + (size_t)cb0 * cb_stride + lane;
    const uint4 *a0 = act + gt.act_off[grp] + (size_t)(pass * TT) * nkb * 64 + lane;

    floatx16 acc[CBW][TT];
#pragma unroll
    for (int cw = 0; cw < CBW; ++cw)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) zero16(acc[cw][tt]);

    if (TT == 1 || ntl == 1) down_stream<TT, 1, CBW, UNR>(w2, cb_stride, a0, nkb, k0, k1, acc);
    else if (TT == 2 || ntl == 2) down_stream<TT, 2, CBW, UNR>(w2, cb_stride, a0, nkb, k0, k1, acc);
    else if (ntl == 3) down_stream<TT, (TT > 2 ? 3 : TT), CBW, UNR>(w2, cb_stride, a0, nkb, k0, k1, acc);
    else down_stream<TT, TT, CBW, UNR>(w2, cb_stride, a0, nkb, k0, k1, acc);

    // The four waves' partial tiles meet in LDS; every wave then sums a quarter of the tile in the fixed
    // order (p0 + p2) + (p1 + p3) and stores that quarter, so the adds and the stores of the epilogue run on
    // all four waves instead of a three-step tree that leaves one wave to store everything.  Passes of four
    // token tiles take two such rounds of two tiles (the partials of all four would not fit the LDS budget).
    // A lane holds token lane % 32 and, per accumulator quad q, output columns 8q + 4 (lane / 32) .. + 3.
    const int g = lane >> 5;
    float *Yp = Y + (size_t)kslice * y_plane;
    constexpr int UNITS = CBW * TH * 4;           // 64-lane slices of 16 bytes of a round's tile; a quarter per wave
    static_assert(UNITS % 4 == 0, "the tile is dealt to four waves");
#pragma unroll
    for (int round = 0; round < TT / TH; ++round) {
        if (round > 0) __syncthreads();           // the previous round's partials have been read
#pragma unroll
        for (int cw = 0; cw < CBW; ++cw)
#pragma unroll
            for (int th = 0; th < TH; ++th)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const floatx16 &v = acc[cw][round * TH + th];
                    red[wave * REGION + ((cw * TH + th) * 4 + q) * 64 + lane] =
                        make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
                }
        __syncthreads();
#pragma unroll
        for (int qq = 0; qq < UNITS / 4; ++qq) {
            const int u = wave * (UNITS / 4) + qq;
            const int cw = u / (TH * 4), tt = round * TH + (u / 4) % TH, q = u % 4;
            const float4 *r = red + u * 64 + lane;
            const float4 p0 = r[0], p1 = r[REGION], p2 = r[2 * REGION], p3 = r[3 * REGION];
            const float4 sum = make_float4((p0.x + p2.x) + (p1.x + p3.x), (p0.y + p2.y) + (p1.y + p3.y),
                                           (p0.z + p2.z) + (p1.z + p3.z), (p0.w + p2.w) + (p1.w + p3.w));
            if (tt >= ntl) continue;
            const int col = (cb0 + cw) * 32 + 8 * q + 4 * g;
            const int tl = (pass * TT + tt) * kTile + (lane & 31);
            if (tl < gt.count[grp]) *reinterpret_cast<float4 *>(Yp + (size_t)(gt.row_offset[grp] + tl) * d + col) = sum;
        }
    }
}

hipError_t launch_ffn_down(const GroupTable &gt, int total_wgs, int tiles_per_pass, int ksg, const void *act,
                           float *y, long long y_plane, int d, hipStream_t s) {
    if (total_wgs <= 0) return hipSuccess;
    const uint4 *a = reinterpret_cast<const uint4 *>(act);
    if (tiles_per_pass == 1)
        hipLaunchKernelGGL((ffn_down_kernel<1>), dim3(total_wgs), dim3(256), 0, s, gt, a, y, d, ksg, y_plane);
    else if (tiles_per_pass == 2)
        hipLaunchKernelGGL((ffn_down_kernel<2>), dim3(total_wgs), dim3(256), 0, s, gt, a, y, d, ksg, y_plane);
    else if (tiles_per_pass == 4)
        hipLaunchKernelGGL((ffn_down_kernel<4>), dim3(total_wgs), dim3(256), 0, s, gt, a, y, d, ksg, y_plane);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// weighted un-permute: out[t] = sum_j w[t,j] * (sum over the K-slice planes of expert ids[t,j] of Y[inv_perm[t*k+j]])
//                               (+ the dense shared FFN's row of token t)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ Y, PlaneTable planes, long long y_plane,
                                                      const float *__restrict__ w, const int32_t *__restrict__ ids,
                                                      const int32_t *__restrict__ inv_perm, int T, int k, int d,
                                                      long long shared_row0, float *__restrict__ out) {
    const int t = blockIdx.x;
    const int c = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (c >= d) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < k; ++j) {
        const int a = t * k + j;
        const float wj = w[a];
        const int np = planes.routed[ids[a]];
        const float *row = Y + (size_t)inv_perm[a] * d + c;
        float4 y = *reinterpret_cast<const float4 *>(row);
        for (int p = 1; p < np; ++p) {
            const float4 z = *reinterpret_cast<const float4 *>(row + (size_t)p * y_plane);
            y.x += z.x; y.y += z.y; y.z += z.z; y.w += z.w;
        }
        acc.x += wj * y.x; acc.y += wj * y.y; acc.z += wj * y.z; acc.w += wj * y.w;
    }
    if (shared_row0 >= 0) {
        const float *row = Y + (size_t)(shared_row0 + t) * d + c;
        float4 y = *reinterpret_cast<const float4 *>(row);
        for (int p = 1; p < planes.shared; ++p) {
            const float4 z = *reinterpret_cast<const float4 *>(row + (size_t)p * y_plane);
            y.x += z.x; y.y += z.y; y.z += z.z; y.w += z.w;
        }
        acc.x += y.x; acc.y += y.y; acc.z += y.z; acc.w += y.w;
    }
    *reinterpret_cast<float4 *>(out + (size_t)t * d + c) = acc;
}

// `done` (may be null): an event that completes with this kernel.  It rides on the kernel's own completion
// signal, which costs the stream nothing, where a separate event record behind the kernel costs 2-3 us.
hipError_t launch_combine(const float *y, const PlaneTable &planes, long long y_plane, const float *w,
                          const int32_t *ids, const int32_t *inv_perm, int T, int k, int d, long long shared_row0,
                          float *out, hipEvent_t done, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    if (done)
        hipExtLaunchKernelGGL(combine_kernel, dim3(T, (d + 1023) / 1024), dim3(256), 0, s, nullptr, done, 0, y, planes,
                              y_plane, w, ids, inv_perm, T, k, d, shared_row0, out);
    else
        hipLaunchKernelGGL(combine_kernel, dim3(T, (d + 1023) / 1024), dim3(256), 0, s, y, planes, y_plane, w, ids,
                           inv_perm, T, k, d, shared_row0, out);
    return hipGetLastError();
}

}  // namespace ef
