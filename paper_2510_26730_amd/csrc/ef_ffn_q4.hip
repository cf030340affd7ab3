// Grouped SwiGLU expert FFN with 4-bit expert weights (w = (q - 8) * s, one bf16 scale per matrix row
// and group of 128 inputs), for groups of any size.
//
// With 4-bit weights a byte of weights meets four times as many token bytes as with bf16, so the
// re-reads of the token (or activation) fragments, not the weight stream, would bound a kernel in
// which every wave fetches its own copy.  Here the four waves of a workgroup work on the same
// tokens and the same K range (different weight rows / output columns): each wave fetches a quarter
// of the token fragments of a stage, the workgroup shares them through a small LDS ring, and only
// the weight stream is private to a wave.  A stage is one "quad" of weights per matrix (four
// k-steps, 64 inputs); weight quads, scales and the wave's share of token fragments sit in a
// register ring of kDepth stages filled that many stages ahead with unconditional loads (clamped
// addresses), one barrier per stage.  Dequantisation happens on the operand fragment, where a lane
// holds one matrix row (column) and therefore needs one scale per group, and in fp16: the codes
// become the fp16 numbers 1024 + q (or 64 + q) by one bit operation, a packed subtraction gives q - 8 exactly and
// a packed multiplication (q - 8) * s: three vector instructions per pair of weights where an fp32
// route costs seven, which is what keeps these kernels on the memory side of the balance.  The
// matrix cores therefore run in fp16 (fp32 accumulation): the packed tokens of a 4-bit context and
// the intermediate activations are fp16 fragments (tokens convert exactly from bf16 for
// 2^-14 <= |x| < 65504).
#include <algorithm>

#include "ef_device.h"
#include "ef_kernels.h"

namespace ef {

typedef _Float16 q4_half2 __attribute__((ext_vector_type(2)));
typedef _Float16 q4_half8 __attribute__((ext_vector_type(8)));

// dword x = eight codes of one lane for one k-step, code t at bits 4*(t/2) + 16*(t%2);
// s2 = the lane's scale in both halves.  Codes in mantissa bits 0..3 under the exponent of 1024 (unit in the
// last place 1) are the fp16 numbers 1024 + q, codes in mantissa bits 4..7 under the exponent of 64 (unit
// 1/16) are 64 + q: x & 0x000F000F | 0x64006400 is the pair t = 0, 1, x & 0x00F000F0 | 0x54005400 the pair
// t = 2, 3, and x >> 8 gives the other two pairs the same way (one shift per dword instead of three).  Minus
// 1032 (72) is q - 8 exactly; times s rounds once to fp16 (11 significant bits for a 4-bit integer times an
// 8-bit mantissa: relative error <= 2^-12).
__device__ __forceinline__ u32x4_t dequant_q4(uint32_t x, q4_half2 s2) {
    const q4_half2 off_lo = {(_Float16)-1032.f, (_Float16)-1032.f}, off_hi = {(_Float16)-72.f, (_Float16)-72.f};
    const uint32_t y = x >> 8;
    // the masks live in vector registers the compiler cannot see through: "and" and "or" then fit one
    // three-operand instruction (it takes a single literal, here the exponent pattern)
    uint32_t m_lo = 0x000F000Fu, m_hi = 0x00F000F0u;
    asm("" : "+v"(m_lo));
    asm("" : "+v"(m_hi));
    const uint32_t pr[4] = {(x & m_lo) | 0x64006400u, (x & m_hi) | 0x54005400u,
                            (y & m_lo) | 0x64006400u, (y & m_hi) | 0x54005400u};
    u32x4_t out;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const q4_half2 w = (__builtin_bit_cast(q4_half2, pr[p]) + ((p & 1) ? off_hi : off_lo)) * s2;
        out[p] = __builtin_bit_cast(uint32_t, w);
    }
    return out;
}

// bf16 scale (exact in fp16 for 2^-14 <= |s| < 65504) in both halves of a packed pair
__device__ __forceinline__ q4_half2 q4_scale(uint16_t b) {
    const _Float16 h = (_Float16)__builtin_bit_cast(float, (uint32_t)b << 16);
    return q4_half2{h, h};
}

// register ring: stages in flight per wave (four were measured slower than six with two token tiles per pass
// and one wave per SIMD)
template <int TT> constexpr int q4_depth() { return 6; }
constexpr int kQ4Lds = 4;     // LDS ring of shared token / activation fragments (stages)

// ------------------------------------------------------------------------------------------
// first half: act = silu(X W1^T) * (X W3^T).  Workgroup = (group, pass of TT token tiles, four
// consecutive 32-row blocks of F), wave = one row block and one of KH halves of the K range.
//
// OCC = 2: registers for two workgroups per compute unit (launches with more workgroups than compute units).
// KH = 2: eight waves, two per SIMD.  A wave issues in order, so with one wave per SIMD its dequantising
// vector instructions (about 40 % of its cycles), its waits for LDS and barriers (25 %) and its issue stalls
// add up; a second wave on the SIMD fills them.  A launch rarely has enough row blocks for that (two Mixtral-
// shaped experts: 896 for 1024 SIMDs), so the second wave comes from the K range: the four waves of a half
// share their token fragments as before (a ring per half), and at the end the upper half hands its partial
// sums to the lower one through LDS (the ring's space).
// ------------------------------------------------------------------------------------------
template <int TT, int KH, int OCC>
__global__ __launch_bounds__(256 * KH, OCC) void ffn_gate_up_q4_kernel(GroupTable gt, const uint4 *__restrict__ xp,
                                                                       uint4 *__restrict__ act, int d) {
    constexpr int D = (KH == 2 || OCC == 2) ? 4 : q4_depth<TT>();   // 3 and 6 measured slower with two waves per SIMD
    __shared__ __attribute__((aligned(16))) u32x4_t xs[KH][kQ4Lds][TT * 4][64];
    const int wg = blockIdx.x;
    int grp = 0;
    while (grp + 1 < gt.n_groups && gt.wg_start[grp + 1] <= wg) ++grp;
    const int local = wg - gt.wg_start[grp];
    const int F = gt.F[grp];
    const int rbw = (F >> 5) >> 2;               // workgroups per pass (F is a multiple of 128)
    const int pass = local / rbw;
    const int wave = (threadIdx.x >> 6) & 3, kh = threadIdx.x >> 8, lane = threadIdx.x & 63;
    const int rb = (local % rbw) * 4 + wave;
    int ntl = gt.n_tiles[grp] - pass * TT;
    if (ntl > TT) ntl = TT;
    const int nkb = d >> 4, nq = d >> 6;
    // stages [k0, k0 + nloc) of this wave's half (the launcher checks that the halves are equal: every wave
    // passes the same barriers)
    const int nloc = nq / KH, k0 = kh * nloc;

    const char *blob = reinterpret_cast<const char *>(gt.blob[grp]);
    const uint4 *w13 = reinterpret_cast<const uint4 *>(blob) + (size_t)rb * nq * 128 + lane;
    const uint16_t *sA = reinterpret_cast<const uint16_t *>(blob + (size_t)3 * d * F / 2) +
                         (size_t)rb * (d >> 7) * 64 + (lane & 31);
    // this wave's share of the token fragments of a stage: k-step `wave` of each tile (tiles past the
    // group's last one repeat it; their results are dropped)
    const uint4 *xsrc[TT];
#pragma unroll
    for (int u = 0; u < TT; ++u)
        xsrc[u] = xp + (size_t)(gt.tile_start[grp] + pass * TT + min(u, ntl - 1)) * nkb * 64 + lane;

    floatx16 G[TT], U[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) { zero16(G[tt]); zero16(U[tt]); }

    u32x4_t qa[D], qb[D], xr[D][TT];
    uint16_t sa[D], sb[D];
#define EF_Q4U_LOAD(slot, kq)                                                                             \
    {                                                                                                     \
        const int kc_ = k0 + min((kq), nloc - 1);                                                         \
        _Pragma("unroll") for (int u = 0; u < TT; ++u)                                                    \
            xr[slot][u] = *reinterpret_cast<const u32x4_t *>(xsrc[u] + (size_t)(4 * kc_ + wave) * 64);    \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        qa[slot] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(w13 + (size_t)kc_ * 128));       \
        qb[slot] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(w13 + (size_t)kc_ * 128 + 64));  \
        sa[slot] = sA[(size_t)(kc_ >> 1) * 64];                                                           \
        sb[slot] = sA[(size_t)(kc_ >> 1) * 64 + 32];                                                      \
    }
#define EF_Q4U_SHARE(slot, st)                                                                            \
    {                                                                                                     \
        _Pragma("unroll") for (int u = 0; u < TT; ++u) xs[kh][(st) & (kQ4Lds - 1)][u * 4 + wave][lane] = xr[slot][u]; \
    }
    // The MFMAs of a k-step are issued between the vector instructions that dequantise the next
    // k-step's fragments (one MFMA, then a share of the ~40 vector instructions), so the matrix
    // cores work while the wave converts: a wave issues in order and has the SIMD to itself, nothing
    // else would overlap the two.
#define EF_Q4U_COMPUTE(slot, st)                                                                          \
    {                                                                                                     \
        const q4_half2 f1_ = q4_scale(sa[slot]), f3_ = q4_scale(sb[slot]);                                \
        u32x4_t xb_[TT][4];                                                                               \
        _Pragma("unroll") for (int tt = 0; tt < TT; ++tt)                                                 \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) xb_[tt][j] = xs[kh][(st) & (kQ4Lds - 1)][tt * 4 + j][lane]; \
        u32x4_t a1_ = dequant_q4(qa[slot][0], f1_), a3_ = dequant_q4(qb[slot][0], f3_);                   \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                   \
            u32x4_t n1_ = a1_, n3_ = a3_;                                                                 \
            if (j < 3) { n1_ = dequant_q4(qa[slot][j + 1], f1_); n3_ = dequant_q4(qb[slot][j + 1], f3_); } \
            _Pragma("unroll") for (int tt = 0; tt < TT; ++tt) {                                           \
                G[tt] = mfma32h(a1_, xb_[tt][j], G[tt]);                                                  \
                U[tt] = mfma32h(a3_, xb_[tt][j], U[tt]);                                                  \
            }                                                                                             \
            if (j < 3) {                                                                                  \
                _Pragma("unroll") for (int q_ = 0; q_ < 2 * TT; ++q_) {                                   \
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                    \
                    __builtin_amdgcn_sched_group_barrier(0x002, 40 / (2 * TT), 0);                        \
                }                                                                                         \
            }                                                                                             \
            a1_ = n1_; a3_ = n3_;                                                                         \
        }                                                                                                 \
    }
    // one stage: hand the next stage's token fragments to the workgroup, compute this one, refill the
    // register slot just used, barrier (the next stage's fragments are visible; this stage's LDS
    // buffer is overwritten three stages from now)
#define EF_Q4U_STAGE(slot, next_slot, st)                                                                 \
    {                                                                                                     \
        EF_Q4U_SHARE(next_slot, (st) + 1)                                                                 \
        EF_Q4U_COMPUTE(slot, st)                                                                          \
        EF_Q4U_LOAD(slot, (st) + D)                                                                       \
        __syncthreads();                                                                                  \
    }
#pragma unroll
    for (int ring_ = 0; ring_ < D; ++ring_) EF_Q4U_LOAD(ring_, ring_)
    EF_Q4U_SHARE(0, 0)
    __syncthreads();
    int st = 0;
    for (; st + D <= nloc; st += D) {
#pragma unroll
        for (int ring_ = 0; ring_ < D; ++ring_) EF_Q4U_STAGE(ring_, (ring_ + 1) % D, st + ring_)
    }
#pragma unroll
    for (int ring_ = 0; ring_ < D - 1; ++ring_)
        if (st + ring_ < nloc) EF_Q4U_STAGE(ring_, ring_ + 1, st + ring_)
#undef EF_Q4U_LOAD
#undef EF_Q4U_SHARE
#undef EF_Q4U_COMPUTE
#undef EF_Q4U_STAGE

    if constexpr (KH == 2) {
        // every stage ends with a barrier: the ring is no longer read.  Lower half + upper half, in this order.
        float4 *red = reinterpret_cast<float4 *>(&xs[0][0][0][0]) + (size_t)wave * (2 * TT * 4) * 64 + lane;
        static_assert(sizeof(xs) >= (size_t)4 * (2 * TT * 4) * 64 * sizeof(float4), "partial sums fit the ring's space");
        if (kh == 1) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    red[((tt * 2) * 4 + q) * 64] = make_float4(G[tt][4 * q], G[tt][4 * q + 1], G[tt][4 * q + 2], G[tt][4 * q + 3]);
                    red[((tt * 2 + 1) * 4 + q) * 64] = make_float4(U[tt][4 * q], U[tt][4 * q + 1], U[tt][4 * q + 2], U[tt][4 * q + 3]);
                }
        }
        __syncthreads();
        if (kh == 1) return;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 g = red[((tt * 2) * 4 + q) * 64], u = red[((tt * 2 + 1) * 4 + q) * 64];
                G[tt][4 * q] += g.x; G[tt][4 * q + 1] += g.y; G[tt][4 * q + 2] += g.z; G[tt][4 * q + 3] += g.w;
                U[tt][4 * q] += u.x; U[tt][4 * q + 1] += u.y; U[tt][4 * q + 2] += u.z; U[tt][4 * q + 3] += u.w;
            }
    }
    // a lane holds 16 F-values of one token: the two paired-order fragments (fp16) the second half consumes
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
                pk[q] = __builtin_bit_cast(uint32_t, q4_half2{(_Float16)v0, (_Float16)v1});
            }
            dst[(size_t)s * 64] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        }
    }
}

hipError_t launch_ffn_gate_up_q4(const GroupTable &gt, int total_wgs, int tiles_per_pass, const void *xp, void *act,
                                 int d, hipStream_t s) {
    if (total_wgs <= 0) return hipSuccess;
    if (d % 128 != 0) return hipErrorInvalidValue;
    for (int i = 0; i < gt.n_groups; ++i)
        if (gt.F[i] % 128 != 0 || gt.n_tiles[i] <= 0 ||
            gt.wg_start[i + 1] - gt.wg_start[i] != ffn_gate_up_q4_wgs(gt.F[i], gt.n_tiles[i], tiles_per_pass))
            return hipErrorInvalidValue;
    if (gt.wg_start[gt.n_groups] != total_wgs) return hipErrorInvalidValue;
    const uint4 *x = reinterpret_cast<const uint4 *>(xp);
    uint4 *a = reinterpret_cast<uint4 *>(act);
    // two K halves per workgroup when each half keeps a few stages (d / 64 stages in all, an even number)
    const bool halves = (d >> 6) % 2 == 0 && (d >> 6) >= 8;
    // more workgroups than compute units: two of them per unit instead (whole K range each, the short register ring);
    // their waves stall at different times, where the halves of one workgroup meet at the same barriers
    // (seven Mixtral-shaped experts: 127 against 135 us, Qwen-shaped batch 52 against 60 us)
    const bool many = total_wgs > 256;
    if (tiles_per_pass == 1 && many) hipLaunchKernelGGL((ffn_gate_up_q4_kernel<1, 1, 2>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else if (tiles_per_pass == 2 && many) hipLaunchKernelGGL((ffn_gate_up_q4_kernel<2, 1, 2>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else if (tiles_per_pass == 1 && halves) hipLaunchKernelGGL((ffn_gate_up_q4_kernel<1, 2, 1>), dim3(total_wgs), dim3(512), 0, s, gt, x, a, d);
    else if (tiles_per_pass == 1) hipLaunchKernelGGL((ffn_gate_up_q4_kernel<1, 1, 1>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else if (tiles_per_pass == 2 && halves) hipLaunchKernelGGL((ffn_gate_up_q4_kernel<2, 2, 1>), dim3(total_wgs), dim3(512), 0, s, gt, x, a, d);
    else if (tiles_per_pass == 2) hipLaunchKernelGGL((ffn_gate_up_q4_kernel<2, 1, 1>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// second half: Y = act W2^T.  Workgroup = (group, pass of TT token tiles, eight consecutive
// 32-column blocks of d, one of `ksg` K-slices), wave = two column blocks.  Activations are operand
// A (rows = tokens), shared through LDS; W2 quads operand B (a lane holds one output column).
// Each K-slice writes its own partial Y plane; the un-permute sums the planes in order.
// ------------------------------------------------------------------------------------------
template <int TT>
__global__ __launch_bounds__(256, 1) void ffn_down_q4_kernel(GroupTable gt, const uint4 *__restrict__ act,
                                                             float *__restrict__ Y, int d, int ksg,
                                                             long long y_plane) {
    constexpr int D = q4_depth<TT>(), CBW = 2;
    __shared__ __attribute__((aligned(16))) u32x4_t as[kQ4Lds][TT * 4][64];
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
    const int nkb = F >> 4, nq = F >> 6;
    const int q0 = (int)((long long)kslice * nq / ksg), q1 = (int)((long long)(kslice + 1) * nq / ksg);
    int ntl = gt.n_tiles[grp] - pass * TT;
    if (ntl > TT) ntl = TT;

    const char *blob = reinterpret_cast<const char *>(gt.blob[grp]);
    const size_t qstride = (size_t)nq * 64, sstride = (size_t)(F >> 7) * 32;
    const uint4 *w2q = reinterpret_cast<const uint4 *>(blob + (size_t)d * F) + (size_t)cbc * qstride + lane;
    const uint16_t *sB = reinterpret_cast<const uint16_t *>(blob + (size_t)3 * d * F / 2 + (size_t)d * F / 32) +
                         (size_t)cbc * sstride + (lane & 31);
    const uint4 *asrc[TT];
#pragma unroll
    for (int u = 0; u < TT; ++u)
        asrc[u] = act + gt.act_off[grp] + (size_t)(pass * TT + min(u, ntl - 1)) * nkb * 64 + lane;

    floatx16 acc[CBW][TT];
#pragma unroll
    for (int cw = 0; cw < CBW; ++cw)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) zero16(acc[cw][tt]);

    u32x4_t qw[D][CBW], ar[D][TT];
    uint16_t sc[D][CBW];
#define EF_Q4D_LOAD(slot, kq)                                                                             \
    {                                                                                                     \
        const int kc_ = min((kq), nq - 1);                                                                \
        _Pragma("unroll") for (int u = 0; u < TT; ++u)                                                    \
            ar[slot][u] = *reinterpret_cast<const u32x4_t *>(asrc[u] + (size_t)(4 * kc_ + wave) * 64);    \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        _Pragma("unroll") for (int cw = 0; cw < CBW; ++cw) {                                              \
            qw[slot][cw] = __builtin_nontemporal_load(                                                    \
                reinterpret_cast<const u32x4_t *>(w2q + cw * qstride + (size_t)kc_ * 64));                \
            sc[slot][cw] = sB[cw * sstride + (size_t)(kc_ >> 1) * 32];                                    \
        }                                                                                                 \
    }
#define EF_Q4D_SHARE(slot, st)                                                                            \
    {                                                                                                     \
        _Pragma("unroll") for (int u = 0; u < TT; ++u) as[(st) & (kQ4Lds - 1)][u * 4 + wave][lane] = ar[slot][u]; \
    }
    // as in the first half: the MFMAs of one weight fragment are issued between the vector
    // instructions that dequantise the next one
#define EF_Q4D_COMPUTE(slot, st)                                                                          \
    {                                                                                                     \
        u32x4_t af_[TT][4];                                                                               \
        _Pragma("unroll") for (int tt = 0; tt < TT; ++tt)                                                 \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) af_[tt][j] = as[(st) & (kQ4Lds - 1)][tt * 4 + j][lane]; \
        q4_half2 f_[CBW];                                                                                 \
        _Pragma("unroll") for (int cw = 0; cw < CBW; ++cw) f_[cw] = q4_scale(sc[slot][cw]);               \
        u32x4_t w_ = dequant_q4(qw[slot][0][0], f_[0]);                                                   \
        _Pragma("unroll") for (int idx = 0; idx < CBW * 4; ++idx) {                                       \
            const int cw = idx >> 2, j = idx & 3;                                                         \
            u32x4_t n_ = w_;                                                                              \
            if (idx + 1 < CBW * 4) n_ = dequant_q4(qw[slot][(idx + 1) >> 2][(idx + 1) & 3], f_[(idx + 1) >> 2]); \
            _Pragma("unroll") for (int tt = 0; tt < TT; ++tt) acc[cw][tt] = mfma32h(w_, af_[tt][j], acc[cw][tt]); \
            if (idx + 1 < CBW * 4) {                                                                      \
                _Pragma("unroll") for (int q_ = 0; q_ < TT; ++q_) {                                       \
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                    \
                    __builtin_amdgcn_sched_group_barrier(0x002, 20 / TT, 0);                              \
                }                                                                                         \
            }                                                                                             \
            w_ = n_;                                                                                      \
        }                                                                                                 \
    }
#define EF_Q4D_STAGE(slot, next_slot, st)                                                                 \
    {                                                                                                     \
        EF_Q4D_SHARE(next_slot, (st) + 1)                                                                 \
        EF_Q4D_COMPUTE(slot, st)                                                                          \
        EF_Q4D_LOAD(slot, (st) + D)                                                                       \
        __syncthreads();                                                                                  \
    }
#pragma unroll
    for (int ring_ = 0; ring_ < D; ++ring_) EF_Q4D_LOAD(ring_, q0 + ring_)
    EF_Q4D_SHARE(0, q0)
    __syncthreads();
    int st = q0;
    for (; st + D <= q1; st += D) {
#pragma unroll
        for (int ring_ = 0; ring_ < D; ++ring_) EF_Q4D_STAGE(ring_, (ring_ + 1) % D, st + ring_)
    }
#pragma unroll
    for (int ring_ = 0; ring_ < D - 1; ++ring_)
        if (st + ring_ < q1) EF_Q4D_STAGE(ring_, ring_ + 1, st + ring_)
#undef EF_Q4D_LOAD
#undef EF_Q4D_SHARE
#undef EF_Q4D_COMPUTE
#undef EF_Q4D_STAGE

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

hipError_t launch_ffn_down_q4(const GroupTable &gt, int total_wgs, int tiles_per_pass, int ksg, const void *act,
                              float *y, long long y_plane, int d, hipStream_t s) {
    if (total_wgs <= 0) return hipSuccess;
    if (d % 128 != 0 || ksg < 1) return hipErrorInvalidValue;
    for (int i = 0; i < gt.n_groups; ++i)
        if (gt.F[i] % 128 != 0 || gt.n_tiles[i] <= 0 ||
            gt.wg_start[i + 1] - gt.wg_start[i] != ffn_down_q4_wgs(d, gt.n_tiles[i], tiles_per_pass, ksg))
            return hipErrorInvalidValue;
    if (gt.wg_start[gt.n_groups] != total_wgs) return hipErrorInvalidValue;
    const uint4 *a = reinterpret_cast<const uint4 *>(act);
    if (tiles_per_pass == 1)
        hipLaunchKernelGGL((ffn_down_q4_kernel<1>), dim3(total_wgs), dim3(256), 0, s, gt, a, y, d, ksg, y_plane);
    else if (tiles_per_pass == 2)
        hipLaunchKernelGGL((ffn_down_q4_kernel<2>), dim3(total_wgs), dim3(256), 0, s, gt, a, y, d, ksg, y_plane);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// 4-bit blob -> 16-bit blob of the bf16 layout holding the fp16 numbers (q - 8) * s.
// One wave per quad position: (rb, kq) of W1 and W3 together (two quads in, eight fragments out), then
// (cb, kq) of W2 (one quad in, four fragments out).  A quad's dword j of lane l is the fragment of k-step
// 4*kq + j of the same lane, so reads and writes are whole 1 KiB rows of 64 lanes.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dequant_q4_kernel(DequantTable t, int d) {
    const int grp = blockIdx.y;
    const int F = t.F[grp];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int nq = d >> 6, nq2 = F >> 6, nkb = d >> 4, nkb2 = F >> 4;
    const int nA = (F >> 5) * nq, nB = (d >> 5) * nq2;
    const int u = blockIdx.x * 4 + wave;
    if (u >= nA + nB) return;
    const char *blob = reinterpret_cast<const char *>(t.src[grp]);
    uint4 *out = reinterpret_cast<uint4 *>(t.dst[grp]);
    if (u < nA) {
        const int rb = u / nq, kq = u - rb * nq;
        const uint4 *q = reinterpret_cast<const uint4 *>(blob) + ((size_t)rb * nq + kq) * 128 + lane;
        const uint16_t *sc = reinterpret_cast<const uint16_t *>(blob + (size_t)3 * d * F / 2) +
                             ((size_t)rb * (d >> 7) + (kq >> 1)) * 64 + (lane & 31);
        const uint4 q1 = q[0], q3 = q[64];
        const q4_half2 f1 = q4_scale(sc[0]), f3 = q4_scale(sc[32]);
        uint4 *o1 = out + ((size_t)rb * 2 * nkb + 4 * kq) * 64 + lane;
        uint4 *o3 = o1 + (size_t)nkb * 64;
        const uint32_t c1[4] = {q1.x, q1.y, q1.z, q1.w}, c3[4] = {q3.x, q3.y, q3.z, q3.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u32x4_t a = dequant_q4(c1[j], f1), b = dequant_q4(c3[j], f3);
            o1[(size_t)j * 64] = make_uint4(a[0], a[1], a[2], a[3]);
            o3[(size_t)j * 64] = make_uint4(b[0], b[1], b[2], b[3]);
        }
    } else {
        const int v = u - nA;
        const int cb = v / nq2, kq = v - cb * nq2;
        const uint4 *q = reinterpret_cast<const uint4 *>(blob + (size_t)d * F) + ((size_t)cb * nq2 + kq) * 64 + lane;
        const uint16_t *sc = reinterpret_cast<const uint16_t *>(blob + (size_t)3 * d * F / 2 + (size_t)d * F / 32) +
                             ((size_t)cb * (F >> 7) + (kq >> 1)) * 32 + (lane & 31);
        const uint4 q2 = q[0];
        const q4_half2 f2 = q4_scale(sc[0]);
        uint4 *o2 = reinterpret_cast<uint4 *>(reinterpret_cast<char *>(out) + (size_t)4 * d * F) +
                    ((size_t)cb * nkb2 + 4 * kq) * 64 + lane;
        const uint32_t c2[4] = {q2.x, q2.y, q2.z, q2.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u32x4_t a = dequant_q4(c2[j], f2);
            o2[(size_t)j * 64] = make_uint4(a[0], a[1], a[2], a[3]);
        }
    }
}

hipError_t launch_dequant_q4(const DequantTable &t, int d, hipStream_t s) {
    if (t.n <= 0) return hipSuccess;
    if (t.n > kMaxGroups || d <= 0 || d % 128 != 0) return hipErrorInvalidValue;
    int units = 0;
    for (int i = 0; i < t.n; ++i) {
        if (t.F[i] <= 0 || t.F[i] % 128 != 0 || !t.src[i] || !t.dst[i]) return hipErrorInvalidValue;
        units = std::max(units, (t.F[i] / 32) * (d / 64) + (d / 32) * (t.F[i] / 64));
    }
    hipLaunchKernelGGL(dequant_q4_kernel, dim3((units + 3) / 4, t.n), dim3(256), 0, s, t, d);
    return hipGetLastError();
}

}  // namespace ef
