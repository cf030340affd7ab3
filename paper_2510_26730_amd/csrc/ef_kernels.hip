// gfx950 kernels of the cache-aware MoE-layer hot path.
//
// Matrix-core tiles use v_mfma_f32_32x32x16_bf16 (wave64): operand A is 32 rows x 16 k, operand B
// is 16 k x 32 columns, each lane l = 32*g + i carries 8 bf16 of row/column i, k-group g; the
// accumulator lane l holds column l%32 and rows 8*(v/4) + 4*(l/32) + v%4 for v = 0..15.
// Every operand fragment is therefore 64 lanes x 16 bytes = one contiguous 1 KiB read when the
// data is stored in fragment order (expert weights, packed tokens, activations).
#include "ef_kernels.h"

namespace ef {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// streaming (read-once) 16-byte load: keeps expert weights from displacing reused data in L2
__device__ __forceinline__ uint4 load_stream(const uint4 *p) {
    u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ floatx16 mfma32(uint4 a, uint4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// ------------------------------------------------------------------------------------------
// small fill (used instead of memset so that callers may capture the stream in a graph)
// ------------------------------------------------------------------------------------------
__global__ void fill_i32_kernel(int32_t *p, int n, int32_t v) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

hipError_t launch_fill_i32(int32_t *p, int n, int32_t v, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n, v);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// gate: logits of G gate matrices on one 32-token tile per workgroup, then per-token softmax,
// biased top-k, combine weights and per-tile expert counts.
//
// The four waves split the K dimension in 64-element chunks; lane (g,i) reads the 64 contiguous
// bytes [c*64 + 32*g, +32) elements of its row, which feed four MFMA steps (the k order inside a
// step is the same for both operands, so the sum is the plain dot product).
// ------------------------------------------------------------------------------------------
template <int NB>
__global__ __launch_bounds__(256) void gate_kernel(GateArgs a) {
    __shared__ float logits[kTile][NB * 32 + 1];
    __shared__ int cnt[kMaxGates * kMaxE];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 5, i = lane & 31;
    const int t0 = blockIdx.x * kTile;
    const int N = a.G * a.E;

    for (int x = tid; x < kMaxGates * kMaxE; x += 256) cnt[x] = 0;

    const bool tvalid = (t0 + i) < a.T;
    const uint4 *arow = reinterpret_cast<const uint4 *>(a.h + (size_t)(tvalid ? t0 + i : 0) * a.d);
    const uint4 *brow[NB];
    bool bvalid[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        int n = nb * 32 + i;
        bvalid[nb] = n < N;
        int gate = bvalid[nb] ? n / a.E : 0, e = bvalid[nb] ? n % a.E : 0;
        brow[nb] = reinterpret_cast<const uint4 *>(a.Wg[gate] + (size_t)e * a.d);
    }

    floatx16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0.f;

    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    const int nchunk = a.d >> 6;
    for (int c = wave; c < nchunk; c += 4) {
        const int off = c * 8 + g * 4;  // in uint4 units (8 bf16 each)
        uint4 av[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) av[m] = tvalid ? arow[off + m] : zero4;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            uint4 bv[4];
#pragma unroll
            for (int m = 0; m < 4; ++m) bv[m] = bvalid[nb] ? brow[nb][off + m] : zero4;
#pragma unroll
            for (int m = 0; m < 4; ++m) acc[nb] = mfma32(av[m], bv[m], acc[nb]);
        }
    }

    // fixed-order reduction of the four K-partials (wave 0, 1, 2, 3) through LDS
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int row = 8 * (v >> 2) + 4 * g + (v & 3);
                    if (w == 0) logits[row][nb * 32 + i] = acc[nb][v];
                    else logits[row][nb * 32 + i] += acc[nb][v];
                }
        }
        __syncthreads();
    }

    // per-token epilogue: a sub-group of W lanes (W = power of two >= E) owns one (token, gate)
    int W = 8;
    while (W < a.E) W <<= 1;
    const int per_wave = 64 / W;
    const int sub = lane / W, e = lane % W;
    const int total = kTile * a.G;
    const bool evalid = e < a.E;
    const float NEG_INF = -__builtin_inff();

    for (int base = wave * per_wave; base < total; base += 4 * per_wave) {
        const int task = base + sub;
        const int ti = task % kTile, gi = task / kTile;
        const int t = t0 + ti;
        const bool live = task < total && t < a.T;
        float z = NEG_INF;
        if (live && evalid) {
            z = logits[ti][gi * a.E + e];
            if (a.bias[gi]) z += a.bias[gi][e];
        }
        const bool want_w = (a.w != nullptr) && gi == 0;   // uniform per sub-group
        float p = 0.f;
        {
            float m = z;
            for (int s = W >> 1; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
            float ex = (live && evalid) ? expf(z - m) : 0.f;
            float sum = ex;
            for (int s = W >> 1; s >= 1; s >>= 1) sum += __shfl_xor(sum, s);
            p = live ? ex / sum : 0.f;
        }
        float sc = z;
        if (live && evalid) {
            if ((a.resident[gi] >> e) & 1ull) sc += a.beta;
            if (a.delta) {
                int req = a.tok2req ? a.tok2req[t] : 0;
                sc += a.delta[(size_t)req * a.delta_req_stride + gi * a.E + e];
            }
        }
        bool sel = false;
        float cur = sc;
        for (int r = 0; r < a.k; ++r) {
            float bv = cur;
            int bi = e;
            for (int s = W >> 1; s >= 1; s >>= 1) {
                float ov = __shfl_xor(bv, s);
                int oi = __shfl_xor(bi, s);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if (bi == e) { sel = true; cur = NEG_INF; }
        }
        sel = sel && live && evalid;
        const unsigned long long ball = __ballot(sel);
        const unsigned long long submask = (W == 64) ? ball : ((ball >> (sub * W)) & ((1ull << W) - 1ull));
        const int rank = __popcll(submask & ((1ull << e) - 1ull));
        float psel = sel ? p : 0.f;
        float psum = psel;
        for (int s = W >> 1; s >= 1; s >>= 1) psum += __shfl_xor(psum, s);
        if (sel) {
            a.ids[((size_t)gi * a.T + t) * a.k + rank] = e;
            if (want_w) {
                float wv = a.renorm ? p / psum : p;
                a.w[(size_t)t * a.k + rank] = wv * a.routed_scale;
            }
            atomicAdd(&cnt[gi * a.E + e], 1);
        }
    }
    __syncthreads();
    for (int x = tid; x < N; x += 256) {
        if (a.hist && cnt[x] > 0) atomicAdd(&a.hist[x], cnt[x]);
        if (a.blockcounts && x < a.E) a.blockcounts[(size_t)blockIdx.x * a.E + x] = cnt[x];
    }
}

template <int NB>
static hipError_t launch_gate_nb(const GateArgs &a, hipStream_t s) {
    int ntiles = (a.T + kTile - 1) / kTile;
    hipLaunchKernelGGL((gate_kernel<NB>), dim3(ntiles), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_gate(const GateArgs &a, hipStream_t s) {
    if (a.T <= 0) return hipSuccess;
    int nb = (a.G * a.E + 31) / 32;
    switch (nb) {
        case 1: return launch_gate_nb<1>(a, s);
        case 2: return launch_gate_nb<2>(a, s);
        case 3: return launch_gate_nb<3>(a, s);
        case 4: return launch_gate_nb<4>(a, s);
        case 5: return launch_gate_nb<5>(a, s);
        case 6: return launch_gate_nb<6>(a, s);
        case 7: return launch_gate_nb<7>(a, s);
        case 8: return launch_gate_nb<8>(a, s);
        case 9: case 10: return launch_gate_nb<10>(a, s);
        default: return hipErrorInvalidValue;   // callers split wider launches over the gates
    }
}

// ------------------------------------------------------------------------------------------
// stable grouping by expert: per-tile counts (from the gate kernel) -> scan -> scatter
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void group_scan_kernel(const int32_t *__restrict__ bc, int ntiles, int E,
                                                          int32_t *__restrict__ blockbase,
                                                          int32_t *__restrict__ counts,
                                                          int32_t *__restrict__ offsets) {
    __shared__ int total[kMaxE];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int e = wave; e < E; e += 16) {
        int carry = 0;
        for (int c0 = 0; c0 < ntiles; c0 += 64) {
            int b = c0 + lane;
            int v = b < ntiles ? bc[(size_t)b * E + e] : 0;
            int incl = v;
            for (int off = 1; off < 64; off <<= 1) {
                int o = __shfl_up(incl, off);
                if (lane >= off) incl += o;
            }
            if (b < ntiles) blockbase[(size_t)b * E + e] = carry + incl - v;
            carry += __shfl(incl, 63);
        }
        if (lane == 0) total[e] = carry;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) {
            counts[e] = total[e];
            offsets[e] = run;
            run += total[e];
        }
        offsets[E] = run;
    }
}

hipError_t launch_group_scan(const int32_t *blockcounts, int ntiles, int E, int32_t *blockbase,
                             int32_t *counts, int32_t *offsets, hipStream_t s) {
    hipLaunchKernelGGL(group_scan_kernel, dim3(1), dim3(1024), 0, s, blockcounts, ntiles, E, blockbase,
                       counts, offsets);
    return hipGetLastError();
}

__global__ __launch_bounds__(64) void group_scatter_kernel(const int32_t *__restrict__ ids, int T, int k, int E,
                                                           const int32_t *__restrict__ blockbase,
                                                           const int32_t *__restrict__ offsets,
                                                           int32_t *__restrict__ perm,
                                                           int32_t *__restrict__ inv_perm) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int tok0 = b * kTile;
    const int ntok = min(kTile, T - tok0);
    const int a0 = tok0 * k, n = ntok * k;
    // lane e keeps the next free position of expert e for this tile
    int next = (lane < E) ? offsets[lane] + blockbase[(size_t)b * E + lane] : 0;
    for (int c0 = 0; c0 < n; c0 += 64) {
        const int idx = c0 + lane;
        const bool valid = idx < n;
        const int e = valid ? ids[a0 + idx] : 0;
        unsigned long long todo = __ballot(valid);
        int pos = 0;
        while (todo) {
            const int leader = __ffsll((long long)todo) - 1;
            const int le = __shfl(e, leader);
            const bool mine = valid && e == le;
            const unsigned long long m = __ballot(mine);
            const int start = __shfl(next, le);
            if (mine) pos = start + __popcll(m & ((1ull << lane) - 1ull));
            if (lane == le) next += __popcll(m);
            todo &= ~m;
        }
        if (valid) {
            perm[pos] = a0 + idx;
            inv_perm[a0 + idx] = pos;
        }
    }
}

hipError_t launch_group_scatter(const int32_t *ids, int T, int k, int E, const int32_t *blockbase,
                                const int32_t *offsets, int32_t *perm, int32_t *inv_perm, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    int ntiles = (T + kTile - 1) / kTile;
    hipLaunchKernelGGL(group_scatter_kernel, dim3(ntiles), dim3(64), 0, s, ids, T, k, E, blockbase, offsets,
                       perm, inv_perm);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// token permutation into per-expert groups, written directly in operand-fragment order:
// xp[tile][kb][lane (g,i)] = 8 bf16 of row i of the tile, columns kb*16 + 8g .. +8
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_x_kernel(PackTable pt, const uint16_t *__restrict__ h, int d, int k,
                                                     const int32_t *__restrict__ perm, uint4 *__restrict__ xp) {
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
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    for (int kb = wave; kb < nkb; kb += 4) dst[(size_t)kb * 64] = valid ? src[kb * 2 + g] : zero4;
}

hipError_t launch_pack_x(const PackTable &pt, int total_tiles, const uint16_t *h, int d, int k,
                         const int32_t *perm, void *xp, hipStream_t s) {
    if (total_tiles <= 0) return hipSuccess;
    hipLaunchKernelGGL(pack_x_kernel, dim3(total_tiles), dim3(256), 0, s, pt, h, d, k, perm,
                       reinterpret_cast<uint4 *>(xp));
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// grouped FFN, first half: act = silu(X W1^T) * (X W3^T), one wave per (group, 32 F-rows, pass of
// TT token tiles).  Weights are operand A (rows = F index), packed tokens operand B (columns =
// tokens), so a lane ends with 16 F-values of one token: exactly the two paired-order fragments
// the second half consumes.  No LDS, no barriers: each wave streams its own contiguous weights.
// ------------------------------------------------------------------------------------------
template <int TT>
__global__ __launch_bounds__(256) void ffn_gate_up_kernel(GroupTable gt, const uint4 *__restrict__ xp,
                                                          uint4 *__restrict__ act, int d) {
    const int wg = blockIdx.x;
    int grp = 0;
    while (grp + 1 < gt.n_groups && gt.wg_start[grp + 1] <= wg) ++grp;
    const int local = wg - gt.wg_start[grp];
    const int F = gt.F[grp];
    const int nrb = F >> 5, rbw = (nrb + 3) >> 2;
    const int pass = local / rbw;
    const int rb = (local % rbw) * 4 + (threadIdx.x >> 6);
    if (rb >= nrb) return;
    const int lane = threadIdx.x & 63;
    int ntl = gt.n_tiles[grp] - pass * TT;
    if (ntl > TT) ntl = TT;
    const int nkb = d >> 4;
    const uint4 *w1 = reinterpret_cast<const uint4 *>(gt.blob[grp]) + (size_t)rb * 2 * nkb * 64 + lane;
    const uint4 *w3 = w1 + (size_t)nkb * 64;
    const uint4 *x0 = xp + (size_t)(gt.tile_start[grp] + pass * TT) * nkb * 64 + lane;

    floatx16 G[TT], U[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int v = 0; v < 16; ++v) { G[tt][v] = 0.f; U[tt][v] = 0.f; }

    constexpr int UNR = 4;
    for (int kb = 0; kb < nkb; kb += UNR) {
        uint4 a1[UNR], a3[UNR], xb[TT][UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            a1[u] = load_stream(w1 + (size_t)(kb + u) * 64);
            a3[u] = load_stream(w3 + (size_t)(kb + u) * 64);
        }
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
            if (tt < ntl) {
#pragma unroll
                for (int u = 0; u < UNR; ++u) xb[tt][u] = x0[((size_t)tt * nkb + kb + u) * 64];
            }
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                if (tt < ntl) {
                    G[tt] = mfma32(a1[u], xb[tt][u], G[tt]);
                    U[tt] = mfma32(a3[u], xb[tt][u], U[tt]);
                }
    }

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
                float g0 = G[tt][8 * s + 2 * q], g1 = G[tt][8 * s + 2 * q + 1];
                float a0 = g0 / (1.f + __expf(-g0)) * U[tt][8 * s + 2 * q];
                float a1v = g1 / (1.f + __expf(-g1)) * U[tt][8 * s + 2 * q + 1];
                pk[q] = f32_to_bf16_bits(a0) | (f32_to_bf16_bits(a1v) << 16);
            }
            dst[(size_t)s * 64] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        }
    }
}

hipError_t launch_ffn_gate_up(const GroupTable &gt, int total_wgs, int tiles_per_pass, const void *xp, void *act,
                              int d, hipStream_t s) {
    if (total_wgs <= 0) return hipSuccess;
    const uint4 *x = reinterpret_cast<const uint4 *>(xp);
    uint4 *a = reinterpret_cast<uint4 *>(act);
    if (tiles_per_pass == 1) hipLaunchKernelGGL((ffn_gate_up_kernel<1>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else if (tiles_per_pass == 2) hipLaunchKernelGGL((ffn_gate_up_kernel<2>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else if (tiles_per_pass == 4) hipLaunchKernelGGL((ffn_gate_up_kernel<4>), dim3(total_wgs), dim3(256), 0, s, gt, x, a, d);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// grouped FFN, second half: Y = act W2^T.  A workgroup owns (group, pass of TT token tiles, 32
// output columns); its four waves split K = F and are summed in fixed order through LDS.
// Activations are operand A (rows = tokens), W2 fragments operand B (columns = output features).
// ------------------------------------------------------------------------------------------
template <int TT>
__global__ __launch_bounds__(256) void ffn_down_kernel(GroupTable gt, const uint4 *__restrict__ act,
                                                       float *__restrict__ Y, int d) {
    __shared__ float red[4][TT][16][64];
    const int wg = blockIdx.x;
    int grp = 0;
    while (grp + 1 < gt.n_groups && gt.wg_start[grp + 1] <= wg) ++grp;
    const int local = wg - gt.wg_start[grp];
    const int ncb = d >> 5;
    const int pass = local / ncb, cb = local % ncb;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int F = gt.F[grp];
    const int nkb = F >> 4;
    const int k0 = (int)((long long)wave * nkb / 4), k1 = (int)((long long)(wave + 1) * nkb / 4);
    int ntl = gt.n_tiles[grp] - pass * TT;
    if (ntl > TT) ntl = TT;
    const uint4 *w2 = reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(gt.blob[grp]) +
                                                      (size_t)4 * d * F) + (size_t)cb * nkb * 64 + lane;
    const uint4 *a0 = act + gt.act_off[grp] + (size_t)(pass * TT) * nkb * 64 + lane;

    floatx16 acc[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[tt][v] = 0.f;

    constexpr int UNR = 4;
    int kb = k0;
    for (; kb + UNR <= k1; kb += UNR) {
        uint4 b[UNR], a[TT][UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) b[u] = load_stream(w2 + (size_t)(kb + u) * 64);
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
            if (tt < ntl) {
#pragma unroll
                for (int u = 0; u < UNR; ++u) a[tt][u] = a0[((size_t)tt * nkb + kb + u) * 64];
            }
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                if (tt < ntl) acc[tt] = mfma32(a[tt][u], b[u], acc[tt]);
    }
    for (; kb < k1; ++kb) {
        uint4 b = w2[(size_t)kb * 64];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
            if (tt < ntl) acc[tt] = mfma32(a0[((size_t)tt * nkb + kb) * 64], b, acc[tt]);
    }

#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave][tt][v][lane] = acc[tt][v];
    __syncthreads();

    const int g = lane >> 5, col = cb * 32 + (lane & 31);
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        if (tt >= ntl) break;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int v = 4 * wave + r;
            float sum = red[0][tt][v][lane];
            sum += red[1][tt][v][lane];
            sum += red[2][tt][v][lane];
            sum += red[3][tt][v][lane];
            const int tl = (pass * TT + tt) * kTile + 8 * wave + 4 * g + r;
            if (tl < gt.count[grp]) Y[(size_t)(gt.row_offset[grp] + tl) * d + col] = sum;
        }
    }
}

hipError_t launch_ffn_down(const GroupTable &gt, int total_wgs, int tiles_per_pass, const void *act, float *y,
                           int d, hipStream_t s) {
    if (total_wgs <= 0) return hipSuccess;
    const uint4 *a = reinterpret_cast<const uint4 *>(act);
    if (tiles_per_pass == 1) hipLaunchKernelGGL((ffn_down_kernel<1>), dim3(total_wgs), dim3(256), 0, s, gt, a, y, d);
    else if (tiles_per_pass == 2) hipLaunchKernelGGL((ffn_down_kernel<2>), dim3(total_wgs), dim3(256), 0, s, gt, a, y, d);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// weighted un-permute: out[t] = sum_j w[t,j] * Y[inv_perm[t*k+j]] (+ shared FFN row)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ Y, const float *__restrict__ w,
                                                      const int32_t *__restrict__ inv_perm, int T, int k, int d,
                                                      const float *__restrict__ shared_y, float *__restrict__ out) {
    const int t = blockIdx.x;
    const int c = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (c >= d) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < k; ++j) {
        const int a = t * k + j;
        const float wj = w[a];
        const float4 y = *reinterpret_cast<const float4 *>(Y + (size_t)inv_perm[a] * d + c);
        acc.x += wj * y.x; acc.y += wj * y.y; acc.z += wj * y.z; acc.w += wj * y.w;
    }
    if (shared_y) {
        const float4 y = *reinterpret_cast<const float4 *>(shared_y + (size_t)t * d + c);
        acc.x += y.x; acc.y += y.y; acc.z += y.z; acc.w += y.w;
    }
    *reinterpret_cast<float4 *>(out + (size_t)t * d + c) = acc;
}

hipError_t launch_combine(const float *y, const float *w, const int32_t *inv_perm, int T, int k, int d,
                          const float *shared_y, float *out, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    hipLaunchKernelGGL(combine_kernel, dim3(T, (d + 1023) / 1024), dim3(256), 0, s, y, w, inv_perm, T, k, d,
                       shared_y, out);
    return hipGetLastError();
}

}  // namespace ef
