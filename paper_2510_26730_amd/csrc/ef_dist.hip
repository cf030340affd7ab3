// Intra-batch diversity Dist(t) = sum over token pairs of the Euclidean distance between their
// embeddings (paper Sec. 2.2), computed per token: s[j] = sum_{i<j} ||v_i - v_j||_2.
//
// ||v_i - v_j||^2 = n_i + n_j - 2 <v_i, v_j>: the inner products are one T x T Gram matrix, a dense
// contraction over d that runs on the matrix cores from the packed (operand-fragment) copy of the
// tokens; only tiles that hold a pair i < j are computed.  Three steps on one stream:
//   1. squared norms n_i in fp32 (bf16 products are exact in fp32), one wave per token;
//   2. Gram tiles: a workgroup owns 128 rows i x 256 columns j, a wave 64 x 128 (2 x 4 MFMA
//      32x32x16 accumulators); the epilogue turns inner products into distances, masks i >= j and
//      columns past T, and adds the 64 rows of the wave per column: one partial per (64-row block,
//      token j), no atomics;
//   3. per token the partials of its row blocks are added in ascending order, and the per-token
//      values are added in fixed order (workgroup tree, then one workgroup over the workgroup
//      sums) into Dist(t) in fp64: the result does not depend on scheduling.
#include "ef_device.h"
#include "ef_kernels.h"
#include "ef_tiled_pipeline.h"

namespace ef {

// one wave per token: n[t] = sum_c x[t,c]^2 in fp32, lanes stride the row in 16-byte pieces
__global__ __launch_bounds__(256) void dist_norm_kernel(const uint16_t *__restrict__ h, int T, int d,
                                                        float *__restrict__ norms, int n_pad) {
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (t >= n_pad) return;
    float acc = 0.f;
    if (t < T) {
        const uint4 *row = reinterpret_cast<const uint4 *>(h + (size_t)t * d);
        for (int c = lane; c < (d >> 3); c += 64) {
            const uint4 v = row[c];
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float lo = __builtin_bit_cast(float, w[q] << 16);
                const float hi = __builtin_bit_cast(float, w[q] & 0xFFFF0000u);
                acc += lo * lo;
                acc += hi * hi;
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) norms[t] = acc;   // rows of the padding up to whole tiles get 0
}

// Decode-sized batches (a few hundred tokens at most): the Gram route would be one or two workgroups walking all of
// d in sequence behind five launches.  Here workgroup j owns token j: wave w of 16 takes the rows i = w, w + 16, ...
// < j, two at a time (their loads are independent), the lanes stride the row pair in 16-byte pieces and add
// (x_i - x_j)^2 in fp32 (no norms, no cancellation), a shuffle tree adds the lanes, the root is added to the wave's
// sum in fp64 in ascending i; the waves' sums are added in order.  Everything in a fixed order: the result does not
// depend on scheduling.
constexpr int kDistSmallWaves = 16;
__device__ __forceinline__ float dist_sq_piece(uint4 a, uint4 b) {
    const uint32_t wa[4] = {a.x, a.y, a.z, a.w}, wb[4] = {b.x, b.y, b.z, b.w};
    float acc = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float dl = __builtin_bit_cast(float, wa[q] << 16) - __builtin_bit_cast(float, wb[q] << 16);
        const float dh = __builtin_bit_cast(float, wa[q] & 0xFFFF0000u) - __builtin_bit_cast(float, wb[q] & 0xFFFF0000u);
        acc += dl * dl;
        acc += dh * dh;
    }
    return acc;
}
__global__ __launch_bounds__(64 * kDistSmallWaves) void dist_small_kernel(const uint16_t *__restrict__ h, int T, int d,
                                                                           float *__restrict__ tok_dist,
                                                                           double *__restrict__ wg_sums) {
    __shared__ double red[kDistSmallWaves];
    const int j = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint4 *rj = reinterpret_cast<const uint4 *>(h + (size_t)j * d);
    const int nc = d >> 3;
    double s = 0.0;
    for (int i = wave; i < j; i += 2 * kDistSmallWaves) {
        const int i2 = i + kDistSmallWaves;
        const bool two = i2 < j;
        const uint4 *r0 = reinterpret_cast<const uint4 *>(h + (size_t)i * d);
        const uint4 *r1 = reinterpret_cast<const uint4 *>(h + (size_t)(two ? i2 : i) * d);
        float acc0 = 0.f, acc1 = 0.f;
        for (int c = lane; c < nc; c += 64) {
            const uint4 b = rj[c];
            acc0 += dist_sq_piece(r0[c], b);
            acc1 += dist_sq_piece(r1[c], b);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            acc0 += __shfl_xor(acc0, off);
            acc1 += __shfl_xor(acc1, off);
        }
        s += (double)__builtin_sqrtf(acc0);
        if (two) s += (double)__builtin_sqrtf(acc1);
    }
    if (lane == 0) red[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < kDistSmallWaves; ++w) t += red[w];
        if (tok_dist) tok_dist[j] = (float)t;
        wg_sums[j] = t;
    }
}

constexpr int kDistRowTiles = 4;   // token tiles (32 rows) of operand A per workgroup: 128 rows i
constexpr int kDistColTiles = 8;   // token tiles of operand B per workgroup: 256 columns j

// grid (column blocks, row blocks); xp = packed tokens [tile][d/16][1 KiB]
__global__ __launch_bounds__(256, 2) void dist_tile_kernel(const uint4 *__restrict__ xp,
                                                           const float *__restrict__ norms, int T, int d,
                                                           float *__restrict__ part, int t_pad,
                                                           int n_rowblk) {
    const int JB = blockIdx.x, IB = blockIdx.y;
    if (IB > 2 * JB + 1) return;   // every row of the block is >= every column: no pair i < j
    const int ntiles = (T + kTile - 1) / kTile;
    const int nkb = d >> 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int it0 = IB * kDistRowTiles + (wave >> 1) * 2;    // 2 row tiles of this wave
    const int jt0 = JB * kDistColTiles + (wave & 1) * 4;     // 4 column tiles of this wave
    const uint4 *a_src[2], *b_src[4];
#pragma unroll
    for (int a = 0; a < 2; ++a) a_src[a] = xp + (size_t)min(it0 + a, ntiles - 1) * nkb * 64 + lane;
#pragma unroll
    for (int b = 0; b < 4; ++b) b_src[b] = xp + (size_t)min(jt0 + b, ntiles - 1) * nkb * 64 + lane;

    floatx16 acc[2][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) zero16(acc[a][b]);

    // two register stages of two k-steps each; the prefetch is unconditional (clamped, in bounds)
    constexpr int UNR = 2;
    u32x4_t fa0[2][UNR], fb0[4][UNR], fa1[2][UNR], fb1[4][UNR];
#define EF_DIST_LOAD(fa, fb, kb)                                                                          \
    {                                                                                                     \
        _Pragma("unroll") for (int u = 0; u < UNR; ++u) {                                                 \
            const int kk_ = min((kb) + u, nkb - 1);                                                       \
            _Pragma("unroll") for (int a = 0; a < 2; ++a)                                                 \
                fa[a][u] = *reinterpret_cast<const u32x4_t *>(a_src[a] + (size_t)kk_ * 64);               \
            _Pragma("unroll") for (int b = 0; b < 4; ++b)                                                 \
                fb[b][u] = *reinterpret_cast<const u32x4_t *>(b_src[b] + (size_t)kk_ * 64);               \
        }                                                                                                 \
    }
#define EF_DIST_MMA(fa, fb, kb)                                                                           \
    {                                                                                                     \
        _Pragma("unroll") for (int u = 0; u < UNR; ++u)                                                   \
            if ((kb) + u < nkb) {                                                                         \
                _Pragma("unroll") for (int a = 0; a < 2; ++a)                                             \
                    _Pragma("unroll") for (int b = 0; b < 4; ++b)                                         \
                        acc[a][b] = mfma32v(fa[a][u], fb[b][u], acc[a][b]);                               \
            }                                                                                             \
    }
    EF_DIST_LOAD(fa0, fb0, 0)
    for (int kb = 0; kb < nkb; kb += 2 * UNR) {
        EF_DIST_LOAD(fa1, fb1, kb + UNR)
        EF_DIST_MMA(fa0, fb0, kb)
        EF_DIST_LOAD(fa0, fb0, kb + 2 * UNR)
        EF_DIST_MMA(fa1, fb1, kb + UNR)
    }
#undef EF_DIST_LOAD
#undef EF_DIST_MMA

    // accumulator lane l holds column l%32 and rows 8*(v/4) + 4*(l/32) + v%4: the sum over the
    // wave's 64 rows of one column is 32 in-lane adds and one exchange between the lane halves
    const int g = lane >> 5, c = lane & 31;
    const int rowblk = IB * 2 + (wave >> 1);   // 64-row block of the partials
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int j = (jt0 + b) * kTile + c;
        const float nj = j < T ? norms[j] : 0.f;
        float sum = 0.f;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = (it0 + a) * kTile + 8 * (v >> 2) + 4 * g + (v & 3);
                if (i < j && j < T) {
                    const float sq = norms[i] + nj - 2.f * acc[a][b][v];
                    sum += __builtin_sqrtf(fmaxf(sq, 0.f));
                }
            }
        }
        sum += __shfl_xor(sum, 32);
        if (g == 0 && j < t_pad && rowblk < n_rowblk) part[(size_t)rowblk * t_pad + j] = sum;
    }
}

// ------------------------------------------------------------------------------------------
// Gram tiles through the LDS operand pipeline (large batches): a workgroup owns 256 rows i x 256 columns
// j, both operands are token fragments.  Same accumulation order over k, same epilogue sums and the same
// partials as dist_tile_kernel: the two forms give the same bits.
//
// Only blocks with a pair i < j exist (block row IB <= block column JB).  They are numbered in strips of
// four block rows, column by column within a strip, so that 32 consecutive blocks cover about 4 block
// rows x 8 block columns; runs of 32 go to the XCDs in turn (workgroups with the same index mod 8 share an
// XCD and run side by side on its 32 compute units), so the 64 operand panels of a run are 12 distinct ones
// and an XCD's L2 serves the rest.
// ------------------------------------------------------------------------------------------
constexpr int kGramRun = 32;     // consecutive blocks that one XCD runs side by side
constexpr int kGramStrip = 4;    // block rows per strip

// blocks in the strips before strip R (nB block rows / columns)
__host__ __device__ inline long long gram_blocks_before(int R, int nB) {
    const long long r = kGramStrip * R < nB ? kGramStrip * R : nB;   // block rows before the strip
    return r * nB - r * (r - 1) / 2;                           // row IB holds nB - IB blocks
}
inline long long gram_blocks(int nB) { return (long long)nB * (nB + 1) / 2; }
constexpr long long kDistTiledMinBlocks = 64;

__global__ __launch_bounds__(256, 1) void dist_gram_tiled_kernel(const uint4 *__restrict__ xp,
                                                                  const float *__restrict__ norms, int T, int d,
                                                                  float *__restrict__ part, int t_pad,
                                                                  int n_rowblk, int nB, long long total_whole,
                                                                  int main_grid) {
    constexpr bool kSwapOperands = false;
    constexpr bool HALF = false;   // bf16 token fragments
    __shared__ __attribute__((aligned(16))) u32x4_t lds[kTileStages][kStageFrags][64];
    const int w = blockIdx.x;
    // workgroups [0, main_grid): whole blocks [0, total_whole) in runs over the XCDs; the workgroups after them:
    // the quarters (128 x 128) of the blocks from total_whole on
    long long t;
    int quarter = -1;
    if (w < main_grid) {
        t = ((long long)(w >> 3) / kGramRun * 8 + (w & 7)) * kGramRun + ((w >> 3) % kGramRun);
        if (t >= total_whole) return;
    } else {
        t = total_whole + ((w - main_grid) >> 2);
        quarter = (w - main_grid) & 3;
    }
    // strip R, then the block within the strip: its first h columns hold 1..h blocks (the diagonal), the
    // columns after them h blocks each
    int R = 0;
    while (gram_blocks_before(R + 1, nB) <= t) ++R;
    const int u = (int)(t - gram_blocks_before(R, nB));
    const int h = min(kGramStrip, nB - kGramStrip * R);
    int a, cidx;
    if (u < h * (h + 1) / 2) {
        cidx = 0;
        while ((cidx + 1) * (cidx + 2) / 2 <= u) ++cidx;
        a = u - cidx * (cidx + 1) / 2;
    } else {
        const int v = u - h * (h + 1) / 2;
        cidx = h + v / h;
        a = v % h;
    }
    const int IB = kGramStrip * R + a, JB = kGramStrip * R + cidx;

    const int ntiles = (T + kTile - 1) / kTile;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS DMA targets go through M0
    const int wi = wave & 1, wj = wave >> 1;
    const int nkb = d >> 4;
    const int nstage = nkb / kTileKS;
    const int g = lane >> 5, c = lane & 31;
    const unsigned lds_base = (unsigned)(size_t)&lds[0][0][0];   // LDS byte offset: the low half of its flat address
    const u32x4_t *src[kStageFrags / 4];
    floatx16 acc[4][4];   // [row tile][column tile]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) zero16(acc[i][j]);

    if (quarter < 0) {
        const int it0 = IB * 8, jt0 = JB * 8;
        // operand A slots 0..7 = row tiles it0..it0+7, operand B slots 8..15 = column tiles jt0..jt0+7
#pragma unroll
        for (int q = 0; q < kStageFrags / 4; ++q) {
            const int fi = q * 4 + wave;
            const int ks = fi >> 4, slot = fi & 15;
            const int tile = min(slot < 8 ? it0 + slot : jt0 + slot - 8, ntiles - 1);
            src[q] = reinterpret_cast<const u32x4_t *>(xp + ((size_t)tile * nkb + ks) * 64 + lane);
        }
        const int AOFF = wi * 4, BOFF = wj * 4;
        // column tiles of this wave that exist; none count when every row of the wave is past every column
        // (the lower left quarter of a diagonal block)
        const bool below = it0 + AOFF >= jt0 + BOFF + 4;
        const int live = below ? 0 : max(0, min(4, ntiles - (jt0 + BOFF)));
        EF_TILED_PIPELINE_TILES_B(0, nstage, live)

#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int j = (jt0 + BOFF + b) * kTile + c;
            const float nj = j < T ? norms[j] : 0.f;
#pragma unroll
            for (int rp = 0; rp < 2; ++rp) {   // the wave's two 64-row blocks of the partials
                const int rowblk = IB * 4 + wi * 2 + rp;
                float sum = 0.f;
#pragma unroll
                for (int aa = 0; aa < 2; ++aa) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int i = (it0 + AOFF + 2 * rp + aa) * kTile + 8 * (v >> 2) + 4 * g + (v & 3);
                        if (i < j && j < T) {
                            const float sq = norms[i] + nj - 2.f * acc[2 * rp + aa][b][v];
                            sum += __builtin_sqrtf(fmaxf(sq, 0.f));
                        }
                    }
                }
                sum += __shfl_xor(sum, 32);
                if (g == 0 && j < t_pad && rowblk < n_rowblk) part[(size_t)rowblk * t_pad + j] = sum;
            }
        }
    } else {
        // a quarter: 128 rows x 128 columns, a wave 64 x 64 (2 x 2 accumulators): the same loads and barriers
        // per stage for a quarter of the matrix-core work, for the few blocks that would otherwise be a round
        // of workgroups of their own over a mostly idle chip
        const int it0 = IB * 8 + (quarter >> 1) * 4, jt0 = JB * 8 + (quarter & 1) * 4;
        if (it0 >= jt0 + 4) return;   // every row past every column
        // operand A slots 0..3 = row tiles it0..it0+3, operand B slots 8..11 = column tiles jt0..jt0+3; the other
        // slots repeat them (never read from LDS)
#pragma unroll
        for (int q = 0; q < kStageFrags / 4; ++q) {
            const int fi = q * 4 + wave;
            const int ks = fi >> 4, slot = fi & 15;
            const int tile = min(slot < 8 ? it0 + (slot & 3) : jt0 + (slot & 3), ntiles - 1);
            src[q] = reinterpret_cast<const u32x4_t *>(xp + ((size_t)tile * nkb + ks) * 64 + lane);
        }
        const int AOFF = wi * 2, BOFF = wj * 2;
        EF_TILED_PIPELINE_2X2(0, nstage)

        const int rowblk = (it0 + AOFF) >> 1;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int j = (jt0 + BOFF + b) * kTile + c;
            const float nj = j < T ? norms[j] : 0.f;
            float sum = 0.f;
#pragma unroll
            for (int aa = 0; aa < 2; ++aa) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = (it0 + AOFF + aa) * kTile + 8 * (v >> 2) + 4 * g + (v & 3);
                    if (i < j && j < T) {
                        const float sq = norms[i] + nj - 2.f * acc[aa][b][v];
                        sum += __builtin_sqrtf(fmaxf(sq, 0.f));
                    }
                }
            }
            sum += __shfl_xor(sum, 32);
            if (g == 0 && j < t_pad && rowblk < n_rowblk) part[(size_t)rowblk * t_pad + j] = sum;
        }
    }
}

// s[j] = partials of row blocks 0 .. j/64 in ascending order; workgroup sum in fp64 by a fixed tree
__global__ __launch_bounds__(256) void dist_reduce_kernel(const float *__restrict__ part, int T, int t_pad,
                                                          float *__restrict__ tok_dist,
                                                          double *__restrict__ wg_sums) {
    __shared__ double red[256];
    const int j = blockIdx.x * 256 + threadIdx.x;
    double s = 0.0;
    if (j < T) {
        // eight loads in flight, added in ascending order of the row block
        const int n = (j >> 6) + 1;
        int rb = 0;
        for (; rb + 8 <= n; rb += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = part[(size_t)(rb + u) * t_pad + j];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += (double)v[u];
        }
        for (; rb < n; ++rb) s += (double)part[(size_t)rb * t_pad + j];
        if (tok_dist) tok_dist[j] = (float)s;
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) wg_sums[blockIdx.x] = red[0];
}

__global__ __launch_bounds__(64) void dist_final_kernel(const double *__restrict__ wg_sums, int n,
                                                        double *__restrict__ dist) {
    if (threadIdx.x != 0) return;
    double s = 0.0;
    for (int i = 0; i < n; ++i) s += wg_sums[i];
    *dist = s;
}

size_t dist_scratch_floats(int T) {
    const int t_pad = ((T + kTile - 1) / kTile) * kTile;
    const int n_rowblk = (T + 63) / 64;
    const int n_wg = (T + 255) / 256;
    return (size_t)t_pad + (size_t)n_rowblk * t_pad + 2 * (size_t)n_wg + 2;
}

hipError_t launch_token_dist(const uint16_t *h, int T, int d, const void *xp, float *scratch, float *tok_dist,
                             double *dist, int form, hipStream_t s) {
    if (T <= 0 || d % 64 != 0 || form < 0 || form > 2) return hipErrorInvalidValue;
    const int ntiles = (T + kTile - 1) / kTile;
    const int t_pad = ntiles * kTile;
    const int n_rowblk = (T + 63) / 64;
    const int n_wg = (T + 255) / 256;
    if (!dist_needs_packed(T, form)) {
        // T doubles at the start of the scratch (8-byte aligned: the scratch is), then the usual final sum
        double *sums = reinterpret_cast<double *>(scratch);
        hipLaunchKernelGGL(dist_small_kernel, dim3(T), dim3(64 * kDistSmallWaves), 0, s, h, T, d, tok_dist, sums);
        hipLaunchKernelGGL(dist_final_kernel, dim3(1), dim3(64), 0, s, sums, T, dist);
        return hipGetLastError();
    }
    float *norms = scratch;
    float *part = scratch + t_pad;
    // 8-byte aligned slot for the workgroup sums behind the partials
    size_t off = (size_t)t_pad + (size_t)n_rowblk * t_pad;
    off += off & 1;
    double *wg_sums = reinterpret_cast<double *>(scratch + off);
    hipLaunchKernelGGL(dist_norm_kernel, dim3((t_pad + 3) / 4), dim3(256), 0, s, h, T, d, norms, t_pad);
    // 256 x 256 blocks through LDS once they fill a quarter of the compute units; below that the
    // 128 x 256 blocks of the register-fed kernel, two to a compute unit, spread the batch wider
    const int nB = (ntiles + 7) / 8;
    const long long total = gram_blocks(nB);
    if (form == 2 || (form == 0 && total >= kDistTiledMinBlocks)) {
        // One block per compute unit at a time: the blocks left over after the last full round of 256 would be a
        // round of their own.  Up to 64 of them run as quarters instead (at most 256 workgroups, each with a
        // quarter of the matrix-core work per stage).
        const long long rem = total % 256;
        const long long n_split = total > 256 && rem <= 64 ? rem : 0;
        const long long whole = total - n_split;
        const long long runs = (whole + kGramRun - 1) / kGramRun;
        const long long main_grid = (runs + 7) / 8 * 8 * kGramRun;
        const long long grid = main_grid + 4 * n_split;
        if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
        hipLaunchKernelGGL(dist_gram_tiled_kernel, dim3((unsigned)grid), dim3(256), 0, s,
                           reinterpret_cast<const uint4 *>(xp), norms, T, d, part, t_pad, n_rowblk, nB, whole,
                           (int)main_grid);
    } else {
        const int nJB = (ntiles + kDistColTiles - 1) / kDistColTiles;
        const int nIB = (ntiles + kDistRowTiles - 1) / kDistRowTiles;
        hipLaunchKernelGGL(dist_tile_kernel, dim3(nJB, nIB), dim3(256), 0, s, reinterpret_cast<const uint4 *>(xp),
                           norms, T, d, part, t_pad, n_rowblk);
    }
    hipLaunchKernelGGL(dist_reduce_kernel, dim3(n_wg), dim3(256), 0, s, part, T, t_pad, tok_dist, wg_sums);
    hipLaunchKernelGGL(dist_final_kernel, dim3(1), dim3(64), 0, s, wg_sums, n_wg, dist);
    return hipGetLastError();
}

}  // namespace ef
