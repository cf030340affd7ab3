// Gate / predict kernel (matrix-core logits, wave-level softmax and biased top-k, per-tile expert
// counts, demand histograms) and the stable grouping of assignments by expert.
#include "ef_device.h"
#include "ef_kernels.h"

#include <algorithm>

namespace ef {

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
// gate: logits of a group of gate matrices on one 32-token tile, then per-token softmax, biased
// top-k, combine weights, per-tile expert counts and demand histograms.
//
// grid = (token tiles, gate groups): the G gates of a launch are cut into groups of `gpw` gates
// (at most 128 logit columns); groups are independent, so no workgroup ever waits for or reduces
// with another one.  Hidden states and gate rows are row-major in memory, so a K panel of both is
// first brought into LDS with fully coalesced loads (a wave reads 512 or 256 contiguous bytes of a
// row; reading operand fragments straight from 32 strided rows costs eight times the L1 tag
// look-ups and makes small batches latency-bound); the next panel is prefetched into registers
// while the eight waves run their share of the MFMA steps of the current one from LDS.
// ------------------------------------------------------------------------------------------
constexpr int kGateWaves = 8;
constexpr int kGateMaxSplit = 16;   // K splits of one (tile, gate group) across workgroups

// orders the LDS writes of a wave before its later LDS reads (other lanes' data of the same wave)
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// arr[idx] of a by-value kernel-argument array without forcing the struct into scratch memory
template <class T>
__device__ __forceinline__ T pick(const T (&arr)[kMaxGates], int idx) {
    T v = arr[0];
#pragma unroll
    for (int q = 1; q < kMaxGates; ++q)
        if (idx == q) v = arr[q];
    return v;
}

template <int NB, int NW = kGateWaves>
__device__ __forceinline__ void gate_epilogue(const GateArgs &a, float (*logits)[NB * 32 + 1], int *cnt,
                                              const float *sbias, float (*s_sc)[64],
                                              int tile, int g0, int Gl, int tok_lo, int tok_n, bool shared_tile);

template <int NB>
__global__ __launch_bounds__(64 * kGateWaves) void gate_kernel(GateArgs a) {
    constexpr int NW = kGateWaves, NT = 64 * NW;
    constexpr int KC = NB == 1 ? 256 : 128;            // K panel (elements)
    constexpr int LDK = KC + 8;                        // padded LDS row: 16-byte reads of 16 rows hit 64 banks
    constexpr int C4 = KC / 8;                         // 16-byte units per panel row
    constexpr int A_PER = 32 * C4 / NT;                // 16-byte loads per thread per panel
    constexpr int B_PER = NB * 32 * C4 / NT;
    constexpr int KSW = KC / 16 / NW;                  // MFMA k-steps per wave per panel
    // operand panels; after the K loop the same memory holds the partial tiles of the wave reduction
    constexpr int PANEL_BYTES = (1 + NB) * 32 * LDK * 2;
    constexpr int RED_FLOATS = NB * 16 * 64;           // one wave's partial tile
    constexpr int RED_BYTES = (NW / 2) * RED_FLOATS * 4;
    __shared__ __attribute__((aligned(16))) unsigned char smem[PANEL_BYTES > RED_BYTES ? PANEL_BYTES : RED_BYTES];
    uint16_t *As = reinterpret_cast<uint16_t *>(smem);
    uint16_t *Bs = As + 32 * LDK;
    float *red = reinterpret_cast<float *>(smem);
    __shared__ float logits[kTile][NB * 32 + 1];
    __shared__ int cnt[4 * 32];
    __shared__ float sbias[4 * 32];
    __shared__ __attribute__((aligned(16))) float s_sc[NW][64];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 5, i = lane & 31;
    const int tile = blockIdx.x;
    const int g0 = blockIdx.y * a.gpw;                 // first gate of this workgroup's group
    const int Gl = min(a.gpw, a.G - g0);               // gates in the group
    const int t0 = tile * kTile;
    const int N = Gl * a.E;                            // logit columns of the group (<= NB*32)

    for (int x = tid; x < NB * 32; x += NT) cnt[x] = 0;
    // gate biases go to LDS now, so their latency hides behind the matrix-core phase
    for (int x = tid; x < N; x += NT) {
        const float *bp = pick(a.bias, g0 + x / a.E);
        sbias[x] = bp ? bp[x % a.E] : 0.f;
    }

    // per-thread source rows of the panel loads (fixed over the K loop)
    const uint16_t *asrc[A_PER];
    const uint16_t *bsrc[B_PER];
    bool aok[A_PER], bok[B_PER];
#pragma unroll
    for (int r = 0; r < A_PER; ++r) {
        const int row = (tid + r * NT) / C4;
        aok[r] = t0 + row < a.T;
        asrc[r] = a.h + (size_t)(aok[r] ? t0 + row : 0) * a.d;
    }
#pragma unroll
    for (int r = 0; r < B_PER; ++r) {
        const int n = (tid + r * NT) / C4;
        bok[r] = n < N;
        // columns past N still load (the number of loads in flight stays a compile-time constant), from
        // the valid rows in turn rather than all from one row
        const int nn = n % N;
        bsrc[r] = pick(a.Wg, g0 + nn / a.E) + (size_t)(nn % a.E) * a.d;
    }

    floatx16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) zero16(acc[nb]);

    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    const u32x4_t zero4v = {0u, 0u, 0u, 0u};
    // PF panels are kept in flight in registers: with few token tiles the kernel is bound by memory
    // latency, and one panel per round trip would cost d/KC round trips
    constexpr int PF = 4;
    u32x4_t ra[PF][A_PER], rb[PF][B_PER];
#pragma unroll
    for (int p = 0; p < PF; ++p) {
#pragma unroll
        for (int r = 0; r < A_PER; ++r) ra[p][r] = zero4v;
#pragma unroll
        for (int r = 0; r < B_PER; ++r) rb[p][r] = zero4v;
    }
#define EF_GATE_GLOAD(p, st)                                                                           \
    {                                                                                                  \
        _Pragma("unroll") for (int r = 0; r < A_PER; ++r) {                                            \
            const int col = (st) * KC + ((tid + r * NT) % C4) * 8;                                     \
            ra[p][r] = *reinterpret_cast<const u32x4_t *>(asrc[r] + min(col, a.d - 8));                \
        }                                                                                              \
        _Pragma("unroll") for (int r = 0; r < B_PER; ++r) {                                            \
            const int col = (st) * KC + ((tid + r * NT) % C4) * 8;                                     \
            rb[p][r] = *reinterpret_cast<const u32x4_t *>(bsrc[r] + min(col, a.d - 8));                \
        }                                                                                              \
    }
    // K split across workgroups (grid.z) for batches of few token tiles: each workgroup takes a
    // contiguous range of panels and leaves its partial logits to gate_finish_kernel
    const int nstage_all = (a.d + KC - 1) / KC;
    const int per_split = (nstage_all + a.ksplit - 1) / a.ksplit;
    const int sbeg = blockIdx.z * per_split, nstage = min(nstage_all, sbeg + per_split);
    // Every workgroup walks its panels in a rotated order (start = 5 * tile mod count): with a common
    // order all workgroups would read the same 512-byte column block of their 8 KiB-strided rows at
    // the same time, and those addresses share most of their channel-select bits
    const int nloc = max(nstage - sbeg, 1);
    const int rot0 = (tile * 5) % nloc;
    auto rot = [&](int st) {
        int x = st - sbeg + rot0;
        if (x >= nloc) x -= nloc;
        return sbeg + x;
    };
    // prefetches are unconditional (past the end they re-read the last panel, in bounds) so that the
    // number of loads in flight is known at compile time and only the oldest panel is waited for
    // (issued strictly in panel order: the wait before the first panel's use may then leave the loads of
    // the three younger panels outstanding, on the loop's entry as on its back edge)
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        EF_GATE_GLOAD(p, rot(max(min(sbeg + p, nstage - 1), sbeg)))
        __builtin_amdgcn_sched_barrier(0);
    }
    for (int st0 = sbeg; st0 < nstage; st0 += PF) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int st = st0 + p;
            {   // stages past the end (when nstage is not a multiple of PF) multiply zero panels
#pragma unroll
                for (int r = 0; r < A_PER; ++r) {
                    const int idx = tid + r * NT;   // rows past T and columns past d contribute zeros
                    const bool ok = aok[r] && st < nstage && rot(st) * KC + (idx % C4) * 8 < a.d;
                    *reinterpret_cast<u32x4_t *>(&As[(idx / C4) * LDK + (idx % C4) * 8]) = ok ? ra[p][r] : zero4v;
                }
#pragma unroll
                for (int r = 0; r < B_PER; ++r) {
                    const int idx = tid + r * NT;
                    const bool ok = bok[r] && st < nstage && rot(st) * KC + (idx % C4) * 8 < a.d;
                    *reinterpret_cast<u32x4_t *>(&Bs[(idx / C4) * LDK + (idx % C4) * 8]) = ok ? rb[p][r] : zero4v;
                }
                __syncthreads();
                EF_GATE_GLOAD(p, rot(max(min(st + PF, nstage - 1), sbeg)))
#pragma unroll
                for (int q = 0; q < KSW; ++q) {
                    const int kcol = (wave * KSW + q) * 16 + 8 * g;
                    const uint4 af = *reinterpret_cast<const uint4 *>(&As[i * LDK + kcol]);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const uint4 bf = *reinterpret_cast<const uint4 *>(&Bs[(nb * 32 + i) * LDK + kcol]);
                        acc[nb] = mfma32(af, bf, acc[nb]);
                    }
                }
                __syncthreads();
            }
        }
    }

#undef EF_GATE_GLOAD

    // fixed-order tree over the waves' partial tiles through LDS: (w, w+4), then (w, w+2), then
    // (0, 1); the last barrier of the K loop has retired every read of the operand panels
    static_assert(NW == 8, "the reduction tree below is written for eight waves");
    auto put = [&](int region) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) red[region * RED_FLOATS + (nb * 16 + v) * 64 + lane] = acc[nb][v];
    };
    auto add = [&](int region) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][v] += red[region * RED_FLOATS + (nb * 16 + v) * 64 + lane];
    };
    if (wave >= 4) put(wave - 4);
    __syncthreads();
    if (wave < 4) add(wave);
    __syncthreads();
    if (wave == 2 || wave == 3) put(wave - 2);
    __syncthreads();
    if (wave < 2) add(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave == 0) {
        add(0);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) logits[8 * (v >> 2) + 4 * g + (v & 3)][nb * 32 + i] = acc[nb][v];
    }
    __syncthreads();

    if (a.two_step) {   // partial logits of this K range: [tile][group][split][32][NB*32]
        if (a.tsplit > 1 && a.blockcounts && blockIdx.y == 0 && blockIdx.z == 0)   // added to atomically later
            for (int x = tid; x < a.E; x += NT) a.blockcounts[(size_t)tile * a.E + x] = 0;
        float *dst = a.part + ((((size_t)tile * gridDim.y + blockIdx.y) * a.ksplit + blockIdx.z) * kTile) * (NB * 32);
        for (int x = tid; x < kTile * NB * 32; x += NT) dst[x] = logits[x / (NB * 32)][x % (NB * 32)];
        return;
    }
    gate_epilogue<NB>(a, logits, cnt, sbias, s_sc, tile, g0, Gl, 0, kTile, false);
}

// per-token part of the gate kernels: selection scores, biased top-k, combine weights, counts.
// `logits` holds the tile's router logits without the gate bias (sbias), `cnt` is zeroed.
template <int NB, int NW>
__device__ __forceinline__ void gate_epilogue(const GateArgs &a, float (*logits)[NB * 32 + 1], int *cnt,
                                              const float *sbias, float (*s_sc)[64],
                                              int tile, int g0, int Gl, int tok_lo, int tok_n, bool shared_tile) {
    // tokens tok_lo .. tok_lo + tok_n - 1 of the tile (tok_n a multiple of the tokens per wave round);
    // shared_tile: other workgroups handle the tile's other tokens, so per-tile counts are added
    // atomically to the (zeroed) table instead of stored.  NW waves per workgroup.
    constexpr int NT = 64 * NW;
    // the wave index as a scalar: the gate a round works on is then known to be the same for the whole wave, and
    // its kernel arguments are picked in scalar registers instead of by per-lane loads from the argument block
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int t0 = tile * kTile;
    const int N = Gl * a.E;
    // A sub-group of W lanes (W = power of two >= E) owns one token; a wave
    // handles 64/W tokens of ONE gate per round (the gate index is wave-uniform, so per-gate
    // arguments are scalar loads).  Selection is by rank: lane e counts, from an LDS copy of the
    // token's scores, how many experts beat it (greater score, or equal score and lower id); the k
    // best are those with rank < k.  No dependent shuffle chains: the loops are LDS broadcast reads.
    int W = 8;
    while (W < a.E) W <<= 1;
    const int per_wave = 64 / W;
    const int sub = lane / W, e = lane % W;
    const int chunks_per_gate = tok_n / per_wave;
    const int total_chunks = Gl * chunks_per_gate;
    const bool evalid = e < a.E;
    const float NEG_INF = -__builtin_inff();

    // every wave works on its own row of s_sc: the exchange below needs ordering inside the
    // wave only (LDS operations of one wave execute in order), no workgroup barrier
    for (int it = 0; it * NW < total_chunks; ++it) {
        const int chunk = it * NW + wave;
        const bool cact = chunk < total_chunks;
        const int gl = cact ? chunk / chunks_per_gate : 0;   // gate inside the group
        const int gi = g0 + gl;                              // gate of the launch
        const int ti = tok_lo + (chunk % chunks_per_gate) * per_wave + sub;
        const int t = t0 + ti;
        const bool live = cact && t < a.T;
        const bool want_w = cact && (a.w != nullptr) && gi == 0;  // wave-uniform
        float z = NEG_INF;
        if (live && evalid) z = logits[ti][gl * a.E + e] + sbias[gl * a.E + e];
        float sc = z;
        if (live && evalid) {
            if ((pick(a.resident, gi) >> e) & 1ull) sc += a.beta;
            if (a.delta && gi >= a.delta_gate_begin) {
                int req = a.tok2req ? a.tok2req[t] : 0;
                sc += a.delta[(size_t)req * a.delta_req_stride + (gi - a.delta_gate_begin) * a.E + e];
            }
        }
        s_sc[wave][lane] = sc;
        wave_lds_sync();
        const float4 *srow = reinterpret_cast<const float4 *>(&s_sc[wave][sub * W]);
        int rank = 0;
        for (int j = 0; j < W; j += 4) {
            const float4 v = srow[j >> 2];
            rank += (v.x > sc || (v.x == sc && j + 0 < e)) ? 1 : 0;
            rank += (v.y > sc || (v.y == sc && j + 1 < e)) ? 1 : 0;
            rank += (v.z > sc || (v.z == sc && j + 2 < e)) ? 1 : 0;
            rank += (v.w > sc || (v.w == sc && j + 3 < e)) ? 1 : 0;
        }
        const bool sel = live && evalid && rank < a.k;
        // softmax over all experts in fp32: max, exp and the denominator (all experts, or only the
        // selected ones when the weights are renormalised) by butterfly exchanges inside the token's
        // lane group, a fixed order
        float ex = 0.f, den = 1.f;
        if (want_w) {
            float m = z;   // lanes without an expert hold -inf
            for (int off = W >> 1; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
            ex = (live && evalid) ? __expf(z - m) : 0.f;
            den = (a.renorm && !sel) ? 0.f : ex;
            for (int off = W >> 1; off >= 1; off >>= 1) den += __shfl_xor(den, off);
        }
        const unsigned long long ball = __ballot(sel);
        const unsigned long long submask = (W == 64) ? ball : ((ball >> (sub * W)) & ((1ull << W) - 1ull));
        const int slot = __popcll(submask & ((1ull << e) - 1ull));   // ascending expert id
        if (sel) {
            pick(a.ids, gi)[(size_t)t * a.k + slot] = e;
            if (want_w) a.w[(size_t)t * a.k + slot] = ex / den * a.routed_scale;
            atomicAdd(&cnt[gl * a.E + e], 1);
        }
    }
    __syncthreads();
    for (int x = tid; x < N; x += NT) {
        const int gi = g0 + x / a.E, ee = x % a.E;
        int32_t *hp = pick(a.hist, gi);
        if (hp && cnt[x] > 0) atomicAdd(&hp[ee], cnt[x]);
        if (a.blockcounts && gi == 0) {
            if (!shared_tile) a.blockcounts[(size_t)tile * a.E + ee] = cnt[x];
            else if (cnt[x] > 0) atomicAdd(&a.blockcounts[(size_t)tile * a.E + ee], cnt[x]);
        }
    }
}

// ------------------------------------------------------------------------------------------
// gate for batches of many token tiles (every compute unit has at least one tile of its own, no K split):
// bound by streaming the hidden states from HBM once.  A stage of KC columns of a 32-token tile is brought
// into LDS by direct global -> LDS loads (no staging registers, no LDS store instructions), each wave
// instruction copying 1 KiB (KC = 256: 512 contiguous bytes of two rows; KC = 512: one row), NS stages deep,
// OCC workgroups per compute unit.
// The gate rows of the stage come the same way (only the rows that exist; a workgroup re-reads them from
// L2, a quarter or less of the bytes of its hidden states for E <= 8).  The k-steps of a stage are dealt to
// the four waves, whose partial tiles meet in a fixed-order tree through LDS before the per-token epilogue
// (the one of gate_kernel).  Every workgroup walks the stages in its own rotated order: with a common order
// all workgroups would read the same column block of their 8 KiB-strided rows at the same time, and those
// addresses share most of their channel-select bits.
//
// LDS layout: 1 KiB blocks as the loads deliver them, 1040 bytes apart, so that the 16-byte operand reads of
// 16 consecutive rows cover all 64 banks.  With KC = 256 a block holds the stage's 512 bytes of rows j and
// j + 16 of a 32-row block.  CB = gate-row loads per wave and stage (4 * CB blocks of gate rows per stage).
// ------------------------------------------------------------------------------------------
constexpr int kGsBlock = 1024 + 16;        // bytes between the 1 KiB blocks in LDS
constexpr int kGsWaves = 4;
constexpr int gs_waitcnt(int vm) { return (((vm >> 4) & 3) << 14) | (0x7 << 4) | (0xF << 8) | (vm & 15); }
// as many stages as the LDS of a compute unit holds for OCC workgroups beside the epilogue's arrays, at most 4
constexpr int gs_stages(int NB, int KC, int CB, int OCC) {
    const int stage = (32 / (512 / KC) + 4 * CB) * kGsBlock;
    const int budget = 160 * 1024 / OCC - (kTile * (NB * 32 + 1) * 4 + 2048);
    return budget / stage >= 4 ? 4 : budget / stage;
}

template <int NB, int CB, int KC, int OCC>
__global__ __launch_bounds__(64 * kGsWaves, OCC) void gate_stream_kernel(GateArgs a) {
    constexpr int NW = kGsWaves, NT = 64 * NW;
    constexpr int RPB = 512 / KC;                     // rows per block: 1 (KC = 512) or 2 (KC = 256)
    constexpr int BLOCKS = 32 / RPB;                  // blocks of a 32-row tile
    constexpr int LPR = 64 / RPB;                     // lanes per row in a load
    constexpr int AL = BLOCKS / NW;                   // hidden-state loads per wave and stage
    constexpr int BBLOCKS = 4 * CB;                   // gate-row blocks per stage
    constexpr int A_BYTES = BLOCKS * kGsBlock, STAGE = A_BYTES + BBLOCKS * kGsBlock;
    constexpr int NS = gs_stages(NB, KC, CB, OCC);
    constexpr int LPS = AL + CB;                      // loads per wave and stage
    constexpr int KSW = KC / 16 / NW;                 // k-steps per wave and stage
    constexpr int RED_FLOATS = NB * 16 * 64;          // one wave's partial tile
    static_assert(KC == 256 || KC == 512, "stage width");
    static_assert(BBLOCKS <= NB * BLOCKS, "more gate-row blocks than columns");
    static_assert(NS >= 2 && (NS - 2) * LPS <= 63, "stages / wait count out of range");
    static_assert(2 * RED_FLOATS * 4 <= NS * STAGE, "the reduction reuses the stage buffers");
    __shared__ __attribute__((aligned(16))) unsigned char stage[NS * STAGE];
    __shared__ float logits[kTile][NB * 32 + 1];
    __shared__ int cnt[4 * 32];
    __shared__ float sbias[4 * 32];
    __shared__ __attribute__((aligned(16))) float s_sc[NW][64];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS targets go through M0
    const int g = lane >> 5, i = lane & 31;
    const int tile = blockIdx.x;
    const int g0 = blockIdx.y * a.gpw;
    const int Gl = min(a.gpw, a.G - g0);
    const int t0 = tile * kTile;
    const int N = Gl * a.E;                            // logit columns of the group (<= NB*32)
    const int nstage = a.d / KC;
    const int rot0 = (tile * 5 + (int)blockIdx.y * 3) % nstage;

    for (int x = tid; x < NB * 32; x += NT) cnt[x] = 0;
    for (int x = tid; x < N; x += NT) {
        const float *bp = pick(a.bias, g0 + x / a.E);
        sbias[x] = bp ? bp[x % a.E] : 0.f;
    }

    // per-lane sources of this wave's loads of a stage (column offset of the stage added at issue)
    const int sub = lane / LPR, c8 = (lane % LPR) * 8;
    const uint16_t *srcA[AL];
#pragma unroll
    for (int q = 0; q < AL; ++q) {
        const int row = wave * AL + q + BLOCKS * sub;  // rows past T re-read the last token (results dropped)
        srcA[q] = a.h + (size_t)min(t0 + row, a.T - 1) * a.d + c8;
    }
    const uint16_t *srcB[CB];
#pragma unroll
    for (int q = 0; q < CB; ++q) {
        const int b = wave * CB + q;                   // block b: rows n1 (+ BLOCKS) of 32-row block b / BLOCKS
        const int n1 = (b / BLOCKS) * 32 + b % BLOCKS;
        int n = n1 + BLOCKS * sub;
        if (n >= N) n = n1 < N ? n1 : 0;               // rows that do not exist alias one that does (same cache lines)
        srcB[q] = pick(a.Wg, g0 + n / a.E) + (size_t)(n % a.E) * a.d + c8;
    }
    const unsigned lds_base = (unsigned)(size_t)&stage[0];   // LDS byte offset: the low half of its flat address
#define EF_GS_DMA(gptr, lds_off)                                                                     \
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_off) : "memory")
    // every wave issues LPS loads per stage, unconditionally (past the end the last stage is re-read, in
    // bounds, into a buffer nobody reads any more), so "my loads of stage st have landed" is a constant count
#define EF_GS_ISSUE(st)                                                                              \
    {                                                                                                \
        int stc_ = min((st), nstage - 1) + rot0;                                                     \
        if (stc_ >= nstage) stc_ -= nstage;                                                          \
        const unsigned buf_ = lds_base + (unsigned)(((st) % NS) * STAGE);                            \
        _Pragma("unroll") for (int q = 0; q < AL; ++q)                                               \
            EF_GS_DMA(srcA[q] + stc_ * KC, buf_ + (unsigned)((wave * AL + q) * kGsBlock));           \
        _Pragma("unroll") for (int q = 0; q < CB; ++q)                                               \
            EF_GS_DMA(srcB[q] + stc_ * KC, buf_ + (unsigned)(A_BYTES + (wave * CB + q) * kGsBlock)); \
    }

    floatx16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) zero16(acc[nb]);

#pragma unroll
    for (int p = 0; p < NS - 1; ++p) EF_GS_ISSUE(p)
    // operand reads of lane (g, i): row i of a 32-row block sits in block i % BLOCKS at (i / BLOCKS) * 2 KC bytes;
    // columns 8g.. of a k-step.  Gate rows past the blocks that are loaded read block 0 (their columns are dropped).
    const int a_off = (i % BLOCKS) * kGsBlock + (i / BLOCKS) * (2 * KC) + 16 * g;
    int b_off[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int b = nb * BLOCKS + i % BLOCKS;
        b_off[nb] = A_BYTES + (b < BBLOCKS ? b : 0) * kGsBlock + (i / BLOCKS) * (2 * KC) + 16 * g;
    }
    for (int st = 0; st < nstage; ++st) {
        __builtin_amdgcn_s_waitcnt(gs_waitcnt((NS - 2) * LPS));   // my loads of stage st have landed
        __syncthreads();   // ... and everybody else's; all reads of stage st - 1 are done: its buffer is free
        EF_GS_ISSUE(st + NS - 1)
        const unsigned char *sb = stage + (st % NS) * STAGE;
#pragma unroll
        for (int q = 0; q < KSW; ++q) {
            const int kb = (wave * KSW + q) * 32;          // byte offset of the k-step inside a row
            const u32x4_t af = *reinterpret_cast<const u32x4_t *>(sb + a_off + kb);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const u32x4_t bf = *reinterpret_cast<const u32x4_t *>(sb + b_off[nb] + kb);
                acc[nb] = mfma32v(af, bf, acc[nb]);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(gs_waitcnt(0));   // the re-read stages past the end have landed too
    __syncthreads();
#undef EF_GS_DMA
#undef EF_GS_ISSUE

    // fixed-order tree over the waves' partial tiles through LDS: (w, w+2), then (0, 1)
    float *red = reinterpret_cast<float *>(stage);
    auto put = [&](int region) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) red[region * RED_FLOATS + (nb * 16 + v) * 64 + lane] = acc[nb][v];
    };
    auto add = [&](int region) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][v] += red[region * RED_FLOATS + (nb * 16 + v) * 64 + lane];
    };
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) add(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave == 0) {
        add(0);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) logits[8 * (v >> 2) + 4 * g + (v & 3)][nb * 32 + i] = acc[nb][v];
    }
    __syncthreads();
    gate_epilogue<NB, NW>(a, logits, cnt, sbias, s_sc, tile, g0, Gl, 0, kTile, false);
}

// whether a launch takes the streaming form: no K split or two-step form, whole stages, at most 64 logit
// columns per workgroup, and enough (tile, gate group) pairs that every compute unit streams
bool gate_stream_shape_ok(int T, int d, int G, int E, int gpw) {
    const int ntiles = (T + kTile - 1) / kTile;
    const int ngroups = (G + gpw - 1) / gpw;
    const int nb = (std::min(gpw, G) * E + 31) / 32;
    return d % 256 == 0 && nb <= 2 && (long long)ntiles * ngroups >= 192;
}
bool gate_stream_ok(const GateArgs &a) {
    return !a.two_step && a.ksplit == 1 && a.tsplit == 1 && gate_stream_shape_ok(a.T, a.d, a.G, a.E, a.gpw);
}

static hipError_t launch_gate_stream(const GateArgs &a, hipStream_t s) {
    const int ntiles = (a.T + kTile - 1) / kTile;
    const int ngroups = (a.G + a.gpw - 1) / a.gpw;
    const int n_max = std::min(a.gpw, a.G) * a.E;        // most logit columns of a gate group
    const dim3 grid(ntiles, ngroups), block(64 * kGsWaves);
    // stages of 512 columns (1 KiB per row and load) while the gate rows leave room for three of them in LDS
    // Two workgroups per compute unit wherever two pipelines of at least two stages fit its LDS: one's fill,
    // wave reduction and per-token epilogue then overlap the other's streaming (4.5 -> 6.2 TB/s of hidden states
    // at 131072 tokens and 8 logit columns).  Stages of 256 columns: with 512 the same LDS holds fewer stages
    // and the kernel is slower even at one workgroup per unit (4.5 against 5.0 TB/s).
    // With about one workgroup per compute unit in the launch there is nothing to overlap with, and the deeper
    // pipeline of the single-workgroup form is worth more (8192 tokens with 16 columns: 21 against 23 us); with more
    // than one per unit the single-workgroup form needs a second, mostly empty round over the compute units (9216
    // tokens took 24 us, 10240 tokens in the two-per-unit form 21 us), and two per unit fit the launch into one.
    const bool two = (long long)ntiles * ngroups > 256;
    if (n_max > 32) hipLaunchKernelGGL((gate_stream_kernel<2, 8, 256, 1>), grid, block, 0, s, a);
    else if (n_max > 8) {
        if (two) hipLaunchKernelGGL((gate_stream_kernel<1, 4, 256, 2>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((gate_stream_kernel<1, 4, 256, 1>), grid, block, 0, s, a);
    } else if (n_max > 4) {
        if (two) hipLaunchKernelGGL((gate_stream_kernel<1, 2, 256, 2>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((gate_stream_kernel<1, 2, 256, 1>), grid, block, 0, s, a);
    } else {
        if (two) hipLaunchKernelGGL((gate_stream_kernel<1, 1, 256, 2>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((gate_stream_kernel<1, 1, 256, 1>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

// second step of the K-split form: adds the partial logits of the splits in ascending order
// (fixed, so results do not depend on scheduling) and runs the per-token epilogue
template <int NB>
__global__ __launch_bounds__(64 * kGateWaves) void gate_finish_kernel(GateArgs a) {
    constexpr int NW = kGateWaves, NT = 64 * NW;
    __shared__ float logits[kTile][NB * 32 + 1];
    __shared__ int cnt[4 * 32];
    __shared__ float sbias[4 * 32];
    __shared__ __attribute__((aligned(16))) float s_sc[NW][64];
    const int tid = threadIdx.x;
    const int tile = blockIdx.x;
    const int g0 = blockIdx.y * a.gpw;
    const int Gl = min(a.gpw, a.G - g0);
    const int N = Gl * a.E;
    for (int x = tid; x < NB * 32; x += NT) cnt[x] = 0;
    for (int x = tid; x < N; x += NT) {
        const float *bp = pick(a.bias, g0 + x / a.E);
        sbias[x] = bp ? bp[x % a.E] : 0.f;
    }
    const float *src = a.part + (((size_t)tile * gridDim.y + blockIdx.y) * a.ksplit * kTile) * (NB * 32);
    // only the rows of the tokens this workgroup finishes (a token split leaves the others to its siblings)
    const int tok_n = kTile / a.tsplit, x_lo = blockIdx.z * tok_n * (NB * 32);
    for (int x = x_lo + tid; x < x_lo + tok_n * NB * 32; x += NT) {
        float pz[kGateMaxSplit];   // all loads first (one latency), then the adds in split order
#pragma unroll
        for (int z = 0; z < kGateMaxSplit; ++z)
            pz[z] = z < a.ksplit ? src[(size_t)z * kTile * NB * 32 + x] : 0.f;
        float v = 0.f;
#pragma unroll
        for (int z = 0; z < kGateMaxSplit; ++z) v += pz[z];
        logits[x / (NB * 32)][x % (NB * 32)] = v;
    }
    __syncthreads();
    gate_epilogue<NB>(a, logits, cnt, sbias, s_sc, tile, g0, Gl, blockIdx.z * tok_n, tok_n, a.tsplit > 1);
}

template <int NB>
static hipError_t launch_gate_nb(const GateArgs &a, hipStream_t s) {
    const int ntiles = (a.T + kTile - 1) / kTile;
    const int ngroups = (a.G + a.gpw - 1) / a.gpw;
    hipLaunchKernelGGL((gate_kernel<NB>), dim3(ntiles, ngroups, a.ksplit), dim3(64 * kGateWaves), 0, s, a);
    if (a.two_step)
        hipLaunchKernelGGL((gate_finish_kernel<NB>), dim3(ntiles, ngroups, a.tsplit), dim3(64 * kGateWaves), 0, s,
                           a);
    return hipGetLastError();
}

// K splits of a gate launch: batches of few token tiles are bound by the latency of walking d in
// panels inside one workgroup (the hidden states and gate rows are cold in L2 after the expert
// weights of the previous layer streamed through, and only four panels are in flight), so the
// panels are dealt to several workgroups per (tile, group), four panels each (one round trip),
// whose partial logits a second, short kernel adds up.  `part_floats` is the scratch available.
// Token split of the finishing kernel.  With more than 16 experts a token takes a whole wave round
// of the epilogue (selection by rank costs E^2 compares per token), so the 32 tokens of a tile are
// dealt to up to 4 workgroups when the launch would otherwise leave most of the chip idle.
int gate_pick_tsplit(int T, int G, int E, int gpw) {
    const int ntiles = (T + kTile - 1) / kTile;
    const int ngroups = (G + gpw - 1) / gpw;
    if (E <= 16) return 1;
    int ts = 1;
    while (ts < 4 && ntiles * ngroups * ts < 512) ts *= 2;
    return ts;
}

int gate_pick_ksplit(int T, int d, int G, int E, int gpw, size_t part_floats) {
    const int ntiles = (T + kTile - 1) / kTile;
    const int ngroups = (G + gpw - 1) / gpw;
    const int nb = (std::min(gpw, G) * E + 31) / 32;
    const int kc = nb == 1 ? 256 : 128;
    const int nstage = (d + kc - 1) / kc;
    int ks = 1;
    while (ks < kGateMaxSplit && nstage / (ks * 2) >= 4 && ntiles * ngroups * ks < 64 &&
           (size_t)ntiles * ngroups * (ks * 2) * kTile * nb * 32 <= part_floats)
        ks *= 2;
    return ks;
}

// gates per workgroup: up to 128 logit columns; one 32-column block when there are few token
// tiles (the launch is latency-bound then and more, lighter workgroups finish sooner)
int gate_pick_gpw(int T, int G, int E) {
    const int ntiles = (T + kTile - 1) / kTile;
    const int cols = ntiles < 64 ? 32 : 128;
    int gpw = cols / E;
    if (gpw < 1) gpw = 1;
    if (gpw > G) gpw = G;
    return gpw;
}

hipError_t launch_gate(const GateArgs &a, hipStream_t s) {
    if (a.T <= 0 || a.G <= 0) return hipSuccess;
    if (a.gpw < 1 || a.gpw * a.E > 128 || a.G > kMaxGates) return hipErrorInvalidValue;
    if (a.ksplit < 1 || (a.ksplit > 1 && !a.two_step) || (a.two_step && !a.part)) return hipErrorInvalidValue;
    if (a.tsplit != 1 && a.tsplit != 2 && a.tsplit != 4) return hipErrorInvalidValue;
    if (a.tsplit > 1 && !a.two_step) return hipErrorInvalidValue;
    if (a.stream && gate_stream_ok(a)) return launch_gate_stream(a, s);
    const int nb = (std::min(a.gpw, a.G) * a.E + 31) / 32;
    switch (nb) {
        case 1: return launch_gate_nb<1>(a, s);
        case 2: return launch_gate_nb<2>(a, s);
        case 3: return launch_gate_nb<3>(a, s);
        case 4: return launch_gate_nb<4>(a, s);
        default: return hipErrorInvalidValue;
    }
}

// ------------------------------------------------------------------------------------------
// stable grouping by expert: per-tile counts (from the gate kernel) -> scan -> scatter
// ------------------------------------------------------------------------------------------

// the same scan on counts already in LDS, in place: counts[b*E + e] becomes the exclusive prefix
__device__ __forceinline__ int scan_expert_inplace(int *cnt, int ntiles, int E, int e, int lane) {
    int carry = 0;
    for (int c0 = 0; c0 < ntiles; c0 += 64) {
        const int b = c0 + lane;
        const int v = b < ntiles ? cnt[b * E + e] : 0;
        int incl = v;
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        if (b < ntiles) cnt[b * E + e] = carry + incl - v;
        carry += __shfl(incl, 63);
    }
    return carry;
}

// the same exclusive prefix over the tiles of expert e by one thread, for batches of a few tiles
constexpr int kGroupSerialTiles = 4;
__device__ __forceinline__ int scan_expert_serial(int *cnt, int ntiles, int E, int e) {
    int run = 0;
    for (int b = 0; b < ntiles; ++b) {
        const int v = cnt[b * E + e];
        cnt[b * E + e] = run;
        run += v;
    }
    return run;
}

// one wave: stable scatter of the assignments of token tile b.  nxt [64] (LDS, this wave's own) holds
// the next free position of every expert for this tile.  Per chunk of 64 assignments the lanes with
// the same expert are found with six ballots (one per bit of the expert id, E <= 64): a lane's
// position is its expert's next free one plus the number of lower lanes with the same expert, and
// the lowest such lane advances the expert's entry.  LDS operations of one wave execute in order,
// so the chunks need no barrier between them.
__device__ __forceinline__ void scatter_tile(const int32_t *__restrict__ ids, int T, int k, int b, int lane,
                                             int *nxt, int32_t *__restrict__ perm,
                                             int32_t *__restrict__ inv_perm) {
    const int tok0 = b * kTile;
    const int ntok = min(kTile, T - tok0);
    const int a0 = tok0 * k, n = ntok * k;
    for (int c0 = 0; c0 < n; c0 += 64) {
        const int idx = c0 + lane;
        const bool valid = idx < n;
        const int e = valid ? ids[a0 + idx] : 0;
        unsigned long long same = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 6; ++bit) {
            const bool set = (e >> bit) & 1;
            const unsigned long long bb = __ballot(valid && set);
            same &= set ? bb : ~bb;
        }
        if (valid) {
            const int pos = nxt[e] + __popcll(same & ((1ull << lane) - 1ull));
            perm[pos] = a0 + idx;
            inv_perm[a0 + idx] = pos;
        }
        wave_lds_sync();
        if (valid && (same & ((1ull << lane) - 1ull)) == 0) nxt[e] += __popcll(same);   // lowest lane of its expert
        wave_lds_sync();
    }
}

// Hand the per-expert counts and the predicted demand histograms to the host through host-mapped
// memory.  Every word carries the call's tag (0..254) in its top 8 bits (values are below 2^24), and
// the host polls until all the words it expects show the tag, then overwrites them with tag 255: no
// fence and no separate flag, which would cost the kernel a system-scope fence of about 5 us.
// A word goes to host memory with a system-scope store the wave does not wait for (a volatile store is followed
// by a wait for its completion, about 1 us over the link, in the middle of the kernel's critical path).
__device__ __forceinline__ void host_word(int32_t *p, int32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ void export_meta(const GroupExport &ex, const int *total, int E) {
    if (!ex.host_meta) return;  // uniform
    const int tag = (int)((unsigned)(ex.seq & 0xFF) << 24);
    int32_t *hm = ex.host_meta;
    for (int x = threadIdx.x; x < E; x += blockDim.x) host_word(hm + x, tag | total[x]);
    for (int x = threadIdx.x; x < ex.n_hist; x += blockDim.x) host_word(hm + kMetaHist + x, tag | ex.hist[x]);
    for (int x = threadIdx.x; x < ex.n_clear; x += blockDim.x) ex.hist[x] = 0;   // ready for the next layer
}

// Batches of more than kGroupSmallTiles token tiles: one workgroup per expert forms the exclusive prefix of
// that expert's per-tile counts over the tiles (16 waves, a contiguous range of tiles each: totals first,
// then the scan with the bases of the waves before), and leaves the expert's total in counts[e].
__global__ __launch_bounds__(1024) void group_scan_kernel(const int32_t *__restrict__ bc, int ntiles, int E,
                                                          int32_t *__restrict__ blockbase,
                                                          int32_t *__restrict__ counts) {
    __shared__ int wtot[16];
    const int e = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int per = (((ntiles + 15) / 16 + 63) / 64) * 64;     // tiles per wave, whole chunks of 64
    const int lo = min(ntiles, wave * per), hi = min(ntiles, lo + per);
    int sum = 0;
    for (int b = lo + lane; b < hi; b += 64) sum += bc[(size_t)b * E + e];
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) wtot[wave] = sum;
    __syncthreads();
    int carry = 0, all = 0;
    for (int w = 0; w < 16; ++w) {
        if (w < wave) carry += wtot[w];
        all += wtot[w];
    }
    for (int c0 = lo; c0 < hi; c0 += 64) {
        const int b = c0 + lane;
        const int v = b < hi ? bc[(size_t)b * E + e] : 0;
        int incl = v;
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        if (b < hi) blockbase[(size_t)b * E + e] = carry + incl - v;
        carry += __shfl(incl, 63);
    }
    if (threadIdx.x == 0) counts[e] = all;
}

// ... then one wave per token tile scatters: every wave forms the exclusive prefix of the experts' totals (E <= 64
// lanes) itself; the first workgroup also writes `offsets` and hands counts and histograms to the host.
constexpr int kScatterWaves = 4;
__global__ __launch_bounds__(64 * kScatterWaves) void group_scatter_kernel(const int32_t *__restrict__ ids, int T, int k, int E,
                                                                           int ntiles,
                                                                           const int32_t *__restrict__ blockbase,
                                                                           const int32_t *__restrict__ counts,
                                                                           int32_t *__restrict__ offsets,
                                                                           int32_t *__restrict__ perm,
                                                                           int32_t *__restrict__ inv_perm, GroupExport ex) {
    __shared__ int nxt[kScatterWaves][64];
    __shared__ int total[kMaxE];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t = lane < E ? counts[lane] : 0;
    int incl = t;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
    }
    if (blockIdx.x == 0) {   // uniform over the workgroup
        if (wave == 0) {
            if (lane < E) {
                offsets[lane] = incl - t;
                total[lane] = t;
            }
            if (lane == 63) offsets[E] = incl;
        }
        __syncthreads();
        export_meta(ex, total, E);
    }
    const int b = blockIdx.x * kScatterWaves + wave;
    if (b >= ntiles) return;
    nxt[wave][lane] = (lane < E) ? (incl - t) + blockbase[(size_t)b * E + lane] : 0;
    wave_lds_sync();
    scatter_tile(ids, T, k, b, lane, nxt[wave], perm, inv_perm);
}

// scan + scatter in one workgroup for up to kGroupSmallTiles token tiles (prefixes stay in LDS)
__global__ __launch_bounds__(1024) void group_small_kernel(const int32_t *__restrict__ bc, int ntiles,
                                                           const int32_t *__restrict__ ids, int T, int k, int E,
                                                           int32_t *__restrict__ counts,
                                                           int32_t *__restrict__ offsets,
                                                           int32_t *__restrict__ perm,
                                                           int32_t *__restrict__ inv_perm, GroupExport ex) {
    __shared__ int base[kGroupSmallTiles * kMaxE];
    __shared__ int total[kMaxE];
    __shared__ int offs[kMaxE + 1];
    __shared__ int nxt[16][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // one memory round trip brings the per-tile counts into LDS; the scans then run from there, in place
    for (int x = threadIdx.x; x < ntiles * E; x += blockDim.x) base[x] = bc[x];
    __syncthreads();
    if (ntiles <= kGroupSerialTiles) {   // a few tiles: one thread per expert walks them (no shuffle rounds)
        if (threadIdx.x < (unsigned)E) total[threadIdx.x] = scan_expert_serial(base, ntiles, E, threadIdx.x);
    } else {
        for (int e = wave; e < E; e += 16) {
            int tot = scan_expert_inplace(base, ntiles, E, e, lane);
            if (lane == 0) total[e] = tot;
        }
    }
    __syncthreads();
    if (wave == 0) {   // exclusive scan of the E <= 64 totals across the lanes of one wave
        const int t = lane < E ? total[lane] : 0;
        int incl = t;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        if (lane < E) {
            counts[lane] = t;
            offsets[lane] = incl - t;
            offs[lane] = incl - t;
        }
        if (lane == 63) {
            offsets[E] = incl;
            offs[E] = incl;
        }
    }
    __syncthreads();
    export_meta(ex, total, E);   // the host starts planning while the scatter below still runs
    for (int b = wave; b < ntiles; b += 16) {
        nxt[wave][lane] = (lane < E) ? offs[lane] + base[b * E + lane] : 0;
        wave_lds_sync();
        scatter_tile(ids, T, k, b, lane, nxt[wave], perm, inv_perm);
    }
}

// ------------------------------------------------------------------------------------------
// Decode-sized batches (at most kFusedMaxTiles token tiles) with a K-split gate: the second step of
// the gate (sum of the partial logits, per-token epilogue) for every (tile, gate group) and the
// grouping, in ONE workgroup of 16 waves.  The per-tile expert counts never leave LDS, and one
// kernel launch with its dependency gap and one memory round trip disappear from the layer's
// critical path.  Arithmetic and orders are those of gate_finish_kernel + group_small_kernel.
// Dynamic LDS: the logits of all pairs, [pairs][kTile][NB*32 + 1] floats.
// ------------------------------------------------------------------------------------------
template <int NB>
__global__ __launch_bounds__(1024) void gate_finish_group_kernel(GateArgs a, int32_t *__restrict__ counts,
                                                                 int32_t *__restrict__ offsets,
                                                                 int32_t *__restrict__ perm,
                                                                 int32_t *__restrict__ inv_perm, GroupExport ex) {
    constexpr int NW = 16, NT = 64 * NW, ROW = NB * 32 + 1;
    extern __shared__ float fz_logits[];                       // [pairs][kTile][ROW]
    __shared__ int cnt[kFusedMaxTiles * kMaxGates * kMaxE];    // [(tile, gate)][expert]
    __shared__ float sbias[kMaxGates * kMaxE];                 // [gate][expert]
    __shared__ __attribute__((aligned(16))) float s_sc[NW][64];
    __shared__ int base[kFusedMaxTiles * kMaxE];
    __shared__ int total[kMaxE];
    __shared__ int offs[kMaxE + 1];
    __shared__ int nxt[NW][64];
    __shared__ int32_t s_ids[kFusedMaxTiles * kTile * kMaxK];   // ids of the routed gate, for the scatter below
    // the wave index as a scalar: what is derived from it (the gate a round works on) stays in scalar registers
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int E = a.E, G = a.G;
    const int ntiles = (a.T + kTile - 1) / kTile;
    const int ngroups = (G + a.gpw - 1) / a.gpw;
    const int pairs = ntiles * ngroups;

    for (int x = tid; x < ntiles * G * E; x += NT) cnt[x] = 0;
    for (int x = tid; x < G * E; x += NT) {
        const float *bp = pick(a.bias, x / E);
        sbias[x] = bp ? bp[x % E] : 0.f;
    }
    // partial logits of pair (tile, group): [split][kTile][NB*32], pairs in (tile, group) order
    for (int idx = tid; idx < pairs * kTile * NB * 32; idx += NT) {
        const int pair = idx / (kTile * NB * 32), x = idx % (kTile * NB * 32);
        const float *src = a.part + (size_t)pair * a.ksplit * kTile * (NB * 32);
        float pz[kGateMaxSplit];   // all loads first (one latency), then the adds in split order
#pragma unroll
        for (int z = 0; z < kGateMaxSplit; ++z) pz[z] = z < a.ksplit ? src[(size_t)z * kTile * NB * 32 + x] : 0.f;
        float v = 0.f;
#pragma unroll
        for (int z = 0; z < kGateMaxSplit; ++z) v += pz[z];
        fz_logits[(size_t)(pair * kTile + x / (NB * 32)) * ROW + x % (NB * 32)] = v;
    }
    __syncthreads();

    // per-token epilogue over all (tile, gate, token chunk) triples, dealt to the 16 waves
    {
        int W = 8;
        while (W < E) W <<= 1;
        const int per_wave = 64 / W;
        const int sub = lane / W, e = lane % W;
        const int cpg = kTile / per_wave;                  // chunks per (tile, gate)
        const int total_chunks = ntiles * G * cpg;
        const bool evalid = e < E;
        const float NEG_INF = -__builtin_inff();
        for (int it = 0; it * NW < total_chunks; ++it) {
            const int chunk = it * NW + wave;
            const bool cact = chunk < total_chunks;
            const int tile = cact ? chunk / (G * cpg) : 0;
            const int gi = cact ? (chunk / cpg) % G : 0;
            const int grp = gi / a.gpw, gl = gi - grp * a.gpw;
            const int ti = (chunk % cpg) * per_wave + sub;
            const int t = tile * kTile + ti;
            const bool live = cact && t < a.T;
            const bool want_w = cact && (a.w != nullptr) && gi == 0;  // wave-uniform
            float z = NEG_INF;
            if (live && evalid)
                z = fz_logits[(size_t)((tile * ngroups + grp) * kTile + ti) * ROW + gl * E + e] + sbias[gi * E + e];
            float sc = z;
            if (live && evalid) {
                if ((pick(a.resident, gi) >> e) & 1ull) sc += a.beta;
                if (a.delta && gi >= a.delta_gate_begin) {
                    int req = a.tok2req ? a.tok2req[t] : 0;
                    sc += a.delta[(size_t)req * a.delta_req_stride + (gi - a.delta_gate_begin) * E + e];
                }
            }
            s_sc[wave][lane] = sc;
            wave_lds_sync();
            const float4 *srow = reinterpret_cast<const float4 *>(&s_sc[wave][sub * W]);
            int rank = 0;
            for (int j = 0; j < W; j += 4) {
                const float4 v = srow[j >> 2];
                rank += (v.x > sc || (v.x == sc && j + 0 < e)) ? 1 : 0;
                rank += (v.y > sc || (v.y == sc && j + 1 < e)) ? 1 : 0;
                rank += (v.z > sc || (v.z == sc && j + 2 < e)) ? 1 : 0;
                rank += (v.w > sc || (v.w == sc && j + 3 < e)) ? 1 : 0;
            }
            const bool sel = live && evalid && rank < a.k;
            float exv = 0.f, den = 1.f;
            if (want_w) {
                float m = z;   // lanes without an expert hold -inf
                for (int off = W >> 1; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
                exv = (live && evalid) ? __expf(z - m) : 0.f;
                den = (a.renorm && !sel) ? 0.f : exv;
                for (int off = W >> 1; off >= 1; off >>= 1) den += __shfl_xor(den, off);
            }
            const unsigned long long ball = __ballot(sel);
            const unsigned long long submask = (W == 64) ? ball : ((ball >> (sub * W)) & ((1ull << W) - 1ull));
            const int slot = __popcll(submask & ((1ull << e) - 1ull));   // ascending expert id
            if (sel) {
                pick(a.ids, gi)[(size_t)t * a.k + slot] = e;
                if (gi == 0) s_ids[t * a.k + slot] = e;
                if (want_w) a.w[(size_t)t * a.k + slot] = exv / den * a.routed_scale;
                atomicAdd(&cnt[(tile * G + gi) * E + e], 1);
            }
            wave_lds_sync();   // the wave's row of s_sc is rewritten in the next round
        }
    }
    __syncthreads();

    // demand histograms of the look-ahead gates: to the host hand-over straight from LDS, or added to
    // the caller's (zeroed) device arrays
    const int tag = (int)((unsigned)(ex.seq & 0xFF) << 24);
    for (int x = tid; x < G * E; x += NT) {
        const int gi = x / E, ee = x % E;
        int sum = 0;
        for (int b = 0; b < ntiles; ++b) sum += cnt[(b * G + gi) * E + ee];
        int32_t *hp = pick(a.hist, gi);
        if (!hp) continue;
        if (ex.host_meta) {
            const int at = (int)(hp - ex.hist) + ee;           // position inside the exported histograms
            if (at >= 0 && at < ex.n_hist) host_word(ex.host_meta + kMetaHist + at, tag | sum);
        } else if (sum > 0) {
            atomicAdd(&hp[ee], sum);
        }
    }
    // grouping of the routed gate (gate 0) from its per-tile counts
    for (int x = tid; x < ntiles * E; x += NT) base[x] = cnt[((x / E) * G) * E + x % E];
    __syncthreads();
    if (tid < E) total[tid] = scan_expert_serial(base, ntiles, E, tid);   // at most kFusedMaxTiles tiles
    __syncthreads();
    if (wave == 0) {   // exclusive scan of the E <= 64 totals across the lanes of one wave
        const int t = lane < E ? total[lane] : 0;
        int incl = t;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        if (lane < E) {
            counts[lane] = t;
            offsets[lane] = incl - t;
            offs[lane] = incl - t;
        }
        if (lane == 63) {
            offsets[E] = incl;
            offs[E] = incl;
        }
    }
    __syncthreads();
    if (ex.host_meta)   // the host starts planning while the scatter below still runs
        for (int x = tid; x < E; x += NT) host_word(ex.host_meta + x, tag | total[x]);
    // the scatter reads the routed ids from the copy the epilogue above left in LDS (reading them back from
    // global memory would be one more memory round trip); same workgroup, ordered by the barriers
    for (int b = wave; b < ntiles; b += NW) {
        nxt[wave][lane] = (lane < E) ? offs[lane] + base[b * E + lane] : 0;
        wave_lds_sync();
        scatter_tile(s_ids, a.T, a.k, b, lane, nxt[wave], perm, inv_perm);
    }
}

size_t gate_fused_lds_bytes(int T, int G, int E, int gpw) {
    const int ntiles = (T + kTile - 1) / kTile, ngroups = (G + gpw - 1) / gpw;
    const int nb = (std::min(gpw, G) * E + 31) / 32;
    return (size_t)ntiles * ngroups * kTile * (nb * 32 + 1) * sizeof(float);
}

template <int NB>
static hipError_t launch_gate_fused_nb(const GateArgs &a, int32_t *counts, int32_t *offsets, int32_t *perm,
                                       int32_t *inv_perm, const GroupExport &ex, hipStream_t s) {
    const int ntiles = (a.T + kTile - 1) / kTile;
    const int ngroups = (a.G + a.gpw - 1) / a.gpw;
    hipLaunchKernelGGL((gate_kernel<NB>), dim3(ntiles, ngroups, a.ksplit), dim3(64 * kGateWaves), 0, s, a);
    hipLaunchKernelGGL((gate_finish_group_kernel<NB>), dim3(1), dim3(1024),
                       gate_fused_lds_bytes(a.T, a.G, a.E, a.gpw), s, a, counts, offsets, perm, inv_perm, ex);
    return hipGetLastError();
}

// K-split gate + fused finish/grouping.  The first gate must be the routed one (ids[0], w, renorm).
hipError_t launch_gate_fused(const GateArgs &a, int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                             const GroupExport &ex, hipStream_t s) {
    const int ntiles = (a.T + kTile - 1) / kTile;
    if (a.T <= 0 || ntiles > kFusedMaxTiles || a.G < 1 || a.G > kMaxGates || !a.two_step || a.tsplit != 1 ||
        !a.part || a.ksplit < 1 || a.ksplit > kGateMaxSplit || a.gpw < 1 || a.gpw * a.E > 128 || !a.ids[0] ||
        gate_fused_lds_bytes(a.T, a.G, a.E, a.gpw) > kFusedMaxLds)
        return hipErrorInvalidValue;
    if (ex.host_meta)   // exported histograms must be the arrays the look-ahead gates point at
        for (int gi = 0; gi < a.G; ++gi)
            if (a.hist[gi] && (a.hist[gi] < ex.hist || a.hist[gi] + a.E > ex.hist + ex.n_hist))
                return hipErrorInvalidValue;
    const int nb = (std::min(a.gpw, a.G) * a.E + 31) / 32;
    switch (nb) {
        case 1: return launch_gate_fused_nb<1>(a, counts, offsets, perm, inv_perm, ex, s);
        case 2: return launch_gate_fused_nb<2>(a, counts, offsets, perm, inv_perm, ex, s);
        case 3: return launch_gate_fused_nb<3>(a, counts, offsets, perm, inv_perm, ex, s);
        case 4: return launch_gate_fused_nb<4>(a, counts, offsets, perm, inv_perm, ex, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_group(const int32_t *blockcounts, const int32_t *ids, int T, int k, int E, int32_t *blockbase,
                        int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                        const GroupExport &ex, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    const int ntiles = (T + kTile - 1) / kTile;
    if (ntiles <= kGroupSmallTiles) {
        hipLaunchKernelGGL(group_small_kernel, dim3(1), dim3(1024), 0, s, blockcounts, ntiles, ids, T, k, E,
                           counts, offsets, perm, inv_perm, ex);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(group_scan_kernel, dim3(E), dim3(1024), 0, s, blockcounts, ntiles, E, blockbase, counts);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(group_scatter_kernel, dim3((ntiles + kScatterWaves - 1) / kScatterWaves), dim3(64 * kScatterWaves),
                       0, s, ids, T, k, E, ntiles, blockbase, counts, offsets, perm, inv_perm, ex);
    return hipGetLastError();
}

}  // namespace ef
