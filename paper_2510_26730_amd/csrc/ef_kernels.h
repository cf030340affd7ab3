// Internal launch interface between the C-ABI layer and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace ef {

constexpr int kMaxE = 64;      // experts per layer
constexpr int kMaxK = 8;       // top-k
constexpr int kMaxGates = 8;   // gate matrices per launch (look-ahead + 1)
constexpr int kTile = 32;      // tokens per tile (rows of one matrix-core operand fragment)
constexpr int kMaxGroups = kMaxE + 1;  // routed experts + the dense shared FFN
constexpr int kDownColBlocks = 2;      // 32-column blocks per wave in the second FFN half
constexpr int kGroupSmallTiles = 64;   // token tiles the single-workgroup grouping kernel handles

// Gate / predict launch: G gate matrices applied to the same hidden states.
struct GateArgs {
    const uint16_t *h;             // [T,d] bf16
    int T, d, E, k, G;
    const uint16_t *Wg[kMaxGates]; // [E,d] bf16 each
    const float *bias[kMaxGates];  // [E] or null
    uint64_t resident[kMaxGates];  // bit e: expert e of that gate's layer is in the cache
    float beta;
    const float *delta;            // f32 or null: delta[req*delta_req_stride + (gate-delta_gate_begin)*E + e]
    int delta_req_stride;
    int delta_gate_begin;          // gates below this index take no delta (the current layer's own gate)
    const int32_t *tok2req;        // [T] or null
    int32_t *ids[kMaxGates];       // per gate: [T,k]
    float *w;                      // [T,k] combine weights of gate 0, or null
    int renorm;
    float routed_scale;
    int32_t *hist[kMaxGates];      // per gate: [E] accumulated with integer atomics, or null
    int32_t *blockcounts;          // [ntiles,E] per-tile counts of gate 0, or null
    int gpw;                       // gates per workgroup (gpw * E <= 128 logit columns)
    int ksplit;                    // workgroups that share the K range of one (tile, gate group); >= 1
    int two_step;                  // 1: gate_kernel leaves partial logits, gate_finish_kernel does the per-token part
    int tsplit;                    // two_step: workgroups that share the 32 tokens of a tile in the finish (1, 2, 4)
    float *part;                   // two_step: [tiles][groups][ksplit][32][32 * column blocks] partial logits
    int stream;                    // 1: launches that qualify (gate_stream_ok) take the streaming form of the kernel
};

// Grouped FFN launch: one group per active expert (+ one for the dense shared FFN).
struct GroupTable {
    int n_groups;
    int wg_start[kMaxGroups + 1];  // first workgroup of each group in this launch (cumulative)
    int tile_start[kMaxGroups];    // first 32-row tile of the group in the packed X / activation space
    int n_tiles[kMaxGroups];
    int row_offset[kMaxGroups];    // first row of the group in Y (= offsets[e]; T*k for the shared FFN)
    int count[kMaxGroups];         // rows in the group
    int F[kMaxGroups];             // FFN hidden dim of the group
    long long act_off[kMaxGroups]; // first 16-byte unit of the group's activation fragments
    const void *blob[kMaxGroups];  // packed weights (cache slot or shared blob)
    int xcd_rot[kMaxGroups];       // tiled kernels: the group's first weight panel goes to this XCD (0..7)
};

// Optional hand-over of counts and predicted histograms to the host (host-mapped memory): every word is
// (tag << 24) | value, value < 2^24, tag = `seq` in 0..254 (the caller's sequence number modulo 255; the host
// marks words it has consumed, and the fresh buffer, with tag 255, which no call carries).
constexpr int kMetaHist = kMaxE;                          // hist starts after the E counts
constexpr int kMetaInts = kMaxE + (kMaxGates - 1) * kMaxE;
constexpr int kMetaValueBits = 24;
struct GroupExport {
    int32_t *host_meta;   // device view of the host-mapped buffer, or null
    int32_t *hist;        // [n_hist] device histograms to copy out; [n_clear] is zeroed afterwards
    int n_hist;
    int n_clear;
    int seq;
};

// Describes how rows are gathered into tiles for the X packing kernel.
struct PackTable {
    int n_groups;
    int tile_start[kMaxGroups + 1]; // cumulative over groups
    int row_offset[kMaxGroups];     // offsets[e] (index into perm); -1 = identity (shared FFN: row = token)
    int count[kMaxGroups];
};

hipError_t launch_fill_i32(int32_t *p, int n, int32_t v, hipStream_t s);
int gate_pick_gpw(int T, int G, int E);
int gate_pick_ksplit(int T, int d, int G, int E, int gpw, size_t part_floats);
int gate_pick_tsplit(int T, int G, int E, int gpw);
hipError_t launch_gate(const GateArgs &a, hipStream_t s);
// batches of many token tiles: hidden states streamed through LDS by direct global -> LDS loads
bool gate_stream_ok(const GateArgs &a);
bool gate_stream_shape_ok(int T, int d, int G, int E, int gpw);
// decode-sized batches: K-split gate, then its second step and the grouping fused in one workgroup
constexpr int kFusedMaxTiles = 2;
constexpr size_t kFusedMaxLds = 48 * 1024;   // dynamic LDS of the fused kernel (logits of all pairs)
size_t gate_fused_lds_bytes(int T, int G, int E, int gpw);
hipError_t launch_gate_fused(const GateArgs &a, int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                             const GroupExport &ex, hipStream_t s);
hipError_t launch_group(const int32_t *blockcounts, const int32_t *ids, int T, int k, int E, int32_t *blockbase,
                        int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                        const GroupExport &ex, hipStream_t s);
// f16: write fp16 instead of bf16 fragments (contexts with 4-bit experts)
hipError_t launch_pack_x(const PackTable &pt, int total_tiles, const uint16_t *h, int d, int k,
                         const int32_t *perm, void *xp, bool f16, hipStream_t s);
hipError_t launch_pack_x_dev(const int32_t *counts, const int32_t *offsets, int E, bool has_shared, int T,
                             int max_tiles, const uint16_t *h, int d, int k, const int32_t *perm, void *xp,
                             bool f16, hipStream_t s);
hipError_t launch_ffn_gate_up(const GroupTable &gt, int total_wgs, int tiles_per_pass, int ks, const void *xp,
                              void *act, int d, hipStream_t s);
hipError_t launch_ffn_down(const GroupTable &gt, int total_wgs, int tiles_per_pass, int ksg, const void *act,
                           float *y, long long y_plane, int d, hipStream_t s);
// K-slice planes of Y each expert's rows (and the shared FFN's) were written to: the streamed and the tiled launch
// of a layer choose their slice counts separately
struct PlaneTable {
    uint8_t routed[kMaxE];
    uint8_t shared;
};
hipError_t launch_combine(const float *y, const PlaneTable &planes, long long y_plane, const float *w,
                          const int32_t *ids, const int32_t *inv_perm, int T, int k, int d, long long shared_row0,
                          float *out, hipEvent_t done, hipStream_t s);

// 4-bit expert weights (d and F multiples of 128): a workgroup of the first half takes four 32-row
// blocks of F, one of the second half eight 32-column blocks of d and one of ksg K-slices
inline int ffn_gate_up_q4_wgs(int F, int n_tiles, int tiles_per_pass) {
    return (F / 128) * ((n_tiles + tiles_per_pass - 1) / tiles_per_pass);
}
inline int ffn_down_q4_wgs(int d, int n_tiles, int tiles_per_pass, int ksg) {
    return ((d / 32 + 7) / 8) * ((n_tiles + tiles_per_pass - 1) / tiles_per_pass) * ksg;
}
hipError_t launch_ffn_gate_up_q4(const GroupTable &gt, int total_wgs, int tiles_per_pass, const void *xp, void *act,
                                 int d, hipStream_t s);
hipError_t launch_ffn_down_q4(const GroupTable &gt, int total_wgs, int tiles_per_pass, int ksg, const void *act,
                              float *y, long long y_plane, int d, hipStream_t s);
// Expands 4-bit expert blobs into 16-bit blobs of the bf16 layout whose elements are the fp16 numbers
// (q - 8) * s, the same values the 4-bit kernels form on the fly: large groups then run through the
// tiled matrix-core kernels, which read every weight many times.
struct DequantTable {
    int n;
    int F[kMaxGroups];
    const void *src[kMaxGroups];   // 4-bit blob (cache slot)
    void *dst[kMaxGroups];         // 3*d*F*2 bytes each
};
hipError_t launch_dequant_q4(const DequantTable &t, int d, hipStream_t s);

// Dist(t): scratch floats launch_token_dist needs for T tokens (norms, partials, workgroup sums)
size_t dist_scratch_floats(int T);
// Batches of up to kDistSmallMaxTokens tokens take a kernel that reads the tokens as they are (form 0 only); the Gram
// forms read the packed copy, which the caller writes first.
constexpr int kDistSmallMaxTokens = 256;
inline bool dist_needs_packed(int T, int form) { return !(form == 0 && T <= kDistSmallMaxTokens); }
// `form`: 0 = by batch size, 1 = register-fed 128 x 256 Gram blocks, 2 = 256 x 256 blocks through LDS (same bits)
hipError_t launch_token_dist(const uint16_t *h, int T, int d, const void *xp, float *scratch, float *tok_dist,
                             double *dist, int form, hipStream_t s);

// f16: the W1 / W3 fragments and the packed tokens hold fp16 instead of bf16 (4-bit contexts: the blobs are
// the staging copies launch_dequant_q4 wrote).  Activations and W2 fragments are fp16 in every context.
hipError_t launch_ffn_gate_up_tiled(const GroupTable &gt, int total_wgs, const void *xp, void *act, int d,
                                    bool f16, hipStream_t s);
// `split_grp` (or -1): the group of this launch whose slice count is `split_ksg` instead of `ksg`
hipError_t launch_ffn_down_tiled(const GroupTable &gt, int total_wgs, int ksg, int split_grp, int split_ksg,
                                 const void *act, float *y, long long y_plane, int d, hipStream_t s);

// The tiled (matrix-core bound) kernels take groups of at least kTiledMinTiles token tiles whose shapes
// fit their 256 x 256 workgroup tiles: F a multiple of 128 (4 row blocks), d a multiple of 256 (8 column
// blocks) and of 32 (whole k-step pairs).
constexpr int kTiledMinTiles = 8;
inline bool ffn_tiled_ok(int d, int F, int n_tiles) {
    return n_tiles >= kTiledMinTiles && F % 128 == 0 && d % 256 == 0;
}
// Workgroups are dealt to the 8 XCDs round-robin by index, and each XCD has an L2 of its own.  The
// tiled kernels therefore number a group's workgroups so that those an XCD runs side by side
// (indices congruent mod 8, consecutive) form blocks of kTiledPanelBlock weight panels x all token
// panels: a weight panel is then fetched into one L2 once and read by every token panel there.  The
// count is padded to whole blocks; workgroups that fall past the last weight panel exit at once.
constexpr int kTiledPanelBlock = 2;
// With fewer than 16 weight panels (d = 2048 gives the second half 8) blocks of two would leave half of the
// XCDs without a panel: such launches deal single panels.
__host__ __device__ inline int tiled_panel_block(int npanels) { return npanels >= 8 * kTiledPanelBlock ? kTiledPanelBlock : 1; }
inline int ffn_tiled_wgs(int npanels, int n_tiles) {
    const int per_round = 8 * tiled_panel_block(npanels);
    return ((npanels + per_round - 1) / per_round) * per_round * ((n_tiles + 7) / 8);
}
inline int ffn_gate_up_tiled_wgs(int F, int n_tiles) { return ffn_tiled_wgs(F / 128, n_tiles); }
inline int ffn_down_tiled_wgs(int d, int n_tiles) { return ffn_tiled_wgs(d / 256, n_tiles); }

// workgroups a group needs in the two FFN launches
inline int ffn_gate_up_wgs(int F, int n_tiles, int tiles_per_pass, int ks) {
    int nrb = F / 32, rbw = 4 / ks;
    return ((nrb + rbw - 1) / rbw) * ((n_tiles + tiles_per_pass - 1) / tiles_per_pass);
}
// LDS-shared streaming kernels (groups of a few token tiles, csrc/ef_ffn_shared.hip): a workgroup is four
// 32-row blocks of F (first half) or eight 32-column blocks of d (second half) for one pass of token tiles.
inline int ffn_gate_up_shared_wgs(int F, int n_tiles, int tiles_per_pass) {
    return (F / 128) * ((n_tiles + tiles_per_pass - 1) / tiles_per_pass);
}
inline int ffn_down_shared_wgs(int d, int n_tiles, int tiles_per_pass, int ksg) {
    return ((d / 32 + 7) / 8) * ((n_tiles + tiles_per_pass - 1) / tiles_per_pass) * ksg;
}
hipError_t launch_ffn_gate_up_shared(const GroupTable &gt, int total_wgs, int tiles_per_pass, int occ, const void *xp,
                                     void *act, int d, hipStream_t s);
hipError_t launch_ffn_down_shared(const GroupTable &gt, int total_wgs, int tiles_per_pass, int occ, int ksg, const void *act,
                                  float *y, long long y_plane, int d, hipStream_t s);
inline int ffn_down_wgs(int d, int n_tiles, int tiles_per_pass, int ksg) {
    return (d / 32 / kDownColBlocks) * ((n_tiles + tiles_per_pass - 1) / tiles_per_pass) * ksg;
}

}  // namespace ef
