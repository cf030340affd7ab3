// Launch planner: the gate / grouping launches of routing and prediction, and the grouped FFN of one layer in
// phases (experts that are ready, experts whose copy is in flight, misses that wait for a slot), each phase
// split over the streaming and the tiled kernels.  Declarations and argument contracts of the entry points are
// in include/expertflow.h.
#include "ef_ctx.h"

#include <algorithm>
#include <cmath>

namespace efi {

const ef::GroupExport kNoExport{nullptr, nullptr, 0, 0, 0};

// One pass over `hidden`: optionally the current layer's own gate (routing outputs and grouping)
// and the gates of the next He layers (prediction outputs).  Wide launches are split over the gates.
int run_gates(ef_ctx *c, int layer, const void *hidden, int T, float beta, bool do_route, int He, int H_stride,
              const float *delta, const int32_t *tok2req, int32_t *topk_ids, float *topk_w, int32_t *counts,
              int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *pred_ids, int32_t *pred_hist,
              const ef::GroupExport &ex, const EfRouteScratch &rs, hipStream_t s) {
    const int E = c->cfg.n_experts, k = c->cfg.top_k, d = c->cfg.d_model;
    const int ntiles = (T + ef::kTile - 1) / ef::kTile;
    // the library's own histogram buffer is left zeroed by the hand-over step of the previous layer
    if (He > 0 && !ex.host_meta) EF_HIP(c, ef::launch_fill_i32(pred_hist, He * E, 0, s));
    const int per_launch = ef::kMaxGates;
    const int total_gates = (do_route ? 1 : 0) + He;
    bool grouped = false;
    for (int g0 = 0; g0 < total_gates; g0 += per_launch) {
        ef::GateArgs a{};
        a.h = static_cast<const uint16_t *>(hidden);
        a.T = T; a.d = d; a.E = E; a.k = k;
        a.G = std::min(per_launch, total_gates - g0);
        a.beta = beta;
        a.tok2req = tok2req;
        a.delta = nullptr;
        a.delta_req_stride = H_stride * E;
        a.delta_gate_begin = 0;
        bool first_pred = true;
        for (int gi = 0; gi < a.G; ++gi) {
            const int gg = g0 + gi;                       // index over [route?] + predictions
            const bool is_route = do_route && gg == 0;
            const int j = gg - (do_route ? 1 : 0);        // prediction index (0-based) when !is_route
            const int ly = is_route ? layer : layer + 1 + j;
            const EfLayerReg &L = c->layers[(size_t)ly];
            a.Wg[gi] = L.gate_w;
            a.bias[gi] = L.gate_b;
            a.resident[gi] = resident_mask(c, ly);
            if (is_route) {
                a.ids[gi] = topk_ids;
                a.hist[gi] = nullptr;
                a.w = topk_w;
                a.blockcounts = rs.blockcounts;
                a.renorm = c->cfg.renorm_topk;
                a.routed_scale = c->cfg.routed_scale;
            } else {
                a.ids[gi] = pred_ids + (size_t)j * T * k;
                a.hist[gi] = pred_hist + (size_t)j * E;
                if (first_pred) {
                    a.delta_gate_begin = gi;
                    a.delta = delta ? delta + (size_t)j * E : nullptr;
                    first_pred = false;
                }
            }
        }
        a.gpw = ef::gate_pick_gpw(T, a.G, E);
        a.ksplit = ef::gate_pick_ksplit(T, d, a.G, E, a.gpw, rs.gate_part_floats);
        {
            const int forced = c->tune.gate_k_split;
            if (forced >= 1 && forced <= 16 &&
                (size_t)ntiles * ((a.G + a.gpw - 1) / a.gpw) * forced * ef::kTile * 128 <= rs.gate_part_floats)
                a.ksplit = forced;
        }
        a.part = rs.gate_part;
        a.tsplit = 1;
        // batches of many token tiles stream the hidden states through LDS in one kernel (no second step)
        a.stream = (c->tune.gate_stream != 0 && a.ksplit == 1 && ef::gate_stream_shape_ok(T, d, a.G, E, a.gpw)) ? 1 : 0;
        if (!a.stream) {   // the two-kernel form also pays off without a K split when the per-token part dominates
            const int ts = ef::gate_pick_tsplit(T, a.G, E, a.gpw);
            const size_t need = (size_t)ntiles * ((a.G + a.gpw - 1) / a.gpw) * a.ksplit * ef::kTile * 128;
            if (ts > 1 && need <= rs.gate_part_floats && c->tune.gate_token_split != 0) a.tsplit = ts;
        }
        a.two_step = (a.ksplit > 1 || a.tsplit > 1) ? 1 : 0;
        const bool has_route = do_route && g0 == 0;
        // decode-sized batches with a K-split gate and few experts: its second step and the grouping run as
        // one workgroup (with more than 16 experts a token takes a whole wave round of the epilogue, and the
        // many workgroups of the separate second step are faster: 27 against 36 us at 64 experts)
        const bool fused = has_route && total_gates <= per_launch && ntiles <= ef::kFusedMaxTiles && a.ksplit > 1 &&
                           E <= 16 &&
                           ef::gate_fused_lds_bytes(T, a.G, E, a.gpw) <= ef::kFusedMaxLds &&
                           c->tune.gate_fused_finish != 0;
        if (fused) a.tsplit = 1;
        {
            KernelTimer kt(c, s, has_route ? EF_K_ROUTE : EF_K_PREDICT,
                           (double)T * d * 2 + (double)a.G * E * d * 2 + (double)a.G * T * k * 4 +
                               (has_route ? (double)T * k * 4 + (double)ntiles * E * 4 : 0.0) +
                               (double)(a.G - (has_route ? 1 : 0)) * E * 4 +
                               (fused ? (double)(2 * E + 1) * 4 + (double)T * k * 12 : 0.0));
            if (fused) EF_HIP(c, ef::launch_gate_fused(a, counts, offsets, perm, inv_perm, ex, s));
            else EF_HIP(c, ef::launch_gate(a, s));
        }
        if (fused) grouped = true;
    }
    if (do_route && !grouped) {
        KernelTimer kt(c, s, EF_K_GROUP, (double)ntiles * E * 8 + (double)(2 * E + 1) * 4 + (double)T * k * 12);
        EF_HIP(c, ef::launch_group(rs.blockcounts, topk_ids, T, k, E, rs.blockbase, counts, offsets, perm,
                                   inv_perm, ex, s));
    }
    return EF_OK;
}

int check_predict_args(ef_ctx *c, int layer, int T, int H, int *He_out, const char *who) {
    if (c->fake) return fail(c, EF_ENOSYS, "%s: fake-copy context has no device", who);
    if (H < 0 || H > EF_MAX_HORIZON) return fail(c, EF_EINVAL, "%s: H must be in 0..%d", who, EF_MAX_HORIZON);
    if (T < 0 || T > c->cfg.max_tokens) return fail(c, EF_EINVAL, "%s: T=%d outside 0..max_tokens", who, T);
    int He = std::max(0, std::min(H, c->cfg.n_layers - 1 - layer));
    for (int j = 1; j <= He; ++j)
        if (!c->layers[(size_t)(layer + j)].set)
            return fail(c, EF_EINVAL, "%s: layer %d is not registered", who, layer + j);
    *He_out = He;
    return EF_OK;
}

int open_layer_timer(ef_ctx *c, hipStream_t s) {
    poll_pairs(c, false);
    if ((c->layer_calls++ % kLayerTimerEvery) != 0) return EF_OK;
    c->layer_cur = next_pair(c->layer_ring, c->layer_next, c->layer_pending);
    EF_HIP(c, hipEventRecord(c->layer_cur.a, s));
    c->layer_open = true;
    return EF_OK;
}

}  // namespace efi

using namespace efi;

namespace {

struct PhaseGroup {
    int expert;  // -1: dense shared FFN
    int slot;
};
constexpr int kNoSplit = -2;

// The tiled second half of a layer is `before` workgroups of one time unit each, dealt in order to the 256 compute
// units, then `units` more of the layer's last tiled group.  With that group cut into s K slices its workgroups
// take 1/s of a unit each: the time, in units, until the last one ends.
double tiled_tail_makespan(long long before, long long units, int s) {
    const long long q = before / 256, r = before % 256;   // r compute units are busy until q + 1, the others until q
    for (long long step = 1;; ++step) {
        const long long cap = (256 - r) * step + r * std::max<long long>(0, step - s);
        if (cap >= units * s) return (double)q + (double)step / s;
    }
}

// Build the launch tables of one phase and enqueue both FFN halves.
int launch_phase(ef_ctx *c, int layer, const std::vector<PhaseGroup> &groups, const int32_t *counts_host,
                 const std::vector<int> &offs_host, const std::vector<int> &tile_start,
                 const std::vector<long long> &act_off, int shared_tile_start, long long shared_act_off, int T,
                 int ksg_stream, int ksg_tiled, int split_expert, int split_ksg, ef::PlaneTable &planes, long long y_plane,
                 bool use_tiled, hipStream_t s) {
    // split_expert: the tiled group of the layer (expert id, -1 = shared FFN, kNoSplit = none) whose second half takes
    // split_ksg K slices instead of ksg_tiled; it goes last among the tiled groups of its launch
    if (groups.empty()) return EF_OK;
    const int d = c->cfg.d_model, k = c->cfg.top_k;
    // groups with many tokens go to the tiled (matrix-core bound) kernels, the others to the
    // weight-streaming kernels; at most two launches per FFN half
    ef::GroupTable gu{}, big{};
    ef::DequantTable dq{};
    int n = 0, nb = 0, max_tiles = 1;
    const bool allow_tiled = use_tiled;
    // Workgroups start in index order; groups with the most work go first so that the launch's last round holds
    // the short ones (the groups are independent: the order changes no result)
    std::vector<PhaseGroup> ordered(groups);
    if (c->tune.sort_groups != 0) {
        auto work = [&](const PhaseGroup &pg) {
            const long long cnt = pg.expert < 0 ? T : counts_host[pg.expert];
            const long long F = pg.expert < 0 ? c->cfg.d_ff_shared : c->cfg.d_ff;
            return ((cnt + ef::kTile - 1) / ef::kTile) * F;
        };
        std::stable_sort(ordered.begin(), ordered.end(),
                         [&](const PhaseGroup &a, const PhaseGroup &b) { return work(a) > work(b); });
    }
    if (split_expert != kNoSplit) {
        auto it = std::find_if(ordered.begin(), ordered.end(), [&](const PhaseGroup &pg) { return pg.expert == split_expert; });
        if (it != ordered.end()) std::rotate(it, it + 1, ordered.end());
    }
    int split_grp = -1;
    for (const PhaseGroup &pg : ordered) {
        int cnt, ts, F, ro;
        long long ao;
        const void *blob;
        if (pg.expert < 0) {
            cnt = T; ts = shared_tile_start; F = c->cfg.d_ff_shared; ro = T * k; ao = shared_act_off;
            blob = c->layers[(size_t)layer].shared_blob;
        } else {
            cnt = counts_host[pg.expert]; ts = tile_start[(size_t)pg.expert]; F = c->cfg.d_ff;
            ro = offs_host[(size_t)pg.expert]; ao = act_off[(size_t)pg.expert];
            blob = c->pool + (size_t)pg.slot * c->expert_bytes;
        }
        const int nt = (cnt + ef::kTile - 1) / ef::kTile;
        const bool tiled = allow_tiled && ef::ffn_tiled_ok(d, F, nt) && (pg.expert < 0 || nt >= c->tune.tiled_min_tiles) &&
                           (!c->q4 || nb < c->q4_stage_slots);
        ef::GroupTable &g = tiled ? big : gu;
        int &i = tiled ? nb : n;
        if (tiled && c->q4) {   // the tiled kernels read a 16-bit copy written just before them on the same stream
            void *copy = c->q4_stage + (size_t)nb * c->q4_stage_bytes;
            dq.F[nb] = F; dq.src[nb] = blob; dq.dst[nb] = copy;
            blob = copy;
        }
        const bool split = tiled && split_expert != kNoSplit && pg.expert == split_expert;
        if (split) split_grp = nb;
        (pg.expert < 0 ? planes.shared : planes.routed[pg.expert]) =
            (uint8_t)(split ? split_ksg : tiled ? ksg_tiled : ksg_stream);
        g.tile_start[i] = ts; g.n_tiles[i] = nt; g.row_offset[i] = ro;
        g.count[i] = cnt; g.F[i] = F; g.act_off[i] = ao; g.blob[i] = blob;
        if (!tiled) max_tiles = std::max(max_tiles, nt);
        ++i;
    }
    gu.n_groups = n;
    big.n_groups = nb;
    // weights: 2 bytes each, or half a byte plus one bf16 scale per 128
    const double wb = c->q4 ? 0.5 + 2.0 / 128.0 : 2.0;
    auto alg_bytes = [&](const ef::GroupTable &g, int cnt_groups, double &b_up, double &b_dn) {
        for (int i = 0; i < cnt_groups; ++i) {
            b_up += 2.0 * wb * d * g.F[i] + 2.0 * g.count[i] * d + 2.0 * g.count[i] * g.F[i];
            b_dn += wb * d * g.F[i] + 2.0 * g.count[i] * g.F[i] + 4.0 * g.count[i] * d;
        }
    };
    // Set once this phase's tiled launches have been forked to the side stream.  Whatever path leaves this
    // function afterwards (an error included), the caller's stream is made to wait for the side stream: the
    // caller releases the phase's cache slots behind its own stream, and kernels still running on the side
    // stream read those slots.
    struct SideJoin {
        ef_ctx *c;
        hipStream_t s;
        bool forked = false;
        hipEvent_t join = nullptr;
        hipEvent_t next_event() {
            hipEvent_t ev = c->fork_ring[c->fork_next];
            c->fork_next = (c->fork_next + 1) % c->fork_ring.size();
            return ev;
        }
        hipError_t record() {   // behind the last launch on the side stream
            join = next_event();
            return hipEventRecord(join, c->side_stream);
        }
        hipError_t wait() {
            if (!forked) return hipSuccess;
            hipError_t e = join ? hipSuccess : record();
            if (e == hipSuccess) e = hipStreamWaitEvent(s, join, 0);
            forked = false;
            return e;
        }
        ~SideJoin() { (void)wait(); }
    } side{c, s};
    int tiled_up_wgs = 0;
    if (nb > 0) {
        ef::GroupTable bdn = big;
        int wg_up = 0, wg_dn = 0;
        // Workgroups go to the XCDs round-robin by index and hold one of an XCD's 32 compute units for their whole
        // K loop.  A group's panel blocks (block b -> XCD rot + b) are dealt from the start XCD that leaves the
        // fullest XCD of the first half's launch least full, so groups of a few panels do not pile up on XCD 0.
        int load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        const int rot_on = c->tune.tiled_xcd_rotation;
        for (int i = 0; i < nb; ++i) {
            big.wg_start[i] = wg_up;
            bdn.wg_start[i] = wg_dn;
            const int pu = big.F[i] / 128, pbu = ef::tiled_panel_block(pu), nblk = (pu + pbu - 1) / pbu;
            const int mp = (big.n_tiles[i] + 7) / 8;
            int best = 0, best_max = 1 << 30;
            for (int rot = 0; rot < (rot_on ? 8 : 1); ++rot) {
                int trial[8], mx = 0;
                for (int x = 0; x < 8; ++x) trial[x] = load[x];
                for (int b = 0; b < nblk; ++b) trial[(rot + b) & 7] += std::min(pbu, pu - b * pbu) * mp;
                for (int x = 0; x < 8; ++x) mx = std::max(mx, trial[x]);
                if (mx < best_max) { best_max = mx; best = rot; }
            }
            for (int b = 0; b < nblk; ++b) load[(best + b) & 7] += std::min(pbu, pu - b * pbu) * mp;
            big.xcd_rot[i] = best;
            bdn.xcd_rot[i] = 0;   // the second half's panels cover every XCD (or K slices interleave them)
            wg_up += ef::ffn_gate_up_tiled_wgs(big.F[i], big.n_tiles[i]);
            wg_dn += ef::ffn_down_tiled_wgs(d, big.n_tiles[i]) * (i == split_grp ? split_ksg : ksg_tiled);
        }
        big.wg_start[nb] = wg_up;
        bdn.wg_start[nb] = wg_dn;
        tiled_up_wgs = wg_up;
        double b_up = 0.0, b_dn = 0.0, f_up = 0.0, f_dn = 0.0;
        alg_bytes(big, nb, b_up, b_dn);
        for (int i = 0; i < nb; ++i) {
            f_up += 4.0 * big.count[i] * d * big.F[i];   // two d x F products, 2 flops per multiply-add
            f_dn += 2.0 * big.count[i] * d * big.F[i];
        }
        // A phase with both kinds of groups runs its tiled launches on the side stream, beside the streamed ones:
        // the two touch different groups (tiles of the packed tokens, activations, rows of Y), small tiled launches
        // leave half of the compute units idle, and the streamed kernels are bound by HBM, not by compute units.
        // Fork: the side stream waits for everything enqueued so far (the token packing, the previous layer's
        // un-permute).  Join: the caller's stream waits for the side stream before anything after this phase.
        hipStream_t ts = s;
        if (n > 0 && c->side_stream && c->tune.overlap_tiled != 0) {
            hipEvent_t fork = side.next_event();
            EF_HIP(c, hipEventRecord(fork, s));
            EF_HIP(c, hipStreamWaitEvent(c->side_stream, fork, 0));
            ts = c->side_stream;
            side.forked = true;
        }
        {
            KernelTimer kt(c, ts, EF_K_FFN_UP_TILED, b_up, f_up);   // 4-bit: the expansion is timed with the first half
            if (c->q4) {
                dq.n = nb;
                EF_HIP(c, ef::launch_dequant_q4(dq, d, ts));
            }
            EF_HIP(c, ef::launch_ffn_gate_up_tiled(big, wg_up, c->xp, c->act, d, c->q4, ts));
        }
        {
            KernelTimer kt(c, ts, EF_K_FFN_DOWN_TILED, b_dn, f_dn);
            EF_HIP(c, ef::launch_ffn_down_tiled(bdn, wg_dn, ksg_tiled, split_grp, split_ksg, c->act, c->y, y_plane, d, ts));
        }
        if (side.forked) EF_HIP(c, side.record());
    }
    if (n == 0) return EF_OK;
    ef::GroupTable dn = gu;
    // token tiles per pass over a group's weights: groups of three or more tiles (too few for the tiled
    // kernels) take passes of four, which halves the re-reads of their weights (bf16 kernels only)
    const int tpp = (max_tiles >= 3 && !c->q4 && c->tune.passes_of_four != 0) ? 4 : max_tiles >= 2 ? 2 : 1;
    // K slices inside a workgroup of the first half: split while the launch has too few waves to
    // keep enough weight bytes in flight, as long as a slice keeps >= 16 fragments
    long long units = 0;
    for (int i = 0; i < n; ++i) units += (long long)(gu.F[i] / 32) * ((gu.n_tiles[i] + tpp - 1) / tpp);
    int ks = 1;
    const int want_waves = c->tune.up_want_waves, nkb = d / 16;
    while (ks < 4 && units * ks < want_waves && nkb / (ks * 2) >= 16) ks *= 2;
    if (c->tune.up_k_slices > 0) ks = c->tune.up_k_slices;
    // passes of four tiles: the kernels whose four waves share the token / activation fragments through LDS
    // (per-wave copies of them would be twice the weights' bytes from L2)
    bool shared = tpp == 4 && !c->q4 && c->tune.lds_shared != 0;
    for (int i = 0; i < n && shared; ++i) shared = gu.F[i] % 128 == 0;
    int wg_gu = 0, wg_dn = 0;
    for (int i = 0; i < n; ++i) {
        gu.wg_start[i] = wg_gu;
        dn.wg_start[i] = wg_dn;
        if (shared) {
            wg_gu += ef::ffn_gate_up_shared_wgs(gu.F[i], gu.n_tiles[i], tpp);
            wg_dn += ef::ffn_down_shared_wgs(d, gu.n_tiles[i], tpp, ksg_stream);
            continue;
        }
        wg_gu += c->q4 ? ef::ffn_gate_up_q4_wgs(gu.F[i], gu.n_tiles[i], tpp)
                       : ef::ffn_gate_up_wgs(gu.F[i], gu.n_tiles[i], tpp, ks);
        wg_dn += c->q4 ? ef::ffn_down_q4_wgs(d, gu.n_tiles[i], tpp, ksg_stream)
                       : ef::ffn_down_wgs(d, gu.n_tiles[i], tpp, ksg_stream);
    }
    gu.wg_start[n] = wg_gu;
    dn.wg_start[n] = wg_dn;
    double b_up = 0.0, b_dn = 0.0;
    alg_bytes(gu, n, b_up, b_dn);
    // workgroups per CU of the LDS-shared kernels: one (register ring of three stages) unless the phase's tiled first
    // half runs for well over one round of workgroups over the compute units, in which case two smaller ones (ring of
    // two stages) share each unit as the tiled launch frees it: Qwen-shaped batch (240-290 tiled workgroups) 217 -> 202 us
    // per layer with one, DeepSeek-shaped mixed batch (350-580 tiled workgroups) 304 against 309 us with two
    const int occ = c->tune.lds_shared_occupancy != 0 ? c->tune.lds_shared_occupancy : (tiled_up_wgs > 320 ? 2 : 1);
    {
        KernelTimer kt(c, s, EF_K_FFN_UP, b_up);
        if (shared) EF_HIP(c, ef::launch_ffn_gate_up_shared(gu, wg_gu, tpp, occ, c->xp, c->act, d, s));
        else if (c->q4) EF_HIP(c, ef::launch_ffn_gate_up_q4(gu, wg_gu, tpp, c->xp, c->act, d, s));
        else EF_HIP(c, ef::launch_ffn_gate_up(gu, wg_gu, tpp, ks, c->xp, c->act, d, s));
    }
    {
        KernelTimer kt(c, s, EF_K_FFN_DOWN, b_dn);
        if (shared) EF_HIP(c, ef::launch_ffn_down_shared(dn, wg_dn, tpp, occ, ksg_stream, c->act, c->y, y_plane, d, s));
        else if (c->q4) EF_HIP(c, ef::launch_ffn_down_q4(dn, wg_dn, tpp, ksg_stream, c->act, c->y, y_plane, d, s));
        else EF_HIP(c, ef::launch_ffn_down(dn, wg_dn, tpp, ksg_stream, c->act, c->y, y_plane, d, s));
    }
    EF_HIP(c, side.wait());
    return EF_OK;
}

}  // namespace

extern "C" int ef_moe_ffn(ef_ctx *c, int layer, const void *hidden, int T, const int32_t *topk_ids,
                          const float *topk_w, const int32_t *counts_host, const int32_t *offsets,
                          const int32_t *perm, const int32_t *inv_perm, float *out, void *stream) {
    // set by ef_layer_step for the call it makes right afterwards; never survives this call
    const bool prepacked = c && c->prepacked;
    if (c) c->prepacked = false;
    int rc = check_ctx_layer(c, layer);
    if (rc) return rc;
    if (T < 0 || T > c->cfg.max_tokens) return fail(c, EF_EINVAL, "ef_moe_ffn: T=%d outside 0..max_tokens", T);
    if (!counts_host) return fail(c, EF_EINVAL, "ef_moe_ffn: counts_host is null");
    const int E = c->cfg.n_experts, k = c->cfg.top_k, d = c->cfg.d_model;
    long long tot = 0;
    for (int e = 0; e < E; ++e) {
        if (counts_host[e] < 0 || counts_host[e] > T)
            return fail(c, EF_EINVAL, "ef_moe_ffn: counts_host[%d]=%d outside 0..T", e, counts_host[e]);
        tot += counts_host[e];
    }
    if (tot != (long long)T * k) return fail(c, EF_EINVAL, "ef_moe_ffn: counts_host sums to %lld, not T*k", tot);
    if (!c->fake && T > 0) {
        if (!hidden || !topk_ids || !topk_w || !offsets || !perm || !inv_perm || !out)
            return fail(c, EF_EINVAL, "ef_moe_ffn: null pointer");
        if (!aligned16(hidden) || !aligned16(out)) return fail(c, EF_EINVAL, "ef_moe_ffn: hidden/out must be 16-byte aligned");
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool strict = (c->cfg.flags & EF_FLAG_STRICT_RESIDENT) != 0;
    poll_all_copies(c);
    if (T > 0) {   // how much of what this layer uses had the look-ahead of j layers ago named?
        uint64_t used = 0;
        for (int e = 0; e < E; ++e)
            if (counts_host[e] > 0) used |= 1ull << e;
        for (int j = 0; j < EF_MAX_HORIZON; ++j) {
            const size_t at = (size_t)layer * EF_MAX_HORIZON + j;
            if (!c->pred_valid[at]) continue;
            c->pred_valid[at] = 0;
            c->st.pred_overlap_hits[j] += __builtin_popcountll(used & c->pred_mask[at]);
            c->st.pred_overlap_total[j] += __builtin_popcountll(used);
        }
    }

    // host copies of the group geometry
    std::vector<int> offs_host((size_t)E + 1, 0), tile_start((size_t)E, 0);
    std::vector<long long> act_off((size_t)E, 0);
    int tiles = 0;
    for (int e = 0; e < E; ++e) {
        offs_host[(size_t)e + 1] = offs_host[(size_t)e] + counts_host[e];
        tile_start[(size_t)e] = tiles;
        act_off[(size_t)e] = (long long)tiles * ef::kTile * c->cfg.d_ff / 8;   // 16-byte units
        tiles += (counts_host[e] + ef::kTile - 1) / ef::kTile;
    }
    const bool has_shared = c->cfg.d_ff_shared > 0 && T > 0;
    const int shared_tile_start = tiles;
    const long long shared_act_off = (long long)tiles * ef::kTile * c->cfg.d_ff / 8;
    if (has_shared) tiles += (T + ef::kTile - 1) / ef::kTile;
    if (!c->fake && tiles > c->max_tiles) return fail(c, EF_EINVAL, "ef_moe_ffn: scratch too small (internal)");

    // K slices of the second FFN half across workgroups (one Y plane each, summed by the un-permute):
    // split while the layer's launch would have too few workgroups, a slice keeps >= 32 fragments per
    // wave and the planes fit the scratch.  One value per call: every phase shares the planes.
    const long long y_plane = ((long long)T * k + (has_shared ? T : 0)) * d;
    // Groups of at least 8 token tiles go to the matrix-core tiled kernels.  The two thresholds (total
    // workgroups of the tiled launches) exist for tuning only: on the mixed batches measured (640 tokens
    // with a 2048 x 5632 shared expert, 1056 tokens over 64 experts) the tiled kernels were equal to or
    // 8 % faster than streaming the same groups in several passes, even at 150-200 workgroups.
    bool use_tiled = false;
    long long tiled_dn_wgs = 0, tiled_rows = 0;
    int tiled_stages_min = 1 << 30;   // fewest K stages (32 columns each) among the tiled groups
    int tiled_stages_max = 0;         // ... and most
    if (T > 0 && (!c->q4 || c->q4_stage_slots > 0) && c->tune.tiled != 0) {
        long long wg_up = 0, wg_dn = 0;
        auto add = [&](int F, int cnt, bool routed) {
            const int nt = (cnt + ef::kTile - 1) / ef::kTile;
            if (!ef::ffn_tiled_ok(d, F, nt) || (routed && nt < c->tune.tiled_min_tiles)) return;
            wg_up += ef::ffn_gate_up_tiled_wgs(F, nt);
            wg_dn += ef::ffn_down_tiled_wgs(d, nt);
            tiled_rows += cnt;
            tiled_stages_min = std::min(tiled_stages_min, F / 32);
            tiled_stages_max = std::max(tiled_stages_max, F / 32);
        };
        for (int e = 0; e < E; ++e) add(c->cfg.d_ff, counts_host[e], true);
        if (has_shared) add(c->cfg.d_ff_shared, T, false);
        use_tiled = wg_up >= c->tune.tiled_min_up_wgs && wg_dn >= c->tune.tiled_min_down_wgs;
        tiled_dn_wgs = wg_dn;
    }
    // K slices of the second half (one Y plane each, summed by the un-permute): the streamed launch and the tiled
    // launch of the layer choose separately, each for its own workgroup count
    int ksg = 1, ksg_tiled = 1, split_expert = kNoSplit, split_ksg = 1;
    if (T > 0) {
        long long base_wgs = 0;
        // token tiles per pass of the streamed launch: from the groups that stream (the tiled ones have kernels of
        // their own), with the same rule launch_phase applies to a phase's streamed groups
        int tmax = 1;
        auto streams = [&](int F, int cnt, bool routed) {
            const int nt = (cnt + ef::kTile - 1) / ef::kTile;
            return !(use_tiled && ef::ffn_tiled_ok(d, F, nt) && (!routed || nt >= c->tune.tiled_min_tiles));
        };
        for (int e = 0; e < E; ++e)
            if (counts_host[e] > 0 && streams(c->cfg.d_ff, counts_host[e], true))
                tmax = std::max(tmax, (counts_host[e] + ef::kTile - 1) / ef::kTile);
        if (has_shared && streams(c->cfg.d_ff_shared, T, false)) tmax = std::max(tmax, (T + ef::kTile - 1) / ef::kTile);
        const int tpp = (tmax >= 3 && !c->q4 && c->tune.passes_of_four != 0) ? 4 : tmax >= 2 ? 2 : 1;
        // workgroups of the streamed launch with one slice (groups that take the tiled kernels do not count)
        for (int e = 0; e < E; ++e)
            if (counts_host[e] > 0) {
                const int nt = (counts_host[e] + ef::kTile - 1) / ef::kTile;
                if (use_tiled && ef::ffn_tiled_ok(d, c->cfg.d_ff, nt) && nt >= c->tune.tiled_min_tiles) continue;
                base_wgs += c->q4 ? ef::ffn_down_q4_wgs(d, nt, tpp, 1)
                            : tpp == 4 ? ef::ffn_down_shared_wgs(d, nt, tpp, 1) : ef::ffn_down_wgs(d, nt, tpp, 1);
            }
        if (has_shared && !(use_tiled && ef::ffn_tiled_ok(d, c->cfg.d_ff_shared, (T + ef::kTile - 1) / ef::kTile)))
            base_wgs += c->q4 ? ef::ffn_down_q4_wgs(d, (T + ef::kTile - 1) / ef::kTile, tpp, 1)
                        : tpp == 4 ? ef::ffn_down_shared_wgs(d, (T + ef::kTile - 1) / ef::kTile, tpp, 1)
                                   : ef::ffn_down_wgs(d, (T + ef::kTile - 1) / ef::kTile, tpp, 1);
        // the LDS-shared kernels (passes of four tiles) run two workgroups per compute unit
        const int want = c->tune.down_want_wgs > 0 ? c->tune.down_want_wgs : (tpp == 4 && !c->q4) ? 512 : 256;
        const int nkb_min = std::min(c->cfg.d_ff, has_shared ? c->cfg.d_ff_shared : c->cfg.d_ff) / 16;
        // a slice keeps >= 32 fragments per wave (bf16: four waves split it again), >= 6 quads (4-bit), or >= 8
        // stages of four fragments (LDS-shared kernels: a wave walks the whole slice)
        const int units = c->q4 ? nkb_min / 4 / 6 : tpp == 4 ? nkb_min / 4 / 8 : nkb_min / 4 / 32;
        while (ksg < 8 && base_wgs * ksg < want && units / (ksg * 2) >= 1 && y_plane * (ksg * 2) <= c->y_floats)
            ksg *= 2;
        // A streamed launch of a little more than one round of workgroups (two fit a compute unit: 512 at a time)
        // ends in a round that is mostly empty: 544 workgroups took 28 us where 512 took 22.5.  Twice the slices make
        // the rounds half as long; taken when that saves at least a tenth of a round and a wave keeps >= 8 fragments.
        if (!c->q4 && tpp <= 2 && c->tune.down_tail_split != 0 && c->tune.down_k_slices == 0) {
            const long long slots = 512, w = base_wgs * ksg;
            if (w > slots && ksg < 8 && nkb_min / (ksg * 2 * 4) >= 8 && y_plane * (ksg * 2) <= c->y_floats) {
                const double now = (double)((w + slots - 1) / slots);
                const double halved = (double)((2 * w + slots - 1) / slots) / 2.0;
                if (halved + 0.1 < now) ksg *= 2;
            }
        }
        if (use_tiled) {
            // the tiled second half: slices until its 256 x 256 tiles fill the chip, each slice keeping at least
            // 16 stages
            // (any count from 1 to 8: 40 tiles in 6 slices are 240 workgroups, one round over the 256 compute units
            // at a sixth of the length, where 8 slices are 320 workgroups, two rounds at an eighth; a plane more is
            // priced at what it takes to write and read)
            if (tiled_dn_wgs < 256) {
                const int stages_ref = c->tune.down_slices_by_longest_k ? tiled_stages_max : tiled_stages_min;
                const double plane_pen = (double)tiled_rows * d * 8.0 / 5e12 / (stages_ref * 0.77e-6);
                double best = 0.0;
                for (int ks = 1; ks <= 8; ++ks) {
                    if (ks > 1 && (stages_ref / ks < 16 || y_plane * ks > c->y_floats)) break;
                    const double t = (double)((tiled_dn_wgs * ks + 255) / 256) / ks + (ks - 1) * plane_pen;
                    if (ks == 1 || t < best - 1e-9) { best = t; ksg_tiled = ks; }
                }
            }
            if (c->tune.down_split_slice_counts == 0) ksg = ksg_tiled;   // one slice count for both launches
        }
        int forced = c->tune.down_k_slices;
        if (forced >= 1 && forced <= 8 && y_plane * forced <= c->y_floats) ksg = ksg_tiled = forced;
        // A tiled second half of more than one round of workgroups over the compute units ends in a round that is
        // partly empty (1056 workgroups: four rounds and an eighth; every compute unit holds one at a time).  The
        // layer's last tiled group (the one with the least work; the highest expert among equals) is cut into K
        // slices so that its shorter workgroups fill that round: the slice count with the least modelled time,
        // a Y plane more costing what the second half and the un-permute take to write and read it.  The choice
        // depends on the layer's token counts only, never on what is resident.
        if (use_tiled && ksg_tiled == 1 && forced < 1 && tiled_dn_wgs > 256 && c->tune.tiled_tail_slices != 0) {
            long long best_work = -1, units = 0, rows = 0;
            int F_last = 0;
            auto consider = [&](int expert, int F, int cnt, bool routed) {
                const int nt = (cnt + ef::kTile - 1) / ef::kTile;
                if (!ef::ffn_tiled_ok(d, F, nt) || (routed && nt < c->tune.tiled_min_tiles)) return;
                const long long work = (long long)nt * F;
                if (best_work < 0 || work <= best_work) {
                    best_work = work; split_expert = expert; units = ef::ffn_down_tiled_wgs(d, nt); rows = cnt; F_last = F;
                }
            };
            if (has_shared) consider(-1, c->cfg.d_ff_shared, T, false);
            for (int e = 0; e < E; ++e) consider(e, c->cfg.d_ff, counts_host[e], true);
            if (split_expert != kNoSplit) {
                const double unit_s = (F_last / 32) * 0.77e-6;                        // one workgroup: its K stages
                const double plane_units = (double)rows * d * 8.0 / 5e12 / unit_s;     // write + read of one more plane
                double best = 0.0;
                for (int sl = 1; sl <= 8; sl *= 2) {
                    if (F_last / 32 / sl < 16 || y_plane * sl > c->y_floats) break;
                    const double t = tiled_tail_makespan(tiled_dn_wgs - units, units, sl) + (sl - 1) * plane_units;
                    if (sl == 1 || t < best - 1e-9) { best = t; split_ksg = sl; }
                }
                const int want = c->tune.tiled_tail_slices;   // 1: the modelled best; 2, 4, 8: that count if it fits
                if (want > 1 && F_last / 32 / want >= 16 && y_plane * want <= c->y_floats) split_ksg = want;
                if (split_ksg == 1) split_expert = kNoSplit;
            }
        }
    }
    ef::PlaneTable planes{};

    // classify the needed experts
    std::vector<PhaseGroup> ready, loading;
    std::vector<int> missing;
    bool any_not_ready = false;
    for (int e = 0; e < E; ++e) {
        if (counts_host[e] == 0) continue;
        int slot = c->cache->lookup(layer, e);
        if (slot < 0) {
            if (strict) {
                for (const auto &g : ready) c->cache->pin(g.slot, false);
                for (const auto &g : loading) c->cache->pin(g.slot, false);
                return fail(c, EF_ENOTRESIDENT, "ef_moe_ffn: layer %d expert %d is not resident", layer, e);
            }
            missing.push_back(e);
            any_not_ready = true;
            c->st.misses += 1;
            continue;
        }
        c->st.hits += 1;
        if (c->slots[(size_t)slot].prefetched_unused) {
            c->slots[(size_t)slot].prefetched_unused = false;
            c->st.prefetch_used += 1;
        }
        c->cache->touch(slot);
        c->cache->pin(slot, true);
        if (c->slots[(size_t)slot].copy_pending) { loading.push_back({e, slot}); any_not_ready = true; }
        else ready.push_back({e, slot});
    }
    // feedback counters (paper Sec. 3.2.2): a layer that had to wait counts as a stall, a layer
    // whose experts were all loaded in time counts as an overfetch
    if (T > 0) {
        if (any_not_ready) {
            if (++c->stall_counter >= std::max(1, c->cfg.stall_thresh)) { c->stall_counter = 0; c->fb_adjust += 1; }
        } else {
            if (++c->overfetch_counter >= std::max(1, c->cfg.overfetch_thresh)) { c->overfetch_counter = 0; c->fb_adjust -= 1; }
        }
        c->fb_adjust = std::max(-(c->cfg.h_max - 1), std::min(c->cfg.h_max - 1, c->fb_adjust));
    }

    auto unpin_all = [&](const std::vector<PhaseGroup> &v) {
        for (const auto &g : v)
            if (g.expert >= 0) c->cache->pin(g.slot, false);
    };
    // start what misses can start right now (slots not needed by this layer)
    std::vector<int> deferred;
    for (int e : missing) {
        int slot = -1;
        int r = swap_in_impl(c, layer, e, 1, 0, &slot, nullptr);
        if (r == EF_EBUSY) { deferred.push_back(e); continue; }
        if (r != EF_OK) { unpin_all(ready); unpin_all(loading); return r; }
        c->cache->touch(slot);
        c->cache->pin(slot, true);
        loading.push_back({e, slot});
    }

    // A slot may be overwritten once the kernels that read it have finished: an event recorded behind them
    // is what a later swap-in waits for.  One event behind the layer's last kernel serves every slot of the
    // layer; only when misses are still waiting for a slot (phase C) must each phase's slots be released as
    // soon as that phase's kernels are enqueued.
    const bool eager_marks = !deferred.empty();
    std::vector<int> read_slots;
    // An error return between the phases must not leave the collected slots pinned, and kernels already
    // enqueued may still read them: they are released behind an event on the stream, like on the normal path.
    struct PinGuard {
        ef_ctx *c;
        hipStream_t s;
        std::vector<int> *v;
        ~PinGuard() {
            if (v->empty()) return;
            hipEvent_t ev = nullptr;
            if (!c->fake) {
                ev = c->read_ring[c->read_next];
                c->read_next = (c->read_next + 1) % c->read_ring.size();
                if (hipEventRecord(ev, s) != hipSuccess) ev = nullptr;
            }
            for (int slot : *v) {
                if (ev) c->slots[(size_t)slot].last_read = ev;
                c->cache->pin(slot, false);
            }
        }
    } pin_guard{c, s, &read_slots};
    auto mark_read = [&](const std::vector<PhaseGroup> &v) -> int {
        if (c->fake) { unpin_all(v); return EF_OK; }
        if (!eager_marks) {
            for (const auto &g : v)
                if (g.expert >= 0) read_slots.push_back(g.slot);
            return EF_OK;   // still pinned: released behind the layer's last kernel
        }
        hipEvent_t ev = c->read_ring[c->read_next];
        c->read_next = (c->read_next + 1) % c->read_ring.size();
        EF_HIP(c, hipEventRecord(ev, s));
        for (const auto &g : v)
            if (g.expert >= 0) c->slots[(size_t)g.slot].last_read = ev;
        unpin_all(v);
        return EF_OK;
    };
    auto release_read_slots = [&]() -> int {
        if (read_slots.empty()) return EF_OK;
        hipEvent_t ev = c->read_ring[c->read_next];
        c->read_next = (c->read_next + 1) % c->read_ring.size();
        hipError_t he = hipEventRecord(ev, s);
        for (int slot : read_slots) {
            c->slots[(size_t)slot].last_read = ev;
            c->cache->pin(slot, false);
        }
        read_slots.clear();
        if (he != hipSuccess) return fail(c, EF_EHIP, "hipEventRecord failed: %s", hipGetErrorString(he));
        return EF_OK;
    };
    auto wait_loaded = [&](const std::vector<PhaseGroup> &v) -> int {
        if (v.empty()) return EF_OK;
        std::vector<int> slots;
        for (const auto &g : v) slots.push_back(g.slot);
        if (c->fake) {
            const double need = fake_copy_wait(c, slots.data(), (int)slots.size());
            c->st.stall_seconds += need - c->fake_now;
            c->fake_now = need;
            for (const auto &g : v) poll_copy(c, g.slot);
            return EF_OK;
        }
        EfEventPair p = next_pair(c->stall_ring, c->stall_next, c->stall_pending);
        EF_HIP(c, hipEventRecord(p.a, s));
        // copies still (partly) in the queue become priority copies; once every chunk of them is on the copy
        // stream their ready events exist and the compute stream can wait for them
        int fr = copy_engine_flush(c, slots.data(), (int)slots.size());
        if (fr) return fr;
        for (const auto &g : v) EF_HIP(c, hipStreamWaitEvent(s, c->slots[(size_t)g.slot].ready, 0));
        EF_HIP(c, hipEventRecord(p.b, s));
        c->stall_pending.push_back(p);
        return EF_OK;
    };
    auto run_phase = [&](std::vector<PhaseGroup> &v, bool with_shared) -> int {
        std::vector<PhaseGroup> g = v;
        if (with_shared && has_shared) g.push_back({-1, -1});
        if (!c->fake) {
            int r = launch_phase(c, layer, g, counts_host, offs_host, tile_start, act_off, shared_tile_start,
                                 shared_act_off, T, ksg, ksg_tiled, split_expert, split_ksg, planes, y_plane, use_tiled, s);
            if (r) {   // part of the phase may be enqueued: its slots still get their read marker
                (void)mark_read(v);
                v.clear();   // released: the caller's error path has nothing left to unpin
                return r;
            }
        }
        return mark_read(v);
    };

    if (T > 0) {
        if (!c->fake && !prepacked) {
            // token permutation into per-expert tiles (all groups of this layer in one launch)
            ef::PackTable pt{};
            int n = 0;
            for (int e = 0; e < E; ++e) {
                if (counts_host[e] == 0) continue;
                pt.tile_start[n] = tile_start[(size_t)e];
                pt.row_offset[n] = offs_host[(size_t)e];
                pt.count[n] = counts_host[e];
                ++n;
            }
            if (has_shared) {
                pt.tile_start[n] = shared_tile_start;
                pt.row_offset[n] = -1;
                pt.count[n] = T;
                ++n;
            }
            pt.tile_start[n] = tiles;
            pt.n_groups = n;
            int r = EF_OK;
            long long rows = (long long)T * k + (has_shared ? T : 0);
            KernelTimer kt(c, s, EF_K_PACK, 4.0 * rows * d + 4.0 * T * k);
            hipError_t he = ef::launch_pack_x(pt, tiles, static_cast<const uint16_t *>(hidden), d, k, perm, c->xp, c->q4, s);
            if (he != hipSuccess) r = fail(c, EF_EHIP, "pack_x launch failed: %s", hipGetErrorString(he));
            if (r) { unpin_all(ready); unpin_all(loading); return r; }
        }
        // phase A: experts that are ready (+ the dense shared FFN): tokens whose experts are resident go first
        rc = run_phase(ready, true);
        if (rc) { unpin_all(loading); return rc; }
        // phase B: experts whose copy is in flight (earlier prefetches and the misses started above)
        if (!loading.empty()) {
            rc = wait_loaded(loading);
            if (!rc) rc = run_phase(loading, false);
            if (rc) { unpin_all(loading); return rc; }
        }
        // phase C: misses that had no slot until an earlier phase released one
        size_t next = 0;
        while (next < deferred.size()) {
            std::vector<PhaseGroup> wave;
            while (next < deferred.size()) {
                int slot = -1;
                int r = swap_in_impl(c, layer, deferred[next], 1, 0, &slot, nullptr);
                if (r == EF_EBUSY) break;
                if (r != EF_OK) { unpin_all(wave); return r; }
                c->cache->touch(slot);
                c->cache->pin(slot, true);
                wave.push_back({deferred[next], slot});
                ++next;
            }
            if (wave.empty()) return fail(c, EF_EBUSY, "ef_moe_ffn: no cache slot can be freed for layer %d", layer);
            rc = wait_loaded(wave);
            if (!rc) rc = run_phase(wave, false);
            if (rc) { unpin_all(wave); return rc; }
        }
        if (!c->fake) {
            KernelTimer kt(c, s, EF_K_COMBINE, 4.0 * ((double)T * k + (has_shared ? T : 0)) * d + 4.0 * T * d +
                                                   8.0 * T * k);
            // the layer's last kernel carries the read marker of the slots collected above
            hipEvent_t done = nullptr;
            if (!read_slots.empty()) {
                done = c->read_ring[c->read_next];
                c->read_next = (c->read_next + 1) % c->read_ring.size();
            }
            EF_HIP(c, ef::launch_combine(c->y, planes, y_plane, topk_w, topk_ids, inv_perm, T, k, d,
                                         has_shared ? (long long)T * k : -1ll, out, done, s));
            if (done) {
                for (int slot : read_slots) {
                    c->slots[(size_t)slot].last_read = done;
                    c->cache->pin(slot, false);
                }
                read_slots.clear();
            }
        }
    }
    if ((rc = release_read_slots())) return rc;
    if (!c->fake && c->layer_open) {
        EF_HIP(c, hipEventRecord(c->layer_cur.b, s));
        c->layer_pending.push_back(c->layer_cur);
        c->layer_open = false;
    }
    c->st.layers_run += 1;
    c->st.tokens_run += T;
    c->cache->advance(layer);
    return EF_OK;
}

